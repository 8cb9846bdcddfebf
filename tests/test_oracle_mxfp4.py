"""Pins for the oracle's MXFP4 (e2m1 + e8m0 per 32 elements) quantizer and cache."""
import os

import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "format_words.txt")


def test_e2m1_table_golden_and_exhaustive():
    for line in open(GOLD):
        if line.startswith("e2m1"):
            _, code, val = [s.strip() for s in line.split(";")]
            assert float(O.e2m1_decode(np.array(int(code)))) == float(val)
    # structural definition: sign, 2-bit exponent (bias 1), 1-bit mantissa
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        val = (m * 0.5) if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)
        assert float(O.e2m1_decode(np.array(code))) == (-val if s else val)


def test_e2m1_encode_nearest_ties_saturation():
    grid = [0, .5, 1, 1.5, 2, 3, 4, 6]
    # every representable value encodes to itself (non-negative zero only)
    for code in range(16):
        v = float(O.e2m1_decode(np.array(code)))
        back = int(O.e2m1_encode(np.array(v)))
        assert back == (0 if code == 8 else code)
    # midpoints go to the even code; just off the midpoint goes to the nearer value
    for i in range(7):
        mid = (grid[i] + grid[i + 1]) / 2
        even = i if i % 2 == 0 else i + 1
        assert int(O.e2m1_encode(np.array(mid))) == even
        assert int(O.e2m1_encode(np.array(-mid))) == (even | 8 if even else 0)
        assert int(O.e2m1_encode(np.array(mid - 1e-9))) == i
        assert int(O.e2m1_encode(np.array(mid + 1e-9))) == i + 1
    for v in (6.5, 7.0, 7.99, 100.0):
        assert int(O.e2m1_encode(np.array(v))) == 7 and int(O.e2m1_encode(np.array(-v))) == 15
    assert int(O.e2m1_encode(np.array(-0.0))) == 0 and int(O.e2m1_encode(np.array(-0.2))) == 0


def test_mx_scale_rule():
    rng = np.random.default_rng(0)
    x = W.round_to_bf16(rng.standard_normal((64, 128)).astype(np.float32) * np.float32(3))
    codes, sc = O.mx_quantize(x)
    e = sc.astype(int) - 127
    amax = np.abs(x.reshape(64, 4, 32)).max(-1)
    assert np.all(amax >= 4 * 2.0 ** e) and np.all(amax < 8 * 2.0 ** e)     # amax lands in e2m1's top binade
    xh = O.mx_dequantize(codes, sc)
    # error bound: half a grid step at the top binade (step 2 * 2^e); beyond 6 * 2^e the
    # value saturates, so the error there is below 2 * 2^e
    err = np.abs(xh - x).reshape(64, 4, 32)
    unit = 2.0 ** e[..., None]
    inside = np.abs(x).reshape(64, 4, 32) <= 6 * unit
    assert np.all(err[inside] <= np.broadcast_to(unit, err.shape)[inside])
    assert np.all(err[~inside] < 2 * np.broadcast_to(unit, err.shape)[~inside])
    assert np.all(np.abs(xh).reshape(64, 4, 32)[~inside] == 6 * np.broadcast_to(unit, err.shape)[~inside])
    # idempotent: re-quantizing representable values changes nothing
    c2, s2 = O.mx_quantize(xh)
    assert np.array_equal(O.mx_dequantize(c2, s2), xh)


def test_mx_powers_of_two_and_zero_block():
    x = np.zeros((1, 64), np.float32)
    x[0, :32] = [2.0 ** (k % 4 - 1) for k in range(32)]      # 0.5, 1, 2, 4 -> amax 4 -> e = 0
    codes, sc = O.mx_quantize(x)
    assert sc.tolist() == [[127, 127]]                          # second block all zero -> 127
    assert np.array_equal(O.mx_dequantize(codes, sc), x)
    assert np.all(codes[0, 32:] == 0)
    y = x * np.float32(2.0 ** -20)
    c2, s2 = O.mx_quantize(y)
    assert s2[0, 0] == 107 and np.array_equal(c2, codes) and np.array_equal(O.mx_dequantize(c2, s2), y)


def test_nibble_packing():
    codes = np.arange(16, dtype=np.uint8)
    b = O.pack_nibbles(codes)
    assert b.tolist() == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]
    assert np.array_equal(O.unpack_nibbles(b), codes)


def test_mx_cache_layout_and_append_equals_prefill():
    w = W.scaled(W.CONFIGS["cfg4"], batch=2, n_q_heads=4, n_kv_heads=2, context=300)
    K, V = W.make_kv(w)
    a = O.MxCache(2, 2, 384); a.quant_pack_kv(K[:, :, :250], V[:, :, :250])
    for t in range(250, 300):
        a.append_kv(K[:, :, t], V[:, :, t])
    b = O.MxCache(2, 2, 384); b.quant_pack_kv(K, V)
    for name in ["k_codes", "k_scales", "v_codes", "v_scales"]:
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    # orientation: K bytes along channels of a token, V bytes along tokens of a channel
    kc, ks = O.mx_quantize(K[1, 1, 201]); vc, vs = O.mx_quantize(V[1, 1, 201])
    assert (int(b.k_codes[1, 1, 201, 77 // 2]) >> 4) == kc[77]
    assert (int(b.v_codes[1, 1, 1, 77, (201 - 128) // 2]) >> 4) == vc[77]
    assert np.array_equal(b.v_scales[1, 1, 201], vs)
    # 64 + 4 + 64 + 4 = 136 bytes per token per KV head
    assert (b.k_codes.nbytes + b.k_scales.nbytes + b.v_codes.nbytes + b.v_scales.nbytes) == 136 * 384 * 4
    # attention over the MX cache = attention over independently dequantized values
    q = W.make_q(w)
    out = O.decode_attn(b, q, W.softmax_scale(w), units=[(1, 0)])
    Kd = O.mx_dequantize(*O.mx_quantize(K[1, 0])); Vd = O.mx_dequantize(*O.mx_quantize(V[1, 0]))
    s = W.softmax_scale(w) * (Kd @ q[1, 1].astype(np.float64)); p = np.exp(s - s.max()); p /= p.sum()
    assert np.allclose(out[1, 1], p @ Vd, rtol=1e-12, atol=1e-14)
    assert np.all(np.isnan(out[0]))
