"""Pins for the oracle's int4/int2 quantizer, packer and cache state machine.

None of these re-use the oracle's own formulas: they compare against hand-derived words
(tests/golden/format_words.txt), closed forms, exact rational arithmetic and invariants.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "format_words.txt")


def _gold(kind):
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, a, b = [s.strip() for s in line.split(";")]
        if k == kind:
            rows.append((a, b))
    return rows


@pytest.mark.parametrize("bits", [4, 2])
def test_pack_words_golden(bits):
    for a, b in _gold(f"int{bits}"):
        codes = np.array([int(t) for t in a.split()], np.uint8)
        assert O.pack_words(codes, bits).tolist() == [int(b, 16)]
        assert O.unpack_words(np.array([int(b, 16)], np.uint32), bits).tolist() == codes.tolist()


def test_half2_golden():
    for a, b in _gold("half2"):
        s, z = [float(t) for t in a.split()]
        assert int(O.pack_half2(np.float16(s), np.float16(z))) == int(b, 16)
        s2, z2 = O.unpack_half2(np.array([int(b, 16)], np.uint32))
        assert float(s2[0]) == s and float(z2[0]) == z


@pytest.mark.parametrize("bits", [4, 2])
def test_unpack_pack_identity(bits):
    rng = np.random.default_rng(7)
    codes = rng.integers(0, 1 << bits, size=(5, 128), dtype=np.uint8)
    assert np.array_equal(O.unpack_words(O.pack_words(codes, bits), bits), codes)


@pytest.mark.parametrize("bits", [4, 2])
def test_arithmetic_progression_is_exact(bits):
    """A group {mn + i*s}, s a power of two: scale == s, codes == i, exact round trip."""
    qmax = (1 << bits) - 1
    for s, mn in [(0.5, -2.0), (0.125, 3.0), (2.0, -14.0)]:
        col = np.array([mn + s * (t % (qmax + 1)) for t in range(128)], np.float16)
        blk = np.tile(col[:, None], (1, 128))
        codes, scale, zero = O.quantize_k_block(blk, bits)
        assert np.all(scale == np.float16(s)) and np.all(zero == np.float16(mn))
        assert np.array_equal(codes[:, 0], np.arange(128) % (qmax + 1))
        # the same numbers laid along channels exercise the V (per-token) statistics
        codes_v, scale_v, zero_v = O.quantize_v_block(np.ascontiguousarray(blk.T), bits)
        assert np.all(scale_v == np.float16(s)) and np.all(zero_v == np.float16(mn))
        assert np.array_equal(codes_v[0], np.arange(128) % (qmax + 1))


@pytest.mark.parametrize("bits", [4, 2])
def test_constant_group_and_negative_zero(bits):
    blk = np.full((128, 128), 3.25, np.float16)
    blk[:, 1] = np.float16(-0.0)
    codes, scale, zero = O.quantize_k_block(blk, bits)
    assert np.all(codes == 0) and np.all(scale == 0)
    assert zero[0] == np.float16(3.25)
    assert zero.view(np.uint16)[1] == 0          # -0 minimum stored as +0


@pytest.mark.parametrize("bits", [4, 2])
def test_k_is_per_channel_v_is_per_token(bits):
    """Statistics axis: scaling one channel of K (one token of V) must change only that
    channel's (token's) parameters."""
    rng = np.random.default_rng(3)
    blk = rng.standard_normal((128, 128)).astype(np.float16)
    _, s0, z0 = O.quantize_k_block(blk, bits)
    b2 = blk.copy(); b2[:, 5] *= np.float16(8)
    _, s1, z1 = O.quantize_k_block(b2, bits)
    changed = (s0 != s1) | (z0 != z1)
    assert changed[5] and changed.sum() == 1
    _, s0, z0 = O.quantize_v_block(blk, bits)
    b2 = blk.copy(); b2[9, :] *= np.float16(8)
    _, s1, z1 = O.quantize_v_block(b2, bits)
    changed = (s0 != s1) | (z0 != z1)
    assert changed[9] and changed.sum() == 1


@pytest.mark.parametrize("bits", [4, 2])
def test_roundtrip_bound_extremes_monotone(bits):
    qmax = (1 << bits) - 1
    w = W.scaled(W.CONFIGS["cfg1"], context=256)
    K, V = W.make_kv(w)
    for blk, fn, axis in [(K[0, 3, :128], O.quantize_k_block, 0), (V[0, 5, 128:], O.quantize_v_block, 1)]:
        codes, scale, zero = fn(blk, bits)
        s = scale.astype(np.float64); z = zero.astype(np.float64)
        if axis == 0:
            xhat = codes * s[None, :] + z[None, :]; sb = np.broadcast_to(s[None, :], blk.shape)
        else:
            xhat = codes * s[:, None] + z[:, None]; sb = np.broadcast_to(s[:, None], blk.shape)
        err = np.abs(blk.astype(np.float64) - xhat)
        assert np.all(err <= sb / 2 * (1 + 2.0 ** -10) + 1e-12)
        # min -> code 0, max -> code qmax
        amin = blk.argmin(axis=axis); amax = blk.argmax(axis=axis)
        idx = np.arange(128)
        if axis == 0:
            assert np.all(codes[amin, idx] == 0) and np.all(codes[amax, idx] == qmax)
        else:
            assert np.all(codes[idx, amin] == 0) and np.all(codes[idx, amax] == qmax)
        # monotone inside each group
        order = np.argsort(blk, axis=axis, kind="stable")
        sorted_codes = np.take_along_axis(codes, order, axis=axis)
        assert np.all(np.diff(sorted_codes.astype(int), axis=axis) >= 0)


@pytest.mark.parametrize("bits", [4, 2])
def test_codes_against_exact_rationals(bits):
    """Codes from exact rational arithmetic on the stored fp16 scale/zero: the oracle's fp32
    division may only differ when the exact quotient sits within 1e-6 of a tie."""
    qmax = (1 << bits) - 1
    rng = np.random.default_rng(11)
    blk = (rng.standard_normal((128, 128)) * 3).astype(np.float16)
    codes, scale, zero = O.quantize_k_block(blk, bits)
    for c in range(0, 128, 17):
        s = Fraction(float(scale[c])); z = Fraction(float(zero[c]))
        # scale itself: the fp16 nearest to (max-min)/qmax
        exact_s = (Fraction(float(blk[:, c].max())) - Fraction(float(blk[:, c].min()))) / qmax
        assert abs(Fraction(float(scale[c])) - exact_s) <= Fraction(float(np.spacing(scale[c]))) / 2
        assert z == Fraction(float(blk[:, c].min()))
        for t in range(128):
            r = (Fraction(float(blk[t, c])) - z) / s
            lo = r.numerator // r.denominator
            frac = r - lo
            if abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 6):
                ok = {lo, lo + 1}
            else:
                ok = {lo + (1 if frac > Fraction(1, 2) else 0)}
            ok = {min(max(v, 0), qmax) for v in ok}
            assert int(codes[t, c]) in ok


def test_exact_tie_rounds_to_even():
    """(x - zero)/scale exactly k + 1/2 must go to the even neighbour."""
    col = np.array([0.0, 15.0] + [2.5, 3.5, 0.5, 1.5] + [0.0] * 122, np.float16)   # scale == 1
    blk = np.tile(col[:, None], (1, 128))
    codes, scale, _ = O.quantize_k_block(blk, 4)
    assert scale[0] == 1
    assert codes[2:6, 0].tolist() == [2, 4, 0, 2]


def test_buffer_byte_counts():
    """Per token per KV head the packed cache holds 64+4+64+4 = 136 B at 4 bits and
    32+4+32+4 = 72 B at 2 bits (codes + half2 parameters), against 512 B in fp16."""
    for bits, per_tok in [(4, 136), (2, 72)]:
        c = O.IntCache(1, 1, bits, 256)
        total = c.k_codes.nbytes + c.v_codes.nbytes + c.k_params.nbytes + c.v_params.nbytes
        assert total == per_tok * 256


@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("L,k", [(100, 27), (100, 28), (100, 29), (250, 140), (128, 256), (0, 130)])
def test_append_equals_prefill(bits, L, k):
    """prefill(L) followed by k appends is the same cache, bit for bit, as prefill(L+k),
    for k crossing zero, one and two flushes (partition rule of Sec. IV-B(1))."""
    w = W.scaled(W.CONFIGS["cfg1"], n_q_heads=4, n_kv_heads=2, context=L + k)
    K, V = W.make_kv(w)
    a = O.IntCache(1, 2, bits, 512); a.quant_pack_kv(K[:, :, :L], V[:, :, :L])
    for i in range(k):
        a.append_kv(K[:, :, L + i], V[:, :, L + i])
    b = O.IntCache(1, 2, bits, 512); b.quant_pack_kv(K, V)
    assert (a.packed_len, a.res_len) == (b.packed_len, b.res_len) == ((L + k) // 128 * 128, (L + k) % 128)
    nb = a.packed_len // 128
    for name in ["k_codes", "v_codes", "k_params", "v_params"]:
        assert np.array_equal(getattr(a, name)[:, :, :nb], getattr(b, name)[:, :, :nb]), name
    assert np.array_equal(a.k_res[:, :, :a.res_len], b.k_res[:, :, :b.res_len])
    assert np.array_equal(a.v_res[:, :, :a.res_len], b.v_res[:, :, :b.res_len])


def test_append_capacity():
    w = W.scaled(W.CONFIGS["cfg0"], n_q_heads=1, n_kv_heads=1, context=255)
    K, V = W.make_kv(w)
    c = O.IntCache(1, 1, 4, 128); c.quant_pack_kv(K[:, :, :128], V[:, :, :128])
    for i in range(127):
        c.append_kv(K[:, :, 128 + i], V[:, :, 128 + i])
    with pytest.raises(OverflowError):
        c.append_kv(K[:, :, 0], V[:, :, 0])
    assert (c.packed_len, c.res_len) == (128, 127)


@pytest.mark.parametrize("bits", [4, 2])
def test_layout_orientation(bits):
    """K words run along channels of one token; V words along tokens of one channel."""
    rng = np.random.default_rng(5)
    K = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    V = rng.standard_normal((1, 1, 128, 128)).astype(np.float16)
    c = O.IntCache(1, 1, bits, 128); c.quant_pack_kv(K, V)
    kc, _, _ = O.quantize_k_block(K[0, 0], bits)
    vc, _, _ = O.quantize_v_block(V[0, 0], bits)
    cpw = 32 // bits
    t, ch = 37, 101
    word = int(c.k_codes[0, 0, 0, t, ch // cpw])
    assert (word >> (bits * (ch % cpw))) & ((1 << bits) - 1) == kc[t, ch]
    word = int(c.v_codes[0, 0, 0, ch, t // cpw])
    assert (word >> (bits * (t % cpw))) & ((1 << bits) - 1) == vc[t, ch]


def test_lazy_flush_attends_fp16_and_leaves_the_eager_cache():
    """The Residual Kernel's order (Sec. III-A(1), IV-B(1)): append without flushing keeps a full residual of 128
    tokens in fp16 for that step's attention -- with nothing packed yet the output is textbook softmax
    attention on the raw fp16 K, V (brute force below) -- and flush_if_full() then leaves exactly the cache the
    eager append leaves."""
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=4, n_kv_heads=2, context=127)
    K, V = W.make_kv(w)
    kn, vn = W.make_new_kv(w, 0)
    q = W.make_q(w)
    lazy, eager = O.IntCache(1, 2, 4, 256), O.IntCache(1, 2, 4, 256)
    lazy.quant_pack_kv(K, V); eager.quant_pack_kv(K, V)
    lazy.append_kv(kn, vn, flush=False)
    assert (lazy.packed_len, lazy.res_len) == (0, 128)
    out = O.decode_attn(lazy, q, W.softmax_scale(w))
    Kall = np.concatenate([K, kn[:, :, None, :]], axis=2).astype(np.float64)
    Vall = np.concatenate([V, vn[:, :, None, :]], axis=2).astype(np.float64)
    for hq in range(4):
        h = hq // 2
        s = np.array([W.softmax_scale(w) * sum(float(q[0, hq, c]) * Kall[0, h, t, c] for c in range(128)) for t in range(128)])
        p = np.exp(s - s.max()); p /= p.sum()
        brute = sum(p[t] * Vall[0, h, t] for t in range(128))
        assert np.allclose(out[0, hq], brute, rtol=1e-12, atol=1e-13)
    lazy.flush_if_full()
    eager.append_kv(kn, vn)
    assert (lazy.packed_len, lazy.res_len) == (eager.packed_len, eager.res_len) == (128, 0)
    for name in ("k_codes", "v_codes", "k_params", "v_params"):
        assert np.array_equal(getattr(lazy, name), getattr(eager, name)), name
    # and the eager step's attention sees the quantized block: not the same output
    assert not np.allclose(O.decode_attn(eager, q, W.softmax_scale(w)), out, atol=1e-6)

