"""Pins for the oracle's attention: brute-force loops, closed forms and invariants."""
import math

import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W


def brute_attention(q, K, V, scale):
    """softmax(scale * q.K^T).V for one query, written as scalar Python loops."""
    L, D = len(K), len(q)
    s = [scale * sum(float(q[c]) * float(K[t][c]) for c in range(D)) for t in range(L)]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    tot = sum(e)
    return [sum(e[t] / tot * float(V[t][c]) for t in range(L)) for c in range(D)]


def _small(L, hq, hkv, seed=0):
    w = W.scaled(W.CONFIGS["cfg0"], n_q_heads=hq, n_kv_heads=hkv, context=L, seed=seed)
    K, V = W.make_kv(w)
    return w, K, V, W.make_q(w)


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 1), (8, 2)])
def test_unquantized_matches_brute_force(hq, hkv):
    """L < 128: every token sits in the fp16 residual, so the oracle must equal plain
    attention; also pins the head grouping h_kv = h_q // g_q."""
    w, K, V, q = _small(37, hq, hkv)
    c = O.IntCache(1, hkv, 4, 128); c.quant_pack_kv(K, V)
    assert (c.packed_len, c.res_len) == (0, 37)
    out = O.decode_attn(c, q, 0.25)
    g = hq // hkv
    for h in range(hq):
        ref = brute_attention(q[0, h], K[0, h // g], V[0, h // g], 0.25)
        assert np.allclose(out[0, h], ref, rtol=1e-12, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    w, K, V, q = _small(200, 8, 2)
    a = O.IntCache(1, 2, 4, 256); a.quant_pack_kv(K, V)
    b = O.IntCache(1, 8, 4, 256); b.quant_pack_kv(np.repeat(K, 4, axis=1), np.repeat(V, 4, axis=1))
    assert np.array_equal(O.decode_attn(a, q, 0.1), O.decode_attn(b, q, 0.1))


def test_weights_sum_to_one_and_closed_forms():
    rng = np.random.default_rng(1)
    Kh = rng.standard_normal((300, 128)); q = rng.standard_normal(128)
    wts = O.attention_weights(q, Kh, 0.3)
    assert abs(wts.sum() - 1) < 1e-12 and np.all(wts >= 0)
    # equal keys -> uniform weights -> output is the mean of V
    Kc = np.tile(rng.standard_normal(128), (50, 1))
    assert np.allclose(O.attention_weights(q, Kc, 0.3), 1 / 50, atol=1e-15)
    # one dominant key -> that token's V
    Kd = np.zeros((10, 128)); Kd[4] = q * 1e3
    assert np.argmax(O.attention_weights(q, Kd, 1.0)) == 4
    assert O.attention_weights(q, Kd, 1.0)[4] > 1 - 1e-12
    # sign of the scale: a negative scale prefers the most anti-aligned key
    assert np.argmax(O.attention_weights(q, Kd, -1.0)) != 4


@pytest.mark.parametrize("bits", [4, 2])
def test_quantized_attention_is_attention_on_dequantized_values(bits):
    """Definition (Fig. 2 caption): brute force applied to independently dequantized K', V'."""
    w, K, V, q = _small(300, 4, 1, seed=4)
    c = O.IntCache(1, 1, bits, 384); c.quant_pack_kv(K, V)
    assert (c.packed_len, c.res_len) == (256, 44)
    # independent dequantization straight from the packed words, scalar code
    cpw, mask = 32 // bits, (1 << bits) - 1
    Kd = [[0.0] * 128 for _ in range(300)]; Vd = [[0.0] * 128 for _ in range(300)]
    for t in range(256):
        n, tt = divmod(t, 128)
        for ch in range(128):
            kp = int(c.k_params[0, 0, n, ch]); vp = int(c.v_params[0, 0, n, tt])
            ks = float(np.array([kp & 0xFFFF], np.uint16).view(np.float16)[0])
            kz = float(np.array([kp >> 16], np.uint16).view(np.float16)[0])
            vs = float(np.array([vp & 0xFFFF], np.uint16).view(np.float16)[0])
            vz = float(np.array([vp >> 16], np.uint16).view(np.float16)[0])
            kq = (int(c.k_codes[0, 0, n, tt, ch // cpw]) >> (bits * (ch % cpw))) & mask
            vq = (int(c.v_codes[0, 0, n, ch, tt // cpw]) >> (bits * (tt % cpw))) & mask
            Kd[t][ch] = kq * ks + kz; Vd[t][ch] = vq * vs + vz
    for t in range(256, 300):
        Kd[t] = [float(x) for x in K[0, 0, t]]; Vd[t] = [float(x) for x in V[0, 0, t]]
    out = O.decode_attn(c, q, W.softmax_scale(w))
    for h in (0, 3):
        ref = brute_attention(q[0, h], Kd, Vd, W.softmax_scale(w))
        assert np.allclose(out[0, h], ref, rtol=1e-11, atol=1e-13)


def test_block_permutation_invariance():
    """Softmax attention does not depend on token order: swapping whole packed blocks
    (codes with their parameters) leaves the output unchanged."""
    w, K, V, q = _small(512 + 5, 4, 1, seed=9)
    c = O.IntCache(1, 1, 4, 640); c.quant_pack_kv(K, V)
    out0 = O.decode_attn(c, q, 0.2)
    perm = [2, 0, 3, 1]
    for name in ["k_codes", "v_codes", "k_params", "v_params"]:
        a = getattr(c, name); a[:, :, :4] = a[:, :, perm].copy()
    assert np.allclose(O.decode_attn(c, q, 0.2), out0, rtol=1e-12, atol=1e-14)


def test_online_softmax_recurrence_equals_two_pass():
    """Alg. 1's running max / rescale recurrence, evaluated tile by tile, and a
    log-sum-exp merge of per-split partials both reproduce the oracle's two-pass result."""
    rng = np.random.default_rng(2)
    Kh = rng.standard_normal((1000, 128)); Vh = rng.standard_normal((1000, 128)); q = rng.standard_normal(128)
    ref = O.attention_weights(q, Kh, 0.2) @ Vh
    for nsplit in (1, 2, 3, 7, 8):
        parts = []
        for idx in np.array_split(np.arange(1000), nsplit):
            m, l, acc = -math.inf, 0.0, np.zeros(128)
            for t0 in range(idx[0], idx[-1] + 1, 64):
                t1 = min(t0 + 64, idx[-1] + 1)
                s = 0.2 * (Kh[t0:t1] @ q)
                m_new = max(m, s.max()); p = np.exp(s - m_new)
                acc = acc * math.exp(m - m_new) + p @ Vh[t0:t1]
                l = l * math.exp(m - m_new) + p.sum(); m = m_new
            parts.append((m, l, acc))
        M = max(p[0] for p in parts)
        Lsum = sum(p[1] * math.exp(p[0] - M) for p in parts)
        out = sum(p[2] * math.exp(p[0] - M) for p in parts) / Lsum
        assert np.allclose(out, ref, rtol=1e-12, atol=1e-14)
