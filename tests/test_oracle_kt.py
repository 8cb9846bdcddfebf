"""Pins of the per-token K quantization (the paper's KT setting).  The per-channel path is pinned
in test_oracle_quant; per-token quantization of a square block is per-channel quantization of
its transpose, which ties the two together; the rest are worked examples, bounds and brute force."""
import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W


def _block(seed):
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=1, n_kv_heads=1, context=128, seed=seed)
    K, _ = W.make_kv(w)
    return K[0, 0]


@pytest.mark.parametrize("bits", [4, 2])
def test_per_token_is_per_channel_of_the_transpose(bits):
    X = _block(7)
    c1, s1, z1 = O.quantize_k_block_per_token(X, bits)
    c2, s2, z2 = O.quantize_k_block(np.ascontiguousarray(X.T), bits)
    assert np.array_equal(c1, c2.T) and np.array_equal(s1.view(np.uint16), s2.view(np.uint16))
    assert np.array_equal(z1.view(np.uint16), z2.view(np.uint16))


def test_worked_example_rows():
    """Token rows whose values are an arithmetic progression come back as the codes 0..15 repeated;
    a constant row has scale 0, all codes 0, and dequantizes to the constant."""
    X = np.zeros((128, 128), np.float16)
    X[0] = np.tile(np.arange(16, dtype=np.float16) * np.float16(0.5) - np.float16(3.0), 8)   # -3 .. 4.5
    X[1] = np.float16(2.5)
    X[2, :] = np.float16(-1.0); X[2, 5] = np.float16(14.0)                                    # scale exactly 1
    codes, scale, zero = O.quantize_k_block_per_token(X, 4)
    assert np.array_equal(codes[0], np.tile(np.arange(16), 8)) and scale[0] == np.float16(0.5) and zero[0] == np.float16(-3.0)
    assert scale[1] == 0 and not codes[1].any() and zero[1] == np.float16(2.5)
    assert scale[2] == np.float16(1.0) and codes[2, 5] == 15 and codes[2].sum() == 15


@pytest.mark.parametrize("bits", [4, 2])
def test_brute_force_and_error_bound(bits):
    X = _block(11)
    codes, scale, zero = O.quantize_k_block_per_token(X, bits)
    qmax = (1 << bits) - 1
    for t in (0, 17, 127):
        row = X[t].astype(np.float32)
        mn, mx = row.min(), row.max()
        s = np.float16((mx - mn) / np.float32(qmax))
        assert s == scale[t] and np.float16(mn) == zero[t]
        for c in (0, 63, 127):
            q = (row[c] - np.float32(mn)) / np.float32(s)
            lo = np.floor(q); frac = q - lo
            want = lo + (1 if frac > 0.5 or (frac == 0.5 and int(lo) % 2 == 1) else 0)
            assert codes[t, c] == int(min(max(want, 0), qmax))
    xhat = codes.astype(np.float64) * scale.astype(np.float64)[:, None] + zero.astype(np.float64)[:, None]
    err = np.abs(xhat - X.astype(np.float64))
    # half a step, plus what rounding the scale to fp16 moves the top code by (qmax * 2^-11 * scale)
    assert (err <= (0.5 + qmax * 2.0 ** -11) * scale.astype(np.float64)[:, None] + 1e-12).all()


def test_cache_with_per_token_keys_dequantizes_per_token_and_attends():
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=4, n_kv_heads=1, context=300, seed=13)
    K, V = W.make_kv(w)
    kt = O.IntCache(1, 1, 4, 384, k_per_token=True); kt.quant_pack_kv(K, V)
    kc = O.IntCache(1, 1, 4, 384); kc.quant_pack_kv(K, V)
    assert np.array_equal(kt.v_codes, kc.v_codes) and np.array_equal(kt.k_res, kc.k_res)     # only K's packed part differs
    Kh, Vh = kt.dequant(0, 0)
    codes, scale, zero = O.quantize_k_block_per_token(K[0, 0, 128:256], 4)
    assert np.array_equal(Kh[128:256], codes * scale.astype(np.float64)[:, None] + zero.astype(np.float64)[:, None])
    assert np.array_equal(Kh[256:], K[0, 0, 256:].astype(np.float64))
    # x10 outlier channels stretch every token's range: per-token K is the less accurate of the two
    # settings on such data (why the paper's default is channel-wise K, Sec. IV-B(1))
    q = W.make_q(w)
    ref = O.attention_weights(q[0, 0].astype(np.float64), K[0, 0].astype(np.float64), 0.09) @ V[0, 0].astype(np.float64)
    e_kt = np.abs(O.decode_attn(kt, q, 0.09)[0, 0] - ref).max()
    e_kc = np.abs(O.decode_attn(kc, q, 0.09)[0, 0] - ref).max()
    assert e_kt < 0.5 and e_kc < 0.5
    # appends flush with the same rule
    for step in range(100):
        kn, vn = W.make_new_kv(w, step)
        kt.append_kv(kn, vn)
    assert (kt.packed_len, kt.res_len) == (384, 16)
    c3, s3, z3 = O.quantize_k_block_per_token(kt_res_block := np.concatenate([K[0, 0, 256:], np.stack([W.make_new_kv(w, i)[0][0, 0] for i in range(84)])]), 4)
    assert np.array_equal(O.unpack_words(kt.k_codes[0, 0, 2], 4), c3)
    assert np.array_equal(O.unpack_half2(kt.k_params[0, 0, 2])[0].view(np.uint16), s3.view(np.uint16))
