"""Pins of the smaller quantization groups (32 and 64; K_p of shape (T_n/group, d), V_p of shape
(T_n, d/group), Sec. IV-C(1)).  The group-128 quantizers are pinned in test_oracle_quant; a group of
G tokens (channels) repeated 128/G times is a 128-group with the same minimum and maximum, which
ties the grouped quantizers to them; the rest is brute force with explicit index arithmetic,
bounds, and the cache's layout and state machine."""
import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W


def _blocks(seed):
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=1, n_kv_heads=1, context=128, seed=seed)
    K, V = W.make_kv(w)
    return K[0, 0], V[0, 0]


def _bits_equal(a, b):
    return np.array_equal(np.asarray(a).view(np.uint16), np.asarray(b).view(np.uint16))


@pytest.mark.parametrize("bits", [4, 2])
def test_group_128_is_the_ungrouped_quantizer(bits):
    K, V = _blocks(3)
    c, s, z = O.quantize_k_block_grouped(K, bits, 128)
    c0, s0, z0 = O.quantize_k_block(K, bits)
    assert np.array_equal(c, c0) and _bits_equal(s[0], s0) and _bits_equal(z[0], z0)
    c, s, z = O.quantize_v_block_grouped(V, bits, 128)
    c0, s0, z0 = O.quantize_v_block(V, bits)
    assert np.array_equal(c, c0) and _bits_equal(s[:, 0], s0) and _bits_equal(z[:, 0], z0)


@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("group", [32, 64])
def test_a_group_repeated_to_128_is_a_128_group(bits, group):
    K, V = _blocks(5)
    reps = 128 // group
    kc, ks, kz = O.quantize_k_block_grouped(K, bits, group)
    vc, vs, vz = O.quantize_v_block_grouped(V, bits, group)
    for j in range(reps):
        tiled = np.ascontiguousarray(np.tile(K[j * group:(j + 1) * group], (reps, 1)))
        c0, s0, z0 = O.quantize_k_block(tiled, bits)
        assert np.array_equal(kc[j * group:(j + 1) * group], c0[:group]) and _bits_equal(ks[j], s0) and _bits_equal(kz[j], z0)
        tiled = np.ascontiguousarray(np.tile(V[:, j * group:(j + 1) * group], (1, reps)))
        c0, s0, z0 = O.quantize_v_block(tiled, bits)
        assert np.array_equal(vc[:, j * group:(j + 1) * group], c0[:, :group])
        assert _bits_equal(vs[:, j], s0) and _bits_equal(vz[:, j], z0)


@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("group", [32, 64])
def test_brute_force_bounds_and_nesting(bits, group):
    K, V = _blocks(9)
    qmax = (1 << bits) - 1
    kc, ks, kz = O.quantize_k_block_grouped(K, bits, group)
    vc, vs, vz = O.quantize_v_block_grouped(V, bits, group)

    def check(members, x, scale, zero, code):
        mn, mx = min(members), max(members)
        s = np.float16((np.float32(mx) - np.float32(mn)) / np.float32(qmax))
        assert s == scale and np.float16(mn) == zero
        q = (np.float32(x) - np.float32(mn)) / np.float32(s)
        lo = np.floor(q); frac = q - lo
        want = lo + (1 if frac > 0.5 or (frac == 0.5 and int(lo) % 2 == 1) else 0)
        assert code == int(min(max(want, 0), qmax))

    for t, c in [(0, 0), (31, 5), (32, 64), (77, 127), (127, 33)]:
        j = t // group
        check([float(K[j * group + i, c]) for i in range(group)], K[t, c], ks[j, c], kz[j, c], kc[t, c])
        g = c // group
        check([float(V[t, g * group + i]) for i in range(group)], V[t, c], vs[t, g], vz[t, g], vc[t, c])
    # round trip: half a step of the element's own group (plus the fp16 rounding of the scale)
    khat = kc * np.repeat(ks.astype(np.float64), group, axis=0) + np.repeat(kz.astype(np.float64), group, axis=0)
    vhat = vc * np.repeat(vs.astype(np.float64), group, axis=1) + np.repeat(vz.astype(np.float64), group, axis=1)
    assert (np.abs(khat - K) <= (0.5 + qmax * 2.0 ** -11) * np.repeat(ks.astype(np.float64), group, axis=0) + 1e-12).all()
    assert (np.abs(vhat - V) <= (0.5 + qmax * 2.0 ** -11) * np.repeat(vs.astype(np.float64), group, axis=1) + 1e-12).all()
    # a group's range lies inside the range of the group that contains it
    _, ks2, _ = O.quantize_k_block_grouped(K, bits, 2 * group)
    _, vs2, _ = O.quantize_v_block_grouped(V, bits, 2 * group)
    assert (ks <= np.repeat(ks2, 2, axis=0)).all() and (vs <= np.repeat(vs2, 2, axis=1)).all()


def test_worked_example():
    """Two token groups with different ranges in one channel; a token whose channel groups differ."""
    K = np.zeros((128, 128), np.float16)
    K[:32, 0] = np.tile(np.arange(16, dtype=np.float16), 2)             # 0..15: scale 1, codes = values
    K[32:64, 0] = np.tile(np.arange(16, dtype=np.float16) * np.float16(0.25) + np.float16(2.0), 2)
    codes, scale, zero = O.quantize_k_block_grouped(K, 4, 32)
    assert scale[0, 0] == 1 and zero[0, 0] == 0 and np.array_equal(codes[:32, 0], np.tile(np.arange(16), 2))
    assert scale[1, 0] == np.float16(0.25) and zero[1, 0] == 2 and np.array_equal(codes[32:64, 0], np.tile(np.arange(16), 2))
    assert scale[2, 0] == 0 and not codes[64:, 0].any()
    V = np.zeros((128, 128), np.float16)
    V[7, 32:64] = np.tile(np.array([-3, 0, 3, 6], np.float16), 8)       # 2-bit: scale 3, zero -3
    V[7, 64:96] = np.float16(1.5)
    codes, scale, zero = O.quantize_v_block_grouped(V, 2, 32)
    assert scale[7, 1] == 3 and zero[7, 1] == -3 and np.array_equal(codes[7, 32:64], np.tile(np.arange(4), 8))
    assert scale[7, 2] == 0 and zero[7, 2] == np.float16(1.5) and not codes[7, 64:96].any()


@pytest.mark.parametrize("bits,group", [(4, 32), (2, 64)])
def test_cache_layout_state_machine_and_attention(bits, group):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=4, n_kv_heads=2, context=300, seed=21)
    K, V = W.make_kv(w)
    gc = O.IntCache(2, 2, bits, 512, group=group); gc.quant_pack_kv(K, V)
    base = O.IntCache(2, 2, bits, 512); base.quant_pack_kv(K, V)
    assert gc.k_params.shape == (2, 2, 4, 128 // group, 128) and gc.v_params.shape == (2, 2, 4, 128, 128 // group)
    assert gc.k_codes.shape == base.k_codes.shape and np.array_equal(gc.k_res, base.k_res)
    # block 1 of unit (1, 0) against the block quantizers
    kc, ks, kz = O.quantize_k_block_grouped(K[1, 0, 128:256], bits, group)
    vc, vs, vz = O.quantize_v_block_grouped(V[1, 0, 128:256], bits, group)
    assert np.array_equal(O.unpack_words(gc.k_codes[1, 0, 1], bits), kc)
    assert np.array_equal(O.unpack_words(gc.v_codes[1, 0, 1], bits).T, vc)
    assert np.array_equal(gc.k_params[1, 0, 1], O.pack_half2(ks, kz)) and np.array_equal(gc.v_params[1, 0, 1], O.pack_half2(vs, vz))
    Kh, Vh = gc.dequant(1, 0)
    assert np.array_equal(Kh[128:256], kc * np.repeat(ks.astype(np.float64), group, axis=0) + np.repeat(kz.astype(np.float64), group, axis=0))
    assert np.array_equal(Vh[128:256], vc * np.repeat(vs.astype(np.float64), group, axis=1) + np.repeat(vz.astype(np.float64), group, axis=1))
    assert np.array_equal(Kh[256:], K[1, 0, 256:].astype(np.float64))
    # smaller groups track the data more closely than one group of 128
    q = W.make_q(w)
    exact = np.stack([O.attention_weights(q[1, h].astype(np.float64), K[1, 0].astype(np.float64), 0.09) @ V[1, 0].astype(np.float64)
                      for h in range(2)])
    e_g = np.abs(O.decode_attn(gc, q, 0.09)[1, :2] - exact).max()
    e_b = np.abs(O.decode_attn(base, q, 0.09)[1, :2] - exact).max()
    assert e_g < e_b
    # appends flush with the same rule, and a flushed block equals the prefilled one
    pre = O.IntCache(2, 2, bits, 512, group=group)
    news = [W.make_new_kv(w, i) for i in range(100)]
    for kn, vn in news:
        gc.append_kv(kn, vn)
    assert (gc.packed_len, gc.res_len) == (384, 16)
    K2 = np.concatenate([K, np.stack([kn for kn, _ in news], axis=2)], axis=2)
    V2 = np.concatenate([V, np.stack([vn for _, vn in news], axis=2)], axis=2)
    pre.quant_pack_kv(K2, V2)
    for name in ("k_codes", "v_codes", "k_params", "v_params"):
        assert np.array_equal(getattr(pre, name), getattr(gc, name)), name
    assert np.array_equal(pre.k_res[:, :, :16], gc.k_res[:, :, :16])


# ---- per-token K with channel groups (the KT setting with a group: parameters of shape (T_n, d/group))

@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("group", [32, 64])
def test_per_token_k_groups_brute_force(bits, group):
    """Every element against min / max / scale taken by hand over its own (token, channel group), and the
    transposition symmetry: per-token groups of K are channel-wise groups of K^T."""
    K, _ = _blocks(13)
    kc, ks, kz = O.quantize_k_block_per_token_grouped(K, bits, group)
    assert kc.shape == (128, 128) and ks.shape == kz.shape == (128, 128 // group)
    qmax = 2 ** bits - 1
    rng = np.random.default_rng(5)
    for t, c in zip(rng.integers(0, 128, 300), rng.integers(0, 128, 300)):
        g = c // group
        vals = [float(K[t, g * group + i]) for i in range(group)]
        mn, mx = min(vals), max(vals)
        s = np.float16(np.float32(np.float32(mx) - np.float32(mn)) / np.float32(qmax))
        assert _bits_equal(ks[t, g], s) and float(kz[t, g]) == mn
        code = 0 if s == 0 else int(np.clip(np.rint((np.float32(K[t, c]) - np.float32(mn)) / np.float32(s)), 0, qmax))
        assert kc[t, c] == code
    ct, st, zt = O.quantize_k_block_grouped(np.ascontiguousarray(K.T), bits, group)
    assert np.array_equal(ct.T, kc) and _bits_equal(st.T, ks) and _bits_equal(zt.T, kz)
    # group 128 is the KT quantizer
    c0, s0, z0 = O.quantize_k_block_per_token(K, bits)
    c1, s1, z1 = O.quantize_k_block_per_token_grouped(K, bits, 128)
    assert np.array_equal(c0, c1) and _bits_equal(s0, s1[:, 0]) and _bits_equal(z0, z1[:, 0])


def test_per_token_k_groups_worked_example():
    K = np.zeros((128, 128), np.float16)
    K[5, 64:96] = np.tile(np.arange(16, dtype=np.float16) * np.float16(0.5) - np.float16(1.0), 2)   # scale 0.5, zero -1
    K[5, 96:128] = np.float16(-2.25)                                                                  # constant group
    codes, scale, zero = O.quantize_k_block_per_token_grouped(K, 4, 32)
    assert scale[5, 2] == np.float16(0.5) and zero[5, 2] == -1 and np.array_equal(codes[5, 64:96], np.tile(np.arange(16), 2))
    assert scale[5, 3] == 0 and zero[5, 3] == np.float16(-2.25) and not codes[5, 96:].any()
    assert scale[5, 0] == 0 and zero[5, 0] == 0


@pytest.mark.parametrize("bits,group", [(4, 32), (2, 64)])
def test_per_token_k_groups_cache_and_attention(bits, group):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=4, n_kv_heads=2, context=300, seed=22)
    K, V = W.make_kv(w)
    gc = O.IntCache(2, 2, bits, 512, k_per_token=True, group=group); gc.quant_pack_kv(K, V)
    kt = O.IntCache(2, 2, bits, 512, k_per_token=True); kt.quant_pack_kv(K, V)
    cw = O.IntCache(2, 2, bits, 512, group=group); cw.quant_pack_kv(K, V)
    assert gc.k_params.shape == gc.v_params.shape == (2, 2, 4, 128, 128 // group)
    # V is what the channel-wise grouped cache holds; K differs from both relatives only in its statistics axis
    assert np.array_equal(gc.v_codes, cw.v_codes) and np.array_equal(gc.v_params, cw.v_params)
    assert gc.k_codes.shape == kt.k_codes.shape and np.array_equal(gc.k_res, kt.k_res)
    kc, ks, kz = O.quantize_k_block_per_token_grouped(K[1, 1, 128:256], bits, group)
    assert np.array_equal(O.unpack_words(gc.k_codes[1, 1, 1], bits), kc)
    assert np.array_equal(gc.k_params[1, 1, 1], O.pack_half2(ks, kz))
    Kh, Vh = gc.dequant(1, 1)
    assert np.array_equal(Kh[128:256], kc * np.repeat(ks.astype(np.float64), group, axis=1) + np.repeat(kz.astype(np.float64), group, axis=1))
    assert np.array_equal(Vh, cw.dequant(1, 1)[1])
    # attention over it = brute-force softmax over the dequantized rows
    q = W.make_q(w)
    out = O.decode_attn(gc, q, 0.09)
    for hq in (2, 3):
        s = 0.09 * np.array([sum(float(Kh[t, c]) * float(q[1, hq, c]) for c in range(128)) for t in range(300)])
        p = np.exp(s - s.max())
        ref = (p[:, None] * Vh).sum(axis=0) / p.sum()
        assert np.abs(out[1, hq] - ref).max() < 1e-12
    # smaller K groups track K more closely than one group per token
    exact = np.stack([O.attention_weights(q[1, h].astype(np.float64), K[1, 0].astype(np.float64), 0.09) for h in range(2)])
    w_g = np.stack([O.attention_weights(q[1, h].astype(np.float64), gc.dequant(1, 0)[0], 0.09) for h in range(2)])
    w_t = np.stack([O.attention_weights(q[1, h].astype(np.float64), kt.dequant(1, 0)[0], 0.09) for h in range(2)])
    assert np.abs(w_g - exact).sum() < np.abs(w_t - exact).sum()
    # appends flush with the same rule; a flushed block equals the prefilled one
    pre = O.IntCache(2, 2, bits, 512, k_per_token=True, group=group)
    news = [W.make_new_kv(w, i) for i in range(100)]
    for kn, vn in news:
        gc.append_kv(kn, vn)
    K2 = np.concatenate([K, np.stack([kn for kn, _ in news], axis=2)], axis=2)
    V2 = np.concatenate([V, np.stack([vn for _, vn in news], axis=2)], axis=2)
    pre.quant_pack_kv(K2, V2)
    for name in ("k_codes", "v_codes", "k_params", "v_params"):
        assert np.array_equal(getattr(pre, name), getattr(gc, name)), name


def test_per_token_k_groups_paged_is_a_relocation():
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=4, n_kv_heads=2, context=300, seed=23)
    K, V = W.make_kv(w)
    table = np.array([[5, 2, 7, -1], [0, 6, 1, -1]], np.int32)
    pc = O.PagedIntCache(2, 2, 4, 8, 4, table, k_per_token=True, group=32)
    cc = O.IntCache(2, 2, 4, 512, k_per_token=True, group=32)
    cc.quant_pack_kv(K, V)
    for b in range(2):
        pc.quant_pack_kv(b, K[b], V[b])
    assert pc.k_params.shape == (8, 2, 128, 4)
    for b in range(2):
        for n in range(2):
            assert np.array_equal(pc.k_codes[table[b, n]], cc.k_codes[b, :, n]) and np.array_equal(pc.k_params[table[b, n]], cc.k_params[b, :, n])
    assert np.array_equal(O.decode_attn(pc, W.make_q(w), 0.09), O.decode_attn(cc, W.make_q(w), 0.09))
