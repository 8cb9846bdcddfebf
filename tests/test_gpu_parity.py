"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU oracle on the
same seeded inputs.  Packed bytes and parameters must be bit-exact; attention outputs must be
within 2e-3 max-abs and 1e-3 relative L2 of the float64 oracle."""
import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import binding as B
from paper_2503_18773_amd import workloads as W
from tests.util import assert_attn_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu

BITS = {"int4": 4, "int2": 2, "int4_kt": 4, "int2_kt": 2, "int4_g64": 4, "int4_g32": 4, "int2_g64": 2, "int2_g32": 2,
        "int4_kt_g64": 4, "int4_kt_g32": 4, "int2_kt_g64": 2, "int2_kt_g32": 2}
GROUP = {"int4_g64": 64, "int4_g32": 32, "int2_g64": 64, "int2_g32": 32,
         "int4_kt_g64": 64, "int4_kt_g32": 32, "int2_kt_g64": 64, "int2_kt_g32": 32}
GROUP_FORMATS = sorted(GROUP)


def _int_cache_pair(w, capacity):
    """Oracle cache and GPU cache prefilled from the same K, V."""
    K, V = W.make_kv(w)
    oc = O.IntCache(w.batch, w.n_kv_heads, BITS[w.fmt], capacity, k_per_token="_kt" in w.fmt,
                    group=GROUP.get(w.fmt, 128))
    oc.quant_pack_kv(K, V)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, capacity)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    return K, V, oc, gc


def _assert_int_cache_equal(oc, gc):
    import torch
    torch.cuda.synchronize()
    assert (gc.packed_len, gc.res_len) == (oc.packed_len, oc.res_len)
    nb = oc.packed_len // 128
    names = ["k_codes", "v_codes", "k_params", "v_params"]
    for i, name in enumerate(names):
        ref = getattr(oc, name)
        got = gc.host_buffer(i).view(np.uint32).reshape(ref.shape)
        assert np.array_equal(got[:, :, :nb], ref[:, :, :nb]), name
    for i, name in [(4, "k_res"), (5, "v_res")]:
        ref = getattr(oc, name)
        got = gc.host_buffer(i).view(np.float16).reshape(ref.shape)
        assert np.array_equal(got[:, :, :oc.res_len].view(np.uint16), ref[:, :, :oc.res_len].view(np.uint16)), name


@pytest.mark.parametrize("fmt", ["int4", "int2"])
@pytest.mark.parametrize("L", [128 * 5 + 37, 128 * 3, 90, 0])
def test_quant_pack_bit_exact(fmt, L):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=8, n_kv_heads=2, context=L, fmt=fmt)
    _, _, oc, gc = _int_cache_pair(w, 1024)
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", ["int4", "int2"])
def test_quant_adversarial_values_bit_exact(fmt):
    """Constant groups (scale 0), +-65504, subnormals, -0, exact ties."""
    rng = np.random.default_rng(5)
    K = rng.standard_normal((1, 2, 256, 128)).astype(np.float16)
    V = rng.standard_normal((1, 2, 256, 128)).astype(np.float16)
    K[0, 0, :128, 3] = 1.5                       # constant channel
    K[0, 0, :128, 4] = -0.0                      # all negative zero
    K[0, 0, 0, 5] = 65504; K[0, 0, 1, 5] = -65504
    K[0, 0, :128, 6] = (rng.integers(0, 4, 128) * 6e-8).astype(np.float16)      # subnormals only
    K[0, 0, :128, 7] = np.array([0, 15] + [2.5, 3.5, 0.5, 1.5] * 31 + [7, 7], np.float16)   # exact ties
    V[0, 1, 7, :] = -2.25                        # constant token
    V[0, 1, 8, 0] = 65504; V[0, 1, 8, 1] = -65504
    V[0, 1, 9, :] = (rng.integers(0, 3, 128) * 6e-8).astype(np.float16)
    V[0, 1, 10, :] = np.array([0, 3] + [0.5, 1.5, 2.5, 1.0] * 31 + [2, 2], np.float16)
    w = W.scaled(W.CONFIGS["cfg0"], n_q_heads=2, n_kv_heads=2, context=256, fmt=fmt)
    oc = O.IntCache(1, 2, BITS[fmt], 256); oc.quant_pack_kv(K, V)
    gc = B.KVCache(1, 2, 2, fmt, 256); gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", ["int4", "int2"])
def test_quant_scale_rounding_sweep_bit_exact(fmt):
    """The scale is an fp32 quotient rounded again to fp16, and both roundings must be the oracle's: every
    positive fp16 value as the range of a V group and of a K group (minimum 0, head 0), and ranges that are no
    fp16 value (negative minimum, head 1).  A scale that is one fp16 step off also moves codes."""
    rng = np.random.default_rng(11)
    vals = np.arange(1, 0x7c00, dtype=np.uint16).view(np.float16)        # all positive finite fp16 values
    n = 31744                                                            # 248 blocks of 128
    mx = np.concatenate([vals, vals[:n - vals.size]]).astype(np.float64)
    mn = np.stack([np.zeros(n), -mx[rng.permutation(n)] * 0.37])         # per head
    mn = mn.astype(np.float16).astype(np.float64)
    frac = rng.random((2, n, 128))
    # V: token r is one group; K: (block, channel) is one group -- same values, blocks transposed
    V = (mn[:, :, None] + frac * (mx[None, :, None] - mn[:, :, None])).astype(np.float16)
    V = np.clip(V.astype(np.float64), mn[:, :, None], mx[None, :, None]).astype(np.float16)
    V[:, :, 0] = mn.astype(np.float16); V[:, :, 1] = mx.astype(np.float16)[None]
    K = V.reshape(2, n // 128, 128, 128).transpose(0, 1, 3, 2).reshape(2, n, 128)
    K, V = np.ascontiguousarray(K[None]), np.ascontiguousarray(V[None])
    oc = O.IntCache(1, 2, BITS[fmt], n + 128); oc.quant_pack_kv(K, V)
    gc = B.KVCache(1, 2, 2, fmt, n + 128); gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", ["int4", "int2"])
@pytest.mark.parametrize("L,k", [(100, 27), (100, 28), (200, 190), (0, 130)])
def test_append_state_machine_bit_exact(fmt, L, k):
    w = W.scaled(W.CONFIGS["cfg1"], n_q_heads=8, n_kv_heads=2, context=L, fmt=fmt)
    K, V, oc, gc = _int_cache_pair(w, 512)
    for i in range(k):
        kn, vn = W.make_new_kv(w, i)
        oc.append_kv(kn, vn)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
        assert (gc.packed_len, gc.res_len) == (oc.packed_len, oc.res_len)
    _assert_int_cache_equal(oc, gc)


def test_append_capacity_error_leaves_state():
    w = W.scaled(W.CONFIGS["cfg0"], n_q_heads=1, n_kv_heads=1, context=128 + 127)
    K, V, oc, gc = _int_cache_pair(w, 128)
    kn, vn = W.make_new_kv(w, 0)
    with pytest.raises(B.BitDecodeError) as e:
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    assert e.value.status == -4 and (gc.packed_len, gc.res_len) == (128, 127)


def _decode(gc, w, q, **kw):
    import torch
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16 if w.in_dtype == "fp16" else torch.bfloat16,
                      device="cuda:0")
    gc.decode_attn(to_dev(q, w.in_dtype), W.softmax_scale(w), out, **kw)
    torch.cuda.synchronize()
    return out_to_f64(out)


@pytest.mark.parametrize("fmt", ["int4", "int2"])
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (4, 2)])
@pytest.mark.parametrize("L", [128 * 9 + 37, 128 * 4, 77, 128 * 2 + 127])
def test_decode_matches_oracle(fmt, hq, hkv, L):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=hq, n_kv_heads=hkv, context=L, fmt=fmt)
    _, _, oc, gc = _int_cache_pair(w, 2048)
    q = W.make_q(w)
    ref = O.decode_attn(oc, q, W.softmax_scale(w))
    nb = L // 128
    for ns in sorted({1, 2, 3, 7, max(nb, 1), nb + 5}):
        for fused in (True, False):
            got = _decode(gc, w, q, num_splits=ns, fused=fused)
            assert_attn_close(got, ref, f"{fmt} L={L} splits={ns} fused={fused}")
    got = _decode(gc, w, q)       # library-chosen split factor
    assert_attn_close(got, ref, "auto splits")


def test_decode_empty_cache_gives_zero():
    w = W.scaled(W.CONFIGS["cfg0"], context=0)
    _, _, oc, gc = _int_cache_pair(w, 128)
    got = _decode(gc, w, W.make_q(w), num_splits=3)
    assert np.all(got == 0)


@pytest.mark.parametrize("name", ["cfg0", "cfg1"])
def test_config_decode_steps(name):
    """The configuration as stated: prefill, then decode steps each appending one token
    (cfg0: 1 step; cfg1: its 64 steps are run, outputs checked on a few of them)."""
    w = W.CONFIGS[name]
    K, V, oc, gc = _int_cache_pair(w, w.context + 256)
    check = {0, 1, w.steps - 1}
    for step in range(w.steps):
        kn, vn = W.make_new_kv(w, step)
        oc.append_kv(kn, vn); gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
        if step in check:
            q = W.make_q(w, step)
            ref = O.decode_attn(oc, q, W.softmax_scale(w))
            got = _decode(gc, w, q)
            assert_attn_close(got, ref, f"{name} step {step}")
    _assert_int_cache_equal(oc, gc)


def test_cfg2_int2_batch8_full_size_all_units():
    """Configuration 2 at its full size (batch 8, 32K, int2) in the launch configuration the benchmark
    uses, plus one appended token: the packed bytes and parameters of every (sequence, KV head) unit bit
    for bit, and every output row at the plain bar."""
    w = W.CONFIGS["cfg2"]
    K, V = W.make_kv(w)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, w.context + 128)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    kn, vn = W.make_new_kv(w, 0)
    gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    q = W.make_q(w)
    got = _decode(gc, w, q)
    oc = O.IntCache(w.batch, w.n_kv_heads, 2, w.context + 128)
    oc.quant_pack_kv(K, V)
    oc.append_kv(kn, vn)
    _assert_int_cache_equal(oc, gc)
    ma, rl = assert_attn_close(got, O.decode_attn(oc, q, W.softmax_scale(w)), "cfg2, all 64 units")
    print(f"cfg2 all units: max-abs {ma:.2e} rel-L2 {rl:.2e}")


def test_cfg3_128k_256_steps_all_heads():
    """Configuration 3: 128K context, 256 decode steps (two residual flushes).  Lengths are checked
    every step, the packed bytes of all heads after every flush and the whole cache at the end, the
    outputs of all heads (plain bar) on steps around the flushes and half way between them."""
    w = W.CONFIGS["cfg3"]
    K, V = W.make_kv(w)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, w.context + 512)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    oc = O.IntCache(w.batch, w.n_kv_heads, 4, w.context + 512)
    oc.quant_pack_kv(K, V)
    _assert_int_cache_equal(oc, gc)
    check = {0, 1, 63, 126, 127, 128, 191, 254, 255}
    worst = (0.0, 0.0)
    for step in range(256):
        kn, vn = W.make_new_kv(w, step)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
        oc.append_kv(kn, vn)
        assert (gc.packed_len, gc.res_len) == (oc.packed_len, oc.res_len)
        if gc.res_len == 0:       # a flush happened in this step: the new block of every head
            nb = gc.packed_len // 128
            for i, name in enumerate(["k_codes", "v_codes", "k_params", "v_params"]):
                ref = getattr(oc, name)
                got = gc.host_buffer(i).view(np.uint32).reshape(ref.shape)
                assert np.array_equal(got[:, :, nb - 1], ref[:, :, nb - 1]), (name, step)
        if step in check:
            q = W.make_q(w, step)
            ma, rl = assert_attn_close(_decode(gc, w, q), O.decode_attn(oc, q, W.softmax_scale(w)), f"cfg3 step {step}")
            worst = (max(worst[0], ma), max(worst[1], rl))
    assert (gc.packed_len, gc.res_len) == (131072 + 256, 0)
    _assert_int_cache_equal(oc, gc)
    print(f"cfg3 all heads: worst max-abs {worst[0]:.2e} rel-L2 {worst[1]:.2e}")


# ---------------------------------------------------------------------------- MXFP4

def _mx_pair(w, capacity, L=None):
    K, V = W.make_kv(w, length=L)
    oc = O.MxCache(w.batch, w.n_kv_heads, capacity)
    oc.quant_pack_kv(K, V)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, "mxfp4", capacity)
    gc.quant_pack_kv(to_dev(K, "bf16"), to_dev(V, "bf16"))
    return K, V, oc, gc


def _assert_mx_cache_equal(oc, gc):
    import torch
    torch.cuda.synchronize()
    assert gc.packed_len == oc.length and gc.res_len == 0
    for i, name in enumerate(["k_codes", "v_codes", "k_scales", "v_scales"]):
        ref = getattr(oc, name)
        got = gc.host_buffer(i).reshape(ref.shape)
        if name == "v_codes":
            assert np.array_equal(got, ref), name      # whole buffer: absent tokens are zero nibbles
        else:
            assert np.array_equal(got[:, :, :oc.length], ref[:, :, :oc.length]), name


@pytest.mark.parametrize("L", [128 * 3 + 37, 256, 1, 0])
def test_mx_quant_pack_bit_exact(L):
    w = W.scaled(W.CONFIGS["cfg4"], batch=2, n_q_heads=8, n_kv_heads=2, context=L)
    _, _, oc, gc = _mx_pair(w, 512)
    _assert_mx_cache_equal(oc, gc)


def test_mx_quant_adversarial_bit_exact():
    """Zero blocks, exact ties on the e2m1 grid, saturation, negative zero, huge and tiny magnitudes."""
    rng = np.random.default_rng(3)
    K = W.round_to_bf16(rng.standard_normal((1, 1, 128, 128)).astype(np.float32))
    V = W.round_to_bf16(rng.standard_normal((1, 1, 128, 128)).astype(np.float32))
    K[0, 0, 0, :32] = 0.0
    K[0, 0, 1, :32] = np.array([4.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0] * 4, np.float32)        # ties, amax 5 -> e 0
    K[0, 0, 2, :32] = np.array([-4.0, -0.25, -0.75, -1.25, -1.75, -2.5, -3.5, -5.0] * 4, np.float32)
    K[0, 0, 3, :32] = np.array([7.5, 7.0, 6.5, -7.75] + [0.1, -0.0, -0.1, 0.3] * 7, np.float32)        # saturation
    K[0, 0, 4, :32] = W.round_to_bf16(np.full(32, 3.0e38, np.float32)); K[0, 0, 4, 1] = 1.0
    K[0, 0, 5, :32] = W.round_to_bf16(np.full(32, 1.0e-38, np.float32)); K[0, 0, 5, 3] = -3.0e-39
    # around the switch between the converting instruction and the explicit path (shared exponent -120),
    # with fp32-subnormal elements next to a normal maximum, and negative values that round to zero
    K[0, 0, 6, :32] = np.array([2.0 ** -118, -(2.0 ** -118), 2.0 ** -127, -(2.0 ** -130)] * 8, np.float32)
    K[0, 0, 6, 32:64] = np.array([2.0 ** -119, -(2.0 ** -120), 2.0 ** -126, -(2.0 ** -133)] * 8, np.float32)
    K[0, 0, 6, 64:96] = np.array([1.0, -0.124, -0.0, -0.2] * 8, np.float32)
    V[0, 0, 6, :32] = np.array([-(2.0 ** -117), 1.5 * 2.0 ** -119, -(2.0 ** -121), 2.0 ** -128] * 8, np.float32)
    V[0, 0, 7, 32:64] = 0.0
    V[0, 0, 8, 32:64] = np.array([6.0, 5.0, 1.25, -1.75] * 8, np.float32)
    K, V = W.round_to_bf16(K), W.round_to_bf16(V)
    oc = O.MxCache(1, 1, 128); oc.quant_pack_kv(K, V)
    gc = B.KVCache(1, 1, 1, "mxfp4", 128); gc.quant_pack_kv(to_dev(K, "bf16"), to_dev(V, "bf16"))
    _assert_mx_cache_equal(oc, gc)


@pytest.mark.parametrize("L,k", [(100, 60), (128, 3), (0, 130)])
def test_mx_append_bit_exact(L, k):
    w = W.scaled(W.CONFIGS["cfg4"], batch=2, n_q_heads=8, n_kv_heads=2, context=L)
    _, _, oc, gc = _mx_pair(w, 384)
    for i in range(k):
        kn, vn = W.make_new_kv(w, i)
        oc.append_kv(kn, vn); gc.append_kv(to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    _assert_mx_cache_equal(oc, gc)


def _half_is_rounded_f32(half, f32, what):
    """The bf16 output rows are the fp32 output rows rounded once: within one bf16 step."""
    mask = ~np.isnan(f32)
    assert np.all(np.abs(half - f32)[mask] <= np.abs(f32[mask]) * 2.0 ** -8 + 1e-12), what + " (bf16 rounding)"


def _mx_decode_check(gc, oc_ref, w, q, ns, what, large_outputs=False):
    """bf16 output rounding alone is 2^-9 relative (about 1.1e-3 relative L2), above the bar for the
    kernel's arithmetic.  So the bar (2e-3 max-abs, 1e-3 relative L2 against the float64 oracle) is
    held to the fp32 output rows (bd_cache.out_type = BD_OUT_F32), from the fused call (with one split:
    stored by the attention kernel itself) and from bd_decode_attn + bd_splitk_combine; the bf16 rows
    must be those values rounded once."""
    import torch
    shape = (w.batch, w.n_q_heads, 128)
    qd = to_dev(q, "bf16")
    args = (gc.desc, qd, gc.packed_len, gc.res_len, W.softmax_scale(w), ns, gc.workspace(ns))
    out32, out32b = (torch.full(shape, 9.0, dtype=torch.float32, device="cuda:0") for _ in range(2))
    out16 = torch.full(shape, 9.0, dtype=torch.bfloat16, device="cuda:0")
    mask = ~np.isnan(oc_ref)
    ref = np.where(mask, oc_ref, 0.0)
    try:
        gc.desc.out_type = B.BD_OUT_F32
        B.bd_decode_attn(*args, out32)
        B.bd_decode_attn(*args, None)
        B.bd_splitk_combine(gc.desc, gc.workspace(ns), ns, out32b)
    finally:
        gc.desc.out_type = B.BD_OUT_HALF
    B.bd_decode_attn(*args, out16)
    torch.cuda.synchronize()
    got = np.where(mask, out_to_f64(out32), 0.0)
    ma, rl = assert_attn_close(got, ref, what + " (fp32 out)", large_outputs=large_outputs)
    assert_attn_close(np.where(mask, out_to_f64(out32b), 0.0), ref, what + " (fp32 out, separate merge)",
                      large_outputs=large_outputs)
    _half_is_rounded_f32(np.where(mask, out_to_f64(out16), 0.0), got, what)
    return ma, rl


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 2), (12, 1), (5, 1), (21, 1), (64, 2)])
@pytest.mark.parametrize("L", [128 * 9 + 37, 128 * 4, 77])
def test_mx_decode_matches_oracle(hq, hkv, L):
    w = W.scaled(W.CONFIGS["cfg4"], batch=2, n_q_heads=hq, n_kv_heads=hkv, context=L)
    _, _, oc, gc = _mx_pair(w, 2048)
    q = W.make_q(w)
    ref = O.decode_attn(oc, q, W.softmax_scale(w))
    nb = -(-L // 128)
    for ns in sorted({1, 2, 3, nb, nb + 5, gc.choose_splits()}):
        _mx_decode_check(gc, ref, w, q, ns, f"mx L={L} splits={ns}")


def test_cfg4_mxfp4_full_size_all_units():
    """Configuration 4 at full size (batch 16, 16K, MXFP4) plus one appended token: codes and scales of
    every (sequence, KV head) unit bit for bit, every fp32 output row at the plain bar, the bf16 rows
    those values rounded once.  (The oracle runs unit by unit on the host cores.)"""
    from tests.util import mx_units_on_host_cores
    w = W.CONFIGS["cfg4"]
    K, V = W.make_kv(w)
    cap = w.context + 128
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, "mxfp4", cap)
    gc.quant_pack_kv(to_dev(K, "bf16"), to_dev(V, "bf16"))
    kn, vn = W.make_new_kv(w, 0)
    gc.append_kv(to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    import torch
    torch.cuda.synchronize()
    q = W.make_q(w)
    L, g = w.context + 1, w.g_q
    bufs = [gc.host_buffer(i) for i in range(4)]
    shapes = [(cap, 64), (cap // 128, 128, 64), (cap, 4), (cap, 4)]      # per unit: k_codes, v_codes, k_scales, v_scales
    full = [b.reshape((w.batch, w.n_kv_heads) + sh) for b, sh in zip(bufs, shapes)]
    ref = np.empty((w.batch, w.n_q_heads, 128))
    for b, h, kc, vc, ks, vs, out in mx_units_on_host_cores(K, V, kn, vn, q, W.softmax_scale(w), cap):
        assert np.array_equal(full[0][b, h, :L], kc[:L]), ("k_codes", b, h)
        assert np.array_equal(full[1][b, h], vc), ("v_codes", b, h)      # whole buffer: absent tokens are zero nibbles
        assert np.array_equal(full[2][b, h, :L], ks[:L]), ("k_scales", b, h)
        assert np.array_equal(full[3][b, h, :L], vs[:L]), ("v_scales", b, h)
        ref[b, h * g:(h + 1) * g] = out
    ma, rl = _mx_decode_check(gc, ref, w, q, gc.choose_splits(), "cfg4, all 128 units")
    print(f"cfg4 all units: max-abs {ma:.2e} rel-L2 {rl:.2e}")


# ---------------------------------------------------------------------------- fused step

@pytest.mark.parametrize("fmt", ["int4", "int2", "mxfp4", "int4_g32", "int2_g64", "int4_kt_g32", "int2_kt_g64"])
def test_decode_step_equals_append_then_attention(fmt):
    """bd_decode_step is defined as bd_append_kv + bd_decode_attn: same output bits, same cache,
    same lengths, on ordinary steps, on the step that fills the residual block and after it."""
    import torch
    base = W.CONFIGS["cfg4" if fmt == "mxfp4" else "cfg1"]
    w = W.scaled(base, batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 3 + 120, fmt=fmt)
    dt = w.in_dtype
    K, V = W.make_kv(w)
    a = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, 1024)
    b = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, 1024)
    for c in (a, b):
        c.quant_pack_kv(to_dev(K, dt), to_dev(V, dt))
    tdt = torch.float16 if dt == "fp16" else torch.bfloat16
    oa = torch.empty((w.batch, w.n_q_heads, 128), dtype=tdt, device="cuda:0")
    ob = torch.empty_like(oa)
    ns = 3
    for step in range(12):            # residual 120 -> 127 -> flush -> 4 (int formats)
        kn, vn = W.make_new_kv(w, step)
        q = to_dev(W.make_q(w, step), dt)
        knd, vnd = to_dev(kn, dt), to_dev(vn, dt)
        a.append_kv(knd, vnd)
        a.decode_attn(q, W.softmax_scale(w), oa, num_splits=ns)
        b.decode_step(knd, vnd, q, W.softmax_scale(w), ob, num_splits=ns)
        torch.cuda.synchronize()
        assert (a.packed_len, a.res_len) == (b.packed_len, b.res_len)
        assert torch.equal(oa.view(torch.int16), ob.view(torch.int16)), f"{fmt} step {step}"
    for i in range(6):
        assert np.array_equal(a.host_buffer(i), b.host_buffer(i)), (fmt, i)


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_kt", "int2_kt", "int4_g32", "int2_g64", "int4_kt_g64", "int2_kt_g32"])
@pytest.mark.parametrize("gq", [4, 8, 16, 20])
def test_decode_step_packs_the_full_block_inside_the_attention_launch(fmt, gq):
    """The step that fills the residual block: bd_decode_step (flush first: the workgroup that reads the new
    block quantizes it) against bd_append_kv + bd_decode_attn, bit for bit, for split counts that put the new
    block with different workgroups and waves, short and long caches (both loop structures of the kernel)."""
    import torch
    for nblocks in (1, 6, 37):
        for ns in (1, 2, 5, 16):
            w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=2 * gq, n_kv_heads=2, context=128 * nblocks + 126, fmt=fmt,
                         seed=900 + nblocks)
            K, V = W.make_kv(w)
            cap = 128 * (nblocks + 3)
            a = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, cap)
            b = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, cap)
            for c in (a, b):
                c.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
            oa = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
            ob = torch.empty_like(oa)
            for step in range(3):        # residual 126 -> 127 -> flush -> 1
                kn, vn = (to_dev(x, "fp16") for x in W.make_new_kv(w, step))
                q = to_dev(W.make_q(w, step), "fp16")
                a.append_kv(kn, vn)
                a.decode_attn(q, W.softmax_scale(w), oa, num_splits=ns)
                b.decode_step(kn, vn, q, W.softmax_scale(w), ob, num_splits=ns)
                torch.cuda.synchronize()
                assert (a.packed_len, a.res_len) == (b.packed_len, b.res_len)
                assert torch.equal(oa.view(torch.int16), ob.view(torch.int16)), f"{fmt} gq={gq} blocks {nblocks} ns {ns} step {step}"
            for i in range(6):
                assert np.array_equal(a.host_buffer(i), b.host_buffer(i)), (fmt, gq, nblocks, ns, i)


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_kt", "int4_g32", "int2_g64", "int2_kt_g32"])
@pytest.mark.parametrize("gq", [4, 20])
def test_lazy_decode_step_attends_the_full_residual_in_fp16(fmt, gq):
    """bd_decode_step_lazy (the paper's flush order): on the step that fills the residual block the attention sees
    the block's 128 tokens in fp16 -- the oracle's lazy mode -- and the cache afterwards is the one the eager
    step leaves, bit for bit; every other step equals bd_decode_step bit for bit."""
    import torch
    for nblocks, ns in ((0, 1), (2, 3), (9, 4), (37, 16)):
        w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=2 * gq, n_kv_heads=2, context=128 * nblocks + 126, fmt=fmt,
                     seed=950 + nblocks)
        cap = 128 * (nblocks + 3)
        K, V, oc, lazy = _int_cache_pair(w, cap)
        eager = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, cap)
        eager.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
        ol = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
        oe = torch.empty_like(ol)
        for step in range(3):            # residual 126 -> 127 -> 128 (attended in fp16, then packed) -> 1
            kn, vn = W.make_new_kv(w, step)
            q = W.make_q(w, step)
            knd, vnd, qd = to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16")
            lazy.decode_step(knd, vnd, qd, W.softmax_scale(w), ol, num_splits=ns, lazy=True)
            eager.decode_step(knd, vnd, qd, W.softmax_scale(w), oe, num_splits=ns)
            torch.cuda.synchronize()
            oc.append_kv(kn, vn, flush=False)
            fills = oc.res_len == 128
            ref = O.decode_attn(oc, q, W.softmax_scale(w))
            oc.flush_if_full()
            assert (lazy.packed_len, lazy.res_len) == (eager.packed_len, eager.res_len) == (oc.packed_len, oc.res_len)
            assert_attn_close(out_to_f64(ol), ref, f"lazy {fmt} gq={gq} blocks {nblocks} step {step}", large_outputs=True)
            if not fills:
                assert torch.equal(ol.view(torch.int16), oe.view(torch.int16)), (fmt, gq, nblocks, step)
            _assert_int_cache_equal(oc, lazy)
        for i in range(6):
            assert np.array_equal(lazy.host_buffer(i), eager.host_buffer(i)), (fmt, gq, nblocks, i)


def test_decode_step_matches_oracle_on_cfg1():
    w = W.CONFIGS["cfg1"]
    K, V, oc, gc = _int_cache_pair(w, w.context + 256)
    import torch
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
    for step in range(3):
        kn, vn = W.make_new_kv(w, step)
        q = W.make_q(w, step)
        oc.append_kv(kn, vn)
        gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out)
        torch.cuda.synchronize()
        assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"cfg1 fused step {step}")
    _assert_int_cache_equal(oc, gc)


# ---------------------------------------------------------------------------- paged cache

def _paged_pair(fmt, lens, H, Hq, num_pages, max_pages, seed=31, table=None):
    """Oracle and GPU paged caches prefilled with ragged sequences on scattered pages."""
    B_ = len(lens)
    rng = np.random.default_rng(seed)
    if table is None:
        table = rng.permutation(num_pages)[:B_ * max_pages].reshape(B_, max_pages).astype(np.int32)
    oc = O.PagedIntCache(B_, H, BITS[fmt], num_pages, max_pages, table, k_per_token="_kt" in fmt,
                         group=GROUP.get(fmt, 128))
    gc = B.PagedKVCache(B_, Hq, H, fmt, num_pages, table)
    for b, L in enumerate(lens):
        w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=Hq, n_kv_heads=H, context=max(L, 1), seed=seed + b)
        K, V = W.make_kv(w)
        K, V = np.ascontiguousarray(K[0, :, :L]), np.ascontiguousarray(V[0, :, :L])
        oc.quant_pack_kv(b, K, V)
        gc.quant_pack_kv(b, to_dev(K, "fp16"), to_dev(V, "fp16"))
    return oc, gc, table


def _assert_paged_equal(oc, gc, what):
    import torch
    torch.cuda.synchronize()
    assert list(gc.seq_lens.cpu().numpy()) == list(oc.seq_lens), what
    for i, name in enumerate(["k_codes", "v_codes", "k_params", "v_params"]):
        ref = getattr(oc, name)
        got = gc.host_buffer(i).view(np.uint32).reshape(ref.shape)
        assert np.array_equal(got, ref), (what, name)          # whole pool: untouched pages stay zero
    for i, name in [(4, "k_res"), (5, "v_res")]:
        ref = getattr(oc, name)
        got = gc.host_buffer(i).view(np.float16).reshape(ref.shape)
        for b in range(oc.B):
            r = int(oc.seq_lens[b]) % 128
            assert np.array_equal(got[b, :, :r].view(np.uint16), ref[b, :, :r].view(np.uint16)), (what, name, b)


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_g32", "int2_g64", "int4_g64", "int2_g32", "int4_kt_g32", "int2_kt_g64", "int4_kt_g64", "int2_kt_g32"])
def test_paged_prefill_append_and_decode_match_oracle(fmt):
    """Ragged batch on scattered pages: pool bytes bit-exact after prefill and after appends that
    carry two sequences over a flush; attention within tolerance at several split factors,
    including an empty sequence (zero output)."""
    import torch
    lens = [1000, 0, 126, 128 * 5, 37]
    H, Hq = 2, 8
    oc, gc, _ = _paged_pair(fmt, lens, H, Hq, num_pages=64, max_pages=10)
    _assert_paged_equal(oc, gc, f"{fmt} prefill")
    w = W.scaled(W.CONFIGS["cfg1"], batch=len(lens), n_q_heads=Hq, n_kv_heads=H, context=128, seed=77)
    out = torch.empty((len(lens), Hq, 128), dtype=torch.float16, device="cuda:0")
    for step in range(4):
        kn, vn = W.make_new_kv(w, step)
        oc.append_kv(kn, vn)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
        q = W.make_q(w, step)
        for ns in ((1, 3, 8) if step in (0, 3) else (2,)):
            out.zero_()
            gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, ns)
            torch.cuda.synchronize()
            assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} paged step {step} ns {ns}",
                              large_outputs=True)
    _assert_paged_equal(oc, gc, f"{fmt} after appends")
    assert int(gc.status.item()) == 0
    # the sequence that started empty has 4 residual tokens now and attends only those
    assert int(oc.seq_lens[1]) == 4


def test_paged_bad_table_entries_are_skipped_and_reported():
    """A block whose table entry is outside the pool is neither read nor written: decode flags bit
    0 and attends the remaining blocks; an append that needs such a page flags bit 1 and leaves
    the sequence's length unchanged."""
    import torch
    H, Hq = 1, 4
    table = np.array([[3, 1, 9], [0, 2, -1]], np.int32)     # 9 and -1 are not pages of a pool of 4
    oc, gc, _ = _paged_pair("int4", [255, 255], H, Hq, num_pages=4, max_pages=3, table=np.array([[3, 1, 2], [0, 2, 1]], np.int32))
    # rebuild the GPU cache's table with the bad entries in blocks the sequences do not hold yet
    gc.block_table.copy_(torch.from_numpy(table))
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=Hq, n_kv_heads=H, context=128, seed=5)
    kn, vn = W.make_new_kv(w, 0)
    gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))       # fills block 1 of both: pages 1 and 2, fine
    torch.cuda.synchronize()
    assert list(gc.seq_lens.cpu().numpy()) == [256, 256] and int(gc.status.item()) == 0
    for step in range(1, 128):
        kn, vn = W.make_new_kv(w, step)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    torch.cuda.synchronize()
    assert list(gc.seq_lens.cpu().numpy()) == [383, 383] and int(gc.status.item()) == 0
    kn, vn = W.make_new_kv(w, 128)
    gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    torch.cuda.synchronize()
    # this append needed block 2: entries 9 and -1 -> dropped, flagged, lengths stay at 383
    assert list(gc.seq_lens.cpu().numpy()) == [383, 383]
    assert int(gc.status.item()) == 2
    # decode over a table with a bad entry in a block the sequence does hold
    gc.status.zero_()
    bad = table.copy(); bad[0, 0] = 77
    gc.block_table.copy_(torch.from_numpy(bad))
    out = torch.empty((2, Hq, 128), dtype=torch.float16, device="cuda:0")
    gc.decode_attn(to_dev(W.make_q(w), "fp16"), W.softmax_scale(w), out, 2)
    torch.cuda.synchronize()
    assert int(gc.status.item()) == 1
    assert torch.isfinite(out.float()).all()


def test_paged_long_ragged_batch_sampled_units():
    """LLaMA-3.1-8B head geometry, lengths from 100 tokens to just over 32K, pages scattered over
    one pool, split factor as the library picks it for the longest sequence; outputs checked on
    sampled (sequence, KV head) units."""
    import torch
    lens = [32768 + 5, 8192, 100, 20000 + 127]
    H, Hq = 8, 32
    max_pages = 258
    oc, gc, _ = _paged_pair("int4", lens, H, Hq, num_pages=len(lens) * max_pages + 7, max_pages=max_pages, seed=91)
    w = W.scaled(W.CONFIGS["cfg1"], batch=len(lens), seed=92)
    out = torch.empty((len(lens), Hq, 128), dtype=torch.float16, device="cuda:0")
    shape = B.bd_cache(1, Hq, H, 128, B.BD_FMT_INT4, 128 * max_pages, None, None, None, None, None, None)
    ns = B.bd_choose_splits(shape, 32768)
    kn, vn = W.make_new_kv(w, 0)
    oc.append_kv(kn, vn)                                         # sequence 3 flushes its residual here
    gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    q = W.make_q(w, 1)
    gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, ns)
    torch.cuda.synchronize()
    units = [(0, 0), (0, 5), (1, 7), (2, 3), (3, 1), (3, 6)]
    assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w), units=units), "paged long ragged",
                      large_outputs=True)
    assert list(gc.seq_lens.cpu().numpy()) == [L + 1 for L in lens] and int(gc.status.item()) == 0
    # packed bytes of the flushed block of sequence 3, all heads
    pg = int(oc.block_table[3, lens[3] // 128])
    got = gc.host_buffer(0).view(np.uint32).reshape(oc.k_codes.shape)
    assert np.array_equal(got[pg], oc.k_codes[pg])


def _paged_mx_pair(lens, H, Hq, num_pages, max_pages, seed=41, table=None):
    B_ = len(lens)
    rng = np.random.default_rng(seed)
    if table is None:
        table = rng.permutation(num_pages)[:B_ * max_pages].reshape(B_, max_pages).astype(np.int32)
    oc = O.PagedMxCache(B_, H, num_pages, max_pages, table)
    gc = B.PagedKVCache(B_, Hq, H, "mxfp4", num_pages, table)
    for b, L in enumerate(lens):
        w = W.scaled(W.CONFIGS["cfg4"], batch=1, n_q_heads=Hq, n_kv_heads=H, context=max(L, 1), seed=seed + b)
        K, V = W.make_kv(w)
        K, V = np.ascontiguousarray(K[0, :, :L]), np.ascontiguousarray(V[0, :, :L])
        oc.quant_pack_kv(b, K, V)
        gc.quant_pack_kv(b, to_dev(K, "bf16"), to_dev(V, "bf16"))
    return oc, gc, table


def _assert_paged_mx_equal(oc, gc, what):
    """Lengths, and the bytes of every block a sequence holds (token rows up to its length; the
    channel-major V block whole: absent tokens are zero nibbles)."""
    import torch
    torch.cuda.synchronize()
    assert list(gc.seq_lens.cpu().numpy()) == list(oc.seq_lens), what
    got = {name: gc.host_buffer(i).reshape(getattr(oc, name).shape)
           for i, name in enumerate(["k_codes", "v_codes", "k_scales", "v_scales"])}
    for b in range(oc.B):
        L = int(oc.seq_lens[b])
        for n in range(-(-L // 128)):
            p, m = int(oc.block_table[b, n]), min(128, L - n * 128)
            for name in ("k_codes", "k_scales", "v_scales"):
                assert np.array_equal(got[name][p, :, :m], getattr(oc, name)[p, :, :m]), (what, name, b, n)
            assert np.array_equal(got["v_codes"][p], oc.v_codes[p]), (what, "v_codes", b, n)


def _paged_f32(gc, call, shape):
    """Runs call(out) with fp32 output rows and returns them as float64."""
    import torch
    out32 = torch.full(shape, 9.0, dtype=torch.float32, device="cuda:0")
    try:
        gc.desc.out_type = B.BD_OUT_F32
        call(out32)
    finally:
        gc.desc.out_type = B.BD_OUT_HALF
    torch.cuda.synchronize()
    return out_to_f64(out32)


def _paged_mx_decode_check(gc, oc, w, q, ns, what):
    """Same bar as the contiguous MXFP4 cache: the fp32 output rows against the oracle (any split
    count, one split included), the bf16 rows within one bf16 step of them."""
    import torch
    shape = (w.batch, w.n_q_heads, 128)
    qd = to_dev(q, "bf16")
    got = _paged_f32(gc, lambda o: gc.decode_attn(qd, W.softmax_scale(w), o, ns), shape)
    ref = O.decode_attn(oc, q, W.softmax_scale(w))
    assert_attn_close(got, ref, what + " (fp32 out)", large_outputs=True)
    out = torch.full(shape, 7.0, dtype=torch.bfloat16, device="cuda:0")
    gc.decode_attn(qd, W.softmax_scale(w), out, ns)
    torch.cuda.synchronize()
    _half_is_rounded_f32(out_to_f64(out), got, what)


@pytest.mark.parametrize("hq,hkv", [(8, 2), (12, 1)])
def test_paged_mx_prefill_append_and_decode_match_oracle(hq, hkv):
    """MXFP4 in pages: ragged batch (an empty sequence, one that ends on a block boundary, partial
    last blocks), bytes bit-exact after prefill and after appends that open new pages, attention
    within tolerance at several split factors."""
    lens = [1000, 0, 127, 128 * 5, 37]
    oc, gc, _ = _paged_mx_pair(lens, hkv, hq, num_pages=64, max_pages=10)
    _assert_paged_mx_equal(oc, gc, "mx paged prefill")
    w = W.scaled(W.CONFIGS["cfg4"], batch=len(lens), n_q_heads=hq, n_kv_heads=hkv, context=128, seed=78)
    for ns in (1, 3, 8):
        _paged_mx_decode_check(gc, oc, w, W.make_q(w, 9), ns, f"mx paged prefill ns {ns}")
    for step in range(4):
        kn, vn = W.make_new_kv(w, step)
        oc.append_kv(kn, vn)
        gc.append_kv(to_dev(kn, "bf16"), to_dev(vn, "bf16"))
        for ns in ((1, 3, 8) if step in (0, 3) else (2,)):
            _paged_mx_decode_check(gc, oc, w, W.make_q(w, step), ns, f"mx paged step {step} ns {ns}")
    _assert_paged_mx_equal(oc, gc, "mx paged after appends")
    assert int(gc.status.item()) == 0


def test_paged_mx_bad_table_entries_are_skipped_and_reported():
    """MXFP4 needs a page for every token: an append into a block whose entry is outside the pool is
    dropped and flagged (bit 1), the length stays; decode skips such a block and flags bit 0."""
    import torch
    H, Hq = 1, 4
    good = np.array([[3, 1, 2], [0, 2, 1]], np.int32)
    oc, gc, _ = _paged_mx_pair([255, 200], H, Hq, num_pages=4, max_pages=3, table=good)
    gc.block_table.copy_(torch.from_numpy(np.array([[3, 1, 9], [0, 2, -1]], np.int32)))
    w = W.scaled(W.CONFIGS["cfg4"], batch=2, n_q_heads=Hq, n_kv_heads=H, context=128, seed=5)
    for step in range(3):
        kn, vn = W.make_new_kv(w, step)
        gc.append_kv(to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    torch.cuda.synchronize()
    # sequence 0: token 255 fits block 1, tokens 256 and 257 need block 2 (entry 9): dropped
    assert list(gc.seq_lens.cpu().numpy()) == [256, 203] and int(gc.status.item()) == 2
    gc.status.zero_()
    gc.block_table.copy_(torch.from_numpy(np.array([[77, 1, 2], [0, 2, 1]], np.int32)))
    out = torch.empty((2, Hq, 128), dtype=torch.bfloat16, device="cuda:0")
    gc.decode_attn(to_dev(W.make_q(w), "bf16"), W.softmax_scale(w), out, 2)
    torch.cuda.synchronize()
    assert int(gc.status.item()) == 1 and torch.isfinite(out.float()).all()
    # sequence 1 has only good entries: its output is the oracle's after the same three appends
    for step in range(3):
        kn, vn = W.make_new_kv(w, step)
        oc._store_token(1, int(oc.seq_lens[1]), kn[1], vn[1]); oc.seq_lens[1] += 1
    ref = O.decode_attn(oc, W.make_q(w), W.softmax_scale(w), units=[(1, 0)])
    got = _paged_f32(gc, lambda o: gc.decode_attn(to_dev(W.make_q(w), "bf16"), W.softmax_scale(w), o, 2), (2, Hq, 128))
    assert_attn_close(got, ref, "mx paged, bad table, sequence 1 (fp32 out)")
    _half_is_rounded_f32(out_to_f64(out)[1:], got[1:], "mx paged, bad table")


def test_paged_mx_long_batch_all_units():
    """cfg4 head geometry (g_q = 4), lengths to just over 16K on scattered pages, split factor as
    the library picks it; every unit against the oracle."""
    lens = [16384 + 5, 4096, 100]
    H, Hq = 8, 32
    max_pages = 130
    oc, gc, _ = _paged_mx_pair(lens, H, Hq, num_pages=len(lens) * max_pages + 3, max_pages=max_pages, seed=93)
    w = W.scaled(W.CONFIGS["cfg4"], batch=len(lens), seed=94)
    kn, vn = W.make_new_kv(w, 0)
    oc.append_kv(kn, vn)
    gc.append_kv(to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    shape = B.bd_cache(len(lens), Hq, H, 128, B.BD_FMT_MXFP4, 128 * max_pages, None, None, None, None, None, None)
    ns = B.bd_choose_splits(shape, 16384)
    import torch
    out = torch.empty((len(lens), Hq, 128), dtype=torch.bfloat16, device="cuda:0")
    q = W.make_q(w, 1)
    gc.decode_attn(to_dev(q, "bf16"), W.softmax_scale(w), out, ns)
    got = _paged_f32(gc, lambda o: gc.decode_attn(to_dev(q, "bf16"), W.softmax_scale(w), o, ns), (len(lens), Hq, 128))
    ref = O.decode_attn(oc, q, W.softmax_scale(w))          # every (sequence, KV head) unit
    assert_attn_close(got, ref, "mx paged long (fp32 out)")
    _half_is_rounded_f32(out_to_f64(out), got, "mx paged long")
    assert list(gc.seq_lens.cpu().numpy()) == [L + 1 for L in lens] and int(gc.status.item()) == 0


@pytest.mark.parametrize("fmt", ["int4", "int2", "mxfp4", "int4_g32", "int2_g64", "int4_kt_g32", "int2_kt_g64"])
def test_paged_fused_step_equals_append_then_attention(fmt):
    """bd_paged_decode_step against bd_paged_append_kv + bd_paged_decode_attn on a twin cache:
    outputs, pool bytes and lengths identical bit for bit over steps that cross block
    boundaries, including a sequence whose next page is missing (its token is dropped, it
    attends what it had, bit 1 of the status word); and against the oracle."""
    import torch
    mx = fmt == "mxfp4"
    dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
    H, Hq = 2, 8
    lens = [126, 0, 300, 255]
    table = np.random.default_rng(8).permutation(40)[:4 * 6].reshape(4, 6).astype(np.int32)
    twins = []
    for _ in range(2):
        if mx:
            oc, gc, _ = _paged_mx_pair(lens, H, Hq, num_pages=40, max_pages=6, table=table)
        else:
            oc, gc, _ = _paged_pair(fmt, lens, H, Hq, num_pages=40, max_pages=6, table=table)
        twins.append(gc)
    bad = table.copy(); bad[3, 2] = -5          # sequence 3 (255 tokens) has no page for its third block
    for gc in twins:
        gc.block_table.copy_(torch.from_numpy(bad))
    a, b = twins
    w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=4, n_q_heads=Hq, n_kv_heads=H, context=128, seed=61)
    if mx:      # fp32 output rows: the bar of the oracle applies to them as it stands (bf16 rows: the other step tests)
        a.desc.out_type = b.desc.out_type = B.BD_OUT_F32
        tdt = torch.float32
    outs = [torch.empty((4, Hq, 128), dtype=tdt, device="cuda:0") for _ in range(2)]
    for step in range(5):
        kn, vn, q = (to_dev(x, dt) for x in (*W.make_new_kv(w, step), W.make_q(w, step)))
        ns = (1, 3, 2, 5, 4)[step]
        a.decode_step(kn, vn, q, W.softmax_scale(w), outs[0], ns)
        b.append_kv(kn, vn)
        b.decode_attn(q, W.softmax_scale(w), outs[1], ns)
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int32 if mx else torch.int16), outs[1].view(torch.int32 if mx else torch.int16)), step
        assert torch.equal(a.seq_lens, b.seq_lens), step
    # int formats drop sequence 3's token only when it would fill the residual (token 384 never arrives);
    # MXFP4 needs the page from token 257 on
    assert list(a.seq_lens.cpu().numpy()) == ([131, 5, 305, 256] if mx else [131, 5, 305, 260])
    assert int(a.status.item()) == int(b.status.item()) == (2 if mx else 0)
    for i in range(4 if mx else 6):
        assert torch.equal(a.buffers[i], b.buffers[i]), i
    # against the oracle (sequences 0..2, whose tables are intact)
    for step in range(5):
        kn, vn = W.make_new_kv(w, step)
        for s_ in range(3):
            if mx:
                oc._store_token(s_, int(oc.seq_lens[s_]), kn[s_], vn[s_]); oc.seq_lens[s_] += 1
        if not mx:
            oc.append_kv(kn, vn)
    ref = O.decode_attn(oc, W.make_q(w, 4), W.softmax_scale(w), units=[(s_, h) for s_ in range(3) for h in range(H)])
    assert_attn_close(out_to_f64(outs[0]), ref, f"{fmt} paged fused step", large_outputs=True)


@pytest.mark.parametrize("fmt", ["int4", "int2_kt", "int4_g32", "mxfp4"])
def test_paged_fused_step_drops_the_token_that_has_no_page(fmt):
    """A sequence whose residual the step's token would fill (integer formats), or whose token starts a new
    block (MXFP4), while the table names no page for that block: the token is dropped, the length stays,
    the sequence attends what it had, bit 1 of the status word is set -- the same, bit for bit, from
    bd_paged_decode_step (which appends inside the attention launch for the main integer kernel) and from
    bd_paged_append_kv + bd_paged_decode_attn; the other sequences go on."""
    import torch
    mx = fmt == "mxfp4"
    dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
    H, Hq = 2, 8
    lens = [255, 130, 127] if not mx else [256, 130, 127]
    table = np.random.default_rng(9).permutation(30)[:3 * 5].reshape(3, 5).astype(np.int32)
    twins = []
    for _ in range(2):
        if mx:
            _, gc, _ = _paged_mx_pair(lens, H, Hq, num_pages=30, max_pages=5, table=table)
        else:
            _, gc, _ = _paged_pair(fmt, lens, H, Hq, num_pages=30, max_pages=5, table=table)
        twins.append(gc)
    bad = table.copy(); bad[0, 2 if mx else 1] = 77          # out of the pool: sequence 0 cannot take its next token
    for gc in twins:
        gc.block_table.copy_(torch.from_numpy(bad))
    a, b = twins
    w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=3, n_q_heads=Hq, n_kv_heads=H, context=128, seed=62)
    outs = [torch.empty((3, Hq, 128), dtype=tdt, device="cuda:0") for _ in range(2)]
    for step in range(3):
        kn, vn, q = (to_dev(x, dt) for x in (*W.make_new_kv(w, step), W.make_q(w, step)))
        ns = (2, 1, 3)[step]
        a.decode_step(kn, vn, q, W.softmax_scale(w), outs[0], ns)
        b.append_kv(kn, vn)
        b.decode_attn(q, W.softmax_scale(w), outs[1], ns)
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), step
        assert torch.equal(a.seq_lens, b.seq_lens), step
        assert list(a.seq_lens.cpu().numpy()) == [lens[0], lens[1] + step + 1, lens[2] + step + 1]
        assert int(a.status.item()) == int(b.status.item()) == 2
    for i in range(4 if mx else 6):
        assert torch.equal(a.buffers[i], b.buffers[i]), i


@pytest.mark.parametrize("fmt", ["int4", "int2_kt", "int4_g32", "mxfp4"])
def test_paged_fused_step_on_the_filling_step_for_any_split(fmt):
    """The step that fills a residual (or, MXFP4, lands anywhere in a block) is quantized inside the attention
    launch by the workgroup that reads that block -- whichever split that is: sequences whose next block has
    index 0, 3, 4, 6 and 9, split counts 1 to 8; two steps (the fill, and the step after it) against
    append + attention on a twin, bit for bit, pool included."""
    import torch
    mx = fmt == "mxfp4"
    dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
    H, Hq = 2, 8
    lens = [127, 128 * 3 + 127, 128 * 4 + 127, 128 * 6 + 127, 128 * 9 + 127, 128 * 2 + 5]
    for ns in (1, 2, 3, 5, 8):
        table = np.random.default_rng(20 + ns).permutation(80)[:6 * 12].reshape(6, 12).astype(np.int32)
        twins = []
        for _ in range(2):
            if mx:
                _, gc, _ = _paged_mx_pair(lens, H, Hq, num_pages=80, max_pages=12, table=table)
            else:
                _, gc, _ = _paged_pair(fmt, lens, H, Hq, num_pages=80, max_pages=12, table=table)
            twins.append(gc)
        a, b = twins
        w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=6, n_q_heads=Hq, n_kv_heads=H, context=128, seed=63 + ns)
        outs = [torch.empty((6, Hq, 128), dtype=tdt, device="cuda:0") for _ in range(2)]
        for step in range(2):
            kn, vn, q = (to_dev(x, dt) for x in (*W.make_new_kv(w, step), W.make_q(w, step)))
            a.decode_step(kn, vn, q, W.softmax_scale(w), outs[0], ns)
            b.append_kv(kn, vn)
            b.decode_attn(q, W.softmax_scale(w), outs[1], ns)
            torch.cuda.synchronize()
            assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), (ns, step)
            assert torch.equal(a.seq_lens, b.seq_lens), (ns, step)
        assert list(a.seq_lens.cpu().numpy()) == [L + 2 for L in lens] and int(a.status.item()) == 0
        for i in range(4 if mx else 6):
            assert torch.equal(a.buffers[i], b.buffers[i]), (ns, i)


# ---------------------------------------------------------------------------- quantization groups of 32 / 64

@pytest.mark.parametrize("fmt", GROUP_FORMATS)
@pytest.mark.parametrize("L", [128 * 5 + 37, 128 * 3, 90])
def test_group_quant_pack_bit_exact(fmt, L):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=8, n_kv_heads=2, context=L, fmt=fmt)
    _, _, oc, gc = _int_cache_pair(w, 1024)
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", GROUP_FORMATS)
def test_group_quant_adversarial_and_append_bit_exact(fmt):
    """Constant groups next to live ones, extremes, subnormals and exact ties inside single 32- and
    64-groups; then appends across a flush."""
    rng = np.random.default_rng(6)
    K = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    V = rng.standard_normal((1, 2, 200, 128)).astype(np.float16)
    K[0, 0, 32:64, 3] = 1.5                      # one constant 32-group of a channel
    K[0, 0, 64:128, 4] = -0.0
    K[0, 0, 0, 5] = 65504; K[0, 0, 33, 5] = -65504
    K[0, 0, 96:128, 6] = (rng.integers(0, 4, 32) * 6e-8).astype(np.float16)
    K[0, 0, 0:32, 7] = np.array([0, 15] + [2.5, 3.5, 0.5, 1.5] * 7 + [7, 7], np.float16)
    V[0, 1, 7, 32:64] = -2.25
    V[0, 1, 8, 0] = 65504; V[0, 1, 8, 70] = -65504
    V[0, 1, 9, 64:128] = (rng.integers(0, 3, 64) * 6e-8).astype(np.float16)
    V[0, 1, 10, 96:128] = np.array([0, 3] + [0.5, 1.5, 2.5, 1.0] * 7 + [2, 2], np.float16)
    K[0, 1, 7:11] = V[0, 1, 7:11]               # (the same rows for per-token K groups)
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=2, n_kv_heads=2, context=200, fmt=fmt, seed=9)
    oc = O.IntCache(1, 2, BITS[fmt], 384, k_per_token="_kt" in fmt, group=GROUP[fmt]); oc.quant_pack_kv(K, V)
    gc = B.KVCache(1, 2, 2, fmt, 384); gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    _assert_int_cache_equal(oc, gc)
    for i in range(60):
        kn, vn = W.make_new_kv(w, i)
        oc.append_kv(kn, vn)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    assert (gc.packed_len, gc.res_len) == (256, 4)
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", GROUP_FORMATS)
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (5, 1), (16, 2), (12, 1)])
def test_group_decode_matches_oracle(fmt, hq, hkv):
    """Attention over caches with 32- and 64-groups: several blocks per wave, a ragged residual,
    split factors from 1 to more than there are blocks, then decode steps across a flush."""
    import torch
    L = 128 * 9 + 101
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=hq, n_kv_heads=hkv, context=L, fmt=fmt, seed=70 + hq)
    K, V, oc, gc = _int_cache_pair(w, 128 * 12)
    q = W.make_q(w)
    ref = O.decode_attn(oc, q, W.softmax_scale(w))
    for ns in (1, 2, 3, 9, 14, gc.choose_splits()):
        # (outputs on the x10 outlier channels reach magnitudes where half an fp16 step is 2e-3)
        assert_attn_close(_decode(gc, w, q, num_splits=ns), ref, f"{fmt} {hq}/{hkv} splits={ns}", large_outputs=True)
    out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
    for step in range(30):                      # residual 101 -> 127 -> flush -> 3
        kn, vn = W.make_new_kv(w, step)
        q = W.make_q(w, step + 1)
        oc.append_kv(kn, vn)
        gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=4)
        if step in (0, 25, 26, 27, 29):
            torch.cuda.synchronize()
            assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} step {step}",
                              large_outputs=True)
    assert (gc.packed_len, gc.res_len) == (128 * 10, 3)
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", ["int4_g32", "int2_g64"])
def test_group_decode_short_and_empty(fmt):
    import torch
    for L in (0, 5, 128, 200):
        w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=4, n_kv_heads=1, context=max(L, 1), fmt=fmt, seed=80)
        K, V = W.make_kv(w)
        K, V = np.ascontiguousarray(K[:, :, :L]), np.ascontiguousarray(V[:, :, :L])
        oc = O.IntCache(1, 1, BITS[fmt], 256, k_per_token="_kt" in fmt, group=GROUP[fmt]); oc.quant_pack_kv(K, V)
        gc = B.KVCache(1, 4, 1, fmt, 256); gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
        q = W.make_q(w)
        got = _decode(gc, w, q, num_splits=2)
        if L == 0:
            assert not got.any()
        else:
            assert_attn_close(got, O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} L={L}", large_outputs=True)


@pytest.mark.parametrize("fmt", ["int4_g32", "int4_kt_g32"])
def test_group_full_size_32k_sampled_heads(fmt):
    """cfg1's shape with 32-groups (K channel-wise and per token), split factor as the library picks it; two KV
    heads against the oracle."""
    w = W.scaled(W.CONFIGS["cfg1"], fmt=fmt, context=32768 + 77)
    K, V = W.make_kv(w)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, 32768 + 128)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    q = W.make_q(w)
    got = _decode(gc, w, q)
    for h in (0, 5):
        oc = O.IntCache(1, 1, 4, 32768 + 128, k_per_token="_kt" in fmt, group=32)
        oc.quant_pack_kv(K[:, h:h + 1], V[:, h:h + 1])
        ref = O.decode_attn(oc, q[:, 4 * h:4 * h + 4], W.softmax_scale(w))
        assert_attn_close(got[:, 4 * h:4 * h + 4], ref, f"{fmt} 32K head {h}")


@pytest.mark.parametrize("fmt", ["int4", "mxfp4"])
def test_paged_step_replays_from_one_captured_graph(fmt):
    """Lengths and the flush decision live on the device, so ONE captured bd_paged_decode_step serves
    every later step: the graph is replayed with new inputs copied into its static buffers (eager
    copies and synchronizations between the replays), across a block boundary, and every replay is
    checked against the oracle.  The library enqueues kernels only (no memset or copy nodes)."""
    import torch
    mx = fmt == "mxfp4"
    dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
    H, Hq, lens = 2, 8, [125, 300, 5]
    if mx:
        oc, gc, _ = _paged_mx_pair(lens, H, Hq, num_pages=30, max_pages=5)
    else:
        oc, gc, _ = _paged_pair(fmt, lens, H, Hq, num_pages=30, max_pages=5)
    w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=3, n_q_heads=Hq, n_kv_heads=H, context=128, seed=88)
    kn_s = torch.zeros((3, H, 128), dtype=tdt, device="cuda:0")
    vn_s, q_s = torch.zeros_like(kn_s), torch.zeros((3, Hq, 128), dtype=tdt, device="cuda:0")
    if mx:      # fp32 output rows, which the oracle's bar applies to as it stands
        gc.desc.out_type = B.BD_OUT_F32
    out_s = torch.zeros((3, Hq, 128), dtype=torch.float32 if mx else tdt, device="cuda:0")
    gc.workspace(3)                                   # allocated before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gc.decode_step(kn_s, vn_s, q_s, W.softmax_scale(w), out_s, 3)
    torch.cuda.synchronize()
    assert list(gc.seq_lens.cpu().numpy()) == lens    # capturing runs nothing
    for step in range(6):                             # sequence 0 fills its block at step 2
        kn, vn = W.make_new_kv(w, step)
        q = W.make_q(w, step)
        kn_s.copy_(to_dev(kn, dt)); vn_s.copy_(to_dev(vn, dt)); q_s.copy_(to_dev(q, dt))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        oc.append_kv(kn, vn)
        ref = O.decode_attn(oc, q, W.softmax_scale(w))
        assert_attn_close(out_to_f64(out_s), ref, f"{fmt} replay {step}", large_outputs=True)
        assert list(gc.seq_lens.cpu().numpy()) == [L + step + 1 for L in lens]
    assert int(gc.status.item()) == 0
    if mx:
        _assert_paged_mx_equal(oc, gc, "after replays")
    else:
        _assert_paged_equal(oc, gc, "after replays")


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_kt", "int2_kt"] + GROUP_FORMATS)
@pytest.mark.parametrize("gq", [4, 8, 16])
def test_outputs_do_not_depend_on_the_magnitude_of_k_and_v(fmt, gq):
    """K, V (and Q, inversely, so that the logits stay those of the unit-variance case) scaled by 2^-10 and
    2^10: the fp16 operands of the matrix unit are normalised inside the kernel, so the relative error stays
    where it is at unit scale (the same 1e-3 relative L2; the max-abs bar scales with the outputs)."""
    import torch
    w = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=gq * 2, n_kv_heads=2, context=128 * 33 + 70, fmt=fmt, seed=77)
    K0, V0 = W.make_kv(w)
    q0 = W.make_q(w)
    for ks, vs in [(2.0 ** -10, 2.0 ** -10), (2.0 ** 10, 2.0 ** -10), (2.0 ** -10, 2.0 ** 10), (1.0, 2.0 ** -14), (2.0 ** 10, 2.0 ** 10)]:
        K = (K0.astype(np.float32) * np.float32(min(ks, 2.0 ** 10 / 10))).astype(np.float16)   # (x10 outlier channels: keep fp16 finite)
        V = (V0.astype(np.float32) * np.float32(min(vs, 2.0 ** 10 / 10))).astype(np.float16)
        q = (q0.astype(np.float32) / np.float32(min(ks, 2.0 ** 10 / 10))).astype(np.float16)
        if fmt in GROUP:
            # one channel group of V far smaller than the others, and for a stretch of the sequence smaller still
            V[..., 32:64] = (V[..., 32:64].astype(np.float32) * np.float32(2.0 ** -6)).astype(np.float16)
            V[:, :, :900, 32:64] = (V[:, :, :900, 32:64].astype(np.float32) * np.float32(2.0 ** -4)).astype(np.float16)
        oc = O.IntCache(w.batch, w.n_kv_heads, BITS[fmt], 128 * 35, k_per_token="_kt" in fmt,
                        group=GROUP.get(fmt, 128))
        oc.quant_pack_kv(K, V)
        gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, 128 * 35)
        gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
        _assert_int_cache_equal(oc, gc)
        ref = O.decode_attn(oc, q, W.softmax_scale(w))
        gc.desc.out_type = B.BD_OUT_F32          # (fp16 output rows would underflow at the small scales)
        for ns in (1, 5):
            out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
            gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns)
            torch.cuda.synchronize()
            got = out_to_f64(out)
            rl = np.linalg.norm(got - ref) / np.linalg.norm(ref)
            ma = np.abs(got - ref).max() / np.abs(ref).max()
            assert rl <= 1e-3 and ma <= 2e-3, f"{fmt} gq={gq} K x {ks} V x {vs} splits {ns}: rel-L2 {rl:.2e}, max-abs / max |ref| {ma:.2e}"
            if GROUP.get(fmt) == 32 and np.linalg.norm(ref[..., 32:64]) > 0:
                # the small channel group on its own: its P' is normalised against its own scales
                rg = np.linalg.norm((got - ref)[..., 32:64]) / np.linalg.norm(ref[..., 32:64])
                assert rg <= 1e-3, f"{fmt} gq={gq} K x {ks} V x {vs} splits {ns}: channels 32..63 rel-L2 {rg:.2e}"


@pytest.mark.parametrize("gq", [4, 8, 16])
def test_mx_outputs_do_not_depend_on_the_magnitude_of_k_and_v(gq):
    """MXFP4: K, V scaled by 2^-30 .. 2^30 (and Q inversely): the probabilities meet V's block exponents
    relative to a running exponent, so the error relative to the outputs stays where it is at unit scale."""
    import torch
    w = W.scaled(W.CONFIGS["cfg4"], batch=1, n_q_heads=gq * 2, n_kv_heads=2, context=128 * 20 + 70, seed=79)
    K0, V0 = W.make_kv(w)
    q0 = W.make_q(w)
    for ks, vs in [(2.0 ** -30, 2.0 ** -30), (2.0 ** 20, 2.0 ** -20), (2.0 ** -10, 2.0 ** 30), (1.0, 2.0 ** 20)]:
        K, V, q = (W.round_to_bf16(x) for x in (K0 * np.float32(ks), V0 * np.float32(vs), q0 / np.float32(ks)))
        # (one stretch of the sequence far smaller than the rest: the running exponent has to grow on the way)
        V[:, :, :700] = W.round_to_bf16(V[:, :, :700] * np.float32(2.0 ** -12))
        oc = O.MxCache(w.batch, w.n_kv_heads, 128 * 22)
        oc.quant_pack_kv(K, V)
        gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, "mxfp4", 128 * 22)
        gc.quant_pack_kv(to_dev(K, "bf16"), to_dev(V, "bf16"))
        _assert_mx_cache_equal(oc, gc)
        ref = O.decode_attn(oc, q, W.softmax_scale(w))
        gc.desc.out_type = B.BD_OUT_F32
        for ns in (1, 5):
            out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
            gc.decode_attn(to_dev(q, "bf16"), W.softmax_scale(w), out, num_splits=ns)
            torch.cuda.synchronize()
            got = out_to_f64(out)
            rl = np.linalg.norm(got - ref) / np.linalg.norm(ref)
            ma = np.abs(got - ref).max() / np.abs(ref).max()
            assert rl <= 1e-3 and ma <= 2e-3, f"mxfp4 gq={gq} K x {ks} V x {vs} splits {ns}: rel-L2 {rl:.2e}, max-abs / max |ref| {ma:.2e}"


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_kt", "int4_g32", "int2_g64", "int4_kt_g64", "mxfp4"])
def test_peaked_and_flat_attention(fmt):
    """Queries scaled by 6 (logits of several tens: a handful of tokens take all the weight and the
    running maximum moves across blocks and splits; much larger logits only test the conditioning of
    softmax itself, an fp32 rounding of a logit of 400 moves a weight by 1e-3) and by 1e-3
    (uniform weights over 1500 tokens)."""
    import torch
    mx = fmt == "mxfp4"
    base = "cfg4" if mx else "cfg1"
    L = 128 * 11 + 93
    w = W.scaled(W.CONFIGS[base], batch=2, n_q_heads=8, n_kv_heads=2, context=L, fmt=fmt, seed=123)
    if mx:
        K, V, oc, gc = _mx_pair(w, 128 * 13)
    else:
        K, V, oc, gc = _int_cache_pair(w, 128 * 13)
    for factor in (6.0, 1e-3):
        q = W.make_q(w, 3) * np.float32(factor)
        q = W.round_to_bf16(q) if mx else q.astype(np.float16)
        ref = O.decode_attn(oc, q, W.softmax_scale(w))
        for ns in (1, 4, 12):
            if mx:
                _mx_decode_check(gc, ref, w, q, ns, f"mx q x {factor} splits {ns}")
            else:
                assert_attn_close(_decode(gc, w, q, num_splits=ns), ref, f"{fmt} q x {factor} splits {ns}", large_outputs=True)


@pytest.mark.parametrize("fmt", ["int4", "int2_kt", "int4_g32", "mxfp4"])
@pytest.mark.parametrize("L", [128 * 5 + 77, 0])
def test_one_split_writes_the_output_directly(fmt, L):
    """With one split the attention kernel stores the output itself and no merge kernel runs: bit for
    bit the values the merge kernel computes from that split's partials."""
    import torch
    mx = fmt == "mxfp4"
    w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=3, n_q_heads=12, n_kv_heads=2, context=L, fmt=fmt, seed=17)
    K, V, oc, gc = (_mx_pair(w, 1024) if mx else _int_cache_pair(w, 1024))
    dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
    q = to_dev(W.make_q(w), dt)
    direct = torch.full((3, 12, 128), 3.0, dtype=tdt, device="cuda:0")
    merged = torch.full((3, 12, 128), 5.0, dtype=tdt, device="cuda:0")
    ws = gc.workspace(1)
    B.bd_decode_attn(gc.desc, q, gc.packed_len, gc.res_len, W.softmax_scale(w), 1, ws, direct)
    B.bd_decode_attn(gc.desc, q, gc.packed_len, gc.res_len, W.softmax_scale(w), 1, ws, None)
    B.bd_splitk_combine(gc.desc, ws, 1, merged)
    torch.cuda.synchronize()
    assert torch.equal(direct.view(torch.int16), merged.view(torch.int16))
    if L == 0:
        assert not direct.float().abs().sum().item()


# ---------------------------------------------------------------------------- query groups

@pytest.mark.parametrize("fmt", ["int4", "int2"])
@pytest.mark.parametrize("gq", [1, 3, 5, 8, 12, 16, 20, 32, 40])
def test_query_group_sizes(fmt, gq):
    """Any number of query heads per KV head (Sec. IV-A: the group forms the N dimension of the
    matrix instructions; beyond 16 heads the group is taken 16 at a time): short context (one block per wave) and longer (several), with a
    residual tail, several split factors, and the fused step."""
    import torch
    H = 2
    for L, ns in [(128 * 3 + 70, 2), (128 * 41 + 5, 3)]:
        w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=gq * H, n_kv_heads=H, context=L, fmt=fmt, seed=40 + gq)
        K, V, oc, gc = _int_cache_pair(w, (L // 128 + 2) * 128)
        out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
        q = W.make_q(w)
        gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns)
        torch.cuda.synchronize()
        assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} gq={gq} L={L}",
                          large_outputs=True)
        kn, vn = W.make_new_kv(w, 0)
        q = W.make_q(w, 1)
        oc.append_kv(kn, vn)
        gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns)
        torch.cuda.synchronize()
        assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} gq={gq} L={L} step",
                          large_outputs=True)


@pytest.mark.parametrize("Hq", [16, 48])
def test_paged_with_larger_query_groups(Hq):
    import torch
    lens = [700, 129, 3000]
    H = 2
    oc, gc, _ = _paged_pair("int4", lens, H, Hq, num_pages=80, max_pages=25, seed=55)
    w = W.scaled(W.CONFIGS["cfg1"], batch=len(lens), n_q_heads=Hq, n_kv_heads=H, context=128, seed=56)
    out = torch.empty((len(lens), Hq, 128), dtype=torch.float16, device="cuda:0")
    q = W.make_q(w)
    gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, 4)
    torch.cuda.synchronize()
    assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"paged gq={Hq // 2}", large_outputs=True)


# ---------------------------------------------------------------------------- per-token K (KT)

@pytest.mark.parametrize("fmt", ["int4_kt", "int2_kt"])
@pytest.mark.parametrize("L", [128 * 5 + 37, 128 * 3, 90])
def test_kt_quant_pack_bit_exact(fmt, L):
    w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=8, n_kv_heads=2, context=max(L, 1), fmt=fmt, seed=61)
    K, V, oc, gc = _int_cache_pair(w, 1024)
    _assert_int_cache_equal(oc, gc)


@pytest.mark.parametrize("fmt", ["int4_kt", "int2_kt"])
@pytest.mark.parametrize("gq", [4, 8])
def test_kt_decode_and_steps_match_oracle(fmt, gq):
    """Per-token K: short (one block per wave) and longer contexts, residual tail, fused steps
    over a flush (bit-exact cache afterwards), several split factors."""
    import torch
    H = 2
    for L, ns in [(128 * 4 + 125, 2), (128 * 37 + 5, 3), (128 * 37 + 5, 1)]:
        w = W.scaled(W.CONFIGS["cfg1"], batch=2, n_q_heads=gq * H, n_kv_heads=H, context=L, fmt=fmt, seed=62)
        K, V, oc, gc = _int_cache_pair(w, (L // 128 + 2) * 128)
        out = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
        q = W.make_q(w)
        gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns)
        torch.cuda.synchronize()
        assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), f"{fmt} gq={gq} L={L} ns={ns}",
                          large_outputs=True)
        for step in range(4):
            kn, vn = W.make_new_kv(w, step)
            q = W.make_q(w, step + 1)
            oc.append_kv(kn, vn)
            gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out,
                           num_splits=ns)
            torch.cuda.synchronize()
            assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)),
                              f"{fmt} gq={gq} L={L} step {step}", large_outputs=True)
        _assert_int_cache_equal(oc, gc)


def test_kt_full_size_32k_sampled_heads():
    """cfg1's shape with per-token K: 32K context + residual, all 8 KV heads on the GPU, 3 of them
    through the oracle."""
    import torch
    w = W.scaled(W.CONFIGS["cfg1"], fmt="int4_kt", context=32768 + 77, seed=63)
    K, V = W.make_kv(w)
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, 32768 + 256)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    q = W.make_q(w)
    out = torch.empty((1, 32, 128), dtype=torch.float16, device="cuda:0")
    gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out)
    torch.cuda.synchronize()
    got = out_to_f64(out)
    for h in (0, 3, 7):
        oc = O.IntCache(1, 1, 4, 32768 + 256, k_per_token=True)
        oc.quant_pack_kv(K[:, h:h + 1], V[:, h:h + 1])
        ref = O.decode_attn(oc, q[:, 4 * h:4 * h + 4], W.softmax_scale(w))
        assert_attn_close(got[:, 4 * h:4 * h + 4], ref, f"kt 32K head {h}")


def test_paged_kt():
    import torch
    lens = [700, 129, 1500]
    H, Hq = 2, 8
    rng = np.random.default_rng(3)
    table = rng.permutation(60)[:3 * 14].reshape(3, 14).astype(np.int32)
    oc = O.PagedIntCache(3, H, 4, 60, 14, table, k_per_token=True)
    gc = B.PagedKVCache(3, Hq, H, "int4_kt", 60, table)
    for b, L in enumerate(lens):
        w1 = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=Hq, n_kv_heads=H, context=L, seed=70 + b)
        K, V = W.make_kv(w1)
        K, V = np.ascontiguousarray(K[0]), np.ascontiguousarray(V[0])
        oc.quant_pack_kv(b, K, V)
        gc.quant_pack_kv(b, to_dev(K, "fp16"), to_dev(V, "fp16"))
    w = W.scaled(W.CONFIGS["cfg1"], batch=3, n_q_heads=Hq, n_kv_heads=H, context=128, seed=75)
    for step in range(130):        # every sequence crosses a flush
        kn, vn = W.make_new_kv(w, step)
        oc.append_kv(kn, vn)
        gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
    _assert_paged_equal(oc, gc, "paged kt")
    out = torch.empty((3, Hq, 128), dtype=torch.float16, device="cuda:0")
    q = W.make_q(w)
    gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, 3)
    torch.cuda.synchronize()
    assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), "paged kt", large_outputs=True)


def test_offsets_beyond_two_gigabytes():
    """Forty sequences of 128K tokens: the packed K buffer is 2.7 GB, so byte offsets pass 2^31.  Every
    sequence holds the same tokens (the batch is one sequence repeated on the device), so every output
    row group must equal, bit for bit, the result of a one-sequence cache with the same split factor, and
    so must the last sequence's packed bytes."""
    import torch
    w1 = W.scaled(W.CONFIGS["cfg3"], seed=81)
    K, V = W.make_kv(w1)
    Kd1, Vd1 = to_dev(K, "fp16"), to_dev(V, "fp16")
    nb = 40
    ref_c = B.KVCache(1, 32, 8, "int4", 131072 + 128)
    ref_c.quant_pack_kv(Kd1, Vd1)
    big = B.KVCache(nb, 32, 8, "int4", 131072 + 128)
    assert big.sizes[0] > 2 ** 31
    big.quant_pack_kv(Kd1.expand(nb, -1, -1, -1).contiguous(), Vd1.expand(nb, -1, -1, -1).contiguous())
    q1 = to_dev(W.make_q(w1), "fp16")
    ns = 2
    o1 = torch.empty((1, 32, 128), dtype=torch.float16, device="cuda:0")
    ob = torch.empty((nb, 32, 128), dtype=torch.float16, device="cuda:0")
    ref_c.decode_attn(q1, W.softmax_scale(w1), o1, num_splits=ns)
    big.decode_attn(q1.expand(nb, -1, -1).contiguous(), W.softmax_scale(w1), ob, num_splits=ns)
    torch.cuda.synchronize()
    assert torch.equal(ob.view(torch.int16), o1.view(torch.int16).expand(nb, -1, -1))
    per_seq = ref_c.sizes[0]
    assert torch.equal(big.buffers[0][(nb - 1) * per_seq: nb * per_seq], ref_c.buffers[0][:per_seq])
    per_seq = ref_c.sizes[1]
    assert torch.equal(big.buffers[1][(nb - 1) * per_seq: nb * per_seq], ref_c.buffers[1][:per_seq])


def test_seeded_shape_sweep():
    """Forty seeded random shapes (format, heads per group, batch, KV heads, length, split factor,
    fused or separate step): packed bytes bit-exact, outputs within tolerance."""
    import torch
    rng = np.random.default_rng(2024)
    fmts = ["int4", "int2", "int4_kt", "int2_kt"]
    for case in range(40):
        fmt = fmts[int(rng.integers(4))]
        gq = int(rng.integers(1, 17))
        H = int(rng.integers(1, 4))
        Bn = int(rng.integers(1, 4))
        L = int(rng.integers(1, 128 * 24))
        ns = int(rng.integers(1, 12))
        w = W.scaled(W.CONFIGS["cfg1"], batch=Bn, n_q_heads=gq * H, n_kv_heads=H, context=L, fmt=fmt, seed=1000 + case)
        K, V, oc, gc = _int_cache_pair(w, (L // 128 + 2) * 128)
        _assert_int_cache_equal(oc, gc)
        out = torch.empty((Bn, gq * H, 128), dtype=torch.float16, device="cuda:0")
        what = f"case {case}: {fmt} gq={gq} H={H} B={Bn} L={L} ns={ns}"
        for step in range(2):
            kn, vn = W.make_new_kv(w, step)
            q = W.make_q(w, step)
            oc.append_kv(kn, vn)
            if (case + step) % 2:
                gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out,
                               num_splits=ns)
            else:
                gc.append_kv(to_dev(kn, "fp16"), to_dev(vn, "fp16"))
                gc.decode_attn(to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns, fused=bool(case % 3))
            torch.cuda.synchronize()
            assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), what, large_outputs=True)
        _assert_int_cache_equal(oc, gc)


def test_seeded_shape_sweep_groups_and_large_query_groups():
    """Twenty more seeded shapes over the formats with quantization groups of 64 / 32 and over query
    groups of up to 40 heads."""
    import torch
    rng = np.random.default_rng(2025)
    fmts = GROUP_FORMATS + ["int4", "int2_kt"]
    for case in range(20):
        fmt = fmts[int(rng.integers(len(fmts)))]
        gq = int(rng.integers(1, 41))
        H = int(rng.integers(1, 3))
        Bn = int(rng.integers(1, 3))
        L = int(rng.integers(1, 128 * 20))
        ns = int(rng.integers(1, 12))
        w = W.scaled(W.CONFIGS["cfg1"], batch=Bn, n_q_heads=gq * H, n_kv_heads=H, context=L, fmt=fmt, seed=3000 + case)
        K, V, oc, gc = _int_cache_pair(w, (L // 128 + 2) * 128)
        _assert_int_cache_equal(oc, gc)
        out = torch.empty((Bn, gq * H, 128), dtype=torch.float16, device="cuda:0")
        what = f"case {case}: {fmt} gq={gq} H={H} B={Bn} L={L} ns={ns}"
        for step in range(2):
            kn, vn = W.make_new_kv(w, step)
            q = W.make_q(w, step)
            oc.append_kv(kn, vn)
            gc.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out, num_splits=ns)
            torch.cuda.synchronize()
            assert_attn_close(out_to_f64(out), O.decode_attn(oc, q, W.softmax_scale(w)), what, large_outputs=True)
        _assert_int_cache_equal(oc, gc)


def test_seeded_paged_sweep():
    """Eighteen seeded paged shapes (format incl. MXFP4 and smaller quantization groups, batch, heads, ragged lengths incl. empty
    sequences, scattered pages, split factor; fused step or append + attention)."""
    import torch
    rng = np.random.default_rng(2026)
    fmts = ["int4", "int2", "int4_kt", "mxfp4", "int4_g64", "int2_g32"]
    for case in range(18):
        fmt = fmts[case % 6]
        mx = fmt == "mxfp4"
        dt, tdt = ("bf16", torch.bfloat16) if mx else ("fp16", torch.float16)
        gq = int(rng.integers(1, 13))
        H = int(rng.integers(1, 4))
        Bn = int(rng.integers(1, 5))
        lens = [int(rng.integers(0, 1500)) if rng.random() > 0.15 else 0 for _ in range(Bn)]
        ns = int(rng.integers(1, 9))
        max_pages = 14
        num_pages = Bn * max_pages + int(rng.integers(0, 9))
        if mx:
            oc, gc, _ = _paged_mx_pair(lens, H, gq * H, num_pages, max_pages, seed=4000 + case)
        else:
            table = np.random.default_rng(5000 + case).permutation(num_pages)[:Bn * max_pages].reshape(Bn, max_pages).astype(np.int32)
            oc = O.PagedIntCache(Bn, H, BITS[fmt], num_pages, max_pages, table, k_per_token="_kt" in fmt,
                                 group=GROUP.get(fmt, 128))
            gc = B.PagedKVCache(Bn, gq * H, H, fmt, num_pages, table)
            for b_, L in enumerate(lens):
                wk = W.scaled(W.CONFIGS["cfg1"], batch=1, n_q_heads=gq * H, n_kv_heads=H, context=max(L, 1), seed=4000 + case + b_)
                K, V = W.make_kv(wk)
                K, V = np.ascontiguousarray(K[0, :, :L]), np.ascontiguousarray(V[0, :, :L])
                oc.quant_pack_kv(b_, K, V)
                gc.quant_pack_kv(b_, to_dev(K, "fp16"), to_dev(V, "fp16"))
        w = W.scaled(W.CONFIGS["cfg4" if mx else "cfg1"], batch=Bn, n_q_heads=gq * H, n_kv_heads=H, context=128, seed=6000 + case)
        if mx:      # fp32 output rows, which the oracle's bar applies to as it stands
            gc.desc.out_type = B.BD_OUT_F32
        out = torch.empty((Bn, gq * H, 128), dtype=torch.float32 if mx else tdt, device="cuda:0")
        what = f"case {case}: {fmt} gq={gq} H={H} lens={lens} ns={ns}"
        for step in range(3):
            kn, vn = W.make_new_kv(w, step)
            q = W.make_q(w, step)
            oc.append_kv(kn, vn)
            if (case + step) % 2:
                gc.decode_step(to_dev(kn, dt), to_dev(vn, dt), to_dev(q, dt), W.softmax_scale(w), out, ns)
            else:
                gc.append_kv(to_dev(kn, dt), to_dev(vn, dt))
                gc.decode_attn(to_dev(q, dt), W.softmax_scale(w), out, ns)
            torch.cuda.synchronize()
            ref = O.decode_attn(oc, q, W.softmax_scale(w))
            got = out_to_f64(out)
            assert_attn_close(got, ref, what, large_outputs=True)
        assert list(gc.seq_lens.cpu().numpy()) == [L + 3 for L in lens] and int(gc.status.item()) == 0, what
        if mx:
            _assert_paged_mx_equal(oc, gc, what)
        else:
            _assert_paged_equal(oc, gc, what)


@pytest.mark.parametrize("fmt", ["int4", "int2", "mxfp4", "int4_g32"])
def test_stream_probe_reads_the_cache_and_changes_nothing(fmt):
    """bd_probe_stream_read (measurement aid): runs over an empty, a partly filled and a full cache of every format
    family and leaves every buffer as it was."""
    import torch
    w = W.scaled(W.CONFIGS["cfg4" if fmt == "mxfp4" else "cfg1"], batch=2, n_q_heads=8, n_kv_heads=2, context=128 * 5 + 9, fmt=fmt, seed=3)
    K, V = W.make_kv(w)
    dt = "bf16" if fmt == "mxfp4" else "fp16"
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, 128 * 6)
    gc.quant_pack_kv(to_dev(K, dt), to_dev(V, dt))
    before = [gc.host_buffer(i).copy() for i in range(4)]
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for pl in (0, 128, 128 * 5, 128 * 6):
        B.bd_probe_stream_read(gc.desc, pl, sink)
    torch.cuda.synchronize()
    for i in range(4):
        assert np.array_equal(before[i], gc.host_buffer(i))
    with pytest.raises(B.BitDecodeError):
        B.bd_probe_stream_read(gc.desc, 100)


@pytest.mark.parametrize("fmt", ["int4", "int2", "int4_kt", "int4_g32", "int2_kt_g64"])
@pytest.mark.parametrize("gq", [4, 20])
def test_paged_lazy_step_attends_full_residuals_in_fp16(fmt, gq):
    """bd_paged_decode_step_lazy on a ragged batch: a sequence whose residual the step's token fills is attended
    with its 128 fp16 rows (the oracle's lazy mode), the others as in the eager step; after every step the pool,
    the residual rows in use and the lengths are the eager step's, bit for bit; steps on which no sequence fills
    give the eager step's outputs bit for bit; a sequence without a page for the block it fills drops its token."""
    import torch
    H, Hq = 2, 2 * gq
    lens = [127, 128 * 2 + 126, 40, 128 * 5 + 127, 128 + 127]
    table = np.random.default_rng(12).permutation(60)[:5 * 9].reshape(5, 9).astype(np.int32)
    oc, lz, _ = _paged_pair(fmt, lens, H, Hq, num_pages=60, max_pages=9, table=table)
    _, eg, _ = _paged_pair(fmt, lens, H, Hq, num_pages=60, max_pages=9, table=table)
    bad = table.copy(); bad[4, 1] = 99           # sequence 4 fills its residual at step 0 and has no page for the block
    for gc in (lz, eg):
        gc.block_table.copy_(torch.from_numpy(bad))
    w = W.scaled(W.CONFIGS["cfg1"], batch=5, n_q_heads=Hq, n_kv_heads=H, context=128, seed=64)
    out_l = torch.empty((5, Hq, 128), dtype=torch.float16, device="cuda:0")
    out_e = torch.empty_like(out_l)
    good = [(s_, h) for s_ in range(4) for h in range(H)]
    for step in range(3):        # step 0: sequences 0 and 3 fill (4 drops its token); step 1: sequence 1; step 2: none
        kn, vn, q = W.make_new_kv(w, step), None, W.make_q(w, step)
        kn, vn = kn
        ns = (3, 1, 4)[step]
        lz.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out_l, ns, lazy=True)
        eg.decode_step(to_dev(kn, "fp16"), to_dev(vn, "fp16"), to_dev(q, "fp16"), W.softmax_scale(w), out_e, ns)
        torch.cuda.synchronize()
        # the oracle, lazily (sequence 4 is left out: its table row is broken)
        kn4, vn4 = kn.copy(), vn.copy()
        oc_lens = oc.seq_lens.copy()
        oc.block_table[4, 1] = table[4, 1]       # (the oracle raises on a bad entry; keep its sequence 4 out of the comparison)
        oc.append_kv(kn4, vn4, flush=False)
        ref = O.decode_attn(oc, q, W.softmax_scale(w), units=good)
        oc.flush_if_full()
        got = out_to_f64(out_l)
        assert_attn_close(got[:4], ref[:4], f"{fmt} gq={gq} lazy paged step {step}", large_outputs=True)
        fills = [(int(oc_lens[b]) % 128) == 127 for b in range(5)]
        for b in range(5):
            same = torch.equal(out_l[b].view(torch.int16), out_e[b].view(torch.int16))
            if not fills[b] or b == 4:
                assert same, (step, b)           # (sequence 4's token is dropped by both: it attends what it had)
        assert torch.equal(lz.seq_lens, eg.seq_lens) and int(lz.status.item()) == int(eg.status.item()) == 2
        for i in range(4):
            assert torch.equal(lz.buffers[i], eg.buffers[i]), (step, i)
        lens_now = lz.seq_lens.cpu().numpy()
        for i in (4, 5):
            ra = lz.host_buffer(i).view(np.float16).reshape(5, H, 128, 128)
            rb = eg.host_buffer(i).view(np.float16).reshape(5, H, 128, 128)
            for b in range(5):
                r = int(lens_now[b]) % 128
                assert np.array_equal(ra[b, :, :r].view(np.uint16), rb[b, :, :r].view(np.uint16)), (step, i, b)
    assert list(lz.seq_lens.cpu().numpy()) == [130, 128 * 2 + 129, 43, 128 * 5 + 130, 128 + 127]
