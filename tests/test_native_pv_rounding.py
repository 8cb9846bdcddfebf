"""What a native low-precision second product (O = P V on the scaled fp4/fp8 matrix instruction, P re-quantized:
Sec. II Challenge 2, Sec. IV-D(2)) would do to the outputs, measured with the oracle on the CPU.

V's MX block scales run along channels, so in any formulation they are folded into the probabilities; what is
left to choose is the format P' = p * 2^(e(t, channel block) - E) is rounded to before it meets V's codes:

  fp16                      what the library's MXFP4 kernel does (V codes expanded to fp16, fp16 MFMA)
  e2m1 x 1, own block scale the paper's native route (P re-quantized to fp4)
  e4m3 x n / e2m1 x n       n pieces (each the rounded remainder, each with its own block scale per 32 tokens)

The matrix unit's cost per 128-token block and workgroup column set is 8 channel tiles x n instructions of
16 x 16 x 128; the hardware counters of the library's kernel give 32 cycles for one with an 8-bit operand and the
fp16 path's 32 instructions of 16 x 16 x 32 take 16 cycles each, i.e. 512 cycles.  The test pins the numbers that
decide the design: formats cheaper than 512 cycles (e2m1 x 1..3, e4m3 x 1) miss the parity bar (1e-3 relative
L2) by one to two orders of magnitude, and the cheapest ones that meet it (e4m3 x 2, e2m1 x 4) cost the same 512
cycles and are less accurate than fp16."""
import numpy as np

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import workloads as W

FP16 = (10, -14, 65504.0)
E4M3 = (3, -6, 448.0)
E2M1 = (1, 0, 6.0)


def round_fmt(x, mant, emin, vmax):
    """x rounded to nearest (ties to even) in a binary format with `mant` stored mantissa bits, smallest normal
    exponent emin (subnormals below it) and largest magnitude vmax (saturating)."""
    x = np.asarray(x, np.float64)
    a = np.abs(x)
    e = np.maximum(np.floor(np.log2(np.where(a > 0, a, 1.0))), emin)
    q = np.exp2(e - mant)
    return np.sign(x) * np.minimum(np.round(a / q) * q, vmax)


def pieces(x, fmt, n, top):
    """x [T] as the sum of n numbers of format fmt; every piece has its own power-of-two block scale per 32
    tokens that brings the group's largest remainder just below 2^top."""
    g = x.reshape(-1, 32)
    acc = np.zeros_like(g)
    for _ in range(n):
        rem = g - acc
        mx = np.abs(rem).max(axis=1, keepdims=True)
        sh = np.where(mx > 0, top - 1 - np.floor(np.log2(np.where(mx > 0, mx, 1.0))), 0.0)
        acc = acc + round_fmt(rem * np.exp2(sh), *fmt) * np.exp2(-sh)
    return acc.reshape(x.shape)


VARIANTS = {
    "fp16": lambda x: round_fmt(x * 2.0 ** 13, *FP16) * 2.0 ** -13,
    "e2m1x1": lambda x: pieces(x, E2M1, 1, 2),
    "e2m1x2": lambda x: pieces(x, E2M1, 2, 2),
    "e2m1x3": lambda x: pieces(x, E2M1, 3, 2),
    "e2m1x4": lambda x: pieces(x, E2M1, 4, 2),
    "e4m3x1": lambda x: pieces(x, E4M3, 1, 8),
    "e4m3x2": lambda x: pieces(x, E4M3, 2, 8),
}


def rel_l2_by_variant(context):
    w = W.scaled(W.CONFIGS["cfg4"], batch=1, n_q_heads=8, n_kv_heads=2, context=context, seed=5)
    K, V = W.make_kv(w)
    q = W.make_q(w)
    oc = O.MxCache(1, 2, context)
    oc.quant_pack_kv(K, V)
    num = {k: 0.0 for k in VARIANTS}
    den = 0.0
    for h in range(2):
        Kh, Vh = oc.dequant(0, h)
        codes = O.unpack_nibbles(oc.v_codes[0, h]).transpose(0, 2, 1).reshape(-1, 128)[:context]
        cv = O.e2m1_decode(codes)                                      # [t][c]: V = cv * 2^ex
        ex = oc.v_scales[0, h, :context].astype(np.float64) - 127.0    # [t][channel block]
        assert np.array_equal(cv * np.repeat(np.exp2(ex), 32, axis=1), Vh)
        for j in range(4):
            s = W.softmax_scale(w) * (Kh @ q[0, 4 * h + j].astype(np.float64))
            p = np.exp(s - s.max())
            ref = (p @ Vh) / p.sum()
            den += (ref ** 2).sum()
            for name, rnd in VARIANTS.items():
                out = np.empty(128)
                for cb in range(4):
                    E = ex[:, cb].max()
                    out[32 * cb:32 * cb + 32] = (rnd(p * np.exp2(ex[:, cb] - E)) @ cv[:, 32 * cb:32 * cb + 32]) * 2.0 ** E
                num[name] += ((out / p.sum() - ref) ** 2).sum()
    return {k: float(np.sqrt(v / den)) for k, v in num.items()}


def test_formats_cheaper_than_the_fp16_product_miss_the_parity_bar():
    err = rel_l2_by_variant(128 * 12)
    bar = 1e-3
    assert err["fp16"] < 0.4 * bar, err
    # cheaper than 512 matrix-unit cycles per block: 128 (e2m1), 256, 384 and 256 (e4m3 x 1)
    assert err["e2m1x1"] > 100 * bar, err
    assert err["e2m1x2"] > 10 * bar, err
    assert err["e2m1x3"] > 2 * bar, err
    assert err["e4m3x1"] > 10 * bar, err
    # the same 512 cycles as the fp16 product: inside the bar, yet no better than fp16
    assert err["fp16"] < err["e4m3x2"] < bar, err
    assert err["fp16"] < err["e2m1x4"] < bar, err
