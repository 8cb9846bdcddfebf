"""Helpers shared by the GPU parity tests: host<->device conversion and error metrics."""
import numpy as np

MAX_ABS_TOL = 2e-3     # attention output: max-abs error against the float64 oracle
REL_L2_TOL = 1e-3      # attention output: relative L2 error against the float64 oracle


def to_dev(x: np.ndarray, in_dtype: str):
    """numpy fp16 array, or float32 array of bf16 values, -> torch tensor on cuda:0."""
    import torch
    from paper_2503_18773_amd import workloads as W
    if in_dtype == "fp16":
        return torch.from_numpy(np.ascontiguousarray(x)).cuda()
    bits = W.bf16_bits(x)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def out_to_f64(t) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def attn_errors(got: np.ndarray, ref: np.ndarray):
    d = got - ref
    return float(np.abs(d).max()), float(np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-30))


def assert_attn_close(got: np.ndarray, ref: np.ndarray, what="", large_outputs=False):
    """The bar of the benchmark configurations: max-abs 2e-3 and relative L2 1e-3.  With
    `large_outputs` (sequences of a few tokens or peaked weights, whose outputs are close to single V
    rows: magnitudes of 10 and more with the x10 outlier channels, where half an fp16 step alone is
    8e-3) the max-abs bar is taken per element as 2e-3 + 2^-10 |ref| instead."""
    mask = ~np.isnan(ref)
    ma, rl = attn_errors(got[mask], ref[mask])
    if large_outputs:
        bar = MAX_ABS_TOL + 2.0 ** -10 * np.abs(ref)
        excess = np.abs(got[mask] - ref[mask]) - bar[mask]
        assert excess.max() <= 0 and rl <= REL_L2_TOL, f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e}"
    else:
        assert ma <= MAX_ABS_TOL and rl <= REL_L2_TOL, f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e}"
    return ma, rl


def _mx_unit_job(job):
    """Worker of mx_units_on_host_cores: the oracle on one (sequence, KV head) unit."""
    from oracle import bitdecode_oracle as O
    K, V, kn, vn, q, sm_scale, cap = job
    oc = O.MxCache(1, 1, cap)
    oc.quant_pack_kv(K, V)
    oc.append_kv(kn, vn)
    ref = O.decode_attn(oc, q, sm_scale)
    return oc.k_codes[0, 0], oc.v_codes[0, 0], oc.k_scales[0, 0], oc.v_scales[0, 0], ref[0]


def mx_units_on_host_cores(K, V, kn, vn, q, sm_scale, cap, workers=12):
    """The MXFP4 oracle (prefill, one append, attention) on every (sequence, KV head) unit of a large
    configuration, the independent units spread over host processes (the oracle's nearest-code search
    costs microseconds per element).  Spawned processes: they import numpy and the oracle only and
    never touch the GPU.  Yields (b, h, k_codes, v_codes, k_scales, v_scales, out[g_q, D])."""
    import multiprocessing as mp
    B, H = K.shape[:2]
    g = q.shape[1] // H
    jobs = [(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1],
             q[b:b + 1, h * g:(h + 1) * g], sm_scale, cap) for b in range(B) for h in range(H)]
    with mp.get_context("spawn").Pool(min(workers, len(jobs))) as pool:
        for i, res in enumerate(pool.imap(_mx_unit_job, jobs, chunksize=1)):
            yield (i // H, i % H) + tuple(res)

