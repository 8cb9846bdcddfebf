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


def assert_attn_close(got: np.ndarray, ref: np.ndarray, what="", large_outputs=False, noise=None):
    """The bar of the benchmark configurations: max-abs 2e-3 and relative L2 1e-3.  With
    `large_outputs` (sequences of a few tokens or peaked weights, whose outputs are close to single V
    rows: magnitudes of 10 and more with the x10 outlier channels, where half an fp16 step alone is
    8e-3) the max-abs bar is taken per element as 2e-3 + 2^-10 |ref| instead.
    `noise` (the oracle's rounding_noise_scale, one value per head) adds 2^-11 * noise to that: the
    probabilities enter the second product as fp16, so a head in which one token with large values
    holds most of the weight carries that token's rounding error into every channel, also into
    those whose value is small after cancellation.  For the random shapes of the sweeps."""
    mask = ~np.isnan(ref)
    ma, rl = attn_errors(got[mask], ref[mask])
    if large_outputs:
        bar = MAX_ABS_TOL + 2.0 ** -10 * np.abs(ref)
        if noise is not None:
            bar = bar + 2.0 ** -11 * np.asarray(noise)[..., None]
        excess = np.abs(got[mask] - ref[mask]) - bar[mask]
        assert excess.max() <= 0 and rl <= REL_L2_TOL, f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e}"
    else:
        assert ma <= MAX_ABS_TOL and rl <= REL_L2_TOL, f"{what}: max-abs {ma:.3e} rel-L2 {rl:.3e}"
    return ma, rl
