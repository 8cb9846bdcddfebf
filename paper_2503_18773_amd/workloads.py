"""Seeded synthetic inputs for the low-bit-KV decode-attention path.

This module only draws random tensors of the shapes and value distributions the
benchmark configurations name (LLaMA-3.1-8B attention geometry: 32 query heads,
8 KV heads, head_dim 128; Gaussian activations with a few large-magnitude
"outlier" channels, which is the structure that motivates per-channel K
quantization in the paper's Related Works / Section V-B).  It holds none of the
method's arithmetic (no quantization, packing, softmax), so both the CPU oracle's
tests and the HIP path's tests can feed from it without sharing any code of the
method itself.

All draws come from numpy's counter-based Philox generator, so a (seed, shape)
pair names one tensor on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

HEAD_DIM = 128
BLOCK = 128  # residual block size N_r == quantization group (Eq. 1 evaluates to 128 here)


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    context: int          # tokens resident before the first decode step
    fmt: str              # "int4" | "int2" | "mxfp4" | "int4_kt" | "int2_kt" (K per token)
    steps: int            # decode steps the configuration asks for
    seed: int
    outliers: bool        # 1% of (kv_head, channel) pairs scaled by 10 in K and in V
    head_dim: int = HEAD_DIM

    @property
    def in_dtype(self) -> str:
        return "bf16" if self.fmt == "mxfp4" else "fp16"

    @property
    def g_q(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark configurations (0-based, as listed in the benchmark spec).
CONFIGS = {
    "cfg0": Workload("cfg0", 1, 8, 8, 1024, "int4", 1, 0, False),
    "cfg1": Workload("cfg1", 1, 32, 8, 32768, "int4", 64, 1, True),
    "cfg2": Workload("cfg2", 8, 32, 8, 32768, "int2", 1, 2, True),
    "cfg3": Workload("cfg3", 1, 32, 8, 131072, "int4", 256, 3, True),
    "cfg4": Workload("cfg4", 16, 32, 8, 16384, "mxfp4", 1, 4, False),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a configuration with some fields replaced (smaller parity cases)."""
    return replace(w, **kw)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); result kept as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are exactly representable in bf16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not a bf16"
    return (u >> np.uint32(16)).astype(np.uint16)


def _to_storage(x32: np.ndarray, in_dtype: str) -> np.ndarray:
    if in_dtype == "fp16":
        return x32.astype(np.float16)
    return round_to_bf16(x32)


def outlier_pairs(w: Workload, which: int) -> np.ndarray:
    """(kv_head, channel) pairs whose values are scaled by 10: round(1% of H_kv*D) of them,
    drawn without replacement, independently for K (which=0) and V (which=1)."""
    n = int(round(0.01 * w.n_kv_heads * w.head_dim))
    flat = _rng(w.seed, 100 + which).choice(w.n_kv_heads * w.head_dim, size=n, replace=False)
    return np.stack([flat // w.head_dim, flat % w.head_dim], axis=1)


def make_kv(w: Workload, length: int | None = None, stream: int = 0):
    """K, V of shape [B, H_kv, length, D] ~ N(0,1), outliers applied before rounding to
    the storage type (fp16 as numpy float16; bf16 as float32 holding bf16 values)."""
    L = w.context if length is None else length
    shape = (w.batch, w.n_kv_heads, L, w.head_dim)
    out = []
    for which in (0, 1):
        x = _rng(w.seed, 10 * stream + which).standard_normal(shape, dtype=np.float32)
        if w.outliers:
            for h, c in outlier_pairs(w, which):
                x[:, h, :, c] *= np.float32(10.0)
        out.append(_to_storage(x, w.in_dtype))
    return out[0], out[1]


def make_q(w: Workload, step: int = 0) -> np.ndarray:
    """Query of one decode step, [B, H_q, D] ~ N(0,1)."""
    x = _rng(w.seed, 1000 + step).standard_normal((w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    return _to_storage(x, w.in_dtype)


def make_new_kv(w: Workload, step: int):
    """The K/V token generated at a decode step, each [B, H_kv, D]; same distribution
    (and the same outlier channels) as the prefill tensors."""
    out = []
    for which in (0, 1):
        x = _rng(w.seed, 2000 + 2 * step + which).standard_normal(
            (w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
        if w.outliers:
            for h, c in outlier_pairs(w, which):
                x[:, h, c] *= np.float32(10.0)
        out.append(_to_storage(x, w.in_dtype))
    return out[0], out[1]


def softmax_scale(w: Workload) -> float:
    return 1.0 / float(np.sqrt(w.head_dim))
