"""The allocation-free entry point bd_decode_attn_static (split partials in a static device array of the
library) against bd_decode_attn with a caller's workspace: same kernels, so the same output bits, and both
within the bar of the oracle.  Two calls in a row share the array; the second is smaller, so stale partials
of the first lie behind the ones it writes."""
import ctypes

import numpy as np
import pytest

from oracle import bitdecode_oracle as O
from paper_2503_18773_amd import binding as B
from paper_2503_18773_amd import workloads as W
from tests.util import assert_attn_close, out_to_f64, to_dev

pytestmark = pytest.mark.gpu


def _case(fmt, batch, context, splits, seed):
    import torch
    w = W.scaled(W.CONFIGS["cfg1"], batch=batch, n_q_heads=8, n_kv_heads=2, context=context, fmt=fmt, seed=seed)
    cap = ((context + 127) // 128) * 128 + 128
    K, V = W.make_kv(w)
    q = W.make_q(w)
    oc = O.IntCache(w.batch, w.n_kv_heads, 4 if fmt == "int4" else 2, cap)
    oc.quant_pack_kv(K, V)
    ref = O.decode_attn(oc, q, W.softmax_scale(w))
    gc = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, fmt, cap)
    gc.quant_pack_kv(to_dev(K, "fp16"), to_dev(V, "fp16"))
    qd = to_dev(q, "fp16")
    want = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.float16, device="cuda:0")
    B.bd_decode_attn(gc.desc, qd, gc.packed_len, gc.res_len, W.softmax_scale(w), splits, gc.workspace(splits), want)
    got = torch.full_like(want, float("nan"))
    B.bd_decode_attn_static(gc.desc, qd, gc.packed_len, gc.res_len, W.softmax_scale(w), splits, got)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (fmt, batch, context, splits)
    assert_attn_close(out_to_f64(got), ref, f"static {fmt} L={context} splits={splits}")


def test_static_scratch_matches_workspace_twice_in_a_row():
    _case("int4", 2, 128 * 21 + 77, 6, seed=31)   # 6 splits x 2 sequences x 8 heads of partials
    _case("int4", 1, 128 * 5 + 3, 2, seed=32)     # smaller: stale partials of the first call stay behind
    _case("int2", 1, 128 * 9 + 100, 3, seed=33)
    _case("int4", 1, 128 * 2, 1, seed=34)         # one split: the array is not touched at all


def test_static_scratch_rejects_what_does_not_fit():
    c = B.bd_cache(64, 64, 8, 128, B.BD_FMT_INT4, 4096, None, None, None, None, None, None)
    splits = B.BD_STATIC_SCRATCH_BYTES // (64 * 64 * 130 * 4) + 1
    assert B.lib().bd_decode_attn_static(ctypes.byref(c), 4096, 4096, 0, 0.1, splits, 4096, None) == -4
