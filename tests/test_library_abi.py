"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and
validates arguments before touching the GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2503_18773_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
needs_lib = pytest.mark.skipif(not os.path.exists(B._LIB_PATH), reason="libbitdecode.so not built")


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bitdecode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bd_[a-z_0-9]+)\s*\(", text)))


@needs_lib
def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert hasattr(B.lib(), n), n


def _desc(**kw):
    d = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, format=B.BD_FMT_INT4, capacity=32768)
    d.update(kw)
    return B.bd_cache(d["batch"], d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["format"], d["capacity"],
                      None, None, None, None, None, None)


@needs_lib
def test_cache_bytes_match_the_format():
    c = _desc()
    units, cap = 8, 32768
    assert [B.bd_cache_bytes(c, i) for i in range(6)] == [
        units * cap * 64, units * cap * 64, units * (cap // 128) * 128 * 4, units * cap * 4,
        units * 128 * 128 * 2, units * 128 * 128 * 2]
    c2 = _desc(format=B.BD_FMT_INT2)
    assert B.bd_cache_bytes(c2, 0) == units * cap * 32 and B.bd_cache_bytes(c2, 3) == units * cap * 4
    c4 = _desc(format=B.BD_FMT_MXFP4, batch=16, capacity=16384)
    assert [B.bd_cache_bytes(c4, i) for i in range(6)] == [128 * 16384 * 64, 128 * 16384 * 64, 128 * 16384 * 4,
                                                          128 * 16384 * 4, 0, 0]
    # 136 / 72 / 136 bytes per token per KV head
    for c_, per in [(c, 136), (c2, 72)]:
        assert sum(B.bd_cache_bytes(c_, i) for i in range(4)) == per * units * cap
    assert B.bd_cache_bytes(_desc(head_dim=64), 0) == 0
    assert B.bd_cache_bytes(c, 6) == 0
    # quantization groups of 64 / 32: the codes stay, the parameter arrays grow by 128 / group
    for fmt, per in [(B.BD_FMT_INT4_G64, 144), (B.BD_FMT_INT4_G32, 160), (B.BD_FMT_INT2_G64, 80), (B.BD_FMT_INT2_G32, 96),
                     (B.BD_FMT_INT4_KT_G64, 144), (B.BD_FMT_INT4_KT_G32, 160), (B.BD_FMT_INT2_KT_G64, 80),
                     (B.BD_FMT_INT2_KT_G32, 96)]:
        cg = _desc(format=fmt)
        assert sum(B.bd_cache_bytes(cg, i) for i in range(4)) == per * units * cap
        assert B.bd_cache_bytes(cg, 4) == units * 128 * 128 * 2
    assert B.bd_cache_bytes(_desc(format=13), 0) == 0


@needs_lib
def test_split_heuristic_and_workspace():
    c = _desc()
    for L in (0, 128, 1024, 32768, 131072):
        s = B.bd_choose_splits(c, L)
        assert 1 <= s <= max(1, L // 128)
    assert B.bd_workspace_bytes(c, 64) == 64 * 32 * 130 * 4
    assert B.bd_workspace_bytes(c, 0) == 0


@needs_lib
def test_argument_validation_happens_before_any_launch():
    L = B.lib()
    c = _desc()
    pl, rl = ctypes.c_int32(0), ctypes.c_int32(0)
    # NULL cache buffers
    assert L.bd_quant_pack_kv(ctypes.byref(c), None, None, 128, ctypes.byref(pl), ctypes.byref(rl), None) == -1
    c.k_codes = c.v_codes = c.k_params = c.v_params = c.k_res = c.v_res = 4096
    assert L.bd_quant_pack_kv(ctypes.byref(c), None, None, 128, ctypes.byref(pl), ctypes.byref(rl), None) == -1
    assert L.bd_quant_pack_kv(ctypes.byref(c), 4096, 4096, -1, ctypes.byref(pl), ctypes.byref(rl), None) == -1
    assert L.bd_quant_pack_kv(ctypes.byref(c), 4096, 4100, 128, ctypes.byref(pl), ctypes.byref(rl), None) == -3
    assert L.bd_quant_pack_kv(ctypes.byref(c), 4096, 4096, 32768 + 128, ctypes.byref(pl), ctypes.byref(rl),
                              None) == -4
    # append that would overflow the packed buffers leaves the lengths alone
    pl, rl = ctypes.c_int32(32768), ctypes.c_int32(127)
    assert L.bd_append_kv(ctypes.byref(c), 4096, 4096, ctypes.byref(pl), ctypes.byref(rl), None) == -4
    assert (pl.value, rl.value) == (32768, 127)
    pl, rl = ctypes.c_int32(100), ctypes.c_int32(0)
    assert L.bd_append_kv(ctypes.byref(c), 4096, 4096, ctypes.byref(pl), ctypes.byref(rl), None) == -1
    # decode: bad split count, bad lengths, misaligned workspace
    assert L.bd_decode_attn(ctypes.byref(c), 4096, 1024, 0, 0.1, 0, 4096, 4096, None) == -1
    assert L.bd_decode_attn(ctypes.byref(c), 4096, 1000, 0, 0.1, 4, 4096, 4096, None) == -1
    assert L.bd_decode_attn(ctypes.byref(c), 4096, 1024, 128, 0.1, 4, 4096, 4096, None) == -1
    assert L.bd_decode_attn(ctypes.byref(c), 4096, 1024, 0, 0.1, 4, 4100, 4096, None) == -3
    assert L.bd_splitk_combine(ctypes.byref(c), None, 4, 4096, None) == -1
    # allocation-free variant: `out` is required; partials beyond the static array are refused
    assert L.bd_decode_attn_static(ctypes.byref(c), 4096, 1024, 0, 0.1, 4, None, None) == -1
    too_many = B.BD_STATIC_SCRATCH_BYTES // (c.batch * c.n_q_heads * 130 * 4) + 1
    assert L.bd_decode_attn_static(ctypes.byref(c), 4096, 1024, 0, 0.1, too_many, 4096, None) == -4
    # the streaming-read probe: whole blocks inside the capacity, an aligned sink
    assert L.bd_probe_stream_read(ctypes.byref(c), 1000, None, None) == -1
    assert L.bd_probe_stream_read(ctypes.byref(c), c.capacity + 128, None, None) == -1
    assert L.bd_probe_stream_read(ctypes.byref(c), 1024, 4098, None) == -3
    pl, rl = ctypes.c_int32(1024), ctypes.c_int32(5)
    assert L.bd_decode_step(ctypes.byref(c), 4096, 4096, 4096, ctypes.byref(pl), ctypes.byref(rl), 0.1, 4, 4096,
                            None, None) == -1                       # out is required
    assert L.bd_decode_step(ctypes.byref(c), 4096, 4100, 4096, ctypes.byref(pl), ctypes.byref(rl), 0.1, 4, 4096,
                            4096, None) == -3
    assert (pl.value, rl.value) == (1024, 5)
    # shapes this build has no kernel for
    assert B.bd_cache_bytes(_desc(n_q_heads=64), 0) > 0                # 8 per KV head
    assert B.bd_cache_bytes(_desc(n_q_heads=8 * 40), 0) > 0            # 40 per KV head: 16 at a time
    bad = _desc(n_kv_heads=40000, n_q_heads=40000 * 17)                # 2 x 40000 workgroups per split
    assert L.bd_decode_attn(ctypes.byref(bad), 4096, 1024, 0, 0.1, 4, 4096, 4096, None) == -2
    bad = _desc(batch=65536)                                           # beyond the launch grid
    assert L.bd_decode_attn(ctypes.byref(bad), 4096, 1024, 0, 0.1, 4, 4096, 4096, None) == -2
    assert B.bd_cache_bytes(bad, 0) == 0
    bad = _desc(batch=8192, n_kv_heads=8, n_q_heads=32)                # 65536 (sequence, KV head) units
    assert L.bd_quant_pack_kv(ctypes.byref(bad), 4096, 4096, 128, ctypes.byref(pl), ctypes.byref(rl), None) == -2
    assert B.bd_cache_bytes(_desc(batch=8191, n_kv_heads=8, n_q_heads=32), 0) > 0
    assert L.bd_strerror(-4) == b"cache capacity exceeded"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", "/nonexistent/libbitdecode.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()


def _paged(**kw):
    d = dict(batch=4, n_q_heads=32, n_kv_heads=8, head_dim=128, format=B.BD_FMT_INT4, num_pages=100, max_pages=10)
    d.update(kw)
    return B.bd_paged_cache(d["batch"], d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["format"], d["num_pages"],
                            d["max_pages"])


@needs_lib
def test_paged_sizes_and_argument_validation():
    c = _paged()
    pool = 100 * 8
    assert [B.bd_paged_cache_bytes(c, i) for i in range(8)] == [
        pool * 128 * 64, pool * 128 * 64, pool * 128 * 4, pool * 128 * 4, 4 * 8 * 128 * 128 * 2, 4 * 8 * 128 * 128 * 2,
        4 * 10 * 4, 4 * 4]
    assert B.bd_paged_cache_bytes(_paged(format=B.BD_FMT_INT2), 0) == pool * 128 * 32
    mx = _paged(format=B.BD_FMT_MXFP4)                    # no residual: every token is quantized on arrival
    assert [B.bd_paged_cache_bytes(mx, i) for i in range(8)] == [
        pool * 128 * 64, pool * 128 * 64, pool * 128 * 4, pool * 128 * 4, 0, 0, 4 * 10 * 4, 4 * 4]
    assert B.bd_paged_cache_bytes(_paged(num_pages=0), 0) == 0
    g32 = _paged(format=B.BD_FMT_INT4_G32)               # smaller groups: the parameter arrays grow by 128 / group
    assert [B.bd_paged_cache_bytes(g32, i) for i in range(4)] == [pool * 128 * 64, pool * 128 * 64, pool * 4 * 128 * 4,
                                                                 pool * 128 * 4 * 4]
    assert B.bd_paged_workspace_bytes(c, 16) == 16 * 4 * 32 * 130 * 4
    L = B.lib()
    # NULL buffers are refused before anything is launched
    assert L.bd_paged_append_kv(ctypes.byref(c), 16, 16, None) == -1
    for name in ("k_codes", "v_codes", "k_params", "v_params", "k_res", "v_res", "block_table", "seq_lens"):
        setattr(c, name, 4096)
    assert L.bd_paged_append_kv(ctypes.byref(c), None, 16, None) == -1
    assert L.bd_paged_append_kv(ctypes.byref(c), 8, 16, None) == -3
    assert L.bd_paged_quant_pack_kv(ctypes.byref(c), 4, 16, 16, 10, None) == -1     # sequence out of range
    assert L.bd_paged_quant_pack_kv(ctypes.byref(c), 0, 16, 16, 128 * 11, None) == -4   # more blocks than table columns
    assert L.bd_paged_decode_attn(ctypes.byref(c), 16, ctypes.c_float(0.1), 0, 16, 16, None) == -1
    assert L.bd_paged_decode_attn(ctypes.byref(c), 16, ctypes.c_float(0.1), 4, 16, None, None) == -1
    c.seq_lens = 4098
    assert L.bd_paged_append_kv(ctypes.byref(c), 16, 16, None) == -3
    for name in ("k_codes", "v_codes", "k_params", "v_params", "block_table", "seq_lens"):
        setattr(mx, name, 4096)
    # MXFP4 keeps partly filled blocks in pages: 128 * 10 + 1 tokens need an eleventh table column
    assert L.bd_paged_quant_pack_kv(ctypes.byref(mx), 0, 16, 16, 128 * 10 + 1, None) == -4
    assert L.bd_paged_quant_pack_kv(ctypes.byref(mx), 0, 16, 20, 128, None) == -3


@needs_lib
def test_split_heuristic_properties():
    """One resident round of workgroups: splits x units stays near 512, never exceeds the number of
    4-block quanta, and short contexts get one block per wave at most."""
    for batch, hkv in [(1, 8), (8, 8), (16, 8), (1, 1), (64, 2)]:
        c = _desc(batch=batch, n_q_heads=4 * hkv, n_kv_heads=hkv, capacity=1 << 20)
        prev = 0
        for L in (128, 512, 4096, 32768, 131072, 1 << 20):
            s = B.bd_choose_splits(c, L)
            quanta = (L // 128 + 3) // 4
            assert 1 <= s <= quanta
            assert s * batch * hkv <= max(768, batch * hkv)
            assert s >= prev or s * batch * hkv >= 256        # grows with the context until the chip is full
            prev = s
    assert B.bd_choose_splits(_desc(), 32768) == 64 and B.bd_choose_splits(_desc(), 131072) == 64
    assert B.bd_choose_splits(_desc(batch=8), 32768) == 8
    # a chip already full of units takes one split (no merge kernel) unless the call is long
    assert B.bd_choose_splits(_desc(batch=48), 4096) == 1 and B.bd_choose_splits(_desc(batch=32), 4096) == 1
    assert B.bd_choose_splits(_desc(batch=32), 16384) == 2
    # one block per wave is kept up to three workgroups per compute unit (integer formats, groups <= 8)
    assert B.bd_choose_splits(_desc(), 40960) == 80 and B.bd_choose_splits(_desc(), 49152) == 96
    assert B.bd_choose_splits(_desc(), 57344) == 64                     # beyond that: one round of 512 workgroups
    assert B.bd_choose_splits(_desc(format=B.BD_FMT_MXFP4), 49152) == 64
    assert B.bd_choose_splits(_desc(format=B.BD_FMT_MXFP4), 32768 + 1) == 64   # quanta need not divide evenly
    # one instance of the kernel for smaller quantization groups runs one workgroup per compute unit
    assert B.bd_choose_splits(_desc(format=B.BD_FMT_INT4_G32), 32768) == 64
    assert B.bd_choose_splits(_desc(format=B.BD_FMT_INT4_G32, n_q_heads=64), 32768) == 32
    assert B.bd_choose_splits(_desc(format=B.BD_FMT_INT2_G64, n_q_heads=128), 32768) == 32   # two workgroups per KV head
