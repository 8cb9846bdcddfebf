"""ctypes binding of libbitdecode.so: the same entry points as include/bitdecode.h, argument
marshalling only.  Device memory and streams come from PyTorch; every step of the path runs
in the library's HIP kernels.  There is no fallback: if the library has not been built,
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

BD_FMT_INT4, BD_FMT_INT2, BD_FMT_MXFP4, BD_FMT_INT4_KT, BD_FMT_INT2_KT = 0, 1, 2, 3, 4
BD_FMT_INT4_G64, BD_FMT_INT4_G32, BD_FMT_INT2_G64, BD_FMT_INT2_G32 = 5, 6, 7, 8
BD_FMT_INT4_KT_G64, BD_FMT_INT4_KT_G32, BD_FMT_INT2_KT_G64, BD_FMT_INT2_KT_G32 = 9, 10, 11, 12
FORMATS = {"int4": BD_FMT_INT4, "int2": BD_FMT_INT2, "mxfp4": BD_FMT_MXFP4, "int4_kt": BD_FMT_INT4_KT,
           "int2_kt": BD_FMT_INT2_KT, "int4_g64": BD_FMT_INT4_G64, "int4_g32": BD_FMT_INT4_G32,
           "int2_g64": BD_FMT_INT2_G64, "int2_g32": BD_FMT_INT2_G32,
           "int4_kt_g64": BD_FMT_INT4_KT_G64, "int4_kt_g32": BD_FMT_INT4_KT_G32,
           "int2_kt_g64": BD_FMT_INT2_KT_G64, "int2_kt_g32": BD_FMT_INT2_KT_G32}
BLOCK = 128
BD_OUT_HALF, BD_OUT_F32 = 0, 1
BD_STATIC_SCRATCH_BYTES = 4 << 20   # include/bitdecode.h

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbitdecode.so")
_lib = None


class bd_cache(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("format", ctypes.c_int32), ("capacity", ctypes.c_int32),
        ("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
        ("k_params", ctypes.c_void_p), ("v_params", ctypes.c_void_p),
        ("k_res", ctypes.c_void_p), ("v_res", ctypes.c_void_p),
        ("out_type", ctypes.c_int32),
    ]


class bd_paged_cache(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("format", ctypes.c_int32), ("num_pages", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32),
        ("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
        ("k_params", ctypes.c_void_p), ("v_params", ctypes.c_void_p),
        ("k_res", ctypes.c_void_p), ("v_res", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p), ("status", ctypes.c_void_p),
        ("out_type", ctypes.c_int32),
    ]


class BitDecodeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().bd_strerror(status).decode()
        hip = lib().bd_last_hip_error()
        super().__init__(f"{where}: {msg} (status {status}, hip error {hip})")


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2503_18773_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        P, I, V, F, S = ctypes.POINTER(bd_cache), ctypes.c_int32, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
        IP = ctypes.POINTER(ctypes.c_int32)
        L.bd_cache_bytes.restype, L.bd_cache_bytes.argtypes = S, [P, ctypes.c_int]
        L.bd_choose_splits.restype, L.bd_choose_splits.argtypes = I, [P, I]
        L.bd_workspace_bytes.restype, L.bd_workspace_bytes.argtypes = S, [P, I]
        L.bd_quant_pack_kv.restype, L.bd_quant_pack_kv.argtypes = ctypes.c_int, [P, V, V, I, IP, IP, V]
        L.bd_append_kv.restype, L.bd_append_kv.argtypes = ctypes.c_int, [P, V, V, IP, IP, V]
        L.bd_decode_attn.restype, L.bd_decode_attn.argtypes = ctypes.c_int, [P, V, I, I, F, I, V, V, V]
        L.bd_decode_attn_static.restype, L.bd_decode_attn_static.argtypes = ctypes.c_int, [P, V, I, I, F, I, V, V]
        L.bd_probe_stream_read.restype, L.bd_probe_stream_read.argtypes = ctypes.c_int, [P, I, V, V]
        L.bd_splitk_combine.restype, L.bd_splitk_combine.argtypes = ctypes.c_int, [P, V, I, V, V]
        L.bd_decode_step.restype, L.bd_decode_step.argtypes = ctypes.c_int, [P, V, V, V, IP, IP, F, I, V, V, V]
        L.bd_decode_step_lazy.restype, L.bd_decode_step_lazy.argtypes = ctypes.c_int, [P, V, V, V, IP, IP, F, I, V, V, V]
        PP = ctypes.POINTER(bd_paged_cache)
        L.bd_paged_cache_bytes.restype, L.bd_paged_cache_bytes.argtypes = S, [PP, ctypes.c_int]
        L.bd_paged_workspace_bytes.restype, L.bd_paged_workspace_bytes.argtypes = S, [PP, I]
        L.bd_paged_quant_pack_kv.restype, L.bd_paged_quant_pack_kv.argtypes = ctypes.c_int, [PP, I, V, V, I, V]
        L.bd_paged_append_kv.restype, L.bd_paged_append_kv.argtypes = ctypes.c_int, [PP, V, V, V]
        L.bd_paged_decode_attn.restype, L.bd_paged_decode_attn.argtypes = ctypes.c_int, [PP, V, F, I, V, V, V]
        L.bd_paged_decode_step.restype, L.bd_paged_decode_step.argtypes = ctypes.c_int, [PP, V, V, V, F, I, V, V, V]
        L.bd_paged_decode_step_lazy.restype, L.bd_paged_decode_step_lazy.argtypes = ctypes.c_int, [PP, V, V, V, F, I, V, V, V]
        L.bd_strerror.restype, L.bd_strerror.argtypes = ctypes.c_char_p, [ctypes.c_int]
        L.bd_last_hip_error.restype, L.bd_last_hip_error.argtypes = ctypes.c_int, []
        _lib = L
    return _lib


EXPORTS = ["bd_cache_bytes", "bd_choose_splits", "bd_workspace_bytes", "bd_quant_pack_kv", "bd_append_kv",
           "bd_decode_attn", "bd_decode_attn_static", "bd_probe_stream_read", "bd_decode_step", "bd_decode_step_lazy", "bd_splitk_combine", "bd_strerror", "bd_last_hip_error",
           "bd_paged_cache_bytes", "bd_paged_workspace_bytes", "bd_paged_quant_pack_kv", "bd_paged_append_kv",
           "bd_paged_decode_attn", "bd_paged_decode_step", "bd_paged_decode_step_lazy"]


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise BitDecodeError(status, where)


# ---- the C-ABI, one wrapper per entry point ------------------------------------------------

def bd_cache_bytes(c: bd_cache, which: int) -> int:
    return int(lib().bd_cache_bytes(ctypes.byref(c), which))


def bd_choose_splits(c: bd_cache, packed_len: int) -> int:
    return int(lib().bd_choose_splits(ctypes.byref(c), packed_len))


def bd_workspace_bytes(c: bd_cache, num_splits: int) -> int:
    return int(lib().bd_workspace_bytes(ctypes.byref(c), num_splits))


def bd_quant_pack_kv(c: bd_cache, k, v, L: int, stream=None):
    """Returns (packed_len, res_len)."""
    pl, rl = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().bd_quant_pack_kv(ctypes.byref(c), _ptr(k), _ptr(v), L, ctypes.byref(pl), ctypes.byref(rl),
                                  _stream(stream)), "bd_quant_pack_kv")
    return pl.value, rl.value


def bd_append_kv(c: bd_cache, k_new, v_new, packed_len: int, res_len: int, stream=None):
    """Returns the updated (packed_len, res_len)."""
    pl, rl = ctypes.c_int32(packed_len), ctypes.c_int32(res_len)
    _check(lib().bd_append_kv(ctypes.byref(c), _ptr(k_new), _ptr(v_new), ctypes.byref(pl), ctypes.byref(rl),
                              _stream(stream)), "bd_append_kv")
    return pl.value, rl.value


def bd_decode_attn(c: bd_cache, q, packed_len: int, res_len: int, softmax_scale: float, num_splits: int,
                   workspace, out=None, stream=None):
    _check(lib().bd_decode_attn(ctypes.byref(c), _ptr(q), packed_len, res_len, softmax_scale, num_splits,
                                _ptr(workspace), _ptr(out), _stream(stream)), "bd_decode_attn")


def bd_decode_attn_static(c: bd_cache, q, packed_len: int, res_len: int, softmax_scale: float, num_splits: int, out,
                          stream=None):
    _check(lib().bd_decode_attn_static(ctypes.byref(c), _ptr(q), packed_len, res_len, softmax_scale, num_splits,
                                       _ptr(out), _stream(stream)), "bd_decode_attn_static")


def bd_probe_stream_read(c: bd_cache, packed_len: int, sink=None, stream=None):
    _check(lib().bd_probe_stream_read(ctypes.byref(c), packed_len, _ptr(sink), _stream(stream)), "bd_probe_stream_read")


def bd_decode_step(c: bd_cache, k_new, v_new, q, packed_len: int, res_len: int, softmax_scale: float,
                   num_splits: int, workspace, out, stream=None):
    """Returns the updated (packed_len, res_len)."""
    pl, rl = ctypes.c_int32(packed_len), ctypes.c_int32(res_len)
    _check(lib().bd_decode_step(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _ptr(q), ctypes.byref(pl),
                                ctypes.byref(rl), softmax_scale, num_splits, _ptr(workspace), _ptr(out),
                                _stream(stream)), "bd_decode_step")
    return pl.value, rl.value


def bd_decode_step_lazy(c: bd_cache, k_new, v_new, q, packed_len: int, res_len: int, softmax_scale: float,
                        num_splits: int, workspace, out, stream=None):
    """Returns the updated (packed_len, res_len)."""
    pl, rl = ctypes.c_int32(packed_len), ctypes.c_int32(res_len)
    _check(lib().bd_decode_step_lazy(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _ptr(q), ctypes.byref(pl),
                                     ctypes.byref(rl), softmax_scale, num_splits, _ptr(workspace), _ptr(out),
                                     _stream(stream)), "bd_decode_step_lazy")
    return pl.value, rl.value


def bd_splitk_combine(c: bd_cache, workspace, num_splits: int, out, stream=None):
    _check(lib().bd_splitk_combine(ctypes.byref(c), _ptr(workspace), num_splits, _ptr(out), _stream(stream)),
           "bd_splitk_combine")


def bd_paged_cache_bytes(c: bd_paged_cache, which: int) -> int:
    return int(lib().bd_paged_cache_bytes(ctypes.byref(c), which))


def bd_paged_workspace_bytes(c: bd_paged_cache, num_splits: int) -> int:
    return int(lib().bd_paged_workspace_bytes(ctypes.byref(c), num_splits))


def bd_paged_quant_pack_kv(c: bd_paged_cache, seq: int, k, v, L: int, stream=None):
    _check(lib().bd_paged_quant_pack_kv(ctypes.byref(c), seq, _ptr(k), _ptr(v), L, _stream(stream)),
           "bd_paged_quant_pack_kv")


def bd_paged_append_kv(c: bd_paged_cache, k_new, v_new, stream=None):
    _check(lib().bd_paged_append_kv(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _stream(stream)), "bd_paged_append_kv")


def bd_paged_decode_attn(c: bd_paged_cache, q, softmax_scale: float, num_splits: int, workspace, out, stream=None):
    _check(lib().bd_paged_decode_attn(ctypes.byref(c), _ptr(q), softmax_scale, num_splits, _ptr(workspace), _ptr(out),
                                      _stream(stream)), "bd_paged_decode_attn")


def bd_paged_decode_step(c: bd_paged_cache, k_new, v_new, q, softmax_scale: float, num_splits: int, workspace, out,
                         stream=None):
    _check(lib().bd_paged_decode_step(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _ptr(q), softmax_scale, num_splits,
                                      _ptr(workspace), _ptr(out), _stream(stream)), "bd_paged_decode_step")


def bd_paged_decode_step_lazy(c: bd_paged_cache, k_new, v_new, q, softmax_scale: float, num_splits: int, workspace, out,
                              stream=None):
    _check(lib().bd_paged_decode_step_lazy(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _ptr(q), softmax_scale,
                                           num_splits, _ptr(workspace), _ptr(out), _stream(stream)),
           "bd_paged_decode_step_lazy")


# ---- device-memory plumbing ------------------------------------------------------------------

class KVCache:
    """Owns the six device buffers of one layer's cache as torch tensors (zero-filled) and the
    two host-side lengths; every operation is a call into the library."""

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, fmt: str, capacity: int, device="cuda:0"):
        import torch
        self.fmt = fmt
        self.desc = bd_cache(batch, n_q_heads, n_kv_heads, 128, FORMATS[fmt], capacity, None, None, None, None,
                             None, None)
        sizes = [bd_cache_bytes(self.desc, i) for i in range(6)]
        if sizes[0] == 0:
            raise BitDecodeError(-1, "bd_cache_bytes")
        self.buffers = [torch.zeros(max(n, 16), dtype=torch.uint8, device=device) for n in sizes]
        for name, buf in zip(["k_codes", "v_codes", "k_params", "v_params", "k_res", "v_res"], self.buffers):
            setattr(self.desc, name, buf.data_ptr())
        self.sizes = sizes
        self.packed_len = 0
        self.res_len = 0
        self.device = device
        self._ws = None
        self._retired = []

    @property
    def length(self) -> int:
        return self.packed_len + self.res_len

    def quant_pack_kv(self, k, v, stream=None):
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        self.packed_len, self.res_len = bd_quant_pack_kv(self.desc, k, v, k.shape[2], stream)

    def append_kv(self, k_new, v_new, stream=None):
        self.packed_len, self.res_len = bd_append_kv(self.desc, k_new, v_new, self.packed_len, self.res_len, stream)

    def workspace(self, num_splits: int):
        """A device buffer of at least bd_workspace_bytes(num_splits).  It only grows, and a buffer it
        outgrows is kept alive (kernels queued on any stream may still be writing partials into it)."""
        import torch
        need = bd_workspace_bytes(self.desc, num_splits)
        if self._ws is None or self._ws.numel() < need:
            if self._ws is not None:
                self._retired.append(self._ws)
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def choose_splits(self) -> int:
        return bd_choose_splits(self.desc, self.packed_len)

    def decode_attn(self, q, softmax_scale: float, out, num_splits: int | None = None, fused: bool = True,
                    stream=None):
        ns = self.choose_splits() if num_splits is None else num_splits
        ws = self.workspace(ns)
        if fused:
            bd_decode_attn(self.desc, q, self.packed_len, self.res_len, softmax_scale, ns, ws, out, stream)
        else:
            bd_decode_attn(self.desc, q, self.packed_len, self.res_len, softmax_scale, ns, ws, None, stream)
            bd_splitk_combine(self.desc, ws, ns, out, stream)
        return out

    def decode_step(self, k_new, v_new, q, softmax_scale: float, out, num_splits: int | None = None, stream=None,
                    lazy: bool = False):
        ns = self.choose_splits() if num_splits is None else num_splits
        step = bd_decode_step_lazy if lazy else bd_decode_step
        self.packed_len, self.res_len = step(self.desc, k_new, v_new, q, self.packed_len, self.res_len,
                                             softmax_scale, ns, self.workspace(ns), out, stream)
        return out

    def host_buffer(self, i: int):
        """Buffer i copied to host as a numpy uint8 array (for bit-exact comparisons)."""
        return self.buffers[i][:self.sizes[i]].cpu().numpy()


class PagedKVCache:
    """Device buffers of one layer's paged cache as torch tensors: the page pool, the per-sequence
    residuals, the block table (given by the caller, who owns page allocation), the lengths and
    the status word.  Every operation is a call into the library."""

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, fmt: str, num_pages: int, block_table,
                 device="cuda:0"):
        import torch
        self.fmt = fmt
        max_pages = int(block_table.shape[1])
        assert block_table.shape[0] == batch
        self.desc = bd_paged_cache(batch, n_q_heads, n_kv_heads, 128, FORMATS[fmt], num_pages, max_pages)
        self.sizes = [bd_paged_cache_bytes(self.desc, i) for i in range(8)]
        if self.sizes[0] == 0:
            raise BitDecodeError(-1, "bd_paged_cache_bytes")
        self.buffers = [torch.zeros(max(n, 16), dtype=torch.uint8, device=device) for n in self.sizes[:6]]
        self.block_table = torch.as_tensor(block_table, dtype=torch.int32).contiguous().to(device)
        self.seq_lens = torch.zeros(batch, dtype=torch.int32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        for name, buf in zip(["k_codes", "v_codes", "k_params", "v_params", "k_res", "v_res"], self.buffers):
            setattr(self.desc, name, buf.data_ptr())
        self.desc.block_table = self.block_table.data_ptr()
        self.desc.seq_lens = self.seq_lens.data_ptr()
        self.desc.status = self.status.data_ptr()
        self.device = device
        self._ws = None
        self._retired = []

    def quant_pack_kv(self, seq: int, k, v, stream=None):
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        bd_paged_quant_pack_kv(self.desc, seq, k, v, k.shape[1], stream)

    def append_kv(self, k_new, v_new, stream=None):
        bd_paged_append_kv(self.desc, k_new, v_new, stream)

    def workspace(self, num_splits: int):
        """As KVCache.workspace: grows only, outgrown buffers stay alive."""
        import torch
        need = bd_paged_workspace_bytes(self.desc, num_splits)
        if self._ws is None or self._ws.numel() < need:
            if self._ws is not None:
                self._retired.append(self._ws)
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def decode_attn(self, q, softmax_scale: float, out, num_splits: int, stream=None):
        bd_paged_decode_attn(self.desc, q, softmax_scale, num_splits, self.workspace(num_splits), out, stream)
        return out

    def decode_step(self, k_new, v_new, q, softmax_scale: float, out, num_splits: int, stream=None, lazy: bool = False):
        step = bd_paged_decode_step_lazy if lazy else bd_paged_decode_step
        step(self.desc, k_new, v_new, q, softmax_scale, num_splits, self.workspace(num_splits), out, stream)
        return out

    def host_buffer(self, i: int):
        return self.buffers[i][:self.sizes[i]].cpu().numpy()
