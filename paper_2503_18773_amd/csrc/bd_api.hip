// C-ABI entry points of libbitdecode.so: argument validation and kernel sequencing only.
#include <mutex>

#include "bd_common.h"

namespace bd {
static thread_local int g_last_hip_error = 0;
void note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace bd

// Split partials of bd_decode_attn_static: one array per GPU, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address is looked up once per
// device (static_scratch_ptr) and that pointer is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[BD_STATIC_SCRATCH_BYTES];

using namespace bd;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// workgroups per split and sequence: KV heads x pieces of the query group
long group_workgroups(const bd_cache* c) {
  const int gq = c->n_q_heads / c->n_kv_heads;
  const int pieces = c->format == BD_FMT_MXFP4 ? (gq + 15) / 16
                     : fmt_group(c->format) != kBlock ? (gq + 7) / 8 : (gq + 15) / 16;
  return (long)c->n_kv_heads * pieces;
}

bd_status check_shape(const bd_cache* c) {
  if (!c) return BD_ERR_INVALID_ARG;
  if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->capacity <= 0) return BD_ERR_INVALID_ARG;
  if (c->batch > 65535 || c->n_kv_heads > 65535) return BD_ERR_UNSUPPORTED;   // grid dimensions y and z
  if ((long)c->batch * c->n_kv_heads > 65535) return BD_ERR_UNSUPPORTED;      // the quantizer's grid: (block, sequence x KV head)
  if (!fmt_is_int(c->format) && c->format != BD_FMT_MXFP4) return BD_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads != 0 || c->capacity % kBlock != 0) return BD_ERR_INVALID_ARG;
  if (c->head_dim != kD) return BD_ERR_UNSUPPORTED;
  if (c->out_type != BD_OUT_HALF && c->out_type != BD_OUT_F32) return BD_ERR_INVALID_ARG;
  // query heads per KV head: the int4 / int2 kernels pad the group to 4, 8 or 16 MFMA columns and
  // take larger groups 16 heads per workgroup; the MXFP4 kernels take up to 16 heads per workgroup.
  // The workgroups of one split must fit grid dimension y.
  if (group_workgroups(c) > 65535) return BD_ERR_UNSUPPORTED;
  return BD_OK;
}

bd_status check_buffers(const bd_cache* c) {
  const bool mx = c->format == BD_FMT_MXFP4;
  const void* need[6] = {c->k_codes, c->v_codes, c->k_params, c->v_params, mx ? (void*)16 : c->k_res,
                         mx ? (void*)16 : c->v_res};
  for (const void* p : need) {
    if (!p) return BD_ERR_INVALID_ARG;
    if (!aligned16(p)) return BD_ERR_ALIGNMENT;
  }
  return BD_OK;
}

bd_status hip_status(hipError_t e) {
  if (e == hipSuccess) return BD_OK;
  note_hip_error(e);
  return BD_ERR_HIP;
}

int bits_of(int format) { return fmt_bits(format); }

// Device address of `scratch` on the current device, looked up on the first call per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

bd_status static_scratch_ptr(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_status(e);
  if (dev < 0 || dev >= kMaxDevices) return BD_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_status(e);
    if (!p) return BD_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return BD_OK;
}

}  // namespace

extern "C" {

size_t bd_cache_bytes(const bd_cache* c, int which) {
  if (check_shape(c) != BD_OK || which < 0 || which > 5) return 0;
  const size_t units = (size_t)c->batch * c->n_kv_heads, cap = (size_t)c->capacity;
  if (c->format == BD_FMT_MXFP4) {
    switch (which) {
      case 0: case 1: return units * cap * (kD / 2);
      case 2: case 3: return units * cap * (kD / kMxGroup);
      default: return 0;
    }
  }
  const size_t bits = (size_t)bits_of(c->format);
  const size_t groups = (size_t)(kBlock / fmt_group(c->format));   // K token groups per block, V channel groups per token
  switch (which) {
    case 0: case 1: return units * cap * kD * bits / 8;
    case 2: return units * (cap / kBlock) * groups * kD * 4;
    case 3: return units * cap * groups * 4;
    default: return units * kBlock * kD * 2;
  }
}

int32_t bd_choose_splits(const bd_cache* c, int32_t packed_len) {
  if (check_shape(c) != BD_OK || packed_len <= 0) return 1;
  // Each workgroup runs 4 waves that take 128-token blocks in turn, so the natural work
  // quantum is 4 blocks.  The kernel keeps 2 workgroups resident per compute unit (256 CUs):
  // aim at one full round of 512 workgroups over all (sequence, KV head) units.
  const long units = (long)c->batch * group_workgroups(c);
  const int nb = (packed_len + kBlock - 1) / kBlock;
  const int quanta = (nb + 3) / 4;
  // Up to three workgroups per compute unit fit when no wave has more than one block (that kernel
  // instance needs half the registers; groups of up to 8 heads, integer formats): then one block
  // per wave beats two blocks for some waves and one for others.  Measured at 40K and 48K tokens.
  if (c->format != BD_FMT_MXFP4 && fmt_group(c->format) == kBlock && c->n_q_heads / c->n_kv_heads <= 8 &&
      (long)quanta * units <= 768)
    return quanta;
  // With one workgroup per compute unit already, a single split needs no merge kernel at all; that beats
  // the better occupancy of two splits until the call is long enough to amortize the merge (measured at
  // 256 and 384 units: 30.0 against 32.4 us and 41.9 against 47.1 us at 4K tokens, 99.5 against 94.2 us at 16K).
  // (2-bit codes: the kernel is bound by arithmetic and the second split pays earlier -- 40.7 against 44.6 us
  // at 32 sequences x 8K tokens)
  if (units >= 256 && (long)nb * units <= (fmt_is_int(c->format) && fmt_bits(c->format) == 2 ? 12288 : 16384)) return 1;
  // (some kernel instances run one workgroup per compute unit: groups of 32 with more than 4 query heads
  // per KV head, for 4-bit codes and for per-token K)
  const bool one_wg = fmt_group(c->format) == 32 && (fmt_bits(c->format) == 4 || fmt_kt(c->format)) && c->n_q_heads / c->n_kv_heads > 4;
  const long target = one_wg ? 256 : 512;
  int want = (int)((target + units - 1) / units);
  if (want < 1) want = 1;
  // (no rebalancing: quanta are dealt to the splits round robin, so a count that does not divide them
  // leaves a few workgroups one quantum short, which is faster than fewer workgroups of equal length)
  const int splits = quanta < want ? quanta : want;
  return splits < 1 ? 1 : splits;
}

size_t bd_workspace_bytes(const bd_cache* c, int32_t num_splits) {
  if (check_shape(c) != BD_OK || num_splits < 1) return 0;
  return (size_t)num_splits * c->batch * c->n_q_heads * (kD + 2) * sizeof(float);
}

bd_status bd_quant_pack_kv(const bd_cache* c, const void* k, const void* v, int32_t L, int32_t* packed_len,
                           int32_t* res_len, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_buffers(c)) != BD_OK) return s;
  if (L < 0 || !packed_len || !res_len) return BD_ERR_INVALID_ARG;
  if (L > 0 && (!k || !v)) return BD_ERR_INVALID_ARG;
  if (L > 0 && (!aligned16(k) || !aligned16(v))) return BD_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  const int units = c->batch * c->n_kv_heads;
  const long stride = (long)L * kD;
  if (c->format == BD_FMT_MXFP4) {
    if (L > c->capacity) return BD_ERR_CAPACITY;
    if ((s = hip_status(launch_mx_quant(k, v, stride, L, units, c, 0, st))) != BD_OK) return s;
    *packed_len = L;
    *res_len = 0;
    return BD_OK;
  }
  const int nb = L / kBlock, r = L % kBlock;
  if (nb * kBlock > c->capacity) return BD_ERR_CAPACITY;
  if ((s = hip_status(launch_quant_blocks(k, v, stride, 0, nb, units, c, 0, st))) != BD_OK)
    return s;
  if ((s = hip_status(launch_copy_rows(k, v, stride, nb * kBlock, c->k_res, c->v_res, (long)kBlock * kD, 0, r,
                                       units, st))) != BD_OK)
    return s;
  *packed_len = nb * kBlock;
  *res_len = r;
  return BD_OK;
}

bd_status bd_append_kv(const bd_cache* c, const void* k_new, const void* v_new, int32_t* packed_len,
                       int32_t* res_len, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_buffers(c)) != BD_OK) return s;
  if (!k_new || !v_new || !packed_len || !res_len) return BD_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new)) return BD_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  const int units = c->batch * c->n_kv_heads;
  if (c->format == BD_FMT_MXFP4) {
    if (*packed_len < 0 || *res_len != 0) return BD_ERR_INVALID_ARG;
    if (*packed_len + 1 > c->capacity) return BD_ERR_CAPACITY;
    if ((s = hip_status(launch_mx_quant(k_new, v_new, (long)kD, 1, units, c, *packed_len, st))) != BD_OK) return s;
    *packed_len += 1;
    return BD_OK;
  }
  const int pl = *packed_len, r = *res_len;
  if (pl < 0 || pl % kBlock != 0 || r < 0 || r >= kBlock || pl > c->capacity) return BD_ERR_INVALID_ARG;
  const bool flush = r == kBlock - 1;
  if (flush && pl + kBlock > c->capacity) return BD_ERR_CAPACITY;
  if ((s = hip_status(launch_copy_rows(k_new, v_new, (long)kD, 0, c->k_res, c->v_res, (long)kBlock * kD, r, 1, units,
                                       st))) != BD_OK)
    return s;
  if (flush) {
    // The residual block is full: quantize and pack it as packed block pl/128 (Sec. IV-B(1)).
    if ((s = hip_status(launch_quant_blocks(c->k_res, c->v_res, (long)kBlock * kD, 0, 1, units, c,
                                            pl / kBlock, st))) != BD_OK)
      return s;
    *packed_len = pl + kBlock;
    *res_len = 0;
  } else {
    *res_len = r + 1;
  }
  return BD_OK;
}

bd_status bd_decode_attn(const bd_cache* c, const void* q, int32_t packed_len, int32_t res_len, float softmax_scale,
                         int32_t num_splits, void* workspace, void* out, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_buffers(c)) != BD_OK) return s;
  if (!q || !workspace || num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(workspace) || (out && !aligned16(out))) return BD_ERR_ALIGNMENT;
  if (packed_len < 0 || packed_len > c->capacity) return BD_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  float* part_o = ws_part_o(workspace);
  float* part_ml = ws_part_ml(c, workspace, num_splits);
  if (c->format == BD_FMT_MXFP4) {
    if (res_len != 0) return BD_ERR_INVALID_ARG;
    s = hip_status(launch_decode_mx(c, q, packed_len, softmax_scale, num_splits, part_o, part_ml, nullptr, nullptr, out,
                                    st));
  } else {
    if (packed_len % kBlock != 0 || res_len < 0 || res_len >= kBlock) return BD_ERR_INVALID_ARG;
    if (fmt_group(c->format) != kBlock)
      s = hip_status(launch_decode_grp(c, q, packed_len, res_len, softmax_scale, num_splits, part_o, part_ml, nullptr,
                                       nullptr, out, st));
    else
      s = hip_status(launch_decode_int(c, q, packed_len, res_len, softmax_scale, num_splits, part_o, part_ml,
                                       nullptr, nullptr, out, st));
  }
  if (s != BD_OK) return s;
  // (one split: the attention kernel has written `out` itself, there is nothing to merge)
  if (out && num_splits > 1) s = hip_status(launch_combine(c, part_o, part_ml, num_splits, out, st));
  return s;
}

bd_status bd_decode_attn_static(const bd_cache* c, const void* q, int32_t packed_len, int32_t res_len,
                                float softmax_scale, int32_t num_splits, void* out, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if (!out || num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (bd_workspace_bytes(c, num_splits) > (size_t)BD_STATIC_SCRATCH_BYTES) return BD_ERR_CAPACITY;
  void* ws = nullptr;
  if ((s = static_scratch_ptr(&ws)) != BD_OK) return s;
  // Every partial the merge reads is written by this call's attention launch first (empty splits
  // store m = -inf, l = 0), so nothing of the previous call's contents has to be cleared.
  return bd_decode_attn(c, q, packed_len, res_len, softmax_scale, num_splits, ws, out, stream);
}

bd_status bd_probe_stream_read(const bd_cache* c, int32_t packed_len, void* sink, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_buffers(c)) != BD_OK) return s;
  if ((long)c->batch * c->n_kv_heads > 32767) return BD_ERR_UNSUPPORTED;   // the probe's grid: two rows per unit
  if (packed_len < 0 || packed_len % kBlock != 0 || packed_len > c->capacity) return BD_ERR_INVALID_ARG;
  if (sink && (reinterpret_cast<uintptr_t>(sink) & 3u)) return BD_ERR_ALIGNMENT;
  return hip_status(launch_stream_probe(c, packed_len, sink, (hipStream_t)stream));
}

// One decode step of a contiguous cache.  lazy: the paper's Residual Kernel (Sec. III-A(1), IV-B(1)) -- the
// step that fills the residual block attends its 128 half-precision rows and packs them afterwards;
// otherwise the block is packed first and attended quantized (bd_append_kv + bd_decode_attn).
static bd_status decode_step(const bd_cache* c, const void* k_new, const void* v_new, const void* q,
                             int32_t* packed_len, int32_t* res_len, float softmax_scale, int32_t num_splits,
                             void* workspace, void* out, void* stream, bool lazy) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_buffers(c)) != BD_OK) return s;
  if (!k_new || !v_new || !q || !packed_len || !res_len || !workspace || !out) return BD_ERR_INVALID_ARG;
  if (num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(q) || !aligned16(workspace) || !aligned16(out))
    return BD_ERR_ALIGNMENT;
  const int pl = *packed_len, r = *res_len;
  hipStream_t st = (hipStream_t)stream;
  float* part_o = ws_part_o(workspace);
  float* part_ml = ws_part_ml(c, workspace, num_splits);
  const int gq = c->n_q_heads / c->n_kv_heads;
  if (c->format == BD_FMT_MXFP4) {
    if (pl < 0 || r != 0 || pl > c->capacity) return BD_ERR_INVALID_ARG;
    if (pl + 1 > c->capacity) return BD_ERR_CAPACITY;
    if (gq > 16) {   // several workgroups read the token's block: the append stays a launch of its own
      if ((s = bd_append_kv(c, k_new, v_new, packed_len, res_len, stream)) != BD_OK) return s;
      return bd_decode_attn(c, q, *packed_len, *res_len, softmax_scale, num_splits, workspace, out, stream);
    }
    // one workgroup per split and KV head: the attention launch quantizes the token into the cache itself
    // (the workgroup that reads its block does, first thing)
    if ((s = hip_status(launch_decode_mx(c, q, pl, softmax_scale, num_splits, part_o, part_ml, k_new, v_new, out,
                                         st))) != BD_OK)
      return s;
    if (num_splits > 1 && (s = hip_status(launch_combine(c, part_o, part_ml, num_splits, out, st))) != BD_OK) return s;
    *packed_len = pl + 1;
    return BD_OK;
  }
  if (pl < 0 || pl % kBlock != 0 || r < 0 || r >= kBlock || pl > c->capacity) return BD_ERR_INVALID_ARG;
  const bool fills = r == kBlock - 1;
  if (fills && pl + kBlock > c->capacity) return BD_ERR_CAPACITY;
  const bool grp = fmt_group(c->format) != kBlock;
  if (fills && !lazy && gq > (grp ? 8 : 16)) {
    // several workgroups per split and KV head read the block the step fills, so no single one can pack it
    // inside the attention launch before it is read: the step runs as the calls it is defined by.  (The lazy
    // order has no such reader: its extra workgroup packs the block for any group size.)
    if ((s = bd_append_kv(c, k_new, v_new, packed_len, res_len, stream)) != BD_OK) return s;
    return bd_decode_attn(c, q, *packed_len, *res_len, softmax_scale, num_splits, workspace, out, stream);
  }
  // one attention launch: it reads the new token from k_new / v_new and files it, and on the step that fills
  // the residual block it packs the block as well (before attending it, or, lazy, after)
  const int flush = !fills ? 0 : lazy ? 2 : 1;
  const int att_pl = flush == 1 ? pl + kBlock : pl, att_r = flush == 1 ? 0 : r + 1;
  s = hip_status(grp ? launch_decode_grp(c, q, att_pl, att_r, softmax_scale, num_splits, part_o, part_ml, k_new, v_new, out, st,
                                         flush)
                     : launch_decode_int(c, q, att_pl, att_r, softmax_scale, num_splits, part_o, part_ml, k_new, v_new, out, st,
                                         flush));
  if (s != BD_OK) return s;
  if (num_splits > 1 && (s = hip_status(launch_combine(c, part_o, part_ml, num_splits, out, st))) != BD_OK) return s;
  *packed_len = fills ? pl + kBlock : pl;
  *res_len = fills ? 0 : r + 1;
  return BD_OK;
}

bd_status bd_decode_step(const bd_cache* c, const void* k_new, const void* v_new, const void* q,
                         int32_t* packed_len, int32_t* res_len, float softmax_scale, int32_t num_splits,
                         void* workspace, void* out, void* stream) {
  return decode_step(c, k_new, v_new, q, packed_len, res_len, softmax_scale, num_splits, workspace, out, stream, false);
}

bd_status bd_decode_step_lazy(const bd_cache* c, const void* k_new, const void* v_new, const void* q,
                              int32_t* packed_len, int32_t* res_len, float softmax_scale, int32_t num_splits,
                              void* workspace, void* out, void* stream) {
  return decode_step(c, k_new, v_new, q, packed_len, res_len, softmax_scale, num_splits, workspace, out, stream, true);
}

bd_status bd_splitk_combine(const bd_cache* c, const void* workspace, int32_t num_splits, void* out, void* stream) {
  bd_status s = check_shape(c);
  if (s != BD_OK) return s;
  if (!workspace || !out || num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (!aligned16(workspace) || !aligned16(out)) return BD_ERR_ALIGNMENT;
  void* ws = const_cast<void*>(workspace);
  return hip_status(launch_combine(c, ws_part_o(ws), ws_part_ml(c, ws, num_splits), num_splits, out,
                                   (hipStream_t)stream));
}

// ---- paged cache ------------------------------------------------------------------------------

static bd_cache shape_of(const bd_paged_cache* c) {
  bd_cache s{};
  s.batch = c->batch;
  s.n_q_heads = c->n_q_heads;
  s.n_kv_heads = c->n_kv_heads;
  s.head_dim = c->head_dim;
  s.format = c->format;
  s.capacity = kBlock;
  s.out_type = c->out_type;
  return s;
}

static bd_status check_paged_shape(const bd_paged_cache* c) {
  if (!c) return BD_ERR_INVALID_ARG;
  const bd_cache s = shape_of(c);
  bd_status st = check_shape(&s);
  if (st != BD_OK) return st;
  if (c->num_pages <= 0 || c->max_pages_per_seq <= 0) return BD_ERR_INVALID_ARG;
  return BD_OK;
}

static bd_status check_paged_buffers(const bd_paged_cache* c) {
  const bool mx = c->format == BD_FMT_MXFP4;   // no residual: every token is quantized on arrival
  const void* need[8] = {c->k_codes, c->v_codes, c->k_params, c->v_params, mx ? (void*)16 : c->k_res,
                         mx ? (void*)16 : c->v_res, c->block_table, c->seq_lens};
  for (int i = 0; i < 8; ++i) {
    if (!need[i]) return BD_ERR_INVALID_ARG;
    if (i < 6 ? !aligned16(need[i]) : (reinterpret_cast<uintptr_t>(need[i]) & 3u) != 0) return BD_ERR_ALIGNMENT;
  }
  if (c->status && (reinterpret_cast<uintptr_t>(c->status) & 3u) != 0) return BD_ERR_ALIGNMENT;
  return BD_OK;
}

size_t bd_paged_cache_bytes(const bd_paged_cache* c, int which) {
  if (check_paged_shape(c) != BD_OK || which < 0 || which > 7) return 0;
  const size_t pool = (size_t)c->num_pages * c->n_kv_heads, bits = (size_t)bits_of(c->format);
  if (c->format == BD_FMT_MXFP4) {
    switch (which) {
      case 0: case 1: return pool * kBlock * (kD / 2);
      case 2: case 3: return pool * kBlock * (kD / kMxGroup);
      case 4: case 5: return 0;
      default: break;
    }
  }
  const size_t groups = (size_t)(kBlock / fmt_group(c->format));
  switch (which) {
    case 0: case 1: return pool * kBlock * kD * bits / 8;
    case 2: return pool * groups * kD * 4;
    case 3: return pool * kBlock * groups * 4;
    case 4: case 5: return (size_t)c->batch * c->n_kv_heads * kBlock * kD * 2;
    case 6: return (size_t)c->batch * c->max_pages_per_seq * 4;
    default: return (size_t)c->batch * 4;
  }
}

size_t bd_paged_workspace_bytes(const bd_paged_cache* c, int32_t num_splits) {
  if (check_paged_shape(c) != BD_OK) return 0;
  const bd_cache s = shape_of(c);
  return bd_workspace_bytes(&s, num_splits);
}

bd_status bd_paged_quant_pack_kv(const bd_paged_cache* c, int32_t seq, const void* k, const void* v, int32_t L,
                                 void* stream) {
  bd_status s = check_paged_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_paged_buffers(c)) != BD_OK) return s;
  if (seq < 0 || seq >= c->batch || L < 0) return BD_ERR_INVALID_ARG;
  if (L > 0 && (!k || !v)) return BD_ERR_INVALID_ARG;
  if (L > 0 && (!aligned16(k) || !aligned16(v))) return BD_ERR_ALIGNMENT;
  const int blocks = c->format == BD_FMT_MXFP4 ? (L + kBlock - 1) / kBlock : L / kBlock;
  if (blocks > c->max_pages_per_seq) return BD_ERR_CAPACITY;
  return hip_status(launch_paged_prefill(c, seq, k, v, L, (hipStream_t)stream));
}

bd_status bd_paged_append_kv(const bd_paged_cache* c, const void* k_new, const void* v_new, void* stream) {
  bd_status s = check_paged_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_paged_buffers(c)) != BD_OK) return s;
  if (!k_new || !v_new) return BD_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new)) return BD_ERR_ALIGNMENT;
  return hip_status(launch_paged_append(c, k_new, v_new, true, (hipStream_t)stream));
}

// attention over the paged cache; `step`: the lengths still lack this step's token, and the merge raises
// them.  The token has been filed by a preceding launch_paged_append(bump = false), or, with k_new / v_new
// (main integer kernel only), is appended by the attention launch itself.
static bd_status paged_attention(const bd_paged_cache* c, const void* q, float softmax_scale, int32_t num_splits,
                                 void* workspace, void* out, bool step, hipStream_t st,
                                 const void* k_new = nullptr, const void* v_new = nullptr, bool lazy = false) {
  const bd_cache shape = shape_of(c);
  float* part_o = ws_part_o(workspace);
  float* part_ml = ws_part_ml(&shape, workspace, num_splits);
  // one split: the attention kernel writes `out` itself and no merge runs (a fused step then raises the
  // lengths with the small kernel of bd_paged_append_kv instead of in the merge)
  void* direct = num_splits == 1 ? out : nullptr;
  bd_status s = hip_status(c->format == BD_FMT_MXFP4
                               ? launch_decode_mx_paged(c, q, softmax_scale, num_splits, part_o, part_ml, step, k_new, v_new,
                                                        direct, st)
                           : fmt_group(c->format) != kBlock
                               ? launch_decode_grp_paged(c, q, softmax_scale, num_splits, part_o, part_ml, step, k_new, v_new,
                                                         direct, st, lazy)
                               : launch_decode_paged(c, q, softmax_scale, num_splits, part_o, part_ml, step, k_new, v_new,
                                                     direct, st, lazy));
  if (s != BD_OK) return s;
  if (direct) return step ? hip_status(launch_paged_bump(c, st)) : BD_OK;
  return hip_status(launch_combine(&shape, part_o, part_ml, num_splits, out, st, step ? c : nullptr));
}

bd_status bd_paged_decode_attn(const bd_paged_cache* c, const void* q, float softmax_scale, int32_t num_splits,
                               void* workspace, void* out, void* stream) {
  bd_status s = check_paged_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_paged_buffers(c)) != BD_OK) return s;
  if (!q || !workspace || !out || num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(workspace) || !aligned16(out)) return BD_ERR_ALIGNMENT;
  return paged_attention(c, q, softmax_scale, num_splits, workspace, out, false, (hipStream_t)stream);
}

bd_status bd_paged_decode_step(const bd_paged_cache* c, const void* k_new, const void* v_new, const void* q,
                               float softmax_scale, int32_t num_splits, void* workspace, void* out, void* stream) {
  bd_status s = check_paged_shape(c);
  if (s != BD_OK) return s;
  if ((s = check_paged_buffers(c)) != BD_OK) return s;
  if (!k_new || !v_new || !q || !workspace || !out || num_splits < 1 || num_splits > 65534) return BD_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(q) || !aligned16(workspace) || !aligned16(out))
    return BD_ERR_ALIGNMENT;
  hipStream_t st = (hipStream_t)stream;
  // One workgroup per split and KV head (query groups of up to 16 heads; 8 for the group-64/32 formats):
  // two launches.  The attention kernel reads the new token from the caller's buffers and files it
  // (integer: the workgroup that reads the block a step fills quantizes it first; MXFP4: the workgroup
  // that reads the token's block quantizes the token into it), and the merge raises the lengths.
  // (the kernel of the group-64/32 formats takes 8 heads per workgroup, the others 16)
  if (c->n_q_heads / c->n_kv_heads <= (fmt_is_int(c->format) && fmt_group(c->format) != kBlock ? 8 : 16))
    return paged_attention(c, q, softmax_scale, num_splits, workspace, out, true, st, k_new, v_new);
  // otherwise three launches instead of four: the append leaves the lengths alone, the attention
  // kernel counts the new token in, and the merge, last in line, raises the lengths
  if ((s = hip_status(launch_paged_append(c, k_new, v_new, false, st))) != BD_OK) return s;
  return paged_attention(c, q, softmax_scale, num_splits, workspace, out, true, st);
}

bd_status bd_paged_decode_step_lazy(const bd_paged_cache* c, const void* k_new, const void* v_new, const void* q,
                                    float softmax_scale, int32_t num_splits, void* workspace, void* out, void* stream) {
  bd_status s = check_paged_shape(c);
  if (s != BD_OK) return s;
  if (c->format == BD_FMT_MXFP4)   // no residual: nothing to flush lazily
    return bd_paged_decode_step(c, k_new, v_new, q, softmax_scale, num_splits, workspace, out, stream);
  if ((s = check_paged_buffers(c)) != BD_OK) return s;
  if (!k_new || !v_new || !q || !workspace || !out || num_splits < 1 || num_splits > 65533) return BD_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(q) || !aligned16(workspace) || !aligned16(out))
    return BD_ERR_ALIGNMENT;
  // Two launches for every query group size: no workgroup has to read the block a sequence fills, so the extra
  // workgroup per (sequence, KV head) packs it while the others attend the 128 fp16 rows.
  return paged_attention(c, q, softmax_scale, num_splits, workspace, out, true, (hipStream_t)stream, k_new, v_new, true);
}

const char* bd_strerror(bd_status s) {
  switch (s) {
    case BD_OK: return "ok";
    case BD_ERR_INVALID_ARG: return "invalid argument";
    case BD_ERR_UNSUPPORTED: return "unsupported shape";
    case BD_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
    case BD_ERR_CAPACITY: return "cache capacity exceeded";
    case BD_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int bd_last_hip_error(void) { return bd::g_last_hip_error; }

}  // extern "C"
