// Shared declarations of the HIP sources of libbitdecode.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bitdecode.h"

namespace bd {

constexpr int kD = 128;       // head_dim
constexpr int kBlock = 128;   // residual block N_r (Eq. 1) == quantization group
constexpr int kMxGroup = 32;  // elements per MX block

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
typedef int i8_t __attribute__((ext_vector_type(8)));

// Records a failing HIP call for bd_last_hip_error().
void note_hip_error(hipError_t e);

// Kernel launchers (host side, defined next to their kernels).  All return hipError_t of
// the launch.  `units` = batch * n_kv_heads.
hipError_t launch_quant_blocks(const void* k, const void* v, long src_unit_stride, int src_tok0,
                               int nblocks, int units, const bd_cache* c, int dst_blk0,
                               hipStream_t st);

static inline bool fmt_is_int(int f) { return f != BD_FMT_MXFP4 && f >= BD_FMT_INT4 && f <= BD_FMT_INT2_KT_G32; }
static inline int fmt_bits(int f) {
  return (f == BD_FMT_INT2 || f == BD_FMT_INT2_KT || f == BD_FMT_INT2_G64 || f == BD_FMT_INT2_G32 ||
          f == BD_FMT_INT2_KT_G64 || f == BD_FMT_INT2_KT_G32) ? 2 : 4;
}
static inline bool fmt_kt(int f) { return f == BD_FMT_INT4_KT || f == BD_FMT_INT2_KT || (f >= BD_FMT_INT4_KT_G64 && f <= BD_FMT_INT2_KT_G32); }
// quantization group: tokens per K group and channels per V group
static inline int fmt_group(int f) {
  return (f == BD_FMT_INT4_G64 || f == BD_FMT_INT2_G64 || f == BD_FMT_INT4_KT_G64 || f == BD_FMT_INT2_KT_G64)   ? 64
         : (f == BD_FMT_INT4_G32 || f == BD_FMT_INT2_G32 || f == BD_FMT_INT4_KT_G32 || f == BD_FMT_INT2_KT_G32) ? 32
                                                                                                                : 128;
}
hipError_t launch_copy_rows(const void* ksrc, const void* vsrc, long src_unit_stride, int src_tok0,
                            void* kdst, void* vdst, long dst_unit_stride, int dst_tok0, int ntok,
                            int units, hipStream_t st);
// measurement aid: streams the packed K and V codes of the first packed_len tokens and nothing else
hipError_t launch_stream_probe(const bd_cache* c, int packed_len, void* sink, hipStream_t st);
hipError_t launch_mx_quant(const void* k, const void* v, long src_unit_stride, int ntok, int units,
                           const bd_cache* c, int dst_tok0, hipStream_t st);

hipError_t launch_paged_prefill(const bd_paged_cache* c, int seq, const void* k, const void* v, int L,
                                hipStream_t st);
hipError_t launch_paged_append(const bd_paged_cache* c, const void* k_new, const void* v_new, bool bump,
                               hipStream_t st);
// `out` (all decode launchers): with num_splits == 1 and out != nullptr the kernel writes the final output
// rows itself and no merge is needed; otherwise it writes the split partials.
// raises the length of every sequence whose step's token was appended (launch_paged_append with bump = false)
hipError_t launch_paged_bump(const bd_paged_cache* c, hipStream_t st);
// k_new / v_new non-null (with step): the launch appends the step's token itself -- no launch_paged_append
// before it; query groups of up to 16 heads only
hipError_t launch_decode_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                               float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                               void* out, hipStream_t st, bool lazy = false);

// k_new / v_new non-null: fused step -- residual token res_len-1 is read from k_new / v_new
// ([B][Hkv][128]) and also stored into the residual buffers by the kernel.
// flush (with k_new / v_new, query groups of up to 16 heads): the step's token fills the residual block and
// the launch packs it as well -- 1: before attending it (packed_len counts the block, res_len == 0);
// 2: after attending its 128 fp16 rows (res_len == 128; one more workgroup per KV head does the packing)
hipError_t launch_decode_int(const bd_cache* c, const void* q, int packed_len, int res_len,
                             float softmax_scale, int num_splits, float* part_o, float* part_ml,
                             const void* k_new, const void* v_new, void* out, hipStream_t st, int flush = 0);
// formats with a quantization group of 64 or 32 (k_new / v_new and flush as in launch_decode_int; the flush
// forms for query groups of up to 8 heads only)
hipError_t launch_decode_grp(const bd_cache* c, const void* q, int packed_len, int res_len, float softmax_scale,
                             int num_splits, float* part_o, float* part_ml, const void* k_new, const void* v_new,
                             void* out, hipStream_t st, int flush = 0);
// (k_new / v_new as in launch_decode_paged; query groups of up to 8 heads only)
hipError_t launch_decode_grp_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                                   float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                                   void* out, hipStream_t st, bool lazy = false);
// k_new / v_new non-null: the launch quantizes the step's token into the cache itself (contiguous: at index
// `length`, and attends length + 1 tokens; paged: with `step`); query groups of up to 16 heads only
hipError_t launch_decode_mx_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                                  float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                                  void* out, hipStream_t st);
hipError_t launch_decode_mx(const bd_cache* c, const void* q, int length, float softmax_scale,
                            int num_splits, float* part_o, float* part_ml, const void* k_new, const void* v_new,
                            void* out, hipStream_t st);
// step_of: the paged cache whose fused step this merge ends (it then raises the lengths), or nullptr
hipError_t launch_combine(const bd_cache* c, const float* part_o, const float* part_ml, int nparts,
                          void* out, hipStream_t st, const bd_paged_cache* step_of = nullptr);

static inline float* ws_part_o(void* ws) { return reinterpret_cast<float*>(ws); }
static inline float* ws_part_ml(const bd_cache* c, void* ws, int num_splits) {
  return reinterpret_cast<float*>(ws) + (size_t)num_splits * c->batch * c->n_q_heads * kD;
}

}  // namespace bd
