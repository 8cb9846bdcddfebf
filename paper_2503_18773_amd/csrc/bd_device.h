// Device-side helpers shared by the decode kernels (gfx950, wave64).
#pragma once

#include "bd_common.h"

namespace bd {
namespace {

__device__ __forceinline__ float h2f(uint16_t b) {
  _Float16 h;
  __builtin_memcpy(&h, &b, 2);
  return (float)h;
}
__device__ __forceinline__ uint16_t f2h(float f) {
  _Float16 h = (_Float16)f;
  uint16_t b;
  __builtin_memcpy(&b, &h, 2);
  return b;
}

// DPP lane movement inside rows of 16 lanes.
constexpr int kRowShl4 = 0x104, kRowShl8 = 0x108, kRowShl12 = 0x10C, kRowShr4 = 0x114, kRowShr8 = 0x118, kRowRor4 = 0x124, kRowRor8 = 0x128;
constexpr int kQuadSwap1 = 0xB1 /* [1,0,3,2] */, kQuadSwap2 = 0x4E /* [2,3,0,1] */;
constexpr int kRowHalfMirror = 0x141, kRowMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a row, result in every lane
__device__ __forceinline__ float row_sum16(float x) {
  x += dpp_f<kQuadSwap1>(x);
  x += dpp_f<kQuadSwap2>(x);
  x += dpp_f<kRowHalfMirror>(x);
  x += dpp_f<kRowMirror>(x);
  return x;
}
// 2^e for e in [-126, 127]
__device__ __forceinline__ float pow2i(int e) { return __uint_as_float((uint32_t)(e + 127) << 23); }
// the power of two that brings fp16 magnitudes up to `bits` (the largest one's bit pattern) below 2^top
__device__ __forceinline__ int norm_exponent(uint32_t bits, int top) { return top + 14 - (int)(bits >> 10); }
// Q' = q * scale * position factor goes to the matrix unit as an fp16 high + low pair: queries are brought
// below 2^7 and a block's K scales below 2^8, so |Q'| < 2^15 (finite) and the low pieces of all but
// negligible entries stay above the subnormals.
constexpr int kQTop = 7, kSTop = 8;
__device__ __forceinline__ uint32_t row_max16_u(uint32_t m) {
  m = max(m, dpp_u<kQuadSwap1>(m));
  m = max(m, dpp_u<kQuadSwap2>(m));
  m = max(m, dpp_u<kRowHalfMirror>(m));
  m = max(m, dpp_u<kRowMirror>(m));
  return m;
}
// largest of a non-negative value over the wave, as a wave-uniform result
__device__ __forceinline__ uint32_t wave_max_u(uint32_t m) {
  m = row_max16_u(m);
  return max(max(__builtin_amdgcn_readlane(m, 0), __builtin_amdgcn_readlane(m, 16)),
             max(__builtin_amdgcn_readlane(m, 32), __builtin_amdgcn_readlane(m, 48)));
}
// reductions over the lanes that carry the same head (column % (16 / COPIES)): COPIES column
// groups x 4 lane groups
template <int COPIES>
__device__ __forceinline__ float head_sum(float x) {
  if (COPIES == 4) x += dpp_f<kRowRor4>(x);
  if (COPIES >= 2) x += dpp_f<kRowRor8>(x);
  x += __shfl_xor(x, 16);
  x += __shfl_xor(x, 32);
  return x;
}
template <int COPIES>
__device__ __forceinline__ float head_max(float x) {
  if (COPIES == 4) x = fmaxf(x, dpp_f<kRowRor4>(x));
  if (COPIES >= 2) x = fmaxf(x, dpp_f<kRowRor8>(x));
  x = fmaxf(x, __shfl_xor(x, 16));
  x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}

// Contiguous cache, fused step whose token fills the residual block (Sec. IV-B(1)): how the attention launch
// packs the block (DecodeArgs / GrpArgs flush_mode).
constexpr int kFlushNone = 0, kFlushFirst = 1, kFlushAfter = 2;

// Element type of the output rows: the format's own half type (fp16; bf16 for MXFP4) or fp32
// (bd_cache.out_type).
constexpr int kOutF16 = 0, kOutBf16 = 1, kOutF32 = 2;
__host__ __device__ __forceinline__ int out_kind(int format, int out_type) {
  return out_type == BD_OUT_F32 ? kOutF32 : format == BD_FMT_MXFP4 ? kOutBf16 : kOutF16;
}
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// A launch with one split needs no merge: the workgroup's (L, o) is the result, stored as two
// adjacent outputs o / L at elements idx, idx + 1 of `out`, exactly as the merge kernel would
// compute them (a head that attended nothing, L == 0, gives zeros).
__device__ __forceinline__ void store_final_pair(void* out, size_t idx, int kind, float o0, float o1, float L) {
  const float r0 = L > 0.f ? o0 / L : 0.f, r1 = L > 0.f ? o1 / L : 0.f;
  if (kind == kOutF32) {
    *reinterpret_cast<float2*>(reinterpret_cast<float*>(out) + idx) = make_float2(r0, r1);
    return;
  }
  const uint32_t lo = kind == kOutBf16 ? f2bf(r0) : f2h(r0), hi = kind == kOutBf16 ? f2bf(r1) : f2h(r1);
  *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(out) + idx) = lo | (hi << 16);
}

__device__ __forceinline__ void wave_sync() {
  // LDS operations of one wave execute in order; this only stops the compiler from moving
  // accesses across the exchange point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Makes global stores of this workgroup visible to its own later loads, for data that the workgroup
// writes and then reads back inside one launch: wait until the stores have been written through to
// L2, then meet.  The waves of a workgroup share their compute unit's vector cache, which its own
// stores keep current, so workgroup scope is all this needs -- and all it can afford: measured at one
// such workgroup per (sequence, KV head) and decode step, a device-scope release (__threadfence(),
// which also writes back the XCD's L2) cost 45 us per launch and a device-scope acquire (which
// invalidates the vector cache) 7 us.
__device__ __forceinline__ void workgroup_global_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Index of per-token float2 parameters staged in LDS: lanes that work on different 32-token chunks read
// the same offset of their chunks at once, and entries 32 apart (256 bytes) share their banks, so every
// chunk is shifted by two entries (arrays hold kParSlots entries).
constexpr int kParSlots = 128 + 8;
__device__ __forceinline__ int par_slot(int t) { return t + 2 * (t >> 5); }

}  // namespace
}  // namespace bd
