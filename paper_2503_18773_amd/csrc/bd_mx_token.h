// MXFP4 quantization of single values and of one token (Sec. IV-D(2): e2m1 codes with one shared
// e8m0 exponent per 32 elements), shared by the quantizer kernels and by the attention kernels of
// the fused decode step, which quantize the step's token themselves.
#pragma once

#include "bd_common.h"

namespace bd {
namespace {

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Shared exponent of an MX block from its largest magnitude (> 0): floor(log2(amax)) - 2,
// clamped to [-127, 127].  A subnormal amax has exponent field 0 and clamps to -127.
__device__ __forceinline__ int mx_shared_exp(float amax) {
  int ef = (int)((__float_as_uint(amax) >> 23) & 0xFFu);
  int e = ef - 127 - 2;
  return e < -127 ? -127 : e;
}

// Nearest e2m1 code of x / 2^e: ties to the even code, saturation at 6, no negative zero.
__device__ __forceinline__ uint32_t e2m1_code(float x, int e) {
  float a = fabsf(ldexpf(x, -e));
  uint32_t idx = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u
               : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
  return (x < 0.0f && idx != 0u) ? (idx | 8u) : idx;
}


// One token of one (sequence, KV head), 128 threads (threadIdx.x = channel; whole waves): the MX group
// statistics are wave shuffles over 32 lanes; the K codes (two channels per byte) and the four K and V
// scales go to position i of block bi; the V codes are filed nibble-wise in the channel-major block layout
// (one nibble of byte i/2 of each channel row).
__device__ __forceinline__ void mx_quantize_token(const uint16_t* __restrict__ k_row, const uint16_t* __restrict__ v_row,
                                                  uint8_t* k_codes, uint8_t* k_scales, uint8_t* v_codes,
                                                  uint8_t* v_scales, long bi, int i) {
  const int c = threadIdx.x;
  const float kx = bf16_bits_to_float(k_row[c]);
  const float vx = bf16_bits_to_float(v_row[c]);
  float ka = fabsf(kx), va = fabsf(vx);
#pragma unroll
  for (int off = 1; off < kMxGroup; off <<= 1) {
    ka = fmaxf(ka, __shfl_xor(ka, off));
    va = fmaxf(va, __shfl_xor(va, off));
  }
  const int ke = ka > 0.0f ? mx_shared_exp(ka) : 0, ve = va > 0.0f ? mx_shared_exp(va) : 0;
  const uint32_t kc = ka > 0.0f ? e2m1_code(kx, ke) : 0u, vc = va > 0.0f ? e2m1_code(vx, ve) : 0u;
  const size_t tok = (size_t)bi * kBlock + i;
  if ((c & (kMxGroup - 1)) == 0) {
    k_scales[tok * 4 + c / kMxGroup] = (uint8_t)(ke + 127);
    v_scales[tok * 4 + c / kMxGroup] = (uint8_t)(ve + 127);
  }
  const uint32_t kc_hi = __shfl_down(kc, 1);
  if ((c & 1) == 0) k_codes[tok * (kD / 2) + c / 2] = (uint8_t)(kc | (kc_hi << 4));
  uint8_t* vb = v_codes + ((size_t)bi * kD + c) * 64 + i / 2;
  if ((i & 1) == 0)
    *vb = (uint8_t)vc;                                  // first token of the byte: the other nibble is not there yet
  else
    *vb = (uint8_t)((*vb & 0x0Fu) | (vc << 4));
}

}  // namespace
}  // namespace bd
