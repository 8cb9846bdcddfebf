// The block quantizer of the integer formats: one workgroup of 256 threads turns 128 token rows of
// K and V (fp16) into one packed block -- the quantize half of the paper's Residual Kernel
// (Sec. IV-B) and the prefill quantization (Sec. IV-B(1)).  Shared by the quantizer kernels and by
// the attention kernel of the paged fused step, which quantizes the block that a step fills.
//
// Bit-exactness contract: every stored scale, zero and code is the result of IEEE fp32
// subtract / divide / round-half-even in a fixed order; the instruction sequences below reach
// those results without the division and name every fused multiply-add explicitly, so they do not
// depend on the including file's contraction setting.
#pragma once

#include <type_traits>

#include "bd_common.h"

namespace bd {
namespace {

__device__ __forceinline__ float half_bits_to_float(uint16_t b) {
  _Float16 h;
  __builtin_memcpy(&h, &b, 2);
  return (float)h;
}
__device__ __forceinline__ uint16_t float_to_half_bits(float f) {
  _Float16 h = (_Float16)f;  // round to nearest even, subnormals kept
  uint16_t b;
  __builtin_memcpy(&b, &h, 2);
  return b;
}

// scale / zero of one group from its minimum and maximum (fp16 values held in fp32).
__device__ __forceinline__ void group_params(float mn, float mx, int qmax, float& scale_f, float& zero_f,
                                             uint32_t& packed) {
#pragma clang fp contract(off)
  zero_f = mn + 0.0f;  // -0 -> +0
  // s = (mx - mn) / qmax, correctly rounded, without the division sequence: with c = fl(1 / qmax) the
  // estimate d * c, its exact remainder and one correction give the IEEE quotient (checked on the
  // host for qmax 3 and 15 against d / qmax for every fp32 d in [2^-26, 2^18], which covers every
  // difference of two finite fp16 values)
  const float c = 1.0f / (float)qmax, d = mx - mn;
  const float q0 = d * c;
  float s = __builtin_fmaf(__builtin_fmaf(-(float)qmax, q0, d), c, q0);
  // The scale is this fp32 quotient rounded to fp16 -- two roundings.  Kept opaque here, or the compiler
  // merges the last fma and the conversion into one mixed-precision fma that rounds once.
  asm("" : "+v"(s));
  uint16_t sb = float_to_half_bits(s);
  scale_f = half_bits_to_float(sb);
  packed = (uint32_t)sb | ((uint32_t)float_to_half_bits(zero_f) << 16);
}

// Codes clamp(rint((x - zero) / scale)), the quotient being the IEEE fp32 one, of the 8 fp16 values
// one thread holds of one row (raw[0..4), two per word), one code per byte: lo = codes 0..3, hi =
// codes 4..7 (UNIFORM: one scale / zero for all 8; otherwise one per value).  The hardware's
// division sequence is what would bound this kernel, and an estimate with a test for near ties does
// not help: inputs on the fp16 grid meet exact ties all the time.  Instead the group's reciprocal is
// made correctly rounded once (exact_rcp: one Newton step on v_rcp_f32's 1-ulp value), and then
//     q0 = d * y,   r = fma(-s, q0, d)  (exact),   q = fma(r, y, q0)
// is the correctly rounded quotient d / s for each value (the classical correction step, which
// needs y = RN(1 / s); checked on the host against d / s for every positive fp16 scale, with
// numerators on and within 4 ulps of every half-integer multiple of it and random ones, and with
// reciprocal seeds up to 2 ulps off).  A degenerate group (scale 0) has y = 0 and d = 0: codes 0.
// x >= zero always (zero is the group's minimum) and, for a scale that is a normal fp16 number,
// d / s <= qmax * (1 + 2^-10), so the upper clamp only ever acts for a scale that is an fp16
// subnormal (is_tiny_scale), where d / s <= 1.5 * qmax: such rows are clamped afterwards, on the
// bytes (clamp_code_bytes).  v_cvt_pk_u8_f32 rounds to nearest even, like rintf.

// x - zero for the low / high fp16 of a pair: one mixed-precision fma instead of a conversion and a
// subtraction (same single rounding of the exact difference)
__device__ __forceinline__ float sub_lo(uint32_t pair, float zero) {
  float d;
  asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(zero));
  return d;
}
__device__ __forceinline__ float sub_hi(uint32_t pair, float zero) {
  float d;
  asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(pair), "v"(zero));
  return d;
}

// RN(1 / scale) for a scale that is an fp16 value; 0 for a degenerate group
__device__ __forceinline__ float exact_rcp(float scale_f) {
#pragma clang fp contract(off)
  const float y0 = __builtin_amdgcn_rcpf(scale_f);
  const float y = __builtin_fmaf(__builtin_fmaf(-scale_f, y0, 1.0f), y0, y0);
  return scale_f == 0.0f ? 0.0f : y;
}

template <bool UNIFORM>
__device__ __forceinline__ void code_bytes(const uint32_t* raw, const float* scale, const float* rcp,
                                           const float* zero, uint32_t& lo, uint32_t& hi) {
#pragma clang fp contract(off)
  lo = hi = 0;
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const int i = UNIFORM ? 0 : n;
    const float d = (n & 1) ? sub_hi(raw[n / 2], zero[i]) : sub_lo(raw[n / 2], zero[i]);
    const float q0 = d * rcp[i];
    const float q = __builtin_fmaf(__builtin_fmaf(-scale[i], q0, d), rcp[i], q0);
    if (n < 4) lo = __builtin_amdgcn_cvt_pk_u8_f32(q, n, lo);
    else hi = __builtin_amdgcn_cvt_pk_u8_f32(q, n - 4, hi);
  }
}

// min(code, qmax) on four code bytes at once, for codes <= 1.5 * qmax + 1 (one bit above the field)
template <int BITS>
__device__ __forceinline__ uint32_t clamp_code_bytes(uint32_t b) {
  constexpr uint32_t kOver = BITS == 4 ? 0x10101010u : 0x04040404u, kField = BITS == 4 ? 0x0f0f0f0fu : 0x03030303u;
  const uint32_t t = b & kOver;
  return (b | (t - (t >> BITS))) & kField;
}

__device__ __forceinline__ bool is_tiny_scale(float scale_f) { return scale_f < 0x1p-14f && scale_f > 0.0f; }

// 8 codes, one per byte in lo / hi, as one word of BITS-wide fields (code n at bit BITS * n)
template <int BITS>
__device__ __forceinline__ uint32_t pack_code_bytes(uint32_t lo, uint32_t hi) {
  if constexpr (BITS == 4) {
    lo |= lo >> 4;   // bytes 0 and 2 now hold two codes each
    hi |= hi >> 4;
    return __builtin_amdgcn_perm(hi, lo, 0x06040200u);
  } else {
    lo |= lo >> 6;
    lo |= lo >> 12;  // byte 0 now holds the four codes
    hi |= hi >> 6;
    hi |= hi >> 12;
    return __builtin_amdgcn_perm(hi, lo, 0x0c0c0400u);
  }
}

// b[t] = the codes of 4 channels of token t (one per byte), t = 0..7  ->  w[c] = channel c's 8 codes as
// BITS-wide fields, token t at bit BITS * t
template <int BITS>
__device__ __forceinline__ void transpose_code_bytes(const uint32_t* b, uint32_t* w) {
  if constexpr (BITS == 4) {
    uint32_t p[4];   // byte c = the code pair of tokens 2j, 2j+1 of channel c
#pragma unroll
    for (int j = 0; j < 4; ++j) p[j] = b[2 * j] | (b[2 * j + 1] << 4);
    // 4 x 4 byte transposition in two rounds of byte permutes
    const uint32_t x0 = __builtin_amdgcn_perm(p[1], p[0], 0x05010400u);   // p0.b0 p1.b0 p0.b1 p1.b1
    const uint32_t x1 = __builtin_amdgcn_perm(p[1], p[0], 0x07030602u);   // p0.b2 p1.b2 p0.b3 p1.b3
    const uint32_t y0 = __builtin_amdgcn_perm(p[3], p[2], 0x05010400u);
    const uint32_t y1 = __builtin_amdgcn_perm(p[3], p[2], 0x07030602u);
    w[0] = __builtin_amdgcn_perm(y0, x0, 0x05040100u);
    w[1] = __builtin_amdgcn_perm(y0, x0, 0x07060302u);
    w[2] = __builtin_amdgcn_perm(y1, x1, 0x05040100u);
    w[3] = __builtin_amdgcn_perm(y1, x1, 0x07060302u);
  } else {
    const uint32_t p = b[0] | (b[1] << 2) | (b[2] << 4) | (b[3] << 6);   // byte c = tokens 0..3 of channel c
    const uint32_t q = b[4] | (b[5] << 2) | (b[6] << 4) | (b[7] << 6);   // byte c = tokens 4..7
    w[0] = __builtin_amdgcn_perm(q, p, 0x0c0c0400u);
    w[1] = __builtin_amdgcn_perm(q, p, 0x0c0c0501u);
    w[2] = __builtin_amdgcn_perm(q, p, 0x0c0c0602u);
    w[3] = __builtin_amdgcn_perm(q, p, 0x0c0c0703u);
  }
}

__device__ __forceinline__ h2_t as_h2(uint32_t u) { return __builtin_bit_cast(h2_t, u); }
__device__ __forceinline__ uint32_t as_u32(h2_t h) { return __builtin_bit_cast(uint32_t, h); }

// Packed fp16 minimum / maximum as the bare instruction: the generic form first canonicalizes
// both operands against signalling NaNs, which finite inputs do not need.  Only for values that
// ordinary instructions consume next (no DPP read of the result).
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}

// (minimum, -maximum) of the fp16 pairs in raw[0..NP), as one half2, so that a single packed
// minimum serves both reductions
template <int NP>
__device__ __forceinline__ h2_t min_negmax(const uint32_t* raw) {
  uint32_t l = raw[0], h = raw[0];
#pragma unroll
  for (int i = 1; i < NP; ++i) {
    l = pk_min(l, raw[i]);
    h = pk_max(h, raw[i]);
  }
  const h2_t lo = as_h2(l), hi = as_h2(h);
  const _Float16 mn = lo[0] < lo[1] ? lo[0] : lo[1], mx = hi[0] > hi[1] ? hi[0] : hi[1];
  return (h2_t){mn, (_Float16)(-mx)};
}

// Packed minimum over the N consecutive lanes (N = 8, 16 or 32, aligned) that hold one token
// row; every lane ends up with the result.  DPP inside rows of 16, one shuffle across rows.
template <int CTRL>
__device__ __forceinline__ h2_t dpp_h2(h2_t x) {
  return as_h2((uint32_t)__builtin_amdgcn_update_dpp(0, (int)as_u32(x), CTRL, 0xF, 0xF, true));
}
template <int N>
__device__ __forceinline__ h2_t lanes_min(h2_t m) {
  static_assert(N == 4 || N == 8 || N == 16 || N == 32, "lanes per row group");
  m = __builtin_elementwise_min(m, dpp_h2<0xB1>(m));    // quad_perm [1,0,3,2]
  m = __builtin_elementwise_min(m, dpp_h2<0x4E>(m));    // quad_perm [2,3,0,1]
  if (N >= 8) m = __builtin_elementwise_min(m, dpp_h2<0x141>(m));   // row_half_mirror: the other quad of each 8
  if (N >= 16) m = __builtin_elementwise_min(m, dpp_h2<0x140>(m));   // row_mirror: the other half of the row
  if (N >= 32) m = __builtin_elementwise_min(m, as_h2(__shfl_xor(as_u32(m), 16)));
  return m;
}

// quant_block: the whole workgroup (256 threads) quantizes the 128 token rows at ksrc / vsrc
// ([128][128] fp16) into packed block `dblk` of the four destination arrays.
// KT: K statistics per token (over its 128 channels) instead of per channel (Sec. IV-C(1)).
// G: quantization group (128, 64 or 32): K statistics over G tokens per channel --
//    a wave holds 32 tokens, so the cross-wave step of the ladder joins G/32 waves -- and V
//    statistics over G channels per token; parameters [block][128/G][D] and [block][128][D/G].
//    With KT, K's statistics run over G channels per token like V's ([block][128][D/G]).
// A thread holds 64 values of each tensor: 8 token rows x 8 consecutive channels, i.e. one K word per
// token and one V word per channel at 4 bits, half words at 2 bits.  Minima and maxima are taken on the fp16 pairs as loaded (packed
// instructions), across lanes with shuffles and, for channel-wise K, across waves through LDS
// (the reduction ladder of Sec. IV-B(2)).
template <int BITS, bool KT, int G = kBlock>
__device__ __forceinline__ void quant_block(const uint16_t* __restrict__ ksrc, const uint16_t* __restrict__ vsrc,
                                            uint32_t* __restrict__ k_codes, uint32_t* __restrict__ v_codes,
                                            uint32_t* __restrict__ k_params, uint32_t* __restrict__ v_params,
                                            size_t dblk) {
  constexpr int QMAX = (1 << BITS) - 1;
  constexpr int CPT = 32 / BITS;     // codes per word
  constexpr int NG = kBlock / G;     // K token groups per block == V channel groups per token
  __shared__ uint32_t red_lo[4][kD / 2], red_hi[4][kD / 2];   // per wave: packed fp16 minima / maxima of channel pairs
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  constexpr int C = 8, T = 8, NCG = kD / C;   // 8 rows x 8 channels per thread; 16 lanes per token row
  const int cg = tid % NCG;
  // K: a wave holds 32 consecutive tokens, its four lane groups neighbouring rows, so that one store
  // instruction of the wave covers four consecutive token rows of codes.  V: 8 consecutive tokens per
  // thread (one V word of a channel at 4 bits, half a word at 2 bits).
  auto krow = [&](int t) { return 32 * wave + (lane >> 4) + 4 * t; };
  auto vrow = [&](int t) { return T * (tid / NCG) + t; };
  // Both tensors' rows are requested up front: V arrives while K is being worked on.  (The block's
  // address is the same for the whole workgroup; a thread adds a 32-bit byte offset.  K rows are 4 rows
  // apart, V rows consecutive.)  The source is read once and the codes are not read again by this
  // launch's other workgroups: both go past the caches as streaming (non-temporal) accesses, which
  // at prefill sizes is worth about a tenth of the kernel's time.
  uint32_t kraw[T][C / 2], vraw[T][C / 2];
  const uint32_t koff = (uint32_t)(krow(0) * kD + C * cg) * 2u, voff = (uint32_t)(vrow(0) * kD + C * cg) * 2u;
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const u4_t ld = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(reinterpret_cast<const char*>(ksrc) + koff + t * (4 * kD * 2)));
    kraw[t][0] = ld[0]; kraw[t][1] = ld[1]; kraw[t][2] = ld[2]; kraw[t][3] = ld[3];
  }
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const u4_t ld = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(reinterpret_cast<const char*>(vsrc) + voff + t * (kD * 2)));
    vraw[t][0] = ld[0]; vraw[t][1] = ld[1]; vraw[t][2] = ld[2]; vraw[t][3] = ld[3];
  }

  // Rows with statistics per token (V; K with KT): parameters of each row over the LPG consecutive
  // lanes that hold one group of it, stored by put_params(t, packed); codes one per byte in lo / hi.
  auto token_rows = [&](const uint32_t (*raw)[C / 2], auto lpg_tag, auto put_params, uint32_t* lo, uint32_t* hi) {
    constexpr int LPG = decltype(lpg_tag)::value;
    bool tiny = false;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const h2_t m = lanes_min<LPG>(min_negmax<C / 2>(raw[t]));
      float scale, zero;
      uint32_t packed;
      group_params((float)m[0], -(float)m[1], QMAX, scale, zero, packed);
      const float rcp = exact_rcp(scale);
      put_params(t, packed);
      code_bytes<true>(raw[t], &scale, &rcp, &zero, lo[t], hi[t]);
      tiny |= is_tiny_scale(scale);
    }
    if (__builtin_expect(tiny, 0)) {
#pragma unroll
      for (int t = 0; t < T; ++t) {
        lo[t] = clamp_code_bytes<BITS>(lo[t]);
        hi[t] = clamp_code_bytes<BITS>(hi[t]);
      }
    }
  };

  // ---- K: one K word of a token at 4 bits, half a word at 2 bits (stored as such: the two halves of a
  //      word come from neighbouring lanes)
  {
    auto store_k_row = [&](int t, uint32_t lo, uint32_t hi) {
      const uint32_t w = pack_code_bytes<BITS>(lo, hi);
      const uint32_t at = (uint32_t)(krow(t) * NCG + cg);   // inside the block
      if constexpr (BITS == 4) __builtin_nontemporal_store(w, k_codes + dblk * (kBlock * NCG) + at);
      else __builtin_nontemporal_store((uint16_t)w, reinterpret_cast<uint16_t*>(k_codes) + dblk * (kBlock * NCG) + at);
    };
    if constexpr (KT) {
      uint32_t lo[T], hi[T];
      constexpr int LPG = NCG / NG;   // consecutive lanes that hold one channel group of a token row
      token_rows(kraw, std::integral_constant<int, LPG>{},
                 [&](int t, uint32_t packed) {
                   if (cg % LPG == 0) (k_params + dblk * (kBlock * NG))[(uint32_t)(krow(t) * NG + cg / LPG)] = packed;
                 },
                 lo, hi);
#pragma unroll
      for (int t = 0; t < T; ++t) store_k_row(t, lo[t], hi[t]);
    } else {
      uint32_t mn[C / 2], mx[C / 2];
#pragma unroll
      for (int i = 0; i < C / 2; ++i) {
        mn[i] = mx[i] = kraw[0][i];
#pragma unroll
        for (int t = 1; t < T; ++t) {
          mn[i] = pk_min(mn[i], kraw[t][i]);
          mx[i] = pk_max(mx[i], kraw[t][i]);
        }
        // lanes holding the same channels: the other three token rows of the wave
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
          mn[i] = pk_min(mn[i], __shfl_xor(mn[i], off));
          mx[i] = pk_max(mx[i], __shfl_xor(mx[i], off));
        }
      }
      if (lane < NCG) {
#pragma unroll
        for (int i = 0; i < C / 2; ++i) {
          red_lo[wave][cg * (C / 2) + i] = mn[i];
          red_hi[wave][cg * (C / 2) + i] = mx[i];
        }
      }
      __syncthreads();
      float ks[C], kz[C], kr[C];
      bool tiny = false;
#pragma unroll
      for (int i = 0; i < C / 2; ++i) {
        const int pi = cg * (C / 2) + i;
        // the G/32 waves that hold this wave's token group
        constexpr int WPG = G / 32;
        const int w0 = wave / WPG * WPG;
        uint32_t ua = red_lo[w0][pi], ub = red_hi[w0][pi];
#pragma unroll
        for (int w = 1; w < WPG; ++w) {
          ua = pk_min(ua, red_lo[w0 + w][pi]);
          ub = pk_max(ub, red_hi[w0 + w][pi]);
        }
        const h2_t a = as_h2(ua), b = as_h2(ub);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          uint32_t packed;
          group_params((float)a[e], (float)b[e], QMAX, ks[2 * i + e], kz[2 * i + e], packed);
          kr[2 * i + e] = exact_rcp(ks[2 * i + e]);
          tiny |= is_tiny_scale(ks[2 * i + e]);
          // first thread row of the token group writes its parameters
          if (tid == w0 * 64 + cg) (k_params + dblk * (NG * kD))[(uint32_t)((wave / WPG) * kD + C * cg + 2 * i + e)] = packed;
        }
      }
      // a row's codes leave as soon as they are made
#pragma unroll
      for (int t = 0; t < T; ++t) {
        uint32_t lo, hi;
        code_bytes<false>(kraw[t], ks, kr, kz, lo, hi);
        if (__builtin_expect(tiny, 0)) {
          lo = clamp_code_bytes<BITS>(lo);
          hi = clamp_code_bytes<BITS>(hi);
        }
        store_k_row(t, lo, hi);
      }
    }
  }

  // ---- V: statistics per token.  8 tokens of a channel are one V word at 4 bits and half a word at 2
  //      bits (the halves meet in LDS).
  {
    constexpr int WPC = kBlock / CPT;   // words per channel: 16 at 4 bits, 8 at 2 bits
    constexpr int LPG = NCG / NG;       // consecutive lanes that hold one channel group of a token row
    const int tg = tid / NCG;
    uint32_t lo[T], hi[T];   // per token: the codes of channels 0..3 / 4..7, one per byte
    token_rows(vraw, std::integral_constant<int, LPG>{},
               [&](int t, uint32_t packed) {
                 if (cg % LPG == 0) (v_params + dblk * (kBlock * NG))[(uint32_t)(vrow(t) * NG + cg / LPG)] = packed;
               },
               lo, hi);
    uint32_t words[C];   // channel c: its 8 tokens' codes, token t at bit BITS * t
    transpose_code_bytes<BITS>(lo, words);
    transpose_code_bytes<BITS>(hi, words + 4);
    // Block tokens 8*tg .. 8*tg + 7 of channel C*cg + c: word tg (4 bits), or half tg % 2 of word tg / 2
    // (2 bits).  Through LDS, so that the block's words leave in address order (a thread's own words
    // are WPC apart).
    __shared__ uint32_t vw[kD][WPC + 1];
#pragma unroll
    for (int c = 0; c < C; ++c) {
      if constexpr (BITS == 4) vw[C * cg + c][tg] = words[c];
      else reinterpret_cast<uint16_t*>(&vw[C * cg + c][tg >> 1])[tg & 1] = (uint16_t)words[c];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kD * WPC / 1024; ++k) {
      const int idx = 4 * (tid + 256 * k);
      const uint32_t* row = &vw[idx / WPC][idx % WPC];
      const u4_t w4 = {row[0], row[1], row[2], row[3]};
      u4_t* dstp = reinterpret_cast<u4_t*>(v_codes + dblk * (size_t)(kD * WPC) + (uint32_t)idx);
      __builtin_nontemporal_store(w4, dstp);
    }
  }
}

}  // namespace
}  // namespace bd
