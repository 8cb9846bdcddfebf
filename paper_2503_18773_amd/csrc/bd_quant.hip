// Online quantize-and-pack kernels: the quantize half of the paper's Residual Kernel
// (Sec. IV-B) and the prefill quantization (Sec. IV-B(1)).
//
// Bit-exactness contract: every stored scale, zero and code is the result of IEEE fp32
// subtract / divide / round-half-even in a fixed order, so contraction into FMAs is switched
// off for this file and no fast-math substitution is allowed.
#include <type_traits>

#include "bd_common.h"

#pragma clang fp contract(off)

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
  const float y0 = __builtin_amdgcn_rcpf(scale_f);
  const float y = __builtin_fmaf(__builtin_fmaf(-scale_f, y0, 1.0f), y0, y0);
  return scale_f == 0.0f ? 0.0f : y;
}

template <bool UNIFORM>
__device__ __forceinline__ void code_bytes(const uint32_t* raw, const float* scale, const float* rcp,
                                           const float* zero, uint32_t& lo, uint32_t& hi) {
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
// G: quantization group (128, 64 or 32; not with KT): K statistics over G tokens per channel --
//    a wave holds 32 tokens, so the cross-wave step of the ladder joins G/32 waves -- and V
//    statistics over G channels per token; parameters [block][128/G][D] and [block][128][D/G].
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
  static_assert(!KT || G == kBlock, "per-token K has one group per token");
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
  // apart, V rows consecutive.)
  uint32_t kraw[T][C / 2], vraw[T][C / 2];
  const uint32_t koff = (uint32_t)(krow(0) * kD + C * cg) * 2u, voff = (uint32_t)(vrow(0) * kD + C * cg) * 2u;
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const u4_t ld = *reinterpret_cast<const u4_t*>(reinterpret_cast<const char*>(ksrc) + koff + t * (4 * kD * 2));
    kraw[t][0] = ld[0]; kraw[t][1] = ld[1]; kraw[t][2] = ld[2]; kraw[t][3] = ld[3];
  }
#pragma unroll
  for (int t = 0; t < T; ++t) {
    const u4_t ld = *reinterpret_cast<const u4_t*>(reinterpret_cast<const char*>(vsrc) + voff + t * (kD * 2));
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
      if constexpr (BITS == 4) (k_codes + dblk * (kBlock * NCG))[at] = w;
      else (reinterpret_cast<uint16_t*>(k_codes) + dblk * (kBlock * NCG))[at] = (uint16_t)w;
    };
    if constexpr (KT) {
      uint32_t lo[T], hi[T];
      token_rows(kraw, std::integral_constant<int, NCG>{},
                 [&](int t, uint32_t packed) { if (cg == 0) (k_params + dblk * kBlock)[(uint32_t)krow(t)] = packed; }, lo, hi);
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
    for (int k = 0; k < kD * WPC / 256; ++k) {
      const int idx = tid + 256 * k;
      (v_codes + dblk * (size_t)(kD * WPC))[(uint32_t)idx] = vw[idx / WPC][idx % WPC];
    }
  }
}

// Contiguous cache: block blockIdx.x of unit blockIdx.y.
template <int BITS, bool KT, int G>
__global__ __launch_bounds__(256, KT ? 3 : 4) void quant_block_kernel(const uint16_t* __restrict__ ksrc,
                                                           const uint16_t* __restrict__ vsrc,
                                                           long src_unit_stride, int src_tok0,
                                                           uint32_t* __restrict__ k_codes,
                                                           uint32_t* __restrict__ v_codes,
                                                           uint32_t* __restrict__ k_params,
                                                           uint32_t* __restrict__ v_params, int nbcap,
                                                           int dst_blk0) {
  const int unit = blockIdx.y, blk = blockIdx.x;
  const size_t dblk = (size_t)unit * nbcap + dst_blk0 + blk;
  const size_t src_off = (size_t)unit * src_unit_stride + ((size_t)src_tok0 + (size_t)blk * kBlock) * kD;
  quant_block<BITS, KT, G>(ksrc + src_off, vsrc + src_off, k_codes, v_codes, k_params, v_params, dblk);
}

// ---- paged cache (page = one 128-token block; pool index of (page, head) = page * H + head) ---

struct PagedArgs {
  uint32_t *k_codes, *v_codes, *k_params, *v_params;
  uint16_t *k_res, *v_res;
  const int32_t* block_table;
  int32_t* seq_lens;
  int32_t* status;
  int n_kv_heads, num_pages, max_pages;
};

// Page of block n of sequence b, or -1 (and bit `flag` of *status set) if the table has no
// valid entry for it.
__device__ __forceinline__ int page_of(const PagedArgs& a, int b, int n, int flag) {
  int page = -1;
  if (n < a.max_pages) page = a.block_table[(size_t)b * a.max_pages + n];
  if (page < 0 || page >= a.num_pages) {
    if (a.status && threadIdx.x == 0) atomicOr(a.status, flag);
    return -1;
  }
  return page;
}

// Prefill of one sequence: block blockIdx.x of KV head blockIdx.y, source [H][L][128].
template <int BITS, bool KT, int G>
__global__ __launch_bounds__(256, KT ? 3 : 4) void paged_quant_kernel(PagedArgs a, const uint16_t* __restrict__ ksrc,
                                                           const uint16_t* __restrict__ vsrc, int seq, int L) {
  const int blk = blockIdx.x, h = blockIdx.y;
  const int page = page_of(a, seq, blk, 2);
  if (page < 0) return;
  const size_t src_off = ((size_t)h * L + (size_t)blk * kBlock) * kD;
  quant_block<BITS, KT, G>(ksrc + src_off, vsrc + src_off, a.k_codes, a.v_codes, a.k_params, a.v_params,
                           (size_t)page * a.n_kv_heads + h);
}

// Prefill, rest: the L mod 128 newest tokens of every head go to the sequence's residual and
// the length is recorded.  One workgroup per KV head.
__global__ __launch_bounds__(256) void paged_tail_kernel(PagedArgs a, const u4_t* __restrict__ ksrc,
                                                          const u4_t* __restrict__ vsrc, int seq, int L) {
  const int h = blockIdx.x, r = L % kBlock;
  const size_t so = ((size_t)h * L + (size_t)(L - r)) * (kD / 8);
  const size_t dn = ((size_t)seq * a.n_kv_heads + h) * kBlock * (kD / 8);
  u4_t* kd = reinterpret_cast<u4_t*>(a.k_res);
  u4_t* vd = reinterpret_cast<u4_t*>(a.v_res);
  for (int i = threadIdx.x; i < r * (kD / 8); i += blockDim.x) {
    kd[dn + i] = ksrc[so + i];
    vd[dn + i] = vsrc[so + i];
  }
  if (h == 0 && threadIdx.x == 0) a.seq_lens[seq] = L;
}

// One decode step of sequence blockIdx.y, KV head blockIdx.x: the new token row goes to residual
// slot len mod 128; if that fills the residual it is quantized into the sequence's next page
// (Sec. IV-B(1)).  Lengths are bumped by paged_bump_kernel afterwards, so every workgroup of
// the sequence sees the same length here.
template <int BITS, bool KT, int G>
__global__ __launch_bounds__(256) void paged_append_kernel(PagedArgs a, const uint16_t* __restrict__ k_new,
                                                            const uint16_t* __restrict__ v_new) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int len = a.seq_lens[b];
  if (len < 0) return;
  const int nb = len / kBlock, r = len % kBlock;
  const size_t unit = (size_t)b * a.n_kv_heads + h;
  int page = 0;
  if (r == kBlock - 1) {
    page = page_of(a, b, nb, 2);
    if (page < 0) return;   // the token is dropped; the length stays
  }
  uint16_t* kr = a.k_res + unit * kBlock * kD;
  uint16_t* vr = a.v_res + unit * kBlock * kD;
  if (threadIdx.x < 32) {
    const bool is_v = threadIdx.x >= 16;
    const int c8 = 8 * (threadIdx.x & 15);
    const u4_t val = *reinterpret_cast<const u4_t*>((is_v ? v_new : k_new) + unit * kD + c8);
    *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (size_t)r * kD + c8) = val;
  }
  if (r != kBlock - 1) return;
  // the row just written is read back below by other threads of this workgroup
  __threadfence();
  __syncthreads();
  quant_block<BITS, KT, G>(kr, vr, a.k_codes, a.v_codes, a.k_params, a.v_params, (size_t)page * a.n_kv_heads + h);
}

// seq_lens[b] += 1 for every sequence whose step went through (same test as the append kernel:
// a page is needed when the step fills the residual, or, if `every_token`, by every token).
__global__ void paged_bump_kernel(PagedArgs a, int batch, bool every_token) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  const int len = a.seq_lens[b];
  if (len < 0) return;
  if (every_token || len % kBlock == kBlock - 1) {
    const int n = len / kBlock;
    int page = -1;
    if (n < a.max_pages) page = a.block_table[(size_t)b * a.max_pages + n];
    if (page < 0 || page >= a.num_pages) return;
  }
  a.seq_lens[b] = len + 1;
}

// Copies `ntok` token rows of K and of V between [unit][token][128] arrays of 16-bit values.
__global__ __launch_bounds__(256) void copy_rows_kernel(const u4_t* __restrict__ ksrc,
                                                         const u4_t* __restrict__ vsrc, long src_unit_stride,
                                                         int src_tok0, u4_t* __restrict__ kdst,
                                                         u4_t* __restrict__ vdst, long dst_unit_stride,
                                                         int dst_tok0, int ntok) {
  const int unit = blockIdx.x;
  const size_t so = ((size_t)unit * src_unit_stride + (size_t)src_tok0 * kD) / 8;
  const size_t dn = ((size_t)unit * dst_unit_stride + (size_t)dst_tok0 * kD) / 8;
  const int n = ntok * (kD / 8);
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    kdst[dn + i] = ksrc[so + i];
    vdst[dn + i] = vsrc[so + i];
  }
}

// ---- MXFP4 -------------------------------------------------------------------------------

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

// Where the 128-token blocks of an MXFP4 launch go: block `blk` of unit `u` is block
// u * nbcap + blk of the arrays (contiguous cache), or, for one sequence of a paged cache, block
// page * H + u with page = table_row[blk] (u = KV head).  -1 (and bit 1 of *status) if the table has
// no valid page for it.  Inside a block: K codes [128][64], scales [128][4], V codes [128 ch][64].
struct MxDst {
  uint8_t *k_codes, *k_scales, *v_codes, *v_scales;
  int nbcap;
  const int32_t* table_row;
  int32_t* status;
  int n_kv_heads, num_pages, max_pages;
};
__device__ __forceinline__ long mx_block_index(const MxDst& d, int u, int blk) {
  if (!d.table_row) return (long)u * d.nbcap + blk;
  int page = -1;
  if (blk < d.max_pages) page = d.table_row[blk];
  if (page < 0 || page >= d.num_pages) {
    if (d.status && threadIdx.x == 0) atomicOr(d.status, 2);
    return -1;
  }
  return (long)page * d.n_kv_heads + u;
}

// One workgroup quantizes up to 128 tokens (one V block) of one (batch, kv_head).
// Thread t handles token t: 4 MX groups of K and of V.  K codes go out token-major;
// V codes pass through an LDS tile to be written channel-major, two tokens per byte.
// When `single` (decode append of one token) the V bytes are updated nibble-wise.
__global__ __launch_bounds__(128) void mx_quant_kernel(const uint16_t* __restrict__ ksrc,
                                                        const uint16_t* __restrict__ vsrc,
                                                        long src_unit_stride, int ntok, MxDst d,
                                                        int dst_tok0) {
  constexpr int PITCH = kD + 4;
  __shared__ uint8_t tile[kBlock * PITCH];
  uint8_t *k_codes = d.k_codes, *k_scales = d.k_scales, *v_codes = d.v_codes, *v_scales = d.v_scales;
  const int unit = blockIdx.y;
  // this workgroup covers destination tokens [t_lo, t_hi) of block `dblk`
  const int first_blk = dst_tok0 / kBlock;
  const int dblk = first_blk + blockIdx.x;
  const int t_lo = max(dblk * kBlock, dst_tok0);
  const int t_hi = min((dblk + 1) * kBlock, dst_tok0 + ntok);
  const int t = dblk * kBlock + threadIdx.x;  // destination token of this thread
  const bool live = t >= t_lo && t < t_hi;
  const long bi = mx_block_index(d, unit, dblk);
  if (bi < 0) return;

  if (live) {
    const size_t so = (size_t)unit * src_unit_stride + (size_t)(t - dst_tok0) * kD;
    const size_t tok = (size_t)bi * kBlock + threadIdx.x;
#pragma unroll 1
    for (int which = 0; which < 2; ++which) {
      const uint16_t* src = (which == 0 ? ksrc : vsrc) + so;
      uint32_t scale_word = 0;
#pragma unroll 1
      for (int g = 0; g < kD / kMxGroup; ++g) {
        float xv[kMxGroup];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          u4_t raw = *reinterpret_cast<const u4_t*>(src + g * kMxGroup + 8 * v);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            xv[8 * v + 2 * e] = bf16_bits_to_float((uint16_t)(raw[e] & 0xFFFFu));
            xv[8 * v + 2 * e + 1] = bf16_bits_to_float((uint16_t)(raw[e] >> 16));
          }
        }
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < kMxGroup; ++i) amax = fmaxf(amax, fabsf(xv[i]));
        int e = 0;
        if (amax > 0.0f) e = mx_shared_exp(amax);
        scale_word |= (uint32_t)(e + 127) << (8 * g);
        if (which == 0) {
          u4_t out;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t word = 0;
#pragma unroll
            for (int n = 0; n < 8; ++n)
              word |= (amax > 0.0f ? e2m1_code(xv[8 * w + n], e) : 0u) << (4 * n);
            out[w] = word;
          }
          *reinterpret_cast<u4_t*>(k_codes + tok * (kD / 2) + g * 16) = out;
        } else {
#pragma unroll
          for (int i = 0; i < kMxGroup; ++i)
            tile[threadIdx.x * PITCH + g * kMxGroup + i] =
                (uint8_t)(amax > 0.0f ? e2m1_code(xv[i], e) : 0u);
        }
      }
      *reinterpret_cast<uint32_t*>((which == 0 ? k_scales : v_scales) + tok * 4) = scale_word;
    }
  }
  __syncthreads();
  // V codes, channel-major: byte j of channel c holds block tokens 2j (low), 2j+1 (high).
  uint8_t* vrow = v_codes + (size_t)bi * (size_t)(kD * 64);
  const int j_lo = (t_lo - dblk * kBlock) / 2, j_hi = (t_hi - dblk * kBlock + 1) / 2;
  const int nj = j_hi - j_lo;
  for (int k = threadIdx.x; k < kD * nj; k += 128) {
    const int ch = k / nj, j = j_lo + k % nj;
    const int id = ch * 64 + j;
    const int ta = dblk * kBlock + 2 * j, tb = ta + 1;
    uint8_t old = 0;
    const bool a_new = ta >= t_lo && ta < t_hi, b_new = tb >= t_lo && tb < t_hi;
    if (!(a_new && b_new)) old = vrow[id];       // keep the nibble of a token not in this call
    uint8_t lo = a_new ? tile[(2 * j) * PITCH + ch] : (uint8_t)(old & 0x0F);
    uint8_t hi = b_new ? tile[(2 * j + 1) * PITCH + ch] : (uint8_t)(old >> 4);
    // a token beyond the current end of the cache has never been written: store 0 for it
    if (!b_new && tb >= t_hi) hi = 0;
    vrow[id] = (uint8_t)(lo | (hi << 4));
  }
}

// Whole 128-token blocks of an MXFP4 cache (the bulk of a prefill).  256 threads; a thread takes
// one MX group (32 channels) of a token at a time -- 64 contiguous bytes, neighbouring lanes
// neighbouring groups, so every load and every K store is fully coalesced -- twice per tensor.
// The group maximum is taken on the bf16 magnitudes as loaded (packed 16-bit maxima); codes
// come from v_cvt_scalef32_pk_fp4_f32 (nearest e2m1, ties to the even code, saturating: measured
// identical to the definition) except that it keeps the sign of values that round to zero,
// which is cleared afterwards; groups with a very small maximum (shared exponent below -120,
// where elements can be fp32 subnormals) take the explicit path.  V codes meet their
// neighbouring token's (one byte = two tokens) by a DPP lane shift and reach their
// channel-major place through an LDS tile.
__global__ __launch_bounds__(256) void mx_quant_block_kernel(const uint16_t* __restrict__ ksrc,
                                                              const uint16_t* __restrict__ vsrc,
                                                              long src_unit_stride, MxDst d, int dst_blk0) {
  constexpr int PITCH = 80;   // bytes per channel row of the tile (64 used; 16-byte aligned rows)
  __shared__ __attribute__((aligned(16))) uint8_t tile[kD * PITCH];
  uint8_t *k_codes = d.k_codes, *k_scales = d.k_scales, *v_codes = d.v_codes, *v_scales = d.v_scales;
  const int unit = blockIdx.y, blk = dst_blk0 + blockIdx.x, tid = threadIdx.x, g = tid & 3;
  const long bi = mx_block_index(d, unit, blk);
  if (bi < 0) return;
  const size_t src_blk = (size_t)unit * src_unit_stride + (size_t)blockIdx.x * kBlock * kD;
#pragma unroll 1
  for (int which = 0; which < 2; ++which) {
    const uint16_t* src = (which == 0 ? ksrc : vsrc) + src_blk;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int tl = (tid >> 2) + 64 * i;   // token inside the block
      const size_t tok = (size_t)bi * kBlock + tl;
      const uint16_t* sp = src + (size_t)tl * kD + kMxGroup * g;
      uint32_t raw[16];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const u4_t ld = *reinterpret_cast<const u4_t*>(sp + 8 * v);
        raw[4 * v] = ld[0]; raw[4 * v + 1] = ld[1]; raw[4 * v + 2] = ld[2]; raw[4 * v + 3] = ld[3];
      }
      typedef unsigned short us2_t __attribute__((ext_vector_type(2)));
      us2_t m2 = {0, 0};
#pragma unroll
      for (int w = 0; w < 16; ++w)
        m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(us2_t, raw[w] & 0x7FFF7FFFu));
      const uint32_t mag = m2[0] > m2[1] ? m2[0] : m2[1];   // bf16 bits of the largest magnitude
      int e = 0;
      if (mag != 0) {
        e = (int)(mag >> 7) - 127 - 2;   // floor(log2 amax) - 2 from the exponent field
        e = e < -127 ? -127 : e;
      }
      uint32_t cw[4] = {0u, 0u, 0u, 0u};   // 32 codes: channel 8w + n of the group at nibble n of cw[w]
      if (mag != 0) {
        if (e >= -120) {
          const float scale = __uint_as_float((uint32_t)(e + 127) << 23);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t c = 0;
#define BD_CVT_PAIR(b)                                                                                        \
  c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, __uint_as_float(raw[4 * w + b] << 16),                      \
                                               __uint_as_float(raw[4 * w + b] & 0xFFFF0000u), scale, b)
            BD_CVT_PAIR(0);
            BD_CVT_PAIR(1);
            BD_CVT_PAIR(2);
            BD_CVT_PAIR(3);
#undef BD_CVT_PAIR
            // a value that rounds to zero is stored as +0: drop the sign of nibbles with no magnitude
            const uint32_t m = c & 0x77777777u;
            cw[w] = (((m + 0x77777777u) & c) & 0x88888888u) | m;
          }
        } else {
#pragma unroll
          for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int n = 0; n < 8; ++n) {
              const uint32_t r = raw[4 * w + (n >> 1)];
              const float x = __uint_as_float((n & 1) ? (r & 0xFFFF0000u) : (r << 16));
              cw[w] |= e2m1_code(x, e) << (4 * n);
            }
        }
      }
      if (which == 0) {
        k_scales[tok * 4 + g] = (uint8_t)(e + 127);
        u4_t out = {cw[0], cw[1], cw[2], cw[3]};
        *reinterpret_cast<u4_t*>(k_codes + tok * (kD / 2) + g * 16) = out;
      } else {
        v_scales[tok * 4 + g] = (uint8_t)(e + 127);
        // the next token's codes of the same group sit 4 lanes up
        uint32_t pw[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) pw[w] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)cw[w], 0x104, 0xF, 0xF, true);
        if (((tid >> 2) & 1) == 0) {   // even token: byte j = tl / 2 of 32 channel rows
          const int col = ((tl >> 1) + 16 * g) & 63;   // rows of group g are rotated by 16 g bytes (bank spread)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t be = (cw[w] & 0x0F0F0F0Fu) | ((pw[w] & 0x0F0F0F0Fu) << 4);          // channels 0, 2, 4, 6
            const uint32_t bo = ((cw[w] >> 4) & 0x0F0F0F0Fu) | (pw[w] & 0xF0F0F0F0u);          // channels 1, 3, 5, 7
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const int ch = kMxGroup * g + 8 * w + 2 * k;
              tile[ch * PITCH + col] = (uint8_t)(be >> (8 * k));
              tile[(ch + 1) * PITCH + col] = (uint8_t)(bo >> (8 * k));
            }
          }
        }
      }
    }
  }
  __syncthreads();
  // channel-major V codes of the block: 128 rows of 64 bytes, each thread half a row
  {
    const int row = tid >> 1, hf = tid & 1, gg = row >> 5;
    uint8_t* dst = v_codes + ((size_t)bi * kD + row) * 64 + 32 * hf;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int chunk = 2 * hf + c;
      const u4_t val = *reinterpret_cast<const u4_t*>(&tile[row * PITCH + 16 * ((chunk + gg) & 3)]);
      *reinterpret_cast<u4_t*>(dst + 16 * c) = val;
    }
  }
}


// Decode-step append for MXFP4: one token per (batch, kv_head), thread = channel.  The MX
// group statistics are wave shuffles over 32 lanes; K bytes pair neighbouring channels, V
// bytes are updated nibble-wise in the channel-major block layout.
// One token of one (sequence, KV head): thread c quantizes channel c of the new K and V rows and
// files the codes at position i of block bi (V: one nibble of byte i/2 of its channel row).
__device__ __forceinline__ void mx_append_token(const uint16_t* __restrict__ k_row, const uint16_t* __restrict__ v_row,
                                                const MxDst& d, long bi, int i) {
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
    d.k_scales[tok * 4 + c / kMxGroup] = (uint8_t)(ke + 127);
    d.v_scales[tok * 4 + c / kMxGroup] = (uint8_t)(ve + 127);
  }
  const uint32_t kc_hi = __shfl_down(kc, 1);
  if ((c & 1) == 0) d.k_codes[tok * (kD / 2) + c / 2] = (uint8_t)(kc | (kc_hi << 4));
  uint8_t* vb = d.v_codes + ((size_t)bi * kD + c) * 64 + i / 2;
  if ((i & 1) == 0)
    *vb = (uint8_t)vc;                                  // first token of the byte: the other nibble is not there yet
  else
    *vb = (uint8_t)((*vb & 0x0Fu) | (vc << 4));
}

// Contiguous cache: token t of every unit.
__global__ __launch_bounds__(128) void mx_append_kernel(const uint16_t* __restrict__ k_new,
                                                         const uint16_t* __restrict__ v_new, MxDst d, int t) {
  const int unit = blockIdx.x;
  mx_append_token(k_new + (size_t)unit * kD, v_new + (size_t)unit * kD, d, (long)unit * d.nbcap + t / kBlock,
                  t % kBlock);
}

// Paged cache, one decode step: the token of sequence blockIdx.y, KV head blockIdx.x goes to
// position len mod 128 of the page of block len / 128.  Without a valid page the token is dropped
// (bit 1 of *status) and paged_bump_kernel leaves the length as it is.
__global__ __launch_bounds__(128) void mx_paged_append_kernel(MxDst d, const int32_t* __restrict__ block_table,
                                                               const int32_t* __restrict__ seq_lens,
                                                               const uint16_t* __restrict__ k_new,
                                                               const uint16_t* __restrict__ v_new) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int len = seq_lens[b];
  if (len < 0) return;
  d.table_row = block_table + (size_t)b * d.max_pages;
  const long bi = mx_block_index(d, h, len / kBlock);
  if (bi < 0) return;
  const size_t unit = (size_t)b * d.n_kv_heads + h;
  mx_append_token(k_new + unit * kD, v_new + unit * kD, d, bi, len % kBlock);
}

__global__ void set_len_kernel(int32_t* seq_lens, int seq, int L) {
  if (threadIdx.x == 0 && blockIdx.x == 0) seq_lens[seq] = L;
}

}  // namespace

// Tokens [dst_tok0, dst_tok0 + ntok) of every unit: whole blocks through the block kernel, the
// rest through the general one.
static hipError_t launch_mx_range(const uint16_t* kk, const uint16_t* vv, long src_unit_stride, int ntok, int units,
                           const MxDst& d, int dst_tok0, hipStream_t st) {
  // tokens [t0, t1) of the range that do not fill a block go through the general kernel
  auto partial = [&](int t0, int t1) -> hipError_t {
    if (t1 <= t0) return hipSuccess;
    const size_t off = (size_t)(t0 - dst_tok0) * kD;
    dim3 grid((t1 - 1) / kBlock - t0 / kBlock + 1, units), block(128);
    mx_quant_kernel<<<grid, block, 0, st>>>(kk + off, vv + off, src_unit_stride, t1 - t0, d, t0);
    return hipGetLastError();
  };
  const int end = dst_tok0 + ntok;
  const int full0 = (dst_tok0 + kBlock - 1) / kBlock, full1 = end / kBlock;   // whole blocks [full0, full1)
  if (full1 <= full0) return partial(dst_tok0, end);
  hipError_t e = partial(dst_tok0, full0 * kBlock);
  if (e != hipSuccess) return e;
  const size_t off = (size_t)(full0 * kBlock - dst_tok0) * kD;
  mx_quant_block_kernel<<<dim3(full1 - full0, units), dim3(256), 0, st>>>(kk + off, vv + off, src_unit_stride, d, full0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return partial(full1 * kBlock, end);
}

hipError_t launch_quant_blocks(const void* k, const void* v, long src_unit_stride, int src_tok0, int nblocks,
                               int units, const bd_cache* c, int dst_blk0, hipStream_t st) {
  if (nblocks <= 0) return hipSuccess;
  dim3 grid(nblocks, units), block(256);
  const int nbcap = c->capacity / kBlock;
  const uint16_t *kk = (const uint16_t*)k, *vv = (const uint16_t*)v;
  uint32_t *kc = (uint32_t*)c->k_codes, *vc = (uint32_t*)c->v_codes, *kp = (uint32_t*)c->k_params,
           *vp = (uint32_t*)c->v_params;
#define BD_QUANT_CASE(FMT, BITS, KT, G)                                                                          \
  case FMT:                                                                                                      \
    quant_block_kernel<BITS, KT, G><<<grid, block, 0, st>>>(kk, vv, src_unit_stride, src_tok0, kc, vc, kp, vp, \
                                                            nbcap, dst_blk0);                                    \
    break;
  switch (c->format) {
    BD_QUANT_CASE(BD_FMT_INT4, 4, false, 128)
    BD_QUANT_CASE(BD_FMT_INT2, 2, false, 128)
    BD_QUANT_CASE(BD_FMT_INT4_KT, 4, true, 128)
    BD_QUANT_CASE(BD_FMT_INT2_KT, 2, true, 128)
    BD_QUANT_CASE(BD_FMT_INT4_G64, 4, false, 64)
    BD_QUANT_CASE(BD_FMT_INT4_G32, 4, false, 32)
    BD_QUANT_CASE(BD_FMT_INT2_G64, 2, false, 64)
    BD_QUANT_CASE(BD_FMT_INT2_G32, 2, false, 32)
    default: return hipErrorInvalidValue;
  }
#undef BD_QUANT_CASE
  return hipGetLastError();
}

static PagedArgs paged_args(const bd_paged_cache* c) {
  PagedArgs a;
  a.k_codes = (uint32_t*)c->k_codes;
  a.v_codes = (uint32_t*)c->v_codes;
  a.k_params = (uint32_t*)c->k_params;
  a.v_params = (uint32_t*)c->v_params;
  a.k_res = (uint16_t*)c->k_res;
  a.v_res = (uint16_t*)c->v_res;
  a.block_table = c->block_table;
  a.seq_lens = c->seq_lens;
  a.status = c->status;
  a.n_kv_heads = c->n_kv_heads;
  a.num_pages = c->num_pages;
  a.max_pages = c->max_pages_per_seq;
  return a;
}

static MxDst paged_mx_dst(const bd_paged_cache* c) {
  MxDst d{};
  d.k_codes = (uint8_t*)c->k_codes;
  d.k_scales = (uint8_t*)c->k_params;
  d.v_codes = (uint8_t*)c->v_codes;
  d.v_scales = (uint8_t*)c->v_params;
  d.nbcap = 1;
  d.status = c->status;
  d.n_kv_heads = c->n_kv_heads;
  d.num_pages = c->num_pages;
  d.max_pages = c->max_pages_per_seq;
  return d;
}

hipError_t launch_paged_prefill(const bd_paged_cache* c, int seq, const void* k, const void* v, int L,
                                hipStream_t st) {
  if (c->format == BD_FMT_MXFP4) {
    // every token is quantized on arrival: the last, partly filled block lives in a page as well
    MxDst d = paged_mx_dst(c);
    d.table_row = c->block_table + (size_t)seq * c->max_pages_per_seq;
    if (L > 0) {
      hipError_t e = launch_mx_range((const uint16_t*)k, (const uint16_t*)v, (long)L * kD, L, c->n_kv_heads, d, 0, st);
      if (e != hipSuccess) return e;
    }
    set_len_kernel<<<dim3(1), dim3(64), 0, st>>>(c->seq_lens, seq, L);
    return hipGetLastError();
  }
  const PagedArgs a = paged_args(c);
  const int nb = L / kBlock;
  if (nb > 0) {
    dim3 grid(nb, c->n_kv_heads), block(256);
    const uint16_t *kk = (const uint16_t*)k, *vv = (const uint16_t*)v;
    switch (c->format) {
      case BD_FMT_INT4: paged_quant_kernel<4, false, 128><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT2: paged_quant_kernel<2, false, 128><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT4_KT: paged_quant_kernel<4, true, 128><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT2_KT: paged_quant_kernel<2, true, 128><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT4_G64: paged_quant_kernel<4, false, 64><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT4_G32: paged_quant_kernel<4, false, 32><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT2_G64: paged_quant_kernel<2, false, 64><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      case BD_FMT_INT2_G32: paged_quant_kernel<2, false, 32><<<grid, block, 0, st>>>(a, kk, vv, seq, L); break;
      default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  paged_tail_kernel<<<dim3(c->n_kv_heads), dim3(256), 0, st>>>(a, (const u4_t*)k, (const u4_t*)v, seq, L);
  return hipGetLastError();
}

hipError_t launch_paged_append(const bd_paged_cache* c, const void* k_new, const void* v_new, bool bump,
                               hipStream_t st) {
  const PagedArgs a = paged_args(c);
  dim3 grid(c->n_kv_heads, c->batch), block(256);
  const uint16_t *kk = (const uint16_t*)k_new, *vv = (const uint16_t*)v_new;
  if (c->format == BD_FMT_MXFP4) {
    mx_paged_append_kernel<<<grid, dim3(128), 0, st>>>(paged_mx_dst(c), c->block_table, c->seq_lens, kk, vv);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !bump) return e;
    paged_bump_kernel<<<dim3((c->batch + 63) / 64), dim3(64), 0, st>>>(a, c->batch, true);
    return hipGetLastError();
  }
  switch (c->format) {
    case BD_FMT_INT4: paged_append_kernel<4, false, 128><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT2: paged_append_kernel<2, false, 128><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT4_KT: paged_append_kernel<4, true, 128><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT2_KT: paged_append_kernel<2, true, 128><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT4_G64: paged_append_kernel<4, false, 64><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT4_G32: paged_append_kernel<4, false, 32><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT2_G64: paged_append_kernel<2, false, 64><<<grid, block, 0, st>>>(a, kk, vv); break;
    case BD_FMT_INT2_G32: paged_append_kernel<2, false, 32><<<grid, block, 0, st>>>(a, kk, vv); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !bump) return e;
  paged_bump_kernel<<<dim3((c->batch + 63) / 64), dim3(64), 0, st>>>(a, c->batch, false);
  return hipGetLastError();
}

hipError_t launch_paged_bump(const bd_paged_cache* c, hipStream_t st) {
  paged_bump_kernel<<<dim3((c->batch + 63) / 64), dim3(64), 0, st>>>(paged_args(c), c->batch, c->format == BD_FMT_MXFP4);
  return hipGetLastError();
}

hipError_t launch_copy_rows(const void* ksrc, const void* vsrc, long src_unit_stride, int src_tok0, void* kdst,
                            void* vdst, long dst_unit_stride, int dst_tok0, int ntok, int units,
                            hipStream_t st) {
  if (ntok <= 0) return hipSuccess;
  const int threads = ntok * (kD / 8) >= 256 ? 256 : 64;
  copy_rows_kernel<<<dim3(units), dim3(threads), 0, st>>>((const u4_t*)ksrc, (const u4_t*)vsrc,
                                                          src_unit_stride, src_tok0, (u4_t*)kdst, (u4_t*)vdst,
                                                          dst_unit_stride, dst_tok0, ntok);
  return hipGetLastError();
}

hipError_t launch_mx_quant(const void* k, const void* v, long src_unit_stride, int ntok, int units,
                           const bd_cache* c, int dst_tok0, hipStream_t st) {
  if (ntok <= 0) return hipSuccess;
  MxDst d{};
  d.k_codes = (uint8_t*)c->k_codes;
  d.k_scales = (uint8_t*)c->k_params;
  d.v_codes = (uint8_t*)c->v_codes;
  d.v_scales = (uint8_t*)c->v_params;
  d.nbcap = c->capacity / kBlock;
  const uint16_t *kk = (const uint16_t*)k, *vv = (const uint16_t*)v;
  if (ntok == 1 && src_unit_stride == kD) {
    mx_append_kernel<<<dim3(units), dim3(128), 0, st>>>(kk, vv, d, dst_tok0);
    return hipGetLastError();
  }
  return launch_mx_range(kk, vv, src_unit_stride, ntok, units, d, dst_tok0, st);
}

}  // namespace bd
