// Decode attention over the MXFP4 cache (Sec. IV-D(2): native low-precision matrix
// instructions on packed 4-bit data with block scales, no dequantization for QK^T), gfx950.
//
//   S^T[token, head] = sum_c K[token, c] * Q[head, c]  on v_mfma_scale_f32_16x16x128_f8f6f4:
//     A = the token's 128 e2m1 codes exactly as stored (each lane: one MX block of 32 codes,
//     16 bytes, with its e8m0 scale applied by the instruction); B = Q.  Q stays bf16 in the
//     interface; a bf16 (8 significant bits) is the exact sum of two e4m3 numbers (4 + 4 bits),
//     so B is fed as a high and a low fp8 piece with their own block scales: two MFMAs per
//     16-token tile give the exact products, accumulated in fp32.  (The paper quantizes Q to
//     fp4, Sec. II Challenge 2; keeping it exact costs one more MFMA and no ALU work.)
//   O^T[c, head] = sum_t V[t, c] * P'[t, head]  on v_mfma_f32_16x16x32_f16:
//     V's MX blocks run along channels, i.e. across the M dimension of this product, where the
//     hardware cannot apply them (it scales along the contraction).  So V codes are expanded
//     e2m1 -> fp16 with v_cvt_scalef32_pk_f16_fp4 (scale 1) and the block scale 2^e(t, c/32) is
//     folded into the probabilities instead: four variants of P', one per 32-channel block,
//     each an exact exponent shift of p.  This is the re-quantization of P that the paper
//     names as the new bottleneck of the native path (Sec. II Challenge 2); here it is 8 values
//     per lane and block thanks to the same column-group trick as the integer kernel.
//   V codes are stored channel-major inside each 128-token block (two tokens per byte), so the
//   A operand of the second product is contraction-contiguous: 16-byte loads, no transposition.
#include "bd_common.h"
#include "bd_device.h"
#include "bd_mx_token.h"

namespace bd {
namespace {

constexpr int kWaves = 4;
constexpr float kLog2e = 1.4426950408889634f;

struct MxArgs {
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const uint8_t* k_scales;
  const uint8_t* v_scales;
  const uint16_t* q;
  float* part_o;
  float* part_ml;
  void* out;   // one split only: the output [B][Hq][128], written instead of the partials; else nullptr
  int out_kind;     // element type of `out` (kOutF16 / kOutBf16 / kOutF32)
  int n_q_heads, n_kv_heads, gq;
  int length;      // tokens in the cache
  int capacity;
  int num_splits;
  float scale_log2;
  // paged cache only: block n of sequence b is page block_table[b * max_pages + n]
  const int32_t* block_table;
  const int32_t* seq_lens;
  int32_t* status;
  int max_pages, num_pages;
  int step;   // paged: 1 when this launch is the attention of a fused step
  // fused step without an append launch: the step's token ([B][Hkv][128] bf16), which the workgroup that
  // reads its block quantizes into the cache first (contiguous: at index `length`, and the kernel attends
  // length + 1 tokens; paged: at seq_lens[b], with `step`); nullptr otherwise
  const uint16_t* k_new;
  const uint16_t* v_new;
};

// Fused step: the workgroup that reads block `blk` (the one the step's token falls into; one workgroup per
// split and KV head) quantizes the token into position i of that block (array index bi) before it
// requests anything of the block.
__device__ __forceinline__ void mx_append_here(const MxArgs& a, size_t unit, size_t bi, int i) {
  if (threadIdx.x < 128)
    mx_quantize_token(a.k_new + unit * kD, a.v_new + unit * kD, const_cast<uint8_t*>(a.k_codes),
                      const_cast<uint8_t*>(a.k_scales), const_cast<uint8_t*>(a.v_codes),
                      const_cast<uint8_t*>(a.v_scales), (long)bi, i);
  workgroup_global_sync();   // read back below by other threads of this workgroup
}

struct MergeLdsMx {
  float o[kWaves][4][kD];
  float m[kWaves][4], l[kWaves][4];
};

__device__ __forceinline__ float bf2f(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// The query as the B operand of the scaled MFMA: exact split of each bf16 into two e4m3 pieces.
// P' = p * 2^(e - e_run + kPTop) goes to the second product as fp16, with e the e8m0 exponent of the token's
// channel block and e_run the largest exponent the wave has met so far (a running value, carried like the
// running maximum: the accumulators are rescaled when it grows).  So P' < 2^(kPTop + 1) whatever the
// magnitude of V is, the largest terms sit at the top of the fp16 range, and only blocks far below the
// largest one sink into the subnormals.
constexpr int kPTop = 13;
// largest byte of a u4_t, over all lanes of the wave.  Bytes are compared as the high bytes of 16-bit halves
// (packed 16-bit maxima: the odd bytes of a word as it is, the even ones after a shift by 8; whatever sits in
// the low byte of a half cannot change which high byte wins).
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_pk_max_u16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
template <int N>
__device__ __forceinline__ int wave_max_byte(const u4_t (&x)[N]) {
  uint32_t mo = 0, me = 0;
#pragma unroll
  for (int i = 0; i < N; ++i)
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      mo = pk_max_u16(mo, x[i][d]);
      me = pk_max_u16(me, x[i][d] << 8);
    }
  uint32_t m = max(max(mo >> 24, (mo >> 8) & 0xFFu), max(me >> 24, (me >> 8) & 0xFFu));
  m = max(m, dpp_u<kQuadSwap1>(m));
  m = max(m, dpp_u<kQuadSwap2>(m));
  m = max(m, dpp_u<kRowHalfMirror>(m));
  m = max(m, dpp_u<kRowMirror>(m));
  return (int)max(max(__builtin_amdgcn_readlane(m, 0), __builtin_amdgcn_readlane(m, 16)),
                  max(__builtin_amdgcn_readlane(m, 32), __builtin_amdgcn_readlane(m, 48)));
}
// 2^e as a float, e clamped to the normal range
__device__ __forceinline__ float pow2_clamped(int e) { return __uint_as_float((uint32_t)(min(max(e, -126), 127) + 127) << 23); }

// Operand layout of the 8-bit side (measured): lane (column, g) holds contraction indices
// 16g .. 16g+15 in bytes 0..15 and 64+16g .. 64+16g+15 in bytes 16..31, while the 4-bit
// side holds 32g .. 32g+31 per lane.  One block scale per head (all 128 channels) is used
// for B, so its value does not depend on which lane the instruction reads it from.
// qp: the head's query row + 16 * (lane / 16), or nullptr for a padding column (all zero).
// Every lane of the wave must call this (it exchanges the head's maximum across lane groups).
__device__ __forceinline__ void mx_query_operand(const uint16_t* qp, i8_t& bhi, i8_t& blo, int& sb_hi, int& sb_lo) {
  float x[32];
  u4_t raw[4] = {};
  if (qp) {
    raw[0] = *reinterpret_cast<const u4_t*>(qp);
    raw[1] = *reinterpret_cast<const u4_t*>(qp + 8);
    raw[2] = *reinterpret_cast<const u4_t*>(qp + 64);
    raw[3] = *reinterpret_cast<const u4_t*>(qp + 72);
  }
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    x[i] = bf2f((raw[i >> 3][(i >> 1) & 3] >> (16 * (i & 1))) & 0xFFFFu);
    amax = fmaxf(amax, fabsf(x[i]));
  }
  amax = fmaxf(amax, __shfl_xor(amax, 16));
  amax = fmaxf(amax, __shfl_xor(amax, 32));
  int eb = 0;
  if (amax > 0.0f) eb = (int)((__float_as_uint(amax) >> 23) & 0xFFu) - 127 - 7;   // amax * 2^-eb in [128, 256)
  eb = min(max(eb, -123), 127);
  sb_hi = eb + 127;
  sb_lo = eb - 4 + 127;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    int hi = 0, lo = 0;
    float rem[4];
#pragma unroll
    for (int hw = 0; hw < 2; ++hw) {
      const float x0 = ldexpf(x[4 * v + 2 * hw], -eb), x1 = ldexpf(x[4 * v + 2 * hw + 1], -eb);
      hi = hw ? __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi, true) : __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, hi, false);
      rem[2 * hw] = x0;
      rem[2 * hw + 1] = x1;
    }
    rem[0] = (rem[0] - __builtin_amdgcn_cvt_f32_fp8(hi, 0)) * 16.0f;
    rem[1] = (rem[1] - __builtin_amdgcn_cvt_f32_fp8(hi, 1)) * 16.0f;
    rem[2] = (rem[2] - __builtin_amdgcn_cvt_f32_fp8(hi, 2)) * 16.0f;
    rem[3] = (rem[3] - __builtin_amdgcn_cvt_f32_fp8(hi, 3)) * 16.0f;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(rem[0], rem[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(rem[2], rem[3], lo, true);
    bhi[v] = hi;
    blo[v] = lo;
  }
}

// Query groups of up to 4 heads: the 16 MFMA columns carry the heads four times, and the softmax work
// of a block is shared out over the copies (larger groups: decode_mxg_kernel).
// PAGED: blocks are found through the block table and every sequence has its own length.
template <bool PAGED>
__global__ __launch_bounds__(256, 2) void decode_mx_kernel(MxArgs a) {
  __shared__ MergeLdsMx ml;
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, g = lane >> 4;
  const int head = col & 3, cg = col >> 2;
  const int head0 = hkv * a.gq;                  // first query head of this workgroup
  const int nheads = min(4, a.gq);
  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  int length = a.length;
  long app_bi = -1;   // fused step without an append launch: array index of the block the token goes to
  int app_pos = 0;
  if (PAGED) {
    length = a.seq_lens[b];
    if (a.step && length >= 0) {
      // fused step: this step's token counts if the table names a page for it (a preceding kernel
      // has appended it, or, with a.k_new, this launch does); the length is raised only after this kernel
      const int n = length / kBlock;
      const int e = n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1;
      const bool ok = e >= 0 && e < a.num_pages;
      if (a.k_new) {
        if (ok) {
          app_bi = (long)e * a.n_kv_heads + hkv;
          app_pos = length % kBlock;
        } else if (a.status && tid == 0 && split == 0) {
          atomicOr(a.status, 2);   // the token is dropped
        }
      }
      length += ok ? 1 : 0;
    }
    length = max(0, length);
  } else if (a.k_new) {
    app_bi = (long)(unit * (a.capacity / kBlock) + length / kBlock);
    app_pos = length % kBlock;
    length += 1;
  }
  const int nb = (length + kBlock - 1) / kBlock;
  if (app_bi >= 0 && split == ((nb - 1) / kWaves) % a.num_splits) mx_append_here(a, unit, (size_t)app_bi, app_pos);
  // blocks are dealt to the splits four at a time (one per wave), round robin: the workgroups of a
  // unit read one contiguous window of the cache at any moment
  const int blk0 = split * kWaves, blk1 = nb, bstep = kWaves * a.num_splits;
  const int nbcap = a.capacity / kBlock;
  const int tok_base = 32 * (col >> 2) + (col & 3);   // row `col` of tile T holds token tok_base + 4T

  i8_t bhi, blo;      // Q[head][32g .. 32g+31] as two fp8 (e4m3) pieces
  int sb_hi, sb_lo;   // their e8m0 block scales
  u4_t kraw[8], vraw[8];
  uint32_t ksc[8];
  u4_t vsc[2];
  // A wave keeps 8 KB in flight, not a whole block: keys (and their scales) of the next block
  // are requested when the current block is done, the values of a block when its keys are about
  // to be consumed.  The waves of a compute unit share one in-order memory pipeline; a shorter
  // queue serves everybody sooner and shortens the ramp at both ends of the kernel.
  // bi = index of a 128-token block in the arrays: unit * nbcap + block, or page * H + KV head
  auto issue_k = [&](size_t bi) {
    const size_t tok0 = bi * kBlock;
#pragma unroll
    for (int T = 0; T < 8; ++T) {
      const size_t t = tok0 + tok_base + 4 * T;
      ksc[T] = *reinterpret_cast<const uint32_t*>(a.k_scales + t * 4);
      kraw[T] = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(a.k_codes + t * 64 + 16 * g));
    }
  };
  auto issue_v = [&](size_t bi) {
    const size_t tok0 = bi * kBlock;
#pragma unroll
    for (int half = 0; half < 2; ++half)
      vsc[half] = *reinterpret_cast<const u4_t*>(a.v_scales + (tok0 + 32 * g + 16 * half + 4 * cg) * 4);
    const uint8_t* vp = a.v_codes + bi * (size_t)(kD * 64) + 16 * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
      vraw[mt] = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(vp + (size_t)(16 * mt + col) * 64));
  };
  // Paged: table entry of block n (-1 past the end of the row), and the first block at or after
  // n, in this wave's stride, whose entry names a page of the pool; entries that do not are
  // skipped and reported in *status.
  auto table_entry = [&](int n) { return n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1; };
  auto first_valid = [&](int n, int entry, size_t& bi) {
    while (n < blk1) {
      if (entry >= 0 && entry < a.num_pages) {
        bi = (size_t)entry * a.n_kv_heads + hkv;
        break;
      }
      if (a.status && lane == 0) atomicOr(a.status, 1);
      n += bstep;
      entry = n < blk1 ? table_entry(n) : -1;
    }
    return n;
  };
  int blk = blk0 + wave;
  size_t bi = unit * nbcap + blk;
  if (PAGED) blk = first_valid(blk, blk < blk1 ? table_entry(blk) : -1, bi);
  if (blk < blk1) issue_k(bi);

  mx_query_operand(head < nheads ? a.q + ((size_t)b * a.n_q_heads + head0 + head) * kD + 16 * g : nullptr, bhi, blo,
                   sb_hi, sb_lo);

  float m_run = -INFINITY, l_run = 0.0f;
  int e_run = 0;   // largest V exponent byte so far (biased by 127)
  f4_t oacc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  while (blk < blk1) {
    int nblk = blk + bstep;
    size_t nbi = bi + bstep;
    int next_entry = -1;   // requested a block ahead
    if (PAGED && nblk < blk1) next_entry = table_entry(nblk);
    issue_v(bi);
    // ---- S^T tiles straight from the packed codes; column group cg keeps tiles cg and 4+cg
    float s[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f4_t st[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int T = 4 * half + tt;
        const i8_t ak = {(int)kraw[T][0], (int)kraw[T][1], (int)kraw[T][2], (int)kraw[T][3], 0, 0, 0, 0};
        const int sa = (int)((ksc[T] >> (8 * g)) & 0xFFu);
        f4_t acc = {0.f, 0.f, 0.f, 0.f};
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ak, bhi, acc, 4, 0, 0, sa, 0, sb_hi);
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ak, blo, acc, 4, 0, 0, sa, 0, sb_lo);
        st[tt] = acc;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float lo = cg & 1 ? st[1][r] : st[0][r], hi = cg & 1 ? st[3][r] : st[2][r];
        const int t = blk * kBlock + 32 * g + 16 * half + 4 * cg + r;
        s[half][r] = t < length ? (cg & 2 ? hi : lo) * a.scale_log2 : -INFINITY;   // tokens past the end
      }
    }
    // ---- online softmax (Alg. 1): this lane owns head `head`, tokens 32g + 16*half + 4cg + r
    float bmax = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                       fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    bmax = head_max<4>(bmax);
    const float m_new = fmaxf(m_run, bmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
    const int e_new = max(e_run, wave_max_byte(vsc));
    const float alpha_o = alpha * pow2_clamped(e_run - e_new);
    e_run = e_new;
    if (__any(alpha_o != 1.0f)) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) oacc[mt] *= alpha_o;
    }
    float p[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[half][r] = __builtin_amdgcn_exp2f(s[half][r] - m_new);
        l_run += p[half][r];
      }
    // ---- O^T += V^T P'_cb for the four 32-channel blocks cb (M tiles 2cb, 2cb+1)
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      uint32_t pk[2][2];   // [half][rows 0,1 | rows 2,3] as packed fp16
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        float pe[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int e = (int)((vsc[half][r] >> (8 * cb)) & 0xFFu) - e_run + kPTop;   // <= kPTop
          pe[r] = ldexpf(p[half][r], e);
        }
        pk[half][0] = (uint32_t)f2h(pe[0]) | ((uint32_t)f2h(pe[1]) << 16);
        pk[half][1] = (uint32_t)f2h(pe[2]) | ((uint32_t)f2h(pe[3]) << 16);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int half = j >> 1;
        u4_t pb;
        if ((j & 1) == 0) {
          pb[0] = pk[half][0];
          pb[1] = pk[half][1];
          pb[2] = dpp_u<kRowShl4>(pk[half][0]);
          pb[3] = dpp_u<kRowShl4>(pk[half][1]);
        } else {
          pb[0] = dpp_u<kRowShl8>(pk[half][0]);
          pb[1] = dpp_u<kRowShl8>(pk[half][1]);
          pb[2] = dpp_u<kRowShl12>(pk[half][0]);
          pb[3] = dpp_u<kRowShl12>(pk[half][1]);
        }
        const h8_t bp = __builtin_bit_cast(h8_t, pb);
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const int mt = 2 * cb + mm;
          const uint32_t w = vraw[mt][j];
          h2_t c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0);
          h2_t c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1);
          h2_t c2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2);
          h2_t c3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3);
          const h8_t av = {c0[0], c0[1], c1[0], c1[1], c2[0], c2[1], c3[0], c3[1]};
          oacc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bp, oacc[mt], 0, 0, 0);
        }
      }
    }
    if (PAGED) nblk = first_valid(nblk, next_entry, nbi);
    if (nblk < blk1) issue_k(nbi);
    blk = nblk;
    bi = nbi;
  }

  // ---- merge the waves of the workgroup (the accumulators go back to the true scale first)
  const float back = pow2_clamped(e_run - 127 - kPTop);
  l_run = head_sum<4>(l_run);
  if (col < 4) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) ml.o[wave][col][16 * mt + 4 * g + r] = oacc[mt][r] * back;
    if (g == 0) {
      ml.m[wave][col] = m_run;
      ml.l[wave][col] = l_run;
    }
  }
  __syncthreads();
  {
    const int h = tid >> 6, c0 = 2 * (tid & 63);
    if (h < nheads) {
      float M = ml.m[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) M = fmaxf(M, ml.m[w][h]);
      float L = 0.f, o0 = 0.f, o1 = 0.f;
      if (M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float f = __builtin_amdgcn_exp2f(ml.m[w][h] - M);
          L += f * ml.l[w][h];
          o0 += f * ml.o[w][h][c0];
          o1 += f * ml.o[w][h][c0 + 1];
        }
      }
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + head0 + h;
      if (a.out) {   // one split: row == the output row
        store_final_pair(a.out, row * kD + c0, a.out_kind, o0, o1, L);
      } else {
        float2 o = {o0, o1};
        *reinterpret_cast<float2*>(a.part_o + row * kD + c0) = o;
        if ((tid & 63) == 0) {
          a.part_ml[row * 2] = M;
          a.part_ml[row * 2 + 1] = L;
        }
      }
    }
  }
}


// ---- groups of 5..16 heads per workgroup: GQP = 8 (the 16 MFMA columns carry 8 heads twice) or 16
//
// Every copy of a head's column receives the same S^T.  Copy cg keeps the tiles of its share of
// the block (GQP = 8: the four tiles of half cg, tokens 32g + 16cg .. + 15 of every lane group g;
// GQP = 16: all eight), runs their softmax, and presents their P' as its part of the B operand of
// the second product: the k-steps that contract those tokens, zero in the others.  Nothing moves
// between lanes; the copies' partial O^T are added once, after the loop.  The keys, the values
// and every matrix instruction are shared by all heads, so a group of 8 or 16 costs what a
// group of 4 costs, except for 2x / 4x the softmax work per lane.
template <int GQP>
struct MergeLdsMxG {
  float o[kWaves][GQP][kD];
  float m[kWaves][GQP], l[kWaves][GQP];
};

template <int GQP, bool PAGED>
__global__ __launch_bounds__(256, (GQP == 8 || !PAGED) ? 2 : 1) void decode_mxg_kernel(MxArgs a) {
  constexpr int COPIES = 16 / GQP;     // 2 or 1
  constexpr int NT = 8 / COPIES;       // S^T tiles a lane keeps
  __shared__ MergeLdsMxG<GQP> ml;
  const int nwg = (a.gq + GQP - 1) / GQP;        // workgroups per (split, KV head)
  const int split = blockIdx.x, hkv = blockIdx.y / nwg, sub0 = GQP * (blockIdx.y % nwg), b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, g = lane >> 4;
  const int head = col % GQP, cg = col / GQP;
  const int head0 = hkv * a.gq + sub0;           // first query head of this workgroup
  const int nheads = min(GQP, a.gq - sub0);
  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  int length = a.length;
  long app_bi = -1;   // fused step without an append launch (see decode_mx_kernel)
  int app_pos = 0;
  if (PAGED) {
    length = a.seq_lens[b];
    if (a.step && length >= 0) {
      const int n = length / kBlock;
      const int e = n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1;
      const bool ok = e >= 0 && e < a.num_pages;
      if (a.k_new) {
        if (ok) {
          app_bi = (long)e * a.n_kv_heads + hkv;
          app_pos = length % kBlock;
        } else if (a.status && tid == 0 && split == 0) {
          atomicOr(a.status, 2);   // the token is dropped
        }
      }
      length += ok ? 1 : 0;
    }
    length = max(0, length);
  } else if (a.k_new) {
    app_bi = (long)(unit * (a.capacity / kBlock) + length / kBlock);
    app_pos = length % kBlock;
    length += 1;
  }
  const int nb = (length + kBlock - 1) / kBlock;
  if (app_bi >= 0 && split == ((nb - 1) / kWaves) % a.num_splits) mx_append_here(a, unit, (size_t)app_bi, app_pos);
  // blocks are dealt to the splits four at a time (one per wave), round robin: the workgroups of a
  // unit read one contiguous window of the cache at any moment
  const int blk0 = split * kWaves, blk1 = nb, bstep = kWaves * a.num_splits;
  const int nbcap = a.capacity / kBlock;
  const int tok_base = 32 * (col >> 2) + (col & 3);   // row `col` of tile T holds token tok_base + 4T

  i8_t bhi, blo;
  int sb_hi, sb_lo;
  u4_t kraw[8], vraw[8];
  uint32_t ksc[8];
  u4_t vsc[NT];   // e8m0 scales (4 channel blocks) of this lane's 4 * NT tokens, 4 tokens per register
  auto issue_k = [&](size_t bi) {
    const size_t tok0 = bi * kBlock;
#pragma unroll
    for (int T = 0; T < 8; ++T) {
      const size_t t = tok0 + tok_base + 4 * T;
      ksc[T] = *reinterpret_cast<const uint32_t*>(a.k_scales + t * 4);
      kraw[T] = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(a.k_codes + t * 64 + 16 * g));
    }
  };
  auto issue_v = [&](size_t bi) {
    const size_t tok0 = bi * kBlock;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt)
      vsc[tt] = *reinterpret_cast<const u4_t*>(a.v_scales + (tok0 + 32 * g + 4 * NT * cg + 4 * tt) * 4);
    const uint8_t* vp = a.v_codes + bi * (size_t)(kD * 64) + 16 * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
      vraw[mt] = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(vp + (size_t)(16 * mt + col) * 64));
  };
  auto table_entry = [&](int n) { return n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1; };
  auto first_valid = [&](int n, int entry, size_t& bi) {
    while (n < blk1) {
      if (entry >= 0 && entry < a.num_pages) {
        bi = (size_t)entry * a.n_kv_heads + hkv;
        break;
      }
      if (a.status && lane == 0) atomicOr(a.status, 1);
      n += bstep;
      entry = n < blk1 ? table_entry(n) : -1;
    }
    return n;
  };
  int blk = blk0 + wave;
  size_t bi = unit * nbcap + blk;
  if (PAGED) blk = first_valid(blk, blk < blk1 ? table_entry(blk) : -1, bi);
  if (blk < blk1) issue_k(bi);

  mx_query_operand(head < nheads ? a.q + ((size_t)b * a.n_q_heads + head0 + head) * kD + 16 * g : nullptr, bhi, blo,
                   sb_hi, sb_lo);

  float m_run = -INFINITY, l_run = 0.0f;
  int e_run = 0;   // largest V exponent byte so far (biased by 127)
  f4_t oacc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  while (blk < blk1) {
    int nblk = blk + bstep;
    size_t nbi = bi + bstep;
    int next_entry = -1;
    if (PAGED && nblk < blk1) next_entry = table_entry(nblk);
    issue_v(bi);
    // ---- S^T tiles straight from the packed codes; copy cg keeps tiles NT*cg .. NT*cg + NT-1
    float s[NT][4];
#pragma unroll
    for (int T = 0; T < 8; ++T) {
      const i8_t ak = {(int)kraw[T][0], (int)kraw[T][1], (int)kraw[T][2], (int)kraw[T][3], 0, 0, 0, 0};
      const int sa = (int)((ksc[T] >> (8 * g)) & 0xFFu);
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
      acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ak, bhi, acc, 4, 0, 0, sa, 0, sb_hi);
      acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ak, blo, acc, 4, 0, 0, sa, 0, sb_lo);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = blk * kBlock + 32 * g + 4 * T + r;
        const float v = t < length ? acc[r] * a.scale_log2 : -INFINITY;   // tokens past the end
        if (T < NT) s[T][r] = v;                      // (first half: kept where cg == 0)
        else s[T - NT][r] = cg ? v : s[T - NT][r];    // the second half replaces it in the other copy
      }
    }
    // ---- online softmax (Alg. 1): this lane owns head `head`, tokens 32g + 4*NT*cg + 4tt + r
    float bmax = s[0][0];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt)
#pragma unroll
      for (int r = 0; r < 4; ++r) bmax = fmaxf(bmax, s[tt][r]);
    bmax = head_max<COPIES>(bmax);
    const float m_new = fmaxf(m_run, bmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
    const int e_new = max(e_run, wave_max_byte(vsc));
    const float alpha_o = alpha * pow2_clamped(e_run - e_new);
    e_run = e_new;
    if (__any(alpha_o != 1.0f)) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) oacc[mt] *= alpha_o;
    }
#pragma unroll
    for (int tt = 0; tt < NT; ++tt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[tt][r] = __builtin_amdgcn_exp2f(s[tt][r] - m_new);
        l_run += s[tt][r];
      }
    // ---- O^T += V^T P'_cb for the four 32-channel blocks cb (M tiles 2cb, 2cb+1)
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      uint32_t pk[NT][2];   // [tile][rows 0,1 | rows 2,3] as packed fp16
#pragma unroll
      for (int tt = 0; tt < NT; ++tt) {
        float pe[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int e = (int)((vsc[tt][r] >> (8 * cb)) & 0xFFu) - e_run + kPTop;   // <= kPTop
          pe[r] = ldexpf(s[tt][r], e);
        }
        pk[tt][0] = (uint32_t)f2h(pe[0]) | ((uint32_t)f2h(pe[1]) << 16);
        pk[tt][1] = (uint32_t)f2h(pe[2]) | ((uint32_t)f2h(pe[3]) << 16);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // k-step j contracts tokens 32g + 8j .. + 7: tiles 2j and 2j+1, owned by copy 2j / NT
        const int jo = j % (NT / 2);
        u4_t pb = {pk[2 * jo][0], pk[2 * jo][1], pk[2 * jo + 1][0], pk[2 * jo + 1][1]};
        if (COPIES > 1 && (2 * j) / NT != cg) pb = (u4_t){0u, 0u, 0u, 0u};
        const h8_t bp = __builtin_bit_cast(h8_t, pb);
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const int mt = 2 * cb + mm;
          const uint32_t w = vraw[mt][j];
          h2_t c0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0);
          h2_t c1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1);
          h2_t c2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2);
          h2_t c3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3);
          const h8_t av = {c0[0], c0[1], c1[0], c1[1], c2[0], c2[1], c3[0], c3[1]};
          oacc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bp, oacc[mt], 0, 0, 0);
        }
      }
    }
    if (PAGED) nblk = first_valid(nblk, next_entry, nbi);
    if (nblk < blk1) issue_k(nbi);
    blk = nblk;
    bi = nbi;
  }

  // ---- the copies' partial O^T, then the waves of the workgroup
  const float back = pow2_clamped(e_run - 127 - kPTop);   // the accumulators go back to the true scale
  l_run = head_sum<COPIES>(l_run);
  if (COPIES == 2) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) oacc[mt][r] += dpp_f<kRowShl8>(oacc[mt][r]);
  }
  if (col < GQP) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) ml.o[wave][col][16 * mt + 4 * g + r] = oacc[mt][r] * back;
    if (g == 0) {
      ml.m[wave][col] = m_run;
      ml.l[wave][col] = l_run;
    }
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < GQP / 4; ++p) {
    const int h = 4 * p + (tid >> 6), c0 = 2 * (tid & 63);
    if (h < nheads) {
      float M = ml.m[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) M = fmaxf(M, ml.m[w][h]);
      float L = 0.f, o0 = 0.f, o1 = 0.f;
      if (M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float f = __builtin_amdgcn_exp2f(ml.m[w][h] - M);
          L += f * ml.l[w][h];
          o0 += f * ml.o[w][h][c0];
          o1 += f * ml.o[w][h][c0 + 1];
        }
      }
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + head0 + h;
      if (a.out) {   // one split: row == the output row
        store_final_pair(a.out, row * kD + c0, a.out_kind, o0, o1, L);
      } else {
        float2 o = {o0, o1};
        *reinterpret_cast<float2*>(a.part_o + row * kD + c0) = o;
        if ((tid & 63) == 0) {
          a.part_ml[row * 2] = M;
          a.part_ml[row * 2 + 1] = L;
        }
      }
    }
  }
}

}  // namespace

template <bool PAGED>
static hipError_t launch_mx(const MxArgs& a, int batch, hipStream_t st) {
  dim3 block(256);
  if (a.gq <= 4)
    decode_mx_kernel<PAGED><<<dim3(a.num_splits, a.n_kv_heads, batch), block, 0, st>>>(a);
  else if (a.gq <= 8)
    decode_mxg_kernel<8, PAGED><<<dim3(a.num_splits, a.n_kv_heads, batch), block, 0, st>>>(a);
  else
    decode_mxg_kernel<16, PAGED><<<dim3(a.num_splits, a.n_kv_heads * ((a.gq + 15) / 16), batch), block, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_decode_mx(const bd_cache* c, const void* q, int length, float softmax_scale, int num_splits,
                            float* part_o, float* part_ml, const void* k_new, const void* v_new, void* out,
                            hipStream_t st) {
  MxArgs a{};
  a.k_new = (const uint16_t*)k_new;
  a.v_new = (const uint16_t*)v_new;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
  a.k_codes = (const uint8_t*)c->k_codes;
  a.v_codes = (const uint8_t*)c->v_codes;
  a.k_scales = (const uint8_t*)c->k_params;
  a.v_scales = (const uint8_t*)c->v_params;
  a.q = (const uint16_t*)q;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.n_q_heads = c->n_q_heads;
  a.n_kv_heads = c->n_kv_heads;
  a.gq = c->n_q_heads / c->n_kv_heads;
  a.length = length;
  a.capacity = c->capacity;
  a.num_splits = num_splits;
  a.scale_log2 = softmax_scale * kLog2e;
  return launch_mx<false>(a, c->batch, st);
}

hipError_t launch_decode_mx_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                                  float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                                  void* out, hipStream_t st) {
  MxArgs a{};
  a.k_new = (const uint16_t*)k_new;
  a.v_new = (const uint16_t*)v_new;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
  a.step = step ? 1 : 0;
  a.k_codes = (const uint8_t*)c->k_codes;
  a.v_codes = (const uint8_t*)c->v_codes;
  a.k_scales = (const uint8_t*)c->k_params;
  a.v_scales = (const uint8_t*)c->v_params;
  a.q = (const uint16_t*)q;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.n_q_heads = c->n_q_heads;
  a.n_kv_heads = c->n_kv_heads;
  a.gq = c->n_q_heads / c->n_kv_heads;
  a.capacity = kBlock;
  a.num_splits = num_splits;
  a.scale_log2 = softmax_scale * kLog2e;
  a.block_table = c->block_table;
  a.seq_lens = c->seq_lens;
  a.status = c->status;
  a.max_pages = c->max_pages_per_seq;
  a.num_pages = c->num_pages;
  return launch_mx<true>(a, c->batch, st);
}

}  // namespace bd
