// Decode-step attention over the packed int4 / int2 cache: the paper's Packing Kernel
// (Sec. IV-C: fused dequantize + QK^T + softmax + PV) and the attention half of its
// Residual Kernel (Sec. IV-B), split over the context, for gfx950.
//
// How the contraction is mapped onto v_mfma_f32_16x16x32_f16 (wave64; A and B operands hold,
// per lane, 8 contraction-contiguous fp16 for row/column lane%16; the fp32 result holds rows
// 4*(lane/16)+r, r = 0..3, of column lane%16):
//
//   S^T[token, head] = sum_c K[token, c] * Q'[head, c]      A = K codes (M = 16 tokens),
//                                                           B = Q'^T (N = query group, padded to 16)
//   O^T[c, head]     = sum_t V[t, c] * P'[t, head]          A = V codes^T (M = 16 channels),
//                                                           B = P' (contraction over tokens)
//
// The query group of one KV head forms the N dimension (query transformation, Sec. IV-A).
// Because S^T comes out with 4 consecutive rows (tokens) per lane for one head, it is already
// in the B-operand layout of the second product: probabilities go exp -> fp16 -> MFMA with no
// cross-lane movement and no LDS round trip.  The row -> token assignment of each S^T tile
// and the order of codes inside a word are chosen so that this holds (the analogue, for MFMA,
// of inducing the packed layout from the consumer instruction, Sec. III-A(1)).
//
// Dequantization cost is cut by linearity: K is quantized per channel, so
//   S = sum_c (Q_c s_c) code_c + sum_c Q_c z_c ;  Q' = Q*s (rescaled once per 128-token block,
//   kept as an fp16 hi + lo pair so that it carries ~22 bits), the zero term is one scalar per
//   head and block.  V is quantized per token, so  O = sum_t (P_t s_t) (code_t - c) + sum_t P_t (z_t + c s_t)
//   with c the middle code, so that what P' multiplies is centred on zero.
// The MFMAs therefore consume raw integer codes, produced from the packed words by one
// mask-or per two codes (fp16 bit pattern 0x6400 | code == 1024 + code, Sec. III-A(3)) and one
// packed subtract; codes sitting at bit offsets 4..7 of a byte arrive multiplied by a power
// of two, which is folded into Q' / P'.
#include "bd_common.h"

namespace bd {
namespace {

constexpr int kWaves = 4;          // waves per workgroup, all spread along the token axis (W_m = 1)
constexpr int kQShift = 8;         // Q' is carried as Q' * 2^8 so that its low piece stays a normal fp16
constexpr int kPShift = 8;         // P' likewise
constexpr float kLog2e = 1.4426950408889634f;

struct DecodeArgs {
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const uint32_t* k_params;
  const uint32_t* v_params;
  const uint16_t* k_res;
  const uint16_t* v_res;
  const uint16_t* q;
  float* part_o;    // [nparts][B][Hq][128]
  float* part_ml;   // [nparts][B][Hq][2]   (running max in log2 units, running sum)
  int n_q_heads, n_kv_heads, gq;
  int nb;           // packed 128-token blocks
  int nbcap;
  int res_len;
  int num_splits;
  float scale_log2; // softmax_scale * log2(e)
};

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
__device__ __forceinline__ uint32_t pack_h2(float lo, float hi) {
  return (uint32_t)f2h(lo) | ((uint32_t)f2h(hi) << 16);
}

// ---- format traits ---------------------------------------------------------------------
// WORDS: 32-bit words one lane loads per 16-row tile (32 codes).  k-step j of the 4 k-steps
// of a tile consumes 8 codes: `e`-th code (e = 0..7, VGPR e/2, half e%2) sits at nibble/crumb
// n(j, e) of word wj(j) and arrives multiplied by mult(e).
template <int BITS>
struct Fmt;

template <>
struct Fmt<4> {
  static constexpr int WORDS = 4;
  // position of channel c (0..127) in the permuted Q' array read as B operand
  __device__ static int slot(int c) {
    const int w = c >> 3, n = c & 7;
    return 8 * w + 2 * (n & 3) + (n >> 2);
  }
  // 2^-k factor undoing the scale a code picks up from its bit position
  __device__ static float unmult_of_slot(int slot) { return ((slot >> 1) & 1) ? (1.0f / 16.0f) : 1.0f; }
  // S^T tiles that feed the low / high half of the P' VGPRs of PV k-step j
  __device__ static constexpr int tile_lo(int j) { return 2 * j; }
  __device__ static constexpr int tile_hi(int j) { return 2 * j + 1; }
  __device__ static float unmult_of_row(int r) { return (r & 1) ? (1.0f / 16.0f) : 1.0f; }
  // V codes enter the second product as (code - kCenter): the probabilities then multiply
  // numbers centred on zero, which keeps fp16 rounding of P' from being amplified by the
  // zero-point offset; the shift is returned through the per-token constant term.
  static constexpr int kCenter = 8;
  // 8 codes of k-step j, as fp16 integers minus `center` (times their position factor)
  template <int CENTER>
  __device__ static h8_t dequant(const uint32_t* w, int j) {
    const uint32_t x = w[j], y = x >> 8;
    u4_t r;
    r[0] = (x & 0x000F000Fu) | 0x64006400u;
    r[1] = (x & 0x00F000F0u) | 0x64006400u;
    r[2] = (y & 0x000F000Fu) | 0x64006400u;
    r[3] = (y & 0x00F000F0u) | 0x64006400u;
    const h8_t v = __builtin_bit_cast(h8_t, r);
    constexpr _Float16 c0 = (_Float16)(1024.0f + CENTER), c1 = (_Float16)(1024.0f + 16.0f * CENTER);
    const h8_t bias = {c0, c0, c1, c1, c0, c0, c1, c1};
    return v - bias;
  }
};

template <>
struct Fmt<2> {
  static constexpr int WORDS = 2;
  __device__ static int slot(int c) {
    const int W = c >> 4, n = c & 15;
    return 8 * (2 * W + ((n & 7) >> 2)) + 2 * (n & 3) + (n >> 3);
  }
  __device__ static float unmult_of_slot(int slot) {
    const int v = (slot >> 1) & 3;
    return 1.0f / (float)(1 << (2 * v));
  }
  __device__ static constexpr int tile_lo(int j) { return 4 * (j >> 1) + (j & 1); }
  __device__ static constexpr int tile_hi(int j) { return 4 * (j >> 1) + (j & 1) + 2; }
  __device__ static float unmult_of_row(int r) { return 1.0f / (float)(1 << (2 * r)); }
  static constexpr int kCenter = 2;
  template <int CENTER>
  __device__ static h8_t dequant(const uint32_t* w, int j) {
    const uint32_t x = (j & 1) ? (w[j >> 1] >> 8) : w[j >> 1];
    u4_t r;
    r[0] = (x & 0x00030003u) | 0x64006400u;
    r[1] = (x & 0x000C000Cu) | 0x64006400u;
    r[2] = (x & 0x00300030u) | 0x64006400u;
    r[3] = (x & 0x00C000C0u) | 0x64006400u;
    const h8_t v = __builtin_bit_cast(h8_t, r);
    constexpr _Float16 c0 = (_Float16)(1024.0f + CENTER), c1 = (_Float16)(1024.0f + 4.0f * CENTER),
                       c2 = (_Float16)(1024.0f + 16.0f * CENTER), c3 = (_Float16)(1024.0f + 64.0f * CENTER);
    const h8_t bias = {c0, c0, c1, c1, c2, c2, c3, c3};
    return v - bias;
  }
};

template <int WORDS>
struct RawTile {
  uint32_t w[WORDS];
};

template <int WORDS>
__device__ __forceinline__ RawTile<WORDS> load_raw(const uint32_t* p) {
  RawTile<WORDS> t;
  if constexpr (WORDS == 4) {
    u4_t v = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(p));
    t.w[0] = v[0]; t.w[1] = v[1]; t.w[2] = v[2]; t.w[3] = v[3];
  } else {
    u2_t v = __builtin_nontemporal_load(reinterpret_cast<const u2_t*>(p));
    t.w[0] = v[0]; t.w[1] = v[1];
  }
  return t;
}

// Per-wave LDS scratch.
struct WaveLds {
  uint16_t qhi[4][kD];   // Q' * 2^kQShift, high fp16 piece, permuted to B-operand order
  uint16_t qlo[4][kD];   // low piece
  float2 vpar[kBlock];   // per V token of the block: (scale * 2^kPShift * position factor, zero + center*scale)
  float zq[4];           // sum_c Q_c z_c * scale_log2 * 2^kQShift per head
};
struct MergeLds {
  float o[kWaves][4][kD];
  float m[kWaves][4], l[kWaves][4], z[kWaves][4];
};

constexpr size_t kResidualSmem = 24 * kD * sizeof(float);   // q, scores, partial outputs of the residual path
constexpr size_t cmax(size_t x, size_t y) { return x > y ? x : y; }
constexpr size_t kSmemBytes = cmax(cmax(sizeof(MergeLds), kWaves * sizeof(WaveLds)), kResidualSmem);

__device__ __forceinline__ void wave_sync() {
  // LDS operations of one wave execute in order; this only stops the compiler from moving
  // accesses across the exchange point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Residual tail (Sec. IV-B): plain fp16 tokens, at most 127 of them; written for clarity,
// not speed -- it moves <= 64 KB.
__device__ void residual_part(const DecodeArgs& a, int b, int hkv, float* smem) {
  const int tid = threadIdx.x;
  const int gq = a.gq, R = a.res_len;
  float* sq = smem;                 // [4][128] q * scale_log2
  float* sp = smem + 4 * kD;        // [4][128] scores, then probabilities
  float* sred = smem + 8 * kD;      // [4][4][128] partial outputs per token quarter
  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  const uint16_t* kr = a.k_res + unit * kBlock * kD;
  const uint16_t* vr = a.v_res + unit * kBlock * kD;
  for (int i = tid; i < 4 * kD; i += 256) {
    const int h = i / kD, c = i % kD;
    sq[i] = h < gq ? h2f(a.q[((size_t)b * a.n_q_heads + hkv * gq + h) * kD + c]) * a.scale_log2 : 0.0f;
  }
  __syncthreads();
  if (tid < kBlock) {
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (tid < R) {
      for (int c8 = 0; c8 < kD / 8; ++c8) {
        u4_t raw = *reinterpret_cast<const u4_t*>(kr + (size_t)tid * kD + 8 * c8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float kv = h2f((uint16_t)((raw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu));
#pragma unroll
          for (int h = 0; h < 4; ++h) s[h] += kv * sq[h * kD + 8 * c8 + e];
        }
      }
    }
#pragma unroll
    for (int h = 0; h < 4; ++h) sp[h * kD + tid] = tid < R ? s[h] : -INFINITY;
  }
  __syncthreads();
  // per-head max and sum: wave h handles head h
  const int wave = tid >> 6, lane = tid & 63;
  float m = fmaxf(sp[wave * kD + lane], sp[wave * kD + lane + 64]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  float p0 = 0.f, p1 = 0.f;
  if (R > 0) {
    p0 = exp2f(sp[wave * kD + lane] - m);
    p1 = exp2f(sp[wave * kD + lane + 64] - m);
  }
  float l = p0 + p1;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) l += __shfl_xor(l, off);
  __syncthreads();
  sp[wave * kD + lane] = p0;
  sp[wave * kD + lane + 64] = p1;
  __syncthreads();
  // O[h][c] = sum_t p[h][t] v[t][c]; thread = (token quarter, channel pair)
  {
    const int quarter = tid >> 6, cp = tid & 63;
    float acc[4][2] = {};
    for (int t = quarter * 32; t < quarter * 32 + 32 && t < R; ++t) {
      const uint32_t raw = *reinterpret_cast<const uint32_t*>(vr + (size_t)t * kD + 2 * cp);
      const float v0 = h2f((uint16_t)(raw & 0xFFFFu)), v1 = h2f((uint16_t)(raw >> 16));
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const float p = sp[h * kD + t];
        acc[h][0] += p * v0;
        acc[h][1] += p * v1;
      }
    }
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      sred[(quarter * 4 + h) * kD + 2 * cp] = acc[h][0];
      sred[(quarter * 4 + h) * kD + 2 * cp + 1] = acc[h][1];
    }
  }
  __syncthreads();
  const int part = a.num_splits;  // the residual owns the last partial slot
  const int nbh = gridDim.z * a.n_q_heads;
  for (int i = tid; i < 4 * kD; i += 256) {
    const int h = i / kD, c = i % kD;
    if (h >= gq) continue;
    const float o = sred[(0 * 4 + h) * kD + c] + sred[(1 * 4 + h) * kD + c] + sred[(2 * 4 + h) * kD + c] +
                    sred[(3 * 4 + h) * kD + c];
    const size_t row = (size_t)part * nbh + (size_t)b * a.n_q_heads + hkv * gq + h;
    a.part_o[row * kD + c] = o;
  }
  if (lane == 0 && wave < gq) {
    const size_t row = (size_t)part * nbh + (size_t)b * a.n_q_heads + hkv * gq + wave;
    a.part_ml[row * 2] = R > 0 ? m : -INFINITY;
    a.part_ml[row * 2 + 1] = R > 0 ? l : 0.0f;
  }
}

template <int BITS>
__global__ __launch_bounds__(256) void decode_int_kernel(DecodeArgs a) {
  using F = Fmt<BITS>;
  constexpr int WORDS = F::WORDS;            // words per lane per tile
  constexpr int KROW = kD * BITS / 32;       // K words per token
  constexpr int VROW = kBlock * BITS / 32;   // V words per channel per block

  __shared__ __attribute__((aligned(16))) unsigned char smem_raw[kSmemBytes];

  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  if (split == a.num_splits) {
    residual_part(a, b, hkv, reinterpret_cast<float*>(smem_raw));
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, g = lane >> 4;   // MFMA column (head) and contraction group
  const int gq = a.gq;
  WaveLds& wl = reinterpret_cast<WaveLds*>(smem_raw)[wave];

  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  const int blk0 = (int)(((long)a.nb * split) / a.num_splits);
  const int blk1 = (int)(((long)a.nb * (split + 1)) / a.num_splits);

  // Q of this lane's prep slice: head lane/16, channels 8*(lane%16) .. +7 (zero for padding heads)
  float qv[8];
  {
    const int hh = lane >> 4;
    u4_t raw = {0u, 0u, 0u, 0u};
    if (hh < gq)
      raw = *reinterpret_cast<const u4_t*>(a.q + ((size_t)b * a.n_q_heads + hkv * gq + hh) * kD + 8 * (lane & 15));
#pragma unroll
    for (int e = 0; e < 8; ++e) qv[e] = h2f((uint16_t)((raw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu));
  }

  float m_run = -INFINITY;   // running max of this lane's head (log2 units), equal across g
  float l_run = 0.0f;        // running sum over this lane's own tokens
  float z_run = 0.0f;        // running sum of p * zero_t over this lane's own tokens
  f4_t oacc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  const float qscale = a.scale_log2 * (float)(1 << kQShift);

  for (int blk = blk0 + wave; blk < blk1; blk += kWaves) {
    const size_t gb = unit * a.nbcap + blk;
    // ---- issue the block's loads: 8 K tiles (16 tokens each), 8 V tiles (16 channels each)
    RawTile<WORDS> kraw[8], vraw[8];
    {
      const uint32_t* kp = a.k_codes + gb * (size_t)(kBlock * KROW) + WORDS * g;
      const int tok_base = 32 * (col >> 2) + (col & 3);   // row col of tile T holds token tok_base + 4T
#pragma unroll
      for (int T = 0; T < 8; ++T) kraw[T] = load_raw<WORDS>(kp + (size_t)(tok_base + 4 * T) * KROW);
      const uint32_t* vp = a.v_codes + gb * (size_t)(kD * VROW) + WORDS * g;
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) vraw[mt] = load_raw<WORDS>(vp + (size_t)(16 * mt + col) * VROW);
    }
    // ---- per-block query rescale: Q' = Q * s_c (K is channel-wise), zero term sum_c Q_c z_c
    {
      const int hh = lane >> 4, c0 = 8 * (lane & 15);
      const uint32_t* pp = a.k_params + gb * kD + c0;
      u4_t p0 = *reinterpret_cast<const u4_t*>(pp), p1 = *reinterpret_cast<const u4_t*>(pp + 4);
      float zsum = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t pr = e < 4 ? p0[e] : p1[e - 4];
        const float s = h2f((uint16_t)(pr & 0xFFFFu)), z = h2f((uint16_t)(pr >> 16));
        const int sl = F::slot(c0 + e);
        const float t = qv[e] * s * (qscale * F::unmult_of_slot(sl));
        const uint16_t hi = f2h(t);
        wl.qhi[hh][sl] = hi;
        wl.qlo[hh][sl] = f2h(t - h2f(hi));
        zsum += qv[e] * z;
      }
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) zsum += __shfl_xor(zsum, off);
      if ((lane & 15) == 0) wl.zq[hh] = zsum * qscale;
      // V parameters of the block's 128 tokens
      const u2_t vp2 = *reinterpret_cast<const u2_t*>(a.v_params + gb * kBlock + 2 * lane);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float sv = h2f((uint16_t)(vp2[u] & 0xFFFFu)), zv = h2f((uint16_t)(vp2[u] >> 16));
        const int r = (2 * lane + u) & 3;   // row of the token inside its S^T tile
        wl.vpar[2 * lane + u] = make_float2(sv * ((float)(1 << kPShift) * F::unmult_of_row(r)),
                                            __builtin_fmaf((float)F::kCenter, sv, zv));
      }
    }
    wave_sync();
    h8_t bhi[4], blo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bhi[j] = *reinterpret_cast<const h8_t*>(&wl.qhi[col & 3][8 * (4 * g + j)]);
      blo[j] = *reinterpret_cast<const h8_t*>(&wl.qlo[col & 3][8 * (4 * g + j)]);
    }
    const float zq = wl.zq[col & 3];

    // ---- S^T tiles: rows = tokens 32*(row/4) + 4T + row%4, columns = heads
    f4_t s[8];
#pragma unroll
    for (int T = 0; T < 8; ++T) {
      f4_t acc = {zq, zq, zq, zq};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const h8_t ak = F::template dequant<0>(kraw[T].w, j);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak, bhi[j], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak, blo[j], acc, 0, 0, 0);
      }
      s[T] = acc;
    }
    // ---- online softmax (Alg. 1), this lane: head `col`, tokens 32g + 4T + r
    float bmax = s[0][0];
#pragma unroll
    for (int T = 0; T < 8; ++T)
#pragma unroll
      for (int r = 0; r < 4; ++r) bmax = fmaxf(bmax, s[T][r]);
    bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
    constexpr float kUnQ = 1.0f / (float)(1 << kQShift);
    const float m_new = fmaxf(m_run, bmax * kUnQ);
    const float alpha = exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
    m_run = m_new;
    l_run *= alpha;
    z_run *= alpha;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) oacc[mt] *= alpha;

    float pf[8][4];      // P' = p * scale_t (times the position factor), still fp32
#pragma unroll
    for (int T = 0; T < 8; ++T) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = exp2f(__builtin_fmaf(s[T][r], kUnQ, -m_new));
        const float2 par = wl.vpar[32 * g + 4 * T + r];
        l_run += p;
        z_run = __builtin_fmaf(p, par.y, z_run);
        pf[T][r] = p * par.x;
      }
    }
    // ---- O^T += V^T P' : k-step j contracts 32 tokens (8 per lane group)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int tl = F::tile_lo(j), th = F::tile_hi(j);
      u4_t pb;
#pragma unroll
      for (int v = 0; v < 4; ++v) pb[v] = pack_h2(pf[tl][v], pf[th][v]);
      const h8_t bp = __builtin_bit_cast(h8_t, pb);
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) {
        const h8_t av = F::template dequant<F::kCenter>(vraw[mt].w, j);
        oacc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bp, oacc[mt], 0, 0, 0);
      }
    }
    wave_sync();   // the next block's prep overwrites this wave's LDS scratch
  }

  // ---- merge the waves of the workgroup (cross-wave step of the cooperative softmax)
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  z_run += __shfl_xor(z_run, 16);
  z_run += __shfl_xor(z_run, 32);
  __syncthreads();   // every wave is done with its WaveLds before the space is reused
  MergeLds& ml = *reinterpret_cast<MergeLds*>(smem_raw);
  if (col < 4) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) ml.o[wave][col][16 * mt + 4 * g + r] = oacc[mt][r];
    if (g == 0) {
      ml.m[wave][col] = m_run;
      ml.l[wave][col] = l_run;
      ml.z[wave][col] = z_run;
    }
  }
  __syncthreads();
  {
    const int h = tid >> 6, c0 = 2 * (tid & 63);
    if (h < gq) {
      float M = ml.m[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) M = fmaxf(M, ml.m[w][h]);
      float L = 0.f, Z = 0.f, o0 = 0.f, o1 = 0.f;
      if (M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float f = exp2f(ml.m[w][h] - M);
          L += f * ml.l[w][h];
          Z += f * ml.z[w][h];
          o0 += f * ml.o[w][h][c0];
          o1 += f * ml.o[w][h][c0 + 1];
        }
      }
      constexpr float kUnP = 1.0f / (float)(1 << kPShift);
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + hkv * gq + h;
      float2 o = {o0 * kUnP + Z, o1 * kUnP + Z};
      *reinterpret_cast<float2*>(a.part_o + row * kD + c0) = o;
      if ((tid & 63) == 0) {
        a.part_ml[row * 2] = M;
        a.part_ml[row * 2 + 1] = L;
      }
    }
  }
}

// Log-sum-exp merge of the split partials into the final output row (fp16 or bf16).
template <bool BF16>
__global__ __launch_bounds__(128) void combine_kernel(const float* __restrict__ part_o,
                                                       const float* __restrict__ part_ml, int nparts, int nrows,
                                                       uint16_t* __restrict__ out) {
  const int row = blockIdx.x, c = threadIdx.x;
  float M = -INFINITY;
  for (int p = 0; p < nparts; ++p) M = fmaxf(M, part_ml[((size_t)p * nrows + row) * 2]);
  float L = 0.f, o = 0.f;
  if (M > -INFINITY) {
    for (int p = 0; p < nparts; ++p) {
      const size_t r = (size_t)p * nrows + row;
      const float ms = part_ml[r * 2];
      if (ms == -INFINITY) continue;
      const float f = exp2f(ms - M);
      L += f * part_ml[r * 2 + 1];
      o += f * part_o[r * kD + c];
    }
  }
  const float res = L > 0.f ? o / L : 0.f;
  if (BF16) {
    uint32_t u = __float_as_uint(res);
    u += 0x7FFFu + ((u >> 16) & 1u);
    out[(size_t)row * kD + c] = (uint16_t)(u >> 16);
  } else {
    out[(size_t)row * kD + c] = f2h(res);
  }
}

}  // namespace

hipError_t launch_decode_int(const bd_cache* c, const void* q, int packed_len, int res_len, float softmax_scale,
                             int num_splits, float* part_o, float* part_ml, hipStream_t st) {
  DecodeArgs a;
  a.k_codes = (const uint32_t*)c->k_codes;
  a.v_codes = (const uint32_t*)c->v_codes;
  a.k_params = (const uint32_t*)c->k_params;
  a.v_params = (const uint32_t*)c->v_params;
  a.k_res = (const uint16_t*)c->k_res;
  a.v_res = (const uint16_t*)c->v_res;
  a.q = (const uint16_t*)q;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.n_q_heads = c->n_q_heads;
  a.n_kv_heads = c->n_kv_heads;
  a.gq = c->n_q_heads / c->n_kv_heads;
  a.nb = packed_len / kBlock;
  a.nbcap = c->capacity / kBlock;
  a.res_len = res_len;
  a.num_splits = num_splits;
  a.scale_log2 = softmax_scale * kLog2e;
  dim3 grid(num_splits + 1, c->n_kv_heads, c->batch), block(256);
  if (c->format == BD_FMT_INT4)
    decode_int_kernel<4><<<grid, block, 0, st>>>(a);
  else
    decode_int_kernel<2><<<grid, block, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_combine(const bd_cache* c, const float* part_o, const float* part_ml, int nparts, void* out,
                          hipStream_t st) {
  const int nrows = c->batch * c->n_q_heads;
  if (c->format == BD_FMT_MXFP4)
    combine_kernel<true><<<dim3(nrows), dim3(128), 0, st>>>(part_o, part_ml, nparts, nrows, (uint16_t*)out);
  else
    combine_kernel<false><<<dim3(nrows), dim3(128), 0, st>>>(part_o, part_ml, nparts, nrows, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace bd
