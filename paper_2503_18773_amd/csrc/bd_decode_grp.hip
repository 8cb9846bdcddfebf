// Decode attention over int4 / int2 caches whose quantization group is smaller than the
// 128-token block (Sec. IV-C(1): K_p of shape (T_n/group, d), V_p of shape (T_n, d/group)),
// gfx950.  Same contract as the group-128 kernel (split partials (m, l, O) per query head); a
// plainer schedule, because the parameters now change inside a block:
//
//   S^T[token, head] = sum_c code[token, c] * Q'[c, head] + zq[head],  Q' = Q * s_c * log2(e) / sqrt(d).
//     s_c and z_c belong to (channel, token group), so every 16-token tile lies inside one
//     32-token chunk of the block and the B operand (Q', an fp16 high + low pair: the high piece in
//     the even copies of a head's MFMA column, the low piece in the odd ones, their partial
//     products added with one DPP move) is rebuilt whenever the chunk enters a new token group.
//   O^T[c, head] = sum_t code[t, c] * P'_g[t, head],  P'_g = p * s_(t, g) for the channel group g of
//     c: one variant of P' per channel group, each feeding the M tiles of its channels.  The
//     variants pass through LDS, which also carries them from the lanes that hold a token's
//     score (its row of S^T) to the lanes that need it as contraction index.
//   The centre of each token's codes is taken out of the second product and added back in fp32
//   with the zero terms, as in the group-128 kernel, so that fp16 rounding of P' acts on
//   centred codes.
//   Both fp16 operands are range-normalised by powers of two, so accuracy does not depend on the
//   magnitude of K, V or Q: each head's query is brought below 2^7 and a token group's K scales
//   below 2^8 before Q' is formed (undone when the first product becomes a score), and channel
//   group v's P' carries s * 2^(15 - e_run[v]) with e_run[v] the largest exponent field of the
//   group's V scales so far (accumulators rescaled when it grows, undone before the waves merge).
#include "bd_common.h"
#include "bd_device.h"
#include "bd_fmt.h"
#include "bd_quant_block.h"

namespace bd {
namespace {

constexpr int kWaves = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kTwo24 = 16777216.0f;   // codes enter the MFMAs as code * 2^-24
constexpr int kGrpHeads = 8;            // query heads per workgroup, at most

struct GrpArgs {
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const uint32_t* k_params;
  const uint32_t* v_params;
  const uint16_t* k_res;
  const uint16_t* v_res;
  const uint16_t* q;
  const uint16_t* k_new;   // fused step: the newest token, [B][Hkv][128], not yet in the residual buffers
  const uint16_t* v_new;
  int new_slot;            // its residual slot (res_len - 1), or -1 when the residual buffers are complete
  float* part_o;    // [nparts][B][Hq][128]
  float* part_ml;   // [nparts][B][Hq][2]
  void* out;    // one split only: the output [B][Hq][128], written instead of the partials; else nullptr
  int out_kind;     // element type of `out` (kOutF16 / kOutBf16 / kOutF32)
  int n_q_heads, n_kv_heads, gq;
  int nb, nbcap, res_len, num_splits;
  float scale_log2;
  // paged cache: block n of sequence b is page block_table[b][n], pool index page * Hkv + head;
  // nb and res_len then come from seq_lens[b]
  const int32_t* block_table;
  const int32_t* seq_lens;
  int32_t* status;
  int max_pages, num_pages;
  int step;   // paged: 1 when this launch is the attention of a fused step
  // Contiguous cache, fused step whose token fills the residual block: as in the group-128 kernel
  // (kFlushFirst: the workgroup that reads block flush_blk packs it first; kFlushAfter: the step attends the
  // 128 fp16 rows and one extra workgroup per KV head, blockIdx.x == 0, packs them)
  int flush_mode, flush_blk;
};

template <int GQP, int NV, bool KT>
struct GrpWaveLds {
  __attribute__((aligned(16))) uint16_t zeros[8];   // per-token K: what a lane outside a chain's channel group feeds the matrix unit
  // (rows of qhi, qlo and pbuf padded by 16 bytes: lanes of different heads read the same offset of
  // their rows, and rows a multiple of 256 bytes apart would all fall on the same LDS banks)
  uint16_t qhi[GQP][kD + 8];   // Q' per head, high fp16 piece, in B-operand slot order
  uint16_t qlo[GQP][kD + 8];   // low piece
  float2 vpar[NV][kParSlots];  // per (channel group, token): (scale * position factor, zero + scale * centre code)
  uint16_t c16[NV][kBlock];    // centre code * position factor, in A-operand slot order
  uint16_t pbuf[GQP][kBlock + 8];  // P' of the channel group in work, in B-operand slot order
  float zq[GQP];               // per head: sum_c Q_c z_c of the token group in work
  float ksb[GQP];              // per head: what turns the first product into scores (undoes the range normalisation of Q')
  uint32_t kpar[KT ? 1 : NV][kD];   // K parameters (half2) of the block, per token group and channel
  // per-token K: (scale * 2^24, zero) per (channel group, token) of the block, and per head the sums of the
  // (normalised, scaled) query over each channel group
  float2 ktpar[KT ? NV : 1][kParSlots];
  float qsum[GQP][NV];
};
template <int GQP, int NV>
struct GrpMergeLds {
  float o[kWaves][GQP][kD];
  float m[kWaves][GQP], l[kWaves][GQP], z[kWaves][GQP][NV];
};

constexpr size_t gmax(size_t x, size_t y) { return x > y ? x : y; }

// Every instance fits 256 registers (two waves per SIMD) but those for groups of 32 with more than 4 heads
// per workgroup and 4-bit codes or per-token K, which would spill and run one wave per SIMD instead.
constexpr int grp_waves_per_simd(int bits, int group, int gqp, bool kt) {
  return (bits == 4 || kt) && group == 32 && gqp == 8 ? 1 : 2;
}

// G: quantization group (64 or 32).  GQP: heads per workgroup, padded to 4 or 8 (larger query groups
// take ceil(g_q / 8) workgroups per split and KV head; 16 heads' LDS scratch would not fit); MFMA
// column c carries head c % GQP (the copies compute the same numbers).
// PAGED: blocks are found through the block table and every sequence has its own length.
// KT: K is quantized per token and channel group like V (parameters [token][D/G]):
//   S[t, h] = sum_g s_(t,g) * (sum_{c in g} code_tc Q_c) + sum_g z_(t,g) * (sum_{c in g} Q_c).
//   A lane group holds 32 consecutive channels of a token and the matrix instruction sums over the lane
//   groups, so the channel groups are kept apart in the COLUMNS instead: Q' = Q (normalised, fp16 high + low
//   pair, prepared once per kernel) enters 2 * NG "virtual columns" per head -- (piece, channel group), zero
//   in the lane groups outside that channel group -- which the COPIES copies of the head's column carry in
//   2 * NG / COPIES chains of MFMAs; each partial product is scaled with the (token, channel group)
//   parameters in fp32 and the copies are added with DPP row rotations, after which every copy holds S^T as
//   in the channel-wise case.
template <int BITS, int G, int GQP, bool PAGED, bool KT>
__global__ __launch_bounds__(256, grp_waves_per_simd(BITS, G, GQP, KT)) void decode_grp_kernel(GrpArgs a) {
  // With one wave per SIMD nothing but the wave's own arithmetic hides its memory latency, so it
  // requests a block's values before its keys are consumed and the next block's keys right after
  // ("deep").  With two waves the other one covers and the short queue of the group-128 kernel is
  // better (measured, groups of 64: 13.2 against 13.7 us at 32K, 30.9 against 33.2 us at 128K),
  // except for 2-bit codes, whose blocks are half the bytes (42.9 against 45.3 us at 8 x 32K) -- but not for
  // per-token K in groups of 32 at 2 bits, where the deep queue's registers would spill.
  constexpr bool kDeep = (BITS == 2 && !(KT && G == 32)) || grp_waves_per_simd(BITS, G, GQP, KT) == 1;
  using F = Fmt<BITS>;
  constexpr int WORDS = F::WORDS;
  constexpr int KROW = kD * BITS / 32;       // K words per token
  constexpr int VROW = kBlock * BITS / 32;   // V words per channel per block
  constexpr int NG = kBlock / G;             // token groups per block == channel groups per token
  constexpr int NV = NG;
  constexpr int HP = GQP / 4;
  constexpr int COPIES = 16 / GQP;           // MFMA columns per head
  static_assert(COPIES >= 2 && COPIES % 2 == 0, "the high / low pieces of Q' need an even number of copies");
  constexpr int OWN = 4 / COPIES;            // 32-token chunks whose softmax a lane runs
  using WL = GrpWaveLds<GQP, NV, KT>;
  constexpr int CH = KT ? 2 * NG / COPIES : 0;   // per-token K: MFMA chains per S^T tile
  static_assert(!KT || (2 * NG) % COPIES == 0, "virtual columns per head must fill the copies");
  using ML = GrpMergeLds<GQP, NV>;

  __shared__ __attribute__((aligned(16))) unsigned char smem_raw[gmax(sizeof(ML), kWaves * sizeof(WL))];
  __shared__ float res_s[kBlock][GQP];
  // queries * softmax_scale * log2(e), each head brought below 2^kQTop by a power of two whose inverse is
  // qinv_s[head]; padding heads zero
  __shared__ __attribute__((aligned(16))) float q_s[GQP][kD];
  __shared__ float qinv_s[GQP];

  const int b = blockIdx.z;
  const bool flush_after = a.flush_mode == kFlushAfter;
  const int split = (int)blockIdx.x - (flush_after ? 1 : 0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, g = lane >> 4;
  // Every copy of a head's column receives the same S^T; copy cp keeps the chunks c with
  // c % COPIES == cp, runs their softmax and writes their P', so that work is shared out.
  const int head = col % GQP, cp = col / GQP;
  int hkv = blockIdx.y, head0 = 0;
  if (a.gq > kGrpHeads) {
    const int nchunk = (a.gq + kGrpHeads - 1) / kGrpHeads;
    hkv = blockIdx.y / nchunk;
    head0 = kGrpHeads * (blockIdx.y % nchunk);
  }
  const int gq = min(a.gq - head0, kGrpHeads);
  WL& wl = reinterpret_cast<WL*>(smem_raw)[wave];

  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  int nb = a.nb, res_len = a.res_len;
  int new_slot = a.new_slot;   // fused step: residual slot of the token that is still in the caller's buffer, or -1
  int flush_page = -1;         // paged fused step that fills the residual: the page the block goes to
  if (PAGED) {
    int len = a.seq_lens[b];
    new_slot = -1;
    if (a.step && len >= 0) {
      // fused step: this step's token counts (unless it needs a page the table does not name) and
      // the length is raised only after this kernel.  With a.k_new no kernel has appended the token:
      // it is read from the caller's buffer and filed by this launch, and if it fills the residual,
      // the workgroup that reads the new block quantizes it first (as in the main kernel).
      bool ok = true;
      int e = -1;
      if (len % kBlock == kBlock - 1) {
        const int n = len / kBlock;
        e = n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1;
        ok = e >= 0 && e < a.num_pages;
      }
      if (a.k_new) {
        if (!ok) {
          if (a.status && tid == 0 && split == 0) atomicOr(a.status, 2);   // the token is dropped
        } else if (len % kBlock < kBlock - 1) {
          new_slot = len % kBlock;
        } else {
          flush_page = e;
        }
      }
      len += ok ? 1 : 0;
    }
    len = len < 0 ? 0 : len;
    nb = len / kBlock;
    res_len = len % kBlock;
    if (flush_after && flush_page >= 0) {   // lazy flush: this step attends the 128 residual rows in fp16
      nb -= 1;
      res_len = kBlock;
      new_slot = kBlock - 1;
    }
  }
  // blocks are dealt to the splits four at a time (one per wave), round robin: the workgroups of a
  // unit read one contiguous window of the cache at any moment
  const int blk0 = split * kWaves, blk1 = nb, bstep = kWaves * a.num_splits;
  if (flush_after && split < 0 && head0 != 0) return;   // (one quantizing workgroup per KV head is enough)
  if (!PAGED && a.flush_mode != kFlushNone && head0 == 0 &&
      (flush_after ? split < 0 : split == (a.flush_blk / kWaves) % a.num_splits)) {
    // the step's token completes the residual block: file it, then pack the 128 rows as block flush_blk
    // (kFlushFirst: this workgroup is the block's only reader in this launch -- up to 8 heads per KV head)
    uint16_t* kr = const_cast<uint16_t*>(a.k_res) + unit * kBlock * kD;
    uint16_t* vr = const_cast<uint16_t*>(a.v_res) + unit * kBlock * kD;
    if (tid < 32) {
      const bool is_v = tid >= 16;
      const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
      *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (kBlock - 1) * kD + 8 * (tid & 15)) = *reinterpret_cast<const u4_t*>(src);
    }
    workgroup_global_sync();
    quant_block<BITS, KT, G>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
                             const_cast<uint32_t*>(a.k_params), const_cast<uint32_t*>(a.v_params),
                             unit * a.nbcap + a.flush_blk);
    if (flush_after) return;   // (the whole workgroup: split < 0 is uniform)
    workgroup_global_sync();
  }
  if (PAGED && flush_after && split < 0) {
    // lazy flush: the extra workgroup of a (sequence, KV head) packs the 128 rows into the page if this
    // step's token completes them, and does nothing else
    if (flush_page >= 0 && head0 == 0) {
      uint16_t* kr = const_cast<uint16_t*>(a.k_res) + unit * kBlock * kD;
      uint16_t* vr = const_cast<uint16_t*>(a.v_res) + unit * kBlock * kD;
      if (tid < 32) {
        const bool is_v = tid >= 16;
        const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
        *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (kBlock - 1) * kD + 8 * (tid & 15)) = *reinterpret_cast<const u4_t*>(src);
      }
      workgroup_global_sync();
      quant_block<BITS, KT, G>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
                               const_cast<uint32_t*>(a.k_params), const_cast<uint32_t*>(a.v_params),
                               (size_t)flush_page * a.n_kv_heads + hkv);
    }
    return;
  }
  if (PAGED && !flush_after && flush_page >= 0 && split == ((nb - 1) / kWaves) % a.num_splits) {
    // the 128 residual rows become block nb - 1, which this workgroup alone reads in this launch (one
    // workgroup per split and KV head: the host takes this path for up to 8 heads per KV head)
    uint16_t* kr = const_cast<uint16_t*>(a.k_res) + unit * kBlock * kD;
    uint16_t* vr = const_cast<uint16_t*>(a.v_res) + unit * kBlock * kD;
    if (tid < 32) {
      const bool is_v = tid >= 16;
      const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
      *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (kBlock - 1) * kD + 8 * (tid & 15)) = *reinterpret_cast<const u4_t*>(src);
    }
    workgroup_global_sync();
    quant_block<BITS, KT, G>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
                                const_cast<uint32_t*>(a.k_params), const_cast<uint32_t*>(a.v_params),
                                (size_t)flush_page * a.n_kv_heads + hkv);
    workgroup_global_sync();
  }
  const int rt0 = (res_len * split) / a.num_splits, rt1 = (res_len * (split + 1)) / a.num_splits;
  const uint16_t* qbase = a.q + ((size_t)b * a.n_q_heads + hkv * a.gq + head0) * kD;

  // ---- queries, scaled, for everybody in the workgroup
#pragma unroll
  for (int p = 0; p < HP; ++p) {
    const int h = 4 * p + wave;
    const uint32_t raw = h < gq ? *reinterpret_cast<const uint32_t*>(qbase + h * kD + 2 * lane) : 0u;
    float2 qq = {h2f((uint16_t)(raw & 0xFFFFu)) * a.scale_log2, h2f((uint16_t)(raw >> 16)) * a.scale_log2};
    const uint32_t mb = wave_max_u(max(__float_as_uint(fabsf(qq.x)), __float_as_uint(fabsf(qq.y))));
    const int kq = mb ? min(max(kQTop - 1 - ((int)(mb >> 23) - 127), -60), 60) : 0;   // max |q| * 2^kq < 2^kQTop
    const float up = pow2i(kq);
    qq.x *= up;
    qq.y *= up;
    *reinterpret_cast<float2*>(&q_s[h][2 * lane]) = qq;
    if (lane == 0) qinv_s[h] = pow2i(-kq);
  }

  // ---- residual slice, part 1: scores of this workgroup's fp16 tokens, 16 per MFMA chain
  const int nres = rt1 - rt0, nres_groups = (nres + 15) >> 4;
  if (wave < nres_groups) {
    h8_t res_q[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const h8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
      res_q[j] = col < gq ? *reinterpret_cast<const h8_t*>(qbase + col * kD + 32 * j + 8 * g) : zero;
    }
    for (int grp = wave; grp < nres_groups; grp += kWaves) {
      const int t = min(rt0 + 16 * grp + col, rt1 - 1);   // rows past the slice repeat its last token
      // (the newest token of a fused step is read from where the caller left it)
      const uint16_t* row = (t == new_slot ? a.k_new + unit * kD : a.k_res + (unit * kBlock + t) * kD) + 8 * g;
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const h8_t*>(row + 32 * j), res_q[j], acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int tt = 16 * grp + 4 * g + r;
        if (tt < nres && col < GQP) res_s[tt][col] = acc[r] * a.scale_log2;
      }
    }
  }
  if (new_slot >= 0 && split == 0 && head0 == 0 && tid < 32 && res_len < kBlock && (PAGED || a.flush_mode == kFlushNone)) {   // fused step: file the new token for later steps
    const bool is_v = tid >= 16;
    const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
    uint16_t* dst = const_cast<uint16_t*>(is_v ? a.v_res : a.k_res) + (unit * kBlock + new_slot) * kD + 8 * (tid & 15);
    *reinterpret_cast<u4_t*>(dst) = *reinterpret_cast<const u4_t*>(src);
  }
  __syncthreads();   // q_s and res_s are complete

  float m_run = -INFINITY, l_run = 0.0f;
  float z_run[NV];
  // Channel group v's products accumulate in units of 2^(e_run[v] - 15): e_run is the largest exponent field
  // seen so far among the group's (fp16) V scales, so that scale * 2^(15 - e_run) < 2 whatever the magnitude
  // of V, and the accumulators are rescaled when it grows, together with the softmax's own rescaling.
  int e_run[NV];
  f4_t xacc[NV], oacc[8];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    z_run[v] = 0.0f;
    e_run[v] = 0;
    xacc[v] = (f4_t){0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  // Row rho = 4*gamma + r of S^T tile T = 2*chunk + run holds block token run_base(4*chunk + gamma, run) + r:
  // the tile lies inside one 32-token chunk, and lane group g ends up with exactly the 8 tokens
  // (slot group 4*chunk + g) that one 16-byte piece of the second product's B operand holds.
  const int row_gamma = col >> 2, row_r = col & 3;
  const int prep_sg = lane & 15;
  const int run0 = F::run_base(prep_sg, 0), run1 = F::run_base(prep_sg, 1);
  RawTile<WORDS> kraw[8], vraw[8];
  u4_t kp0, kp1;              // K parameters (half2) of this lane's two channel runs, token group g % NG
  uint32_t vp[2 * NV];        // V parameters (half2) of tokens 2*lane, 2*lane+1, per channel group

  uint32_t ktp[KT ? 2 * NV : 1];   // per-token K: K parameters (half2) of tokens 2*lane, 2*lane+1, per channel group
  auto issue_params = [&](size_t bi) {
    if constexpr (KT) {
      const uint32_t* kpp = a.k_params + (bi * kBlock + 2 * lane) * NV;
      if constexpr (NV == 4) {
        const u4_t x = *reinterpret_cast<const u4_t*>(kpp), y = *reinterpret_cast<const u4_t*>(kpp + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ktp[i] = x[i];
          ktp[4 + i] = y[i];
        }
      } else {
        const u4_t x = *reinterpret_cast<const u4_t*>(kpp);
#pragma unroll
        for (int i = 0; i < 4; ++i) ktp[i] = x[i];
      }
    } else {
      // lane group g fetches token group g % NG (its 16 lanes cover the 128 channels); the token
      // groups meet in LDS, which keeps 8 registers in flight instead of 8 per token group
      const uint32_t* pp = a.k_params + (bi * NG + (g % NG)) * kD;
      kp0 = *reinterpret_cast<const u4_t*>(pp + run0);
      kp1 = *reinterpret_cast<const u4_t*>(pp + run1);
    }
    const uint32_t* vpp = a.v_params + (bi * kBlock + 2 * lane) * NV;
    if constexpr (NV == 4) {
      const u4_t x = *reinterpret_cast<const u4_t*>(vpp), y = *reinterpret_cast<const u4_t*>(vpp + 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        vp[i] = x[i];
        vp[4 + i] = y[i];
      }
    } else {
      const u4_t x = *reinterpret_cast<const u4_t*>(vpp);
#pragma unroll
      for (int i = 0; i < 4; ++i) vp[i] = x[i];
    }
  };
  auto issue_keys = [&](size_t bi) {
    const uint32_t* kp = a.k_codes + bi * (size_t)(kBlock * KROW) + WORDS * g;
#pragma unroll
    for (int T = 0; T < 8; ++T) {
      const int tok = F::run_base(4 * (T >> 1) + row_gamma, T & 1) + row_r;
      kraw[T] = load_raw<WORDS>(kp + (size_t)tok * KROW);
    }
  };
  auto issue_values = [&](size_t bi) {
    const uint32_t* vpp = a.v_codes + bi * (size_t)(kD * VROW) + WORDS * g;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) vraw[mt] = load_raw<WORDS>(vpp + (size_t)(16 * mt + col) * VROW);
  };

  // Q' = Q * s_c as an fp16 high + low pair in B-operand order and the zero term sum_c Q_c z_c, per
  // head, with the K parameters of token group tg: 16 lanes per head (slot group lane % 16).
  auto prep_queries = [&](int tg) {
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int ph = 4 * p + (lane >> 4);
      const f4_t qa = *reinterpret_cast<const f4_t*>(&q_s[ph][run0]);
      const f4_t qb = *reinterpret_cast<const f4_t*>(&q_s[ph][run1]);
      const u4_t ka = *reinterpret_cast<const u4_t*>(&wl.kpar[tg][run0]);
      const u4_t kb = *reinterpret_cast<const u4_t*>(&wl.kpar[tg][run1]);
      // the token group's K scales are brought below 2^kSTop (queries are below 2^kQTop): |Q'| < 2^15
      uint32_t sb = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) sb = max(sb, max(ka[i] & 0xFFFFu, kb[i] & 0xFFFFu));
      const int ek = -norm_exponent(row_max16_u(sb), kSTop);
      const float dn = pow2i(-ek);
      float zsum = 0.0f;
      uint16_t qh[8], ql[8];
#pragma unroll
      for (int run = 0; run < 2; ++run)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float qc = run ? qb[i] : qa[i];
          const uint32_t pr = run ? kb[i] : ka[i];
          const float s = h2f((uint16_t)(pr & 0xFFFFu)), z = h2f((uint16_t)(pr >> 16));
          const float t = qc * (s * dn) * F::un(i);
          const uint16_t hi = f2h(t);
          qh[2 * i + run] = hi;
          ql[2 * i + run] = f2h(t - h2f(hi));
          zsum = __builtin_fmaf(qc, z, zsum);
        }
      const float qinv = qinv_s[ph];
      zsum = row_sum16(zsum) * qinv;
      u4_t phi, plo;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        phi[v] = (uint32_t)qh[2 * v] | ((uint32_t)qh[2 * v + 1] << 16);
        plo[v] = (uint32_t)ql[2 * v] | ((uint32_t)ql[2 * v + 1] << 16);
      }
      *reinterpret_cast<u4_t*>(&wl.qhi[ph][8 * prep_sg]) = phi;
      *reinterpret_cast<u4_t*>(&wl.qlo[ph][8 * prep_sg]) = plo;
      if (prep_sg == 0) {
        wl.zq[ph] = zsum;
        wl.ksb[ph] = pow2i(24 + ek) * qinv;   // codes enter as code * 2^-24
      }
    }
  };

  // Per-token K: Q' = Q * position factor (no K scale in it), once per kernel, and the sums of Q over each
  // channel group for the zero terms.
  float zq_k[KT ? CH : 1];      // chain k of this lane's copy: sum of Q over its channel group if it carries the high piece, else 0
  float qinv = 1.0f;            // undoes the query's normalisation
  constexpr bool kKeepB = CH == 1;     // the chains' B operands stay in registers when there is one chain, else they are read per chunk
  h8_t bqk[1][4];
  auto chain_operand = [&](int k, int j) {
    const int v = k * COPIES + cp;                       // virtual column: piece v & 1, channel group v >> 1
    const bool live = (g >> (G == 64 ? 1 : 0)) == (v >> 1);
    const uint16_t* row = (v & 1) ? &wl.qlo[head][8 * (4 * g + j)] : &wl.qhi[head][8 * (4 * g + j)];
    return *reinterpret_cast<const h8_t*>(live ? row : wl.zeros);
  };
  if constexpr (KT) {
    if (lane < 8) wl.zeros[lane] = 0;
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int ph = 4 * p + (lane >> 4);
      const f4_t qa = *reinterpret_cast<const f4_t*>(&q_s[ph][run0]);
      const f4_t qb = *reinterpret_cast<const f4_t*>(&q_s[ph][run1]);
      uint16_t qh[8], ql[8];
      float part[2] = {0.0f, 0.0f};
#pragma unroll
      for (int run = 0; run < 2; ++run)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float qc = run ? qb[i] : qa[i];
          const float t = qc * F::un(i);
          const uint16_t hi = f2h(t);
          qh[2 * i + run] = hi;
          ql[2 * i + run] = f2h(t - h2f(hi));
          part[run] += qc;
        }
      u4_t phi, plo;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        phi[v] = (uint32_t)qh[2 * v] | ((uint32_t)qh[2 * v + 1] << 16);
        plo[v] = (uint32_t)ql[2 * v] | ((uint32_t)ql[2 * v + 1] << 16);
      }
      *reinterpret_cast<u4_t*>(&wl.qhi[ph][8 * prep_sg]) = phi;
      *reinterpret_cast<u4_t*>(&wl.qlo[ph][8 * prep_sg]) = plo;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const float x = row_sum16((run0 / G == v ? part[0] : 0.0f) + (run1 / G == v ? part[1] : 0.0f));
        if (prep_sg == 0) wl.qsum[ph][v] = x;
      }
    }
    wave_sync();
    qinv = qinv_s[head];
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const int v = k * COPIES + cp;
      zq_k[k] = (v & 1) ? 0.0f : wl.qsum[head][v >> 1];
    }
    if constexpr (kKeepB) {
#pragma unroll
      for (int j = 0; j < 4; ++j) bqk[0][j] = chain_operand(0, j);
    }
  }

  // Paged: table entry of block n (-1 past the end of the row), and the first block at or after
  // n, in this wave's stride, whose entry names a page of the pool; entries that do not are
  // skipped and reported in *status.
  auto table_entry = [&](int n) { return n < a.max_pages ? a.block_table[(size_t)b * a.max_pages + n] : -1; };
  auto first_valid = [&](int n, int entry, size_t& idx) {
    while (n < blk1) {
      if (entry >= 0 && entry < a.num_pages) {
        idx = (size_t)entry * a.n_kv_heads + hkv;
        break;
      }
      if (a.status && lane == 0) atomicOr(a.status, 1);
      n += bstep;
      entry = n < blk1 ? table_entry(n) : -1;
    }
    return n;
  };
  int blk = blk0 + wave;
  size_t bi = unit * a.nbcap + blk;
  if (PAGED) blk = first_valid(blk, blk < blk1 ? table_entry(blk) : -1, bi);
  if (blk < blk1) {
    issue_params(bi);
    issue_keys(bi);
  }
  // this lane's 8 tokens of chunk c are block tokens tok0 + 32*c + {run_base offsets}: slot group 4*c + g
  while (blk < blk1) {
    int nblk = blk + bstep;
    size_t nbi = bi + bstep;
    if (PAGED) nblk = first_valid(nblk, nblk < blk1 ? table_entry(nblk) : -1, nbi);
    const bool has_next = nblk < blk1;
    if constexpr (kDeep) issue_values(bi);
    if constexpr (KT) {   // K parameters of the block's tokens, per channel group
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const uint32_t pr = ktp[u * NV + v];
          wl.ktpar[v][par_slot(2 * lane + u)] = make_float2(h2f((uint16_t)(pr & 0xFFFFu)) * kTwo24, h2f((uint16_t)(pr >> 16)));
        }
    } else if (g < NG) {   // K parameters of the block: every token group from the lane group that fetched it
      *reinterpret_cast<u4_t*>(&wl.kpar[g][run0]) = kp0;
      *reinterpret_cast<u4_t*>(&wl.kpar[g][run1]) = kp1;
    }
    // ---- V parameters of the block's tokens, per channel group
    int e_new[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
      e_new[v] = max(e_run[v], (int)(wave_max_u(max(vp[v] & 0x7FFFu, vp[NV + v] & 0x7FFFu)) >> 10));
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const uint32_t pr = vp[u * NV + v];
        const float sv = h2f((uint16_t)(pr & 0xFFFFu)), zv = h2f((uint16_t)(pr >> 16));
        const int t = 2 * lane + u;
        const int r = t & 3;
        const float ct = sv > 0.0f ? rintf(fminf(fmaxf(-zv * __builtin_amdgcn_rcpf(sv), 0.0f), F::kQmax)) : 0.0f;
        wl.vpar[v][par_slot(t)] = make_float2(sv * pow2i(15 - e_new[v]) * F::un(r), __builtin_fmaf(ct, sv, zv));
        wl.c16[v][F::operand_pos(t)] = (uint16_t)(ct * F::inv_un(r));   // an integer: the fp16 subnormal code * 2^-24
      }
    // ---- S^T, chunk by chunk
    float sc[OWN][2][4];   // [owned chunk][run][row]
    h8_t bq[4];   // the high piece of Q' in the even copies of a head's column, the low piece in the odd ones
    float zq = 0.0f, ksb = 0.0f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (KT) {
        if (c == 0) wave_sync();   // the block's K parameters are staged
        h8_t bload[kKeepB ? 1 : CH][4];
        if constexpr (!kKeepB) {
#pragma unroll
          for (int k = 0; k < CH; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) bload[k][j] = chain_operand(k, j);
        }
        auto bop = [&](int k, int j) -> h8_t {
          if constexpr (!kKeepB) return bload[k][j];
          else return bqk[k][j];
        };
        const bool mine = c % COPIES == cp;
#pragma unroll
        for (int run = 0; run < 2; ++run) {
          const int T = 2 * c + run;
          h8_t ak[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) ak[j] = F::dequant(kraw[T].w, j);
          float val[4] = {0.f, 0.f, 0.f, 0.f};
          const int slot = par_slot(F::run_base(4 * c + g, run));
#pragma unroll
          for (int k = 0; k < CH; ++k) {
            f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak[j], bop(k, j), acc, 0, 0, 0);
            const float2* par = &wl.ktpar[(k * COPIES + cp) >> 1][slot];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float2 sz = par[r];
              val[r] = __builtin_fmaf(sz.x, acc[r], __builtin_fmaf(sz.y, zq_k[k], val[r]));
            }
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float x = val[r];
            if (COPIES == 4) x += dpp_f<kRowRor4>(x);
            if (COPIES >= 2) x += dpp_f<kRowRor8>(x);
            x *= qinv;
            sc[c / COPIES][run][r] = mine ? x : sc[c / COPIES][run][r];
          }
        }
        continue;
      }
      if ((32 * c) % G == 0) {   // the chunk opens a token group: new Q'
        wave_sync();             // the previous Q' has been read by every lane
        prep_queries((32 * c) / G);
        wave_sync();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          bq[j] = *reinterpret_cast<const h8_t*>(cp & 1 ? &wl.qlo[head][8 * (4 * g + j)] : &wl.qhi[head][8 * (4 * g + j)]);
        }
        zq = wl.zq[head];
        ksb = wl.ksb[head];
      }
#pragma unroll
      for (int run = 0; run < 2; ++run) {
        const int T = 2 * c + run;
        f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const h8_t ak = F::dequant(kraw[T].w, j);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak, bq[j], acc, 0, 0, 0);
        }
        // the chunk's owner (copy c % COPIES) adds the other piece's partial product, which the
        // neighbouring copy computed: GQP lanes up for an even owner, GQP lanes down for an odd one
        const bool mine = c % COPIES == cp;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float x = acc[r];
          if (c & 1) x += dpp_f<GQP == 4 ? kRowShr4 : kRowShr8>(x);
          else x += dpp_f<GQP == 4 ? kRowShl4 : kRowShl8>(x);
          const float val = __builtin_fmaf(x, ksb, zq);
          sc[c / COPIES][run][r] = mine ? val : sc[c / COPIES][run][r];
        }
      }
    }
    if constexpr (!kDeep) issue_values(bi);
    if (kDeep && has_next) {   // parameters first: they are the next block's first consumers
      issue_params(nbi);
      issue_keys(nbi);
    }
    // ---- online softmax (Alg. 1) over this lane's 8 * OWN tokens of head `head`
    float bmax = sc[0][0][0];
#pragma unroll
    for (int o = 0; o < OWN; ++o)
#pragma unroll
      for (int run = 0; run < 2; ++run)
#pragma unroll
        for (int r = 0; r < 4; ++r) bmax = fmaxf(bmax, sc[o][run][r]);
    bmax = head_max<COPIES>(bmax);
    const float m_new = fmaxf(m_run, bmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
    m_run = m_new;
    l_run *= alpha;
    bool grew = false;
#pragma unroll
    for (int v = 0; v < NV; ++v) grew |= e_new[v] != e_run[v];
    if (grew || __any(alpha != 1.0f)) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const float av = alpha * pow2i(e_run[v] - e_new[v]);
#pragma unroll
        for (int mm = 0; mm < 8 / NV; ++mm) oacc[v * (8 / NV) + mm] *= av;
        xacc[v] *= av;
        z_run[v] *= alpha;
        e_run[v] = e_new[v];
      }
    }
#pragma unroll
    for (int o = 0; o < OWN; ++o)
#pragma unroll
      for (int run = 0; run < 2; ++run)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          sc[o][run][r] = __builtin_amdgcn_exp2f(sc[o][run][r] - m_new);
          l_run += sc[o][run][r];
        }
    // ---- O^T += V^T P'_v, one channel group after the other
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      __builtin_amdgcn_sched_barrier(0);   // one variant at a time: interleaving them costs a wave per SIMD in registers
      wave_sync();   // the previous variant has been read by every lane
#pragma unroll
      for (int o = 0; o < OWN; ++o) {
        const int sg = 4 * (o * COPIES + cp) + g;   // slot group of this lane's 8 tokens of its o-th chunk
        u4_t w;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          uint32_t hv[2];
#pragma unroll
          for (int run = 0; run < 2; ++run) {
            const float p = sc[o][run][r];
            const float2 par = wl.vpar[v][par_slot(F::run_base(sg, run)) + r];
            z_run[v] = __builtin_fmaf(p, par.y, z_run[v]);
            hv[run] = (uint32_t)f2h(p * par.x);
          }
          w[r] = hv[0] | (hv[1] << 16);   // entries 2r, 2r + 1 of the slot group
        }
        *reinterpret_cast<u4_t*>(&wl.pbuf[head][8 * sg]) = w;   // every (head, slot group) has one owner
      }
      wave_sync();
      h8_t bp[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) bp[j] = *reinterpret_cast<const h8_t*>(&wl.pbuf[head][8 * (4 * g + j)]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const h8_t ac = *reinterpret_cast<const h8_t*>(&wl.c16[v][8 * (4 * g + j)]);
        xacc[v] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ac, bp[j], xacc[v], 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mm = 0; mm < 8 / NV; ++mm) {
          const int mt = v * (8 / NV) + mm;
          oacc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(F::dequant(vraw[mt].w, j), bp[j], oacc[mt], 0, 0, 0);
        }
    }
    if (!kDeep && has_next) {
      issue_params(nbi);
      issue_keys(nbi);
    }
    wave_sync();   // the next block's parameters overwrite this wave's LDS scratch
    blk = nblk;
    bi = nbi;
  }

  // ---- merge the waves of the workgroup (cross-wave step of the cooperative softmax)
  l_run = head_sum<COPIES>(l_run);
#pragma unroll
  for (int v = 0; v < NV; ++v) z_run[v] = head_sum<COPIES>(z_run[v]);
  __syncthreads();   // every wave is done with its per-wave LDS before the space is reused
  ML& ml = *reinterpret_cast<ML*>(smem_raw);
  if (col < GQP) {
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        ml.o[wave][col][16 * mt + 4 * g + r] =
            (oacc[mt][r] - xacc[mt / (8 / NV)][0]) * (kTwo24 * pow2i(e_run[mt / (8 / NV)] - 15));
    if (g == 0) {
      ml.m[wave][col] = m_run;
      ml.l[wave][col] = l_run;
#pragma unroll
      for (int v = 0; v < NV; ++v) ml.z[wave][col][v] = z_run[v];
    }
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < HP; ++p) {
    const int h = 4 * p + wave, c0 = 2 * lane;
    if (h < gq) {
      const int v = c0 / G;   // channel group of channels c0, c0 + 1
      float M = ml.m[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) M = fmaxf(M, ml.m[w][h]);
      for (int t = 0; t < nres; ++t) M = fmaxf(M, res_s[t][h]);
      float L = 0.f, Z = 0.f, o0 = 0.f, o1 = 0.f;
      if (M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float f = __builtin_amdgcn_exp2f(ml.m[w][h] - M);
          L += f * ml.l[w][h];
          Z += f * ml.z[w][h][v];
          o0 += f * ml.o[w][h][c0];
          o1 += f * ml.o[w][h][c0 + 1];
        }
        // residual slice, part 2: fold the fp16 tokens in
        for (int t = 0; t < nres; ++t) {
          const float pr = __builtin_amdgcn_exp2f(res_s[t][h] - M);
          const uint16_t* vrow = rt0 + t == new_slot ? a.v_new + unit * kD : a.v_res + (unit * kBlock + rt0 + t) * kD;
          const uint32_t raw = *reinterpret_cast<const uint32_t*>(vrow + c0);
          L += pr;
          o0 = __builtin_fmaf(pr, h2f((uint16_t)(raw & 0xFFFFu)), o0);
          o1 = __builtin_fmaf(pr, h2f((uint16_t)(raw >> 16)), o1);
        }
      }
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + hkv * a.gq + head0 + h;
      float2 o = {o0 + Z, o1 + Z};
      if (a.out) {   // one split: row == the output row
        store_final_pair(a.out, row * kD + c0, a.out_kind, o.x, o.y, L);
      } else {
        *reinterpret_cast<float2*>(a.part_o + row * kD + c0) = o;
        if (lane == 0) {
          a.part_ml[row * 2] = M;
          a.part_ml[row * 2 + 1] = L;
        }
      }
    }
  }
}

template <int BITS, int G, bool KT = false>
void launch_heads(const GrpArgs& a, bool paged, dim3 grid, hipStream_t st) {
  if (paged) {
    if (a.gq <= 4) decode_grp_kernel<BITS, G, 4, true, KT><<<grid, dim3(256), 0, st>>>(a);
    else decode_grp_kernel<BITS, G, 8, true, KT><<<grid, dim3(256), 0, st>>>(a);
  } else {
    if (a.gq <= 4) decode_grp_kernel<BITS, G, 4, false, KT><<<grid, dim3(256), 0, st>>>(a);
    else decode_grp_kernel<BITS, G, 8, false, KT><<<grid, dim3(256), 0, st>>>(a);
  }
}

hipError_t launch_format(int format, const GrpArgs& a, bool paged, int batch, hipStream_t st) {
  dim3 grid(a.num_splits + (a.flush_mode == kFlushAfter ? 1 : 0), a.n_kv_heads * ((a.gq + kGrpHeads - 1) / kGrpHeads), batch);
  switch (format) {
    case BD_FMT_INT4_G64: launch_heads<4, 64>(a, paged, grid, st); break;
    case BD_FMT_INT4_G32: launch_heads<4, 32>(a, paged, grid, st); break;
    case BD_FMT_INT2_G64: launch_heads<2, 64>(a, paged, grid, st); break;
    case BD_FMT_INT2_G32: launch_heads<2, 32>(a, paged, grid, st); break;
    case BD_FMT_INT4_KT_G64: launch_heads<4, 64, true>(a, paged, grid, st); break;
    case BD_FMT_INT4_KT_G32: launch_heads<4, 32, true>(a, paged, grid, st); break;
    case BD_FMT_INT2_KT_G64: launch_heads<2, 64, true>(a, paged, grid, st); break;
    case BD_FMT_INT2_KT_G32: launch_heads<2, 32, true>(a, paged, grid, st); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_grp(const bd_cache* c, const void* q, int packed_len, int res_len, float softmax_scale,
                             int num_splits, float* part_o, float* part_ml, const void* k_new, const void* v_new,
                             void* out, hipStream_t st, int flush) {
  GrpArgs a;
  a.k_new = (const uint16_t*)k_new;
  a.v_new = (const uint16_t*)v_new;
  // flush 1: the step's token fills the residual block, which this launch packs first (packed_len counts it,
  // res_len is 0); flush 2: ... which this launch attends in fp16 (res_len is 128) and packs as well
  a.flush_mode = flush == 1 ? kFlushFirst : flush == 2 ? kFlushAfter : kFlushNone;
  a.flush_blk = flush == 1 ? packed_len / kBlock - 1 : packed_len / kBlock;
  a.new_slot = k_new && flush != 1 ? res_len - 1 : -1;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
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
  a.block_table = nullptr;
  a.seq_lens = nullptr;
  a.status = nullptr;
  a.max_pages = a.num_pages = a.step = 0;
  return launch_format(c->format, a, false, c->batch, st);
}

hipError_t launch_decode_grp_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                                   float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                                   void* out, hipStream_t st, bool lazy) {
  GrpArgs a;
  a.k_new = (const uint16_t*)k_new;   // non-null: the step's token, which this launch appends itself
  a.v_new = (const uint16_t*)v_new;
  a.new_slot = -1;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
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
  a.nb = a.nbcap = a.res_len = 0;   // per sequence, from seq_lens
  a.num_splits = num_splits;
  a.scale_log2 = softmax_scale * kLog2e;
  a.block_table = c->block_table;
  a.seq_lens = c->seq_lens;
  a.status = c->status;
  a.max_pages = c->max_pages_per_seq;
  a.num_pages = c->num_pages;
  a.step = step ? 1 : 0;
  a.flush_mode = lazy ? kFlushAfter : kFlushNone;   // (as in launch_decode_paged)
  a.flush_blk = 0;
  return launch_format(c->format, a, true, c->batch, st);
}

}  // namespace bd
