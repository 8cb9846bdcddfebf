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
// in the B-operand layout of the second product: probabilities go exp -> fp16 -> MFMA without
// an LDS round trip.  The row -> token assignment of each S^T tile and the order of codes
// inside a word are chosen so that this holds (the analogue, for MFMA, of inducing the packed
// layout from the consumer instruction, Sec. III-A(1)).
//
// The 16 columns carry the <= 4 heads of the group four times over (column c holds head c%4).
// Column group c/4 then keeps only every fourth S^T tile, so the softmax arithmetic runs on
// 8 values per lane per 128-token block instead of 32, with every lane doing useful work; the
// packed probabilities are moved back to columns 0..3 with DPP row shifts.
//
// Dequantization is reduced to masking (Sec. III-A(3) uses lop3 to the same end):
//   * a masked code sitting in the low bits of an fp16 lane IS the fp16 subnormal code * 2^-24
//     (times a power of two when it sits at bit 4..7); gfx950's MFMA takes subnormal inputs
//     exactly, so the MFMAs consume  word & mask  directly: 5 ALU ops per 8 int4 codes,
//     9 per 16 int2 codes; the power-of-two factors are folded into Q' / P'.
//   * K is quantized per channel, so  S = sum_c (Q_c s_c) code_c + sum_c Q_c z_c : the query is
//     rescaled once per 128-token block and the zero term is one scalar per head and block.
//     Q' = Q*s is carried as an fp16 high + low pair (two MFMAs on the same A operand), which
//     keeps ~22 bits: a single fp16 Q' is not enough when a channel holds outliers.
//   * V is quantized per token, so  O = sum_t (P_t s_t) code_t + sum_t P_t z_t.
//   * Raw codes are offset by the token's zero-point, so sum_t P'_t code_t and sum_t P_t z_t are
//     two large numbers that nearly cancel; the fp16 rounding of P' and the last bits of two
//     separately accumulated fp32 sums would then show in the result.  Both are avoided by
//     writing  x_hat = s_t (code - c_t) + (z_t + s_t c_t)  with the integer c_t = rint(-z_t/s_t)
//     (the code of the value 0): a ninth A tile holds c_t for every token, so the same MFMA
//     chain also yields sum_t P'_t c_t, which is subtracted from every channel at the end; what
//     is left outside the MFMAs is sum_t P_t (z_t + s_t c_t), at most half a quantization step
//     per token.
//
// Range.  The fp16 operands are kept clear of overflow and of the subnormals whatever the magnitudes
// of Q, K and V are: every head's queries are scaled by a power of two to below 2^7 before they meet the
// K scales (a column of the B operand may carry any factor; it comes out of that column's scores), so
// |Q'| < 2^15 with the block's K scales normalised likewise; and the per-token V scale is folded into the exponent of the softmax,
// P'_t = 2^(S_t + log2 scale_t - m) with m the running maximum of S + log2 scale, so P' <= 1 with the
// largest term at 1, while the weights proper are P'_t / scale_t in fp32.
//
// The fp16 residual tail (Sec. IV-B) is shared out evenly over the workgroups of a
// (sequence, KV head): each takes a slice of the <= 127 residual tokens, scores them with
// plain dot products and folds them into its partial in the final merge, so no workgroup
// does the tail alone.
#include "bd_common.h"
#include "bd_device.h"
#include "bd_fmt.h"
#include "bd_quant_block.h"

namespace bd {
namespace {

constexpr int kWaves = 4;          // waves per workgroup, all spread along the token axis (W_m = 1)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kTwo24 = 16777216.0f;          // codes enter the MFMAs as code * 2^-24
constexpr float kTwoM24 = 1.0f / 16777216.0f;

struct DecodeArgs {
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
  float* part_ml;   // [nparts][B][Hq][2]   (running max in log2 units, running sum)
  void* out;    // one split only: the output [B][Hq][128], written instead of the partials; else nullptr
  int out_kind;     // element type of `out` (kOutF16 / kOutBf16 / kOutF32)
  int n_q_heads, n_kv_heads, gq;
  int nb;           // packed 128-token blocks
  int nbcap;
  int res_len;
  int num_splits;
  float scale_log2; // softmax_scale * log2(e)
  // paged cache: block n of sequence b is page block_table[b][n], pool index page * Hkv + head;
  // nb and res_len then come from seq_lens[b]
  const int32_t* block_table;
  const int32_t* seq_lens;
  int32_t* status;
  int max_pages, num_pages;
  int step;            // paged: 1 when this launch is the attention of a fused step (see the kernel)
  // Contiguous cache, fused step whose token fills the residual block (Sec. IV-B(1)): the 127 rows of the
  // residual buffers plus k_new / v_new become packed block flush_blk inside this launch.
  //   kFlushFirst: block flush_blk counts as packed (nb includes it); the one workgroup that reads it
  //                quantizes it before it attends (the step is append, flush, then attention).
  //   kFlushAfter: the step attends the 128 fp16 rows (the paper's Residual Kernel: attention on the
  //                half-precision block, quantization of it in the same launch); one extra workgroup per
  //                (sequence, KV head), blockIdx.x == 0, does nothing but quantize.
  int flush_mode, flush_blk;
};

// Per-wave LDS scratch.  GQP = query heads per KV head, padded to 4, 8 or 16.
template <int GQP>
struct WaveLds {
  // (rows padded by 16 bytes: lanes of different heads read the same offset of their rows, and rows a
  // multiple of 256 bytes apart would all fall on the same LDS banks)
  uint16_t qhi[GQP][kD + 8];   // Q' per head, high fp16 piece, in B-operand slot order
  uint16_t qlo[GQP][kD + 8];   // low piece
  float4 vpar[kParSlots];  // per V token of the block: (log2 scale, 1 / scale, value of the centre code / scale, -)
  float2 kpar[kParSlots];  // per-token K only: (scale * 2^24, zero) of the block's tokens
  uint16_t c16[kBlock];    // per V token: centre code * position factor, in the A-operand order of P'
  float zq[GQP];           // per head: sum_c Q_c z_c * 2^-24 (Q as normalised below)
};
template <int GQP>
struct MergeLds {
  float o[kWaves][GQP][kD];
  float m[kWaves][GQP], l[kWaves][GQP], z[kWaves][GQP];
};

constexpr size_t cmax(size_t x, size_t y) { return x > y ? x : y; }

// GQP: the query group padded to 4, 8 or 16 heads; the 16 MFMA columns carry it 16/GQP times
//      (column c holds head c % GQP, "column group" c / GQP) and the softmax work of a block
//      is shared out over the column groups.
//      GQP = 4: column group cg keeps S^T tiles cg and 4 + cg (8 values per lane) and the
//      packed probabilities are moved to columns 0..3 with DPP row shifts, so O^T accumulates
//      in those columns only.
//      GQP = 8, 16: each column group owns 4 / COPIES of the block's four 32-token k-steps of
//      the second product: it keeps the S^T tiles of those tokens, runs their softmax, and
//      presents their P' as its part of the B operand (zero in the k-steps it does not own);
//      no probability moves between lanes, and the column groups' partial O^T are added
//      once, after the loop.
// SINGLE: no wave has more than one block (short contexts); the host picks the instance.
// PAGED: blocks are found through the block table and every sequence has its own length.
// KT: K is quantized per token (Sec. IV-C(1)):  S[t] = s_t * sum_c Q_c code_tc + z_t * sum_c Q_c,
//     so Q' = Q is prepared once per kernel instead of once per block and the per-token scale
//     and zero are applied to the kept S^T values.
template <int BITS, int GQP, bool SINGLE, bool PAGED, bool KT>
__global__ __launch_bounds__(256, 2) void decode_int_kernel(DecodeArgs a) {
  using F = Fmt<BITS>;
  using WL = WaveLds<GQP>;
  using ML = MergeLds<GQP>;
  constexpr int WORDS = F::WORDS;            // words per lane per tile
  constexpr int KROW = kD * BITS / 32;       // K words per token
  constexpr int VROW = kBlock * BITS / 32;   // V words per channel per block
  constexpr int COPIES = 16 / GQP;           // column groups
  constexpr int OWN = 4 / COPIES;            // k-steps owned by a column group
  constexpr int HP = GQP / 4;                // passes over the heads where 16 lanes work on one head

  __shared__ __attribute__((aligned(16))) unsigned char smem_raw[cmax(sizeof(ML), kWaves * sizeof(WL))];
  __shared__ float res_s[kBlock][GQP];       // scores of this workgroup's residual tokens, per head
  __shared__ __attribute__((aligned(16))) float q_s[HP > 1 ? GQP : 1][kD];   // larger groups: queries, normalised; padding heads zero
  __shared__ int kq_s[HP > 1 ? GQP : 1];                                     // larger groups: each head's normalising exponent

  const int b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool flush_after = a.flush_mode == kFlushAfter;
  const int split = (int)blockIdx.x - (flush_after ? 1 : 0);
  const int col = lane & 15, g = lane >> 4;            // MFMA column and contraction group
  const int head = col % GQP, cg = col / GQP;          // head carried by the column; column group
  // Query groups of more than 16 heads are taken 16 at a time by ceil(g_q / 16) workgroups per
  // (split, KV head), each of which reads the cache once.
  int hkv = blockIdx.y, head0 = 0;
  if (GQP == 16 && a.gq > 16) {
    const int nchunk = (a.gq + 15) >> 4;
    hkv = blockIdx.y / nchunk;
    head0 = 16 * (blockIdx.y % nchunk);
  }
  const int gq = min(a.gq - head0, 16);                // heads of this workgroup
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
      // the length is raised only after this kernel.  With a.k_new the token has not been appended
      // by a kernel of its own: it is read from the caller's buffer and filed by this launch, and
      // if it fills the residual, the workgroup that reads the new block quantizes it first.
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
  // Blocks are dealt to the splits four at a time (one per wave), round robin: at any moment the
  // workgroups of a (sequence, KV head) unit read one contiguous window of the cache.  (Contiguous
  // ranges per split put the workgroups' streams a power of two apart for the usual split counts,
  // and then all of them march over the same memory channels.)
  const int blk0 = split * kWaves, blk1 = nb, bstep = kWaves * a.num_splits;
  if (flush_after && split < 0 && head0 != 0) return;   // (one quantizing workgroup per KV head is enough)
  if (!PAGED && a.flush_mode != kFlushNone && head0 == 0 &&
      (flush_after ? split < 0 : split == (a.flush_blk / kWaves) % a.num_splits)) {
    // The step's token completes the residual block: file it, then quantize the 128 rows as block
    // flush_blk.  kFlushFirst: this workgroup is the block's only reader in this launch (one workgroup per
    // split and KV head: query groups of up to 16 heads).  kFlushAfter: nobody reads the block here, and
    // the others read the residual rows, which only gain the row they take from k_new / v_new anyway.
    uint16_t* kr = const_cast<uint16_t*>(a.k_res) + unit * kBlock * kD;
    uint16_t* vr = const_cast<uint16_t*>(a.v_res) + unit * kBlock * kD;
    if (tid < 32) {
      const bool is_v = tid >= 16;
      const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
      *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (kBlock - 1) * kD + 8 * (tid & 15)) = *reinterpret_cast<const u4_t*>(src);
    }
    workgroup_global_sync();
    quant_block<BITS, KT, kBlock>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
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
      quant_block<BITS, KT, kBlock>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
                                    const_cast<uint32_t*>(a.k_params), const_cast<uint32_t*>(a.v_params),
                                    (size_t)flush_page * a.n_kv_heads + hkv);
    }
    return;
  }
  if (PAGED && !flush_after && flush_page >= 0 && split == ((nb - 1) / kWaves) % a.num_splits) {
    // This step's token completes the residual (Sec. IV-B(1)): the 128 rows become block nb - 1, which
    // this workgroup alone reads in this launch.  (One workgroup per split and KV head: the host takes
    // this path only for query groups of up to 16 heads.)
    uint16_t* kr = const_cast<uint16_t*>(a.k_res) + unit * kBlock * kD;
    uint16_t* vr = const_cast<uint16_t*>(a.v_res) + unit * kBlock * kD;
    if (tid < 32) {
      const bool is_v = tid >= 16;
      const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
      *reinterpret_cast<u4_t*>((is_v ? vr : kr) + (kBlock - 1) * kD + 8 * (tid & 15)) = *reinterpret_cast<const u4_t*>(src);
    }
    workgroup_global_sync();   // the row is read back below, and the block further down, by other threads of this workgroup
    quant_block<BITS, KT, kBlock>(kr, vr, const_cast<uint32_t*>(a.k_codes), const_cast<uint32_t*>(a.v_codes),
                                  const_cast<uint32_t*>(a.k_params), const_cast<uint32_t*>(a.v_params),
                                  (size_t)flush_page * a.n_kv_heads + hkv);
    workgroup_global_sync();
  }
  // this workgroup's slice of the fp16 residual tokens
  const int rt0 = (res_len * split) / a.num_splits, rt1 = (res_len * (split + 1)) / a.num_splits;
  const uint16_t* qbase = a.q + ((size_t)b * a.n_q_heads + hkv * a.gq + head0) * kD;

  float m_run = -INFINITY;   // running max of this lane's head (log2 units), equal in all lanes of the head
  float l_run = 0.0f;        // running sum of p over this lane's own tokens
  float z_run = 0.0f;        // running sum of p * zero_t over this lane's own tokens
  f4_t xacc = {0.f, 0.f, 0.f, 0.f};   // sum_t P'_t * centre code of token t (every row the same)
  f4_t oacc[8];
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  // A wave keeps little in flight: the keys of its next block are requested when the current
  // block is done, the values of a block when its keys are about to be consumed.  The eight
  // waves of a compute unit share one in-order memory pipeline, so whatever one wave requests
  // early only delays what the others are waiting for: 8 KB per wave (16 MB over the chip) keeps
  // HBM busy, and a shorter queue shortens the ramp at both ends of the kernel.
  const int prep_sg = lane & 15;
  const int run0 = F::run_base(prep_sg, 0), run1 = F::run_base(prep_sg, 1);
  const int tok_base = 32 * (col >> 2) + (col & 3);   // row `col` of tile T holds token tok_base + 4T
  RawTile<WORDS> kraw[8], vraw[8];
  u4_t kp0, kp1;   // K parameters (half2) of this lane's two channel runs
  u2_t kp2;        // per-token K: parameters of tokens 2*lane, 2*lane+1
  u2_t vp2;        // V parameters (half2) of tokens 2*lane, 2*lane+1
  // All four take the index `bi` of the block in the packed arrays: unit * nbcap + block for the
  // contiguous cache, page * Hkv + head for the paged one.
  auto issue_kpar = [&](size_t bi) {
    if constexpr (KT) {
      kp2 = *reinterpret_cast<const u2_t*>(a.k_params + bi * kBlock + 2 * lane);
    } else {
      const uint32_t* pp = a.k_params + bi * kD;
      kp0 = *reinterpret_cast<const u4_t*>(pp + run0);
      kp1 = *reinterpret_cast<const u4_t*>(pp + run1);
    }
  };
  auto issue_vpar = [&](size_t bi) {
    vp2 = *reinterpret_cast<const u2_t*>(a.v_params + bi * kBlock + 2 * lane);
  };
  auto issue_ktile = [&](size_t bi, int T) {
    const uint32_t* kp = a.k_codes + bi * (size_t)(kBlock * KROW) + WORDS * g;
    kraw[T] = load_raw<WORDS>(kp + (size_t)(tok_base + 4 * T) * KROW);
  };
  auto issue_vtile = [&](size_t bi, int mt) {
    const uint32_t* vp = a.v_codes + bi * (size_t)(kD * VROW) + WORDS * g;
    vraw[mt] = load_raw<WORDS>(vp + (size_t)(16 * mt + col) * VROW);
  };
  // Loads return in order, so what is needed first is requested first: the queries and this
  // wave's first residual key rows, then the first block.
  // A group of up to 4 heads: every lane keeps the query slice it rescales per block (head
  // lane / 16, two runs of 4 channels) in registers.  Larger groups go through LDS (q_s).
  uint32_t qld[HP];
  u2_t qraw0 = {0u, 0u}, qraw1 = {0u, 0u};
  if constexpr (HP == 1) {
    if ((lane >> 4) < gq) {
      qraw0 = *reinterpret_cast<const u2_t*>(qbase + (lane >> 4) * kD + run0);
      qraw1 = *reinterpret_cast<const u2_t*>(qbase + (lane >> 4) * kD + run1);
    }
  } else {
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int h = 4 * p + (tid >> 6);   // thread tid: head h, channels 2*(tid%64), +1
      qld[p] = h < gq ? *reinterpret_cast<const uint32_t*>(qbase + h * kD + 2 * lane) : 0u;
    }
  }
  const uint16_t* kres = a.k_res + unit * kBlock * kD;
  // row t of the residual keys: the newest token of a fused step is read from where the caller left it
  auto kres_row = [&](int t) { return t == new_slot ? a.k_new + unit * kD : kres + (size_t)t * kD; };
  // The residual tokens are scored 16 at a time on the matrix unit: S[token, head] with the fp16
  // key rows as A and the fp16 queries as B, four k-steps of 32 channels.  Wave w takes token
  // groups w, w + 4, ...; the operands of its first group are requested here.
  const int nres = rt1 - rt0, nres_groups = (nres + 15) >> 4;
  const bool has_res = wave < nres_groups;
  h8_t res_a[4], res_q[4];
  auto load_res_keys = [&](int grp) {
    const int t = min(rt0 + 16 * grp + col, rt1 - 1);   // rows past the slice repeat its last token
    const uint16_t* row = kres_row(t) + 8 * g;
#pragma unroll
    for (int j = 0; j < 4; ++j) res_a[j] = *reinterpret_cast<const h8_t*>(row + 32 * j);
  };
  if (has_res) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const h8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
      res_q[j] = col < gq ? *reinterpret_cast<const h8_t*>(qbase + col * kD + 32 * j + 8 * g) : zero;
    }
    load_res_keys(wave);
  }
  if (new_slot >= 0 && split == 0 && head0 == 0 && tid < 32 && res_len < kBlock && (PAGED || a.flush_mode == kFlushNone)) {   // fused step: file the new token for later steps
    const bool is_v = tid >= 16;
    const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
    uint16_t* dst = const_cast<uint16_t*>(is_v ? a.v_res : a.k_res) + (unit * kBlock + new_slot) * kD + 8 * (tid & 15);
    *reinterpret_cast<u4_t*>(dst) = *reinterpret_cast<const u4_t*>(src);
  }
  // (Where exactly the values are requested is fixed at compile time, so that the compiler knows
  // how many loads are in flight behind the one it waits for: half way through QK^T.)
  const int my_blocks = blk1 > blk0 + wave ? (blk1 - blk0 - wave + bstep - 1) / bstep : 0;
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
  size_t bi = unit * a.nbcap + blk;
  if (PAGED) blk = first_valid(blk, blk < blk1 ? table_entry(blk) : -1, bi);
  if (blk < blk1) {   // parameters first: they are the block's first consumers
    issue_kpar(bi);
    issue_vpar(bi);
#pragma unroll
    for (int T = 0; T < 8; ++T) issue_ktile(bi, T);
  }

  // The first residual value rows this workgroup folds in at the very end: requested now, so
  // that the final merge does not wait on memory (thread tid: channels 2*(tid%64), +1).
  constexpr int kResPre = 2;
  auto vres_row = [&](int t) {
    return t == new_slot ? a.v_new + unit * kD : a.v_res + (unit * kBlock + t) * kD;
  };
  uint32_t vres_pre[kResPre];
#pragma unroll
  for (int i = 0; i < kResPre; ++i)
    vres_pre[i] = i < nres ? *reinterpret_cast<const uint32_t*>(vres_row(rt0 + i) + 2 * lane) : 0u;

  // ---- larger groups: the queries, scaled, for everybody in the workgroup
  if constexpr (HP > 1) {
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int h = 4 * p + (tid >> 6);   // this wave holds all 128 channels of head h
      uint32_t qb = row_max16_u(max(qld[p] & 0x7FFFu, (qld[p] >> 16) & 0x7FFFu));
      qb = max(max(__builtin_amdgcn_readlane(qb, 0), __builtin_amdgcn_readlane(qb, 16)),
               max(__builtin_amdgcn_readlane(qb, 32), __builtin_amdgcn_readlane(qb, 48)));
      const int kqh = norm_exponent(qb, kQTop);
      const float f = pow2i(kqh);
      float2 qq = {h2f((uint16_t)(qld[p] & 0xFFFFu)) * f, h2f((uint16_t)(qld[p] >> 16)) * f};
      *reinterpret_cast<float2*>(&q_s[h][2 * lane]) = qq;
      if (lane == 0) kq_s[h] = kqh;
    }
    __syncthreads();
  }

  // ---- residual slice, part 1: scores s[t][h] = q_h . k_t * softmax_scale * log2(e)
  if (has_res) {
    for (int grp = wave; grp < nres_groups; grp += kWaves) {
      if (grp != wave) load_res_keys(grp);
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(res_a[j], res_q[j], acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = 16 * grp + 4 * g + r;   // row 4g + r of the tile
        if (t < nres && col < GQP) res_s[t][col] = acc[r] * a.scale_log2;
      }
    }
  }

  // tokens whose softmax this lane runs: for its o-th owned k-step j = cg * OWN + o, the low
  // (lh = 0) and high (lh = 1) fp16 halves of the P' registers come from tiles tile_lo / tile_hi
  // of half j / 2; token = 32 g + 4 tile + row
  // Every head's queries times the power of two that brings the largest below 1 (kq); the factor comes
  // back out of the scores, together with softmax_scale * log2(e) and the 2^24 of the subnormal codes (kS).
  float qv[2][4];
  int kq_head = 0;   // of the head this lane's column carries
  if constexpr (HP == 1) {
    uint32_t qb = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      qb = max(max(qb, max(qraw0[i] & 0x7FFFu, (qraw0[i] >> 16) & 0x7FFFu)), max(qraw1[i] & 0x7FFFu, (qraw1[i] >> 16) & 0x7FFFu));
    qb = row_max16_u(qb);   // largest |q| of head lane / 16
    const float f = pow2i(norm_exponent(qb, kQTop));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qv[0][i] = h2f((uint16_t)((qraw0[i >> 1] >> (16 * (i & 1))) & 0xFFFFu)) * f;
      qv[1][i] = h2f((uint16_t)((qraw1[i >> 1] >> (16 * (i & 1))) & 0xFFFFu)) * f;
    }
    kq_head = norm_exponent((uint32_t)__shfl((int)qb, 16 * head), kQTop);   // (head h's queries sit in lanes 16h ..)
  } else {
    kq_head = kq_s[head];
  }
  const float kS = a.scale_log2 * pow2i((KT ? 0 : 24) - kq_head);   // what the kept scores still have to be multiplied by
  const float kZ = a.scale_log2 * pow2i(-kq_head);                  // ... and the zero term sum_c Q_c z_c
  int tb[OWN][2];
#pragma unroll
  for (int o = 0; o < OWN; ++o) {
    const int j = cg * OWN + o;
    tb[o][0] = 32 * g + 4 * (4 * (j >> 1) + ((j & 1) ? F::tile_lo(1) : F::tile_lo(0)));
    tb[o][1] = 32 * g + 4 * (4 * (j >> 1) + ((j & 1) ? F::tile_hi(1) : F::tile_hi(0)));
  }
  if (COPIES == 4) {   // tiles cg and 4 + cg
    tb[0][0] = 32 * g + 4 * cg;
    tb[0][1] = 32 * g + 16 + 4 * cg;
  }

  // Q' = Q * s_c as an fp16 high + low pair in B-operand order, and the zero term sum_c Q_c z_c, per
  // head: once per block for channel-wise K (with the block's parameters), once per kernel for
  // per-token K.  16 lanes per head (slot group lane % 16: two runs of 4 consecutive channels).
  // Channel-wise K: the block's scales are first brought below 1 by a power of two (2^-ek, from the largest
  // of the block), so that with |q| < 1 the products neither overflow nor sink into the fp16 subnormals;
  // the factor comes back out of the scores with kS.  Returns ek.
  auto prep_queries = [&]() -> int {
    int ek = 0;
    float nrm[4];   // 2^-ek times the position factor of register i
#pragma unroll
    for (int i = 0; i < 4; ++i) nrm[i] = F::un(i);
    if constexpr (!KT) {
      uint32_t sb = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) sb = max(sb, max(kp0[i] & 0xFFFFu, kp1[i] & 0xFFFFu));
      ek = -norm_exponent(row_max16_u(sb), kSTop);   // scale * 2^-ek < 2^kSTop for every channel of the block
      const float f = pow2i(-ek);
#pragma unroll
      for (int i = 0; i < 4; ++i) nrm[i] = f * F::un(i);
    }
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int ph = 4 * p + (lane >> 4);
      f4_t qa, qb;
      if constexpr (HP == 1) {
        qa = (f4_t){qv[0][0], qv[0][1], qv[0][2], qv[0][3]};
        qb = (f4_t){qv[1][0], qv[1][1], qv[1][2], qv[1][3]};
      } else {
        qa = *reinterpret_cast<const f4_t*>(&q_s[ph][run0]);
        qb = *reinterpret_cast<const f4_t*>(&q_s[ph][run1]);
      }
      float zsum = 0.0f;
      h2_t qh[4], ql[4];   // register i: entries 2i (run 0) and 2i + 1 (run 1)
#pragma unroll
      for (int run = 0; run < 2; ++run)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float qc = run ? qb[i] : qa[i];
          float t = qc;   // per-token K: Q' = Q, and the "zero term" is sum_c Q_c
          float z = 1.0f;
          if constexpr (!KT) {
            const h2_t pr = __builtin_bit_cast(h2_t, run ? kp1[i] : kp0[i]);   // (scale, zero)
            t = qc * (float)pr[0];   // exact: 11 bits times 11 bits
            z = (float)pr[1];
          }
          // high piece, and the rest in one rounding: fma(t, nrm, -high)
          const _Float16 hi = (_Float16)(t * nrm[i]);
          qh[i][run] = hi;
          ql[i][run] = (_Float16)__builtin_fmaf(t, nrm[i], -(float)hi);
          zsum = __builtin_fmaf(qc, z, zsum);
        }
      zsum = row_sum16(zsum);
      u4_t phi, plo;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        phi[v] = __builtin_bit_cast(uint32_t, qh[v]);
        plo[v] = __builtin_bit_cast(uint32_t, ql[v]);
      }
      *reinterpret_cast<u4_t*>(&wl.qhi[ph][8 * prep_sg]) = phi;
      *reinterpret_cast<u4_t*>(&wl.qlo[ph][8 * prep_sg]) = plo;
      if (prep_sg == 0) wl.zq[ph] = zsum;
    }
    return ek;
  };
  // Groups of up to 8 heads: the high piece of Q' goes to the even column groups and the low piece to
  // the odd ones, so one MFMA per k-step produces both partial products (added across the column
  // groups afterwards); groups of 9..16 have no columns to spare and run two MFMAs per k-step.
  constexpr bool kSplitCols = COPIES >= 2;
  h8_t bqh[4], bql[4];
  auto load_bq = [&](int j) {
    if constexpr (kSplitCols) {
      bqh[j] = *reinterpret_cast<const h8_t*>(cg & 1 ? &wl.qlo[head][8 * (4 * g + j)] : &wl.qhi[head][8 * (4 * g + j)]);
    } else {
      bqh[j] = *reinterpret_cast<const h8_t*>(&wl.qhi[head][8 * (4 * g + j)]);
      bql[j] = *reinterpret_cast<const h8_t*>(&wl.qlo[head][8 * (4 * g + j)]);
    }
  };
  float zq = 0.0f, qsum = 0.0f;
  if constexpr (KT) {
    (void)prep_queries();
    wave_sync();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      load_bq(j);
    }
    qsum = wl.zq[head];
  }

  // Two waves of different workgroups share each SIMD and the issue arbiter favours the older
  // one, which then runs a block ahead, finishes early and leaves the other to drain alone with
  // half the loads in flight.  Priority by remaining work keeps the pair in step.
  int done = 0;
  bool first = true;
  while (blk < blk1) {
    int nblk = SINGLE ? blk1 : blk + bstep;
    size_t nbi = bi + bstep;
    int next_entry = -1;   // requested a block ahead, like the parameters
    if (PAGED && nblk < blk1) next_entry = table_entry(nblk);
    if (!SINGLE) {
      const int q4 = (4 * done) / (my_blocks > 0 ? my_blocks : 1);   // quarter of the work done: 0..3
      if (q4 == 0) __builtin_amdgcn_s_setprio(3);
      else if (q4 == 1) __builtin_amdgcn_s_setprio(2);
      else if (q4 == 2) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
      ++done;
    }
    float kSb = kS;   // kS for this block's K exponent
    if constexpr (!KT) kSb = kS * pow2i(prep_queries());
    if constexpr (KT) {   // K parameters of the block's 128 tokens
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float sk = h2f((uint16_t)(kp2[u] & 0xFFFFu)), zk = h2f((uint16_t)(kp2[u] >> 16));
        wl.kpar[par_slot(2 * lane + u)] = make_float2(sk * kTwo24, zk);
      }
    }
    // V parameters of the block's 128 tokens
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const float sv = h2f((uint16_t)(vp2[u] & 0xFFFFu)), zv = h2f((uint16_t)(vp2[u] >> 16));
      const int t = 2 * lane + u;
      const int r = t & 3;                // row of the token inside its S^T tile
      // (a token whose values are all equal has scale 0 and all-zero codes: any scale does, take 1)
      const float se = sv > 0.0f ? sv : 1.0f, rs = __builtin_amdgcn_rcpf(se);
      const float ct = sv > 0.0f ? rintf(fminf(fmaxf(-zv * rs, 0.0f), F::kQmax)) : 0.0f;
      wl.vpar[par_slot(t)] = make_float4(__builtin_amdgcn_logf(se), rs, __builtin_fmaf(ct, sv, zv) * rs, 0.0f);
      wl.c16[F::p_slot(t)] = (uint16_t)(ct * F::inv_un(r));
    }
    wave_sync();
    if constexpr (!KT) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        load_bq(j);
      }
      zq = wl.zq[head];
    }
    bool has_next = !SINGLE && nblk < blk1;
    if (!PAGED && has_next) {   // small, and the next block's first consumers: requested a block ahead
      issue_kpar(nbi);
      issue_vpar(nbi);
    }
    // groups of 9..16 heads: only once the keys' registers are free, which lets two waves fit a SIMD
    constexpr bool kValuesAfterQK = GQP == 16;

    // ---- S^T tiles (rows = tokens 32*(row/4) + 4T + row%4, all 16 columns valid); each lane
    //      keeps the tiles of the k-steps its column group owns: sc[o][low/high half][row]
    float sc[OWN][2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f4_t s[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        f4_t acc = {0.f, 0.f, 0.f, 0.f};   // (the zero term, one number per head, joins in the softmax)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const h8_t ak = F::dequant(kraw[4 * half + tt].w, j);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak, bqh[j], acc, 0, 0, 0);
          if constexpr (!kSplitCols) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ak, bql[j], acc, 0, 0, 0);
        }
        s[tt] = acc;
      }
      if (half == 0 && !kValuesAfterQK) {
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) issue_vtile(bi, mt);
      }
      // k-steps 2*half and 2*half+1 draw on this half's four tiles
      if constexpr (COPIES == 1) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            sc[2 * half + jj][0][r] = s[F::tile_lo(jj)][r];
            sc[2 * half + jj][1][r] = s[F::tile_hi(jj)][r];
          }
      } else if constexpr (COPIES == 2) {   // column group cg owns k-steps 2cg, 2cg+1: half cg
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            // own partial product plus the other column group's (half 0 is kept by group 0, half 1 by group 1)
            float lo = s[F::tile_lo(jj)][r], hi = s[F::tile_hi(jj)][r];
            lo += half == 0 ? dpp_f<kRowShl8>(lo) : dpp_f<kRowShr8>(lo);
            hi += half == 0 ? dpp_f<kRowShl8>(hi) : dpp_f<kRowShr8>(hi);
            sc[jj][0][r] = (half == 0 || cg == 1) ? lo : sc[jj][0][r];
            sc[jj][1][r] = (half == 0 || cg == 1) ? hi : sc[jj][1][r];
          }
      } else {                              // column group cg keeps tile cg of each half: its own partial
                                            // product plus that of the neighbouring column group
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float v0 = s[0][r] + dpp_f<kRowShl4>(s[0][r]), v1 = s[1][r] + dpp_f<kRowShr4>(s[1][r]);
          const float v2 = s[2][r] + dpp_f<kRowShl4>(s[2][r]), v3 = s[3][r] + dpp_f<kRowShr4>(s[3][r]);
          const float lo = cg & 1 ? v1 : v0, hi = cg & 1 ? v3 : v2;
          sc[0][half][r] = cg & 2 ? hi : lo;
        }
      }
    }
    if (kValuesAfterQK) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) issue_vtile(bi, mt);
    }
    if constexpr (KT) {   // per-token scale and zero of K
#pragma unroll
      for (int o = 0; o < OWN; ++o)
#pragma unroll
        for (int lh = 0; lh < 2; ++lh)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float2 kq = wl.kpar[par_slot(tb[o][lh]) + r];
            sc[o][lh][r] = __builtin_fmaf(sc[o][lh][r], kq.x, kq.y * qsum);
          }
    }
    // ---- online softmax (Alg. 1) over this lane's 8 * OWN tokens of head `head`, on S + log2 of the
    //      token's V scale (see "Range" at the top): av = score in log2 units, but for the block's zero term
#pragma unroll
    for (int o = 0; o < OWN; ++o)
#pragma unroll
      for (int lh = 0; lh < 2; ++lh)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sc[o][lh][r] = __builtin_fmaf(sc[o][lh][r], kSb, wl.vpar[par_slot(tb[o][lh]) + r].x);
    float bmax = sc[0][0][0];
#pragma unroll
    for (int o = 0; o < OWN; ++o)
#pragma unroll
      for (int lh = 0; lh < 2; ++lh)
#pragma unroll
        for (int r = 0; r < 4; ++r) bmax = fmaxf(bmax, sc[o][lh][r]);
    bmax = head_max<COPIES>(bmax);
    // channel-wise K: every score of the head still lacks the block's zero term
    const float zqs = zq * kZ;
    const float m_new = fmaxf(m_run, bmax + zqs);
    const float zoff = zqs - m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
    m_run = m_new;
    l_run *= alpha;
    z_run *= alpha;
    if (!SINGLE && !first && __any(alpha != 1.0f)) {   // nothing to rescale on the first block
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) oacc[mt] *= alpha;
      xacc *= alpha;
    }
    u4_t pb[4];   // P' as the B operand of the 4 k-steps of O^T += V^T P'
    if constexpr (COPIES == 4) {   // valid in columns 0..3
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float e = __builtin_amdgcn_exp2f(sc[0][half][r] + zoff);   // P' = weight * V scale, <= 1
          const float4& par = wl.vpar[par_slot(tb[0][half]) + r];
          l_run = __builtin_fmaf(e, par.y, l_run);
          z_run = __builtin_fmaf(e, par.z, z_run);
          // gather the column groups' fp16 values into the B-operand register pairs
          const uint32_t x = (uint32_t)f2h(e * F::un(r));
          const uint32_t pr = x | dpp_u<F::kPairShift>(x << 16);
          pb[2 * half][r] = pr;
          pb[2 * half + 1][r] = dpp_u<F::kStepShift>(pr);
        }
    } else {                       // zero where another column group owns the k-step
      u4_t pair[OWN];
#pragma unroll
      for (int o = 0; o < OWN; ++o)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          uint32_t hv[2];
#pragma unroll
          for (int lh = 0; lh < 2; ++lh) {
            const float e = __builtin_amdgcn_exp2f(sc[o][lh][r] + zoff);
            const float4& par = wl.vpar[par_slot(tb[o][lh]) + r];
            l_run = __builtin_fmaf(e, par.y, l_run);
            z_run = __builtin_fmaf(e, par.z, z_run);
            hv[lh] = (uint32_t)f2h(e * F::un(r));
          }
          pair[o][r] = hv[0] | (hv[1] << 16);
        }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if constexpr (COPIES == 1) pb[j][r] = pair[j][r];
          else pb[j][r] = cg == (j >> 1) ? pair[j & 1][r] : 0u;
        }
    }
    // ---- O^T += V^T P' : k-step j contracts 32 tokens (8 per lane group)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const h8_t ac = *reinterpret_cast<const h8_t*>(&wl.c16[8 * (4 * g + j)]);
      xacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ac, __builtin_bit_cast(h8_t, pb[j]), xacc, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {   // k-step outermost: consecutive MFMAs go to different accumulators
      const h8_t bp = __builtin_bit_cast(h8_t, pb[j]);
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
        oacc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(F::dequant(vraw[mt].w, j), bp, oacc[mt], 0, 0, 0);
    }
    if (PAGED && has_next) {
      nblk = first_valid(nblk, next_entry, nbi);
      has_next = nblk < blk1;
      if (has_next) {
        issue_kpar(nbi);
        issue_vpar(nbi);
      }
    }
    if (has_next) {
#pragma unroll
      for (int T = 0; T < 8; ++T) issue_ktile(nbi, T);
    }
    // Both sums grow with the number of tokens, their difference (the signal) with its square root: every
    // 16 blocks the centre sum is taken out of the accumulators and starts again from zero.
    if (!SINGLE && (done & 15) == 0) {
#pragma unroll
      for (int mt = 0; mt < 8; ++mt) oacc[mt] -= xacc[0];
      xacc = (f4_t){0.f, 0.f, 0.f, 0.f};
    }
    wave_sync();   // the next block's prep overwrites this wave's LDS scratch
    first = false;
    blk = nblk;
    bi = nbi;
  }

  // ---- merge the column groups (groups of 8 heads), then the waves of the workgroup
  //      (cross-wave step of the cooperative softmax)
  l_run = head_sum<COPIES>(l_run);
  z_run = head_sum<COPIES>(z_run);
  __syncthreads();   // every wave is done with its WaveLds before the space is reused
  ML& ml = *reinterpret_cast<ML*>(smem_raw);
  // (all lane movement first, in passes over independent values, then one predicated run of stores)
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) oacc[mt] -= xacc[0];
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
      for (int r = 0; r < 4; ++r) ml.o[wave][col][16 * mt + 4 * g + r] = oacc[mt][r] * kTwo24;
    if (g == 0) {
      ml.m[wave][col] = m_run;
      ml.l[wave][col] = l_run;
      ml.z[wave][col] = z_run;
    }
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < HP; ++p) {
    const int h = 4 * p + (tid >> 6), c0 = 2 * (tid & 63);
    if (h < gq) {
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
          Z += f * ml.z[w][h];
          o0 += f * ml.o[w][h][c0];
          o1 += f * ml.o[w][h][c0 + 1];
        }
        // residual slice, part 2: fold the fp16 tokens in (the first rows were requested at the
        // start of the kernel, any further ones are read here)
        auto fold = [&](int t, uint32_t raw) {
          const float p = __builtin_amdgcn_exp2f(res_s[t][h] - M);
          L += p;
          o0 = __builtin_fmaf(p, h2f((uint16_t)(raw & 0xFFFFu)), o0);
          o1 = __builtin_fmaf(p, h2f((uint16_t)(raw >> 16)), o1);
        };
#pragma unroll
        for (int t = 0; t < kResPre; ++t)
          if (t < nres) fold(t, vres_pre[t]);
        for (int t = kResPre; t < nres; ++t) fold(t, *reinterpret_cast<const uint32_t*>(vres_row(rt0 + t) + c0));
      }
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + hkv * a.gq + head0 + h;
      float2 o = {o0 + Z, o1 + Z};
      if (a.out) {   // one split: row == the output row
        store_final_pair(a.out, row * kD + c0, a.out_kind, o.x, o.y, L);
      } else {
        *reinterpret_cast<float2*>(a.part_o + row * kD + c0) = o;
        if ((tid & 63) == 0) {
          a.part_ml[row * 2] = M;
          a.part_ml[row * 2 + 1] = L;
        }
      }
    }
  }
}

// Log-sum-exp merge of the split partials into the final output rows (fp16 or bf16).
// One workgroup per output row: 128 channels x kGroups interleaved groups of partials.  The
// kernel is pure latency (a few hundred KB in total), so every thread issues all its loads at
// once -- up to kBatch partials per round, one round for up to kGroups * kBatch partials -- and
// merges them with a running maximum; the groups meet in LDS.
constexpr int kCombineGroups = 8, kCombineBatch = 8;
// Fused step of a paged cache: the merge is the last kernel of the step, so it also raises the
// length of every sequence whose token was appended (same test as the append kernel).
struct StepBump {
  int32_t* seq_lens;            // nullptr: nothing to raise
  const int32_t* block_table;
  int n_q_heads, max_pages, num_pages;
  int every_token;              // a page is needed by every token (MXFP4), not only by the 128th
};

template <int G>
__global__ __launch_bounds__(128 * G) void combine_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_ml,
                                                           int nparts, int nrows,
                                                           void* __restrict__ out, int kind, StepBump bump) {
  constexpr int kBatch = kCombineBatch;
  __shared__ float sm[G][128], sl[G][128], so[G][128];
  const int row = blockIdx.x, tid = threadIdx.x, c = tid & 127, grp = tid >> 7;
  if (bump.seq_lens && tid == 128 * G - 1 && row % bump.n_q_heads == 0) {   // one thread per sequence
    const int b = row / bump.n_q_heads;
    const int len = bump.seq_lens[b];
    if (len >= 0) {
      bool ok = true;
      if (bump.every_token || len % kBlock == kBlock - 1) {
        const int n = len / kBlock;
        const int e = n < bump.max_pages ? bump.block_table[(size_t)b * bump.max_pages + n] : -1;
        ok = e >= 0 && e < bump.num_pages;
      }
      if (ok) bump.seq_lens[b] = len + 1;
    }
  }
  float M = -INFINITY, L = 0.f, o = 0.f;
  for (int p0 = grp; p0 < nparts; p0 += G * kBatch) {
    float2 ml[kBatch];
    float ov[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int p = p0 + G * i;
      const size_t r = (size_t)(p < nparts ? p : 0) * nrows + row;
      ml[i] = *reinterpret_cast<const float2*>(part_ml + r * 2);
      ov[i] = part_o[r * kD + c];
      if (p >= nparts) ml[i].x = -INFINITY;
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const float Mn = fmaxf(M, ml[i].x);
      const bool live = ml[i].x > -INFINITY;
      const float fo = live ? __builtin_amdgcn_exp2f(M - Mn) : 1.0f;
      const float fn = live ? __builtin_amdgcn_exp2f(ml[i].x - Mn) : 0.0f;
      L = L * fo + fn * ml[i].y;
      o = o * fo + fn * ov[i];
      M = Mn;
    }
  }
  sm[grp][c] = M;
  sl[grp][c] = L;
  so[grp][c] = o;
  __syncthreads();
  if (tid < 128) {
    float Mt = sm[0][c];
#pragma unroll
    for (int g = 1; g < G; ++g) Mt = fmaxf(Mt, sm[g][c]);
    float res = 0.f;
    if (Mt > -INFINITY) {
      float Lt = 0.f, ot = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float Mg = sm[g][c];
        const float f = Mg > -INFINITY ? __builtin_amdgcn_exp2f(Mg - Mt) : 0.f;
        Lt += f * sl[g][c];
        ot += f * so[g][c];
      }
      res = Lt > 0.f ? ot / Lt : 0.f;
    }
    const size_t idx = (size_t)row * kD + c;
    if (kind == kOutF32) reinterpret_cast<float*>(out)[idx] = res;
    else reinterpret_cast<uint16_t*>(out)[idx] = kind == kOutBf16 ? f2bf(res) : f2h(res);
  }
}

}  // namespace

namespace {

template <int BITS, int GQP, bool KT>
void launch_mode(bool single, bool paged, const DecodeArgs& a, dim3 grid, dim3 block, hipStream_t st) {
  if (paged) decode_int_kernel<BITS, GQP, false, true, KT><<<grid, block, 0, st>>>(a);
  else if (single) decode_int_kernel<BITS, GQP, true, false, KT><<<grid, block, 0, st>>>(a);
  else decode_int_kernel<BITS, GQP, false, false, KT><<<grid, block, 0, st>>>(a);
}

template <int BITS, bool KT>
void launch_group(int gq, bool single, bool paged, const DecodeArgs& a, dim3 grid, dim3 block, hipStream_t st) {
  if (gq <= 4) launch_mode<BITS, 4, KT>(single, paged, a, grid, block, st);
  else if (gq <= 8) launch_mode<BITS, 8, KT>(single, paged, a, grid, block, st);
  else launch_mode<BITS, 16, KT>(single, paged, a, grid, block, st);
}

// picks the kernel instance: format, query group padded to 4 / 8 / 16 heads, loop structure
void launch_instance(int format, int gq, bool single, bool paged, const DecodeArgs& a, dim3 grid, dim3 block,
                     hipStream_t st) {
  switch (format) {
    case BD_FMT_INT4: launch_group<4, false>(gq, single, paged, a, grid, block, st); break;
    case BD_FMT_INT2: launch_group<2, false>(gq, single, paged, a, grid, block, st); break;
    case BD_FMT_INT4_KT: launch_group<4, true>(gq, single, paged, a, grid, block, st); break;
    default: launch_group<2, true>(gq, single, paged, a, grid, block, st); break;
  }
}

}  // namespace

hipError_t launch_decode_int(const bd_cache* c, const void* q, int packed_len, int res_len, float softmax_scale,
                             int num_splits, float* part_o, float* part_ml, const void* k_new, const void* v_new,
                             void* out, hipStream_t st, int flush) {
  DecodeArgs a;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
  a.k_codes = (const uint32_t*)c->k_codes;
  a.v_codes = (const uint32_t*)c->v_codes;
  a.k_params = (const uint32_t*)c->k_params;
  a.v_params = (const uint32_t*)c->v_params;
  a.k_res = (const uint16_t*)c->k_res;
  a.v_res = (const uint16_t*)c->v_res;
  a.q = (const uint16_t*)q;
  a.k_new = (const uint16_t*)k_new;
  a.v_new = (const uint16_t*)v_new;
  // flush 1: the step's token fills the residual block, which this launch packs first (packed_len counts it,
  // res_len is 0); flush 2: ... which this launch attends in fp16 (res_len is 128) and packs as well
  a.flush_mode = flush == 1 ? kFlushFirst : flush == 2 ? kFlushAfter : kFlushNone;
  a.flush_blk = flush == 1 ? packed_len / kBlock - 1 : packed_len / kBlock;
  a.new_slot = k_new && flush != 1 ? res_len - 1 : -1;
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
  a.max_pages = a.num_pages = 0;
  a.step = 0;
  dim3 grid(num_splits + (flush == 2 ? 1 : 0), c->n_kv_heads * ((a.gq + 15) / 16), c->batch), block(256);
  const bool single = (a.nb + num_splits - 1) / num_splits <= kWaves;   // at most one block per wave
  launch_instance(c->format, a.gq, single, false, a, grid, block, st);
  return hipGetLastError();
}

hipError_t launch_decode_paged(const bd_paged_cache* c, const void* q, float softmax_scale, int num_splits,
                               float* part_o, float* part_ml, bool step, const void* k_new, const void* v_new,
                               void* out, hipStream_t st, bool lazy) {
  DecodeArgs a;
  a.step = step ? 1 : 0;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
  a.k_codes = (const uint32_t*)c->k_codes;
  a.v_codes = (const uint32_t*)c->v_codes;
  a.k_params = (const uint32_t*)c->k_params;
  a.v_params = (const uint32_t*)c->v_params;
  a.k_res = (const uint16_t*)c->k_res;
  a.v_res = (const uint16_t*)c->v_res;
  a.q = (const uint16_t*)q;
  a.k_new = (const uint16_t*)k_new;   // non-null: the step's token, which this launch appends itself
  a.v_new = (const uint16_t*)v_new;
  a.new_slot = -1;
  // lazy: a sequence whose residual this step's token fills is attended with its 128 fp16 rows, and one extra
  // workgroup per (sequence, KV head), blockIdx.x == 0, packs them into the sequence's next page
  a.flush_mode = lazy ? kFlushAfter : kFlushNone;
  a.flush_blk = 0;
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
  dim3 grid(num_splits + (lazy ? 1 : 0), c->n_kv_heads * ((a.gq + 15) / 16), c->batch), block(256);
  launch_instance(c->format, a.gq, false, true, a, grid, block, st);
  return hipGetLastError();
}

hipError_t launch_combine(const bd_cache* c, const float* part_o, const float* part_ml, int nparts, void* out,
                          hipStream_t st, const bd_paged_cache* step_of) {
  const int nrows = c->batch * c->n_q_heads;
  StepBump bump{};
  if (step_of) {
    bump.seq_lens = step_of->seq_lens;
    bump.block_table = step_of->block_table;
    bump.n_q_heads = step_of->n_q_heads;
    bump.max_pages = step_of->max_pages_per_seq;
    bump.num_pages = step_of->num_pages;
    bump.every_token = step_of->format == BD_FMT_MXFP4;
  }
  // thread groups per row: enough to request every partial in one round (8 per group), no more -- a launch of
  // 1024-thread workgroups costs about a microsecond more than one of 128-thread workgroups
  const int kind = out_kind(c->format, c->out_type);
#define BD_COMBINE(G) combine_kernel<G><<<dim3(nrows), dim3(128 * G), 0, st>>>(part_o, part_ml, nparts, nrows, out, kind, bump)
  if (nparts <= kCombineBatch) BD_COMBINE(1);
  else if (nparts <= 2 * kCombineBatch) BD_COMBINE(2);
  else if (nparts <= 4 * kCombineBatch) BD_COMBINE(4);
  else BD_COMBINE(kCombineGroups);
#undef BD_COMBINE
  return hipGetLastError();
}

}  // namespace bd
