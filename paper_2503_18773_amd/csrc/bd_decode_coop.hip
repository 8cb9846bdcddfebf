// Decode-step attention over the packed int4 / int2 cache for query groups of up to 4 heads
// (channel-wise K, contiguous cache): the four waves of a workgroup work on ONE 128-token block at
// a time and share its softmax -- the paper's layout of warps along the token axis with a
// cooperative softmax (Sec. III-B(1), III-B(2), Alg. 1; Sec. IV-C) -- instead of each wave owning a
// block of its own as in decode_int_kernel.  The chain a workgroup still has to run after its last
// bytes arrive is a quarter as long, which is what a 32K-token call (two blocks per SIMD) is bound by.
//
// Per block (matrix instruction and operand layouts as in bd_decode.hip):
//   QK^T    wave w scores tokens 32w .. 32w+31: two S^T tiles of 16 tokens, A = K codes (masked, fp16
//           subnormals), B = Q' = Q * scale as an fp16 high + low pair in alternating column groups.
//           Q' of the block is prepared by all four waves, a quarter of the channels each, in LDS.
//   softmax every lane ends up with 2 scores; the block maximum per head goes through LDS (one
//           barrier), so all waves use the same running maximum and P' of the whole block is on one
//           scale (Alg. 1 with the cross-warp reduction of Sec. III-B(2)).
//   P'      = p * scale_t (V is quantized per token) goes to LDS as fp16 in the B-operand order of
//           the second product (one barrier): the paper's sAcc round trip.
//   PV      wave w accumulates O^T for channels 32w .. 32w+31 over all 128 tokens: A = V codes.
//           Every wave owns its channels, so nothing is merged between waves at the end.
// Two barriers per block; Q' of the next block is prepared between them.
//
// Range: fp16 operands hold Q' and P' only after a power-of-two normalisation -- Q' by the exponent
// of the block's largest K scale, P' by a running exponent of the largest V scale seen (carried like
// the running maximum: the accumulators are rescaled when it grows) -- so the result does not depend
// on the magnitude of K and V.
#include "bd_common.h"
#include "bd_device.h"
#include "bd_fmt.h"

namespace bd {
namespace {

constexpr int kCoopWaves = 4;
constexpr float kLog2eC = 1.4426950408889634f;
constexpr int kRowPad = 8;          // fp16 elements of padding per LDS row (bank spread between heads)
constexpr int kPShift = 13;         // P' = p * scale * 2^(kPShift - E) < 2^14 for p <= 1

struct CoopArgs {
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const uint32_t* k_params;
  const uint32_t* v_params;
  const uint16_t* k_res;
  const uint16_t* v_res;
  const uint16_t* q;
  const uint16_t* k_new;   // fused step: the newest token, [B][Hkv][128], not yet in the residual buffers
  const uint16_t* v_new;
  int new_slot;            // its residual slot (res_len - 1), or -1
  float* part_o;           // [num_splits][B][Hq][128]
  float* part_ml;          // [num_splits][B][Hq][2]  (running max in log2 units, running sum)
  void* out;               // one split only: the output rows, written instead of the partials; else nullptr
  int out_kind;
  int n_q_heads, n_kv_heads, gq;
  int nb, nbcap, res_len, num_splits;
  float scale_log2;        // softmax_scale * log2(e)
};

// one block's loads of one lane
template <int WORDS>
struct BlockRegs {
  RawTile<WORDS> k[2];   // K rows of this wave's two S^T tiles
  RawTile<WORDS> v[2];   // V rows (channels) of this wave's two O^T tiles
  u2_t kpw;              // K parameters of channels 2 * lane, 2 * lane + 1 (for the block's largest scale)
  u2_t vpw;              // V parameters of tokens 2 * lane, 2 * lane + 1   (likewise)
  uint32_t kp[2];        // K parameters of the two channels whose Q' this lane prepares
  uint32_t vp[2];        // V parameters of the two tokens whose probabilities this lane computes
};

// largest of the fp16 bit patterns (non-negative values) in the low halves of x[0], x[1] over the wave
__device__ __forceinline__ uint32_t wave_max_half_bits(u2_t x) {
  uint32_t m = max(x[0] & 0xFFFFu, x[1] & 0xFFFFu);
  m = max(m, dpp_u<kQuadSwap1>(m));
  m = max(m, dpp_u<kQuadSwap2>(m));
  m = max(m, dpp_u<kRowHalfMirror>(m));
  m = max(m, dpp_u<kRowMirror>(m));
  const uint32_t a = __builtin_amdgcn_readlane(m, 0), b = __builtin_amdgcn_readlane(m, 16);
  const uint32_t c = __builtin_amdgcn_readlane(m, 32), d = __builtin_amdgcn_readlane(m, 48);
  return max(max(a, b), max(c, d));
}
// binary exponent of a positive fp16 given by its bits (subnormals and zero: -15)
__device__ __forceinline__ int half_exponent(uint32_t bits) { return (int)(bits >> 10) - 15; }
__device__ __forceinline__ float pow2i(int e) {   // 2^e, e in [-126, 127]
  return __uint_as_float((uint32_t)(e + 127) << 23);
}

template <int BITS>
__global__ __launch_bounds__(256, 2) void decode_coop_kernel(CoopArgs a) {
  using F = Fmt<BITS>;
  constexpr int WORDS = F::WORDS;
  constexpr int KROW = kD * BITS / 32;       // K words per token
  constexpr int VROW = kBlock * BITS / 32;   // V words per channel per block
  using Regs = BlockRegs<WORDS>;

  __shared__ __attribute__((aligned(16))) uint16_t q_hi[4][kD + kRowPad];   // Q' high piece, B-operand order
  __shared__ __attribute__((aligned(16))) uint16_t q_lo[4][kD + kRowPad];
  __shared__ __attribute__((aligned(16))) uint16_t p_s[4][kBlock + kRowPad];   // P' of the block, B-operand order
  __shared__ __attribute__((aligned(16))) uint16_t c_s[kBlock];   // centre code (times its position factor) of every token of the block, same order
  __shared__ __attribute__((aligned(16))) float zpart[4][kCoopWaves];   // per head: sum_c Q_c zero_c, by wave
  __shared__ __attribute__((aligned(16))) float smax[4][kCoopWaves];    // per head: largest raw score, by wave
  __shared__ __attribute__((aligned(16))) float red[2][4][kCoopWaves];  // epilogue: l, z sums per head, by wave
  __shared__ float res_s[kBlock][4];                                    // scores of this workgroup's residual tokens

  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, g = lane >> 4;
  const int head = col & 3, cg = col >> 2;
  const int gq = a.gq;
  const size_t unit = (size_t)b * a.n_kv_heads + hkv;
  const int nb = a.nb, res_len = a.res_len, new_slot = a.new_slot;
  // blocks of this workgroup: split, split + num_splits, ...
  const int cnt = nb > split ? (nb - split + a.num_splits - 1) / a.num_splits : 0;
  // this workgroup's slice of the fp16 residual tokens
  const int rt0 = (res_len * split) / a.num_splits, rt1 = (res_len * (split + 1)) / a.num_splits;
  const int nres = rt1 - rt0;
  const uint16_t* qbase = a.q + ((size_t)b * a.n_q_heads + (size_t)hkv * gq) * kD;

  // ---- what this lane does in each role
  // Q' preparation: head lane / 16, slot group 4 * wave + (lane / 4) % 4, entries 2i, 2i+1 (i = lane % 4):
  // the i-th channel of each of the slot group's two runs
  const int prep_head = lane >> 4, prep_sg = 4 * wave + ((lane >> 2) & 3), prep_i = lane & 3;
  const int prep_c0 = F::run_base(prep_sg, 0) + prep_i, prep_c1 = F::run_base(prep_sg, 1) + prep_i;
  // softmax: tile cg / 2 of this wave's two, rows 4g + 2 (cg % 2) + {0, 1}: operand entries e0, e0 + 1 of
  // the 8-token group (wave, g)
  const int my_tile = cg >> 1, e0 = 4 * my_tile + 2 * (cg & 1);
  const int tok0 = 32 * wave + F::tok_of_entry(g, e0), tok1 = 32 * wave + F::tok_of_entry(g, e0 + 1);
  const float un0 = F::un_entry(e0), un1 = F::un_entry(e0 + 1);
  const float iun0 = F::inv_un_entry(e0), iun1 = F::inv_un_entry(e0 + 1);

  // ---- loads of one block
  auto issue = [&](Regs& r, int k) {
    if (k >= cnt) return;
    const size_t bi = unit * a.nbcap + (size_t)(split + k * a.num_splits);
    const uint32_t* kp = a.k_params + bi * kD;
    const uint32_t* vp = a.v_params + bi * kBlock;
    r.kpw = *reinterpret_cast<const u2_t*>(kp + 2 * lane);
    r.kp[0] = kp[prep_c0];
    r.kp[1] = kp[prep_c1];
    r.vpw = *reinterpret_cast<const u2_t*>(vp + 2 * lane);
    r.vp[0] = vp[tok0];
    r.vp[1] = vp[tok1];
    const uint32_t* kc = a.k_codes + bi * (size_t)(kBlock * KROW) + WORDS * g;
#pragma unroll
    for (int T = 0; T < 2; ++T) {   // A-operand row `col` of tile T: token 32 wave + entry 4T + col % 4 of group col / 4
      const int tok = 32 * wave + F::tok_of_entry(col >> 2, 4 * T + (col & 3));
      r.k[T] = load_raw<WORDS>(kc + (size_t)tok * KROW);
    }
    const uint32_t* vc = a.v_codes + bi * (size_t)(kD * VROW) + WORDS * g;
#pragma unroll
    for (int T = 0; T < 2; ++T) r.v[T] = load_raw<WORDS>(vc + (size_t)(32 * wave + 16 * T + col) * VROW);
  };

  // The queries this lane rescales every block: head prep_head, channels prep_c0 / prep_c1.  Every head's
  // queries are first brought to the top of the fp16 range by a power of two of their own (a column of
  // the B operand may carry any factor: it comes out of that column's scores), so that the low pieces of
  // Q' keep their bits whatever the magnitudes of Q and of the K scales are: |q| * 2^kq < 2^13.
  uint32_t qbits = 0;
  if (prep_head < gq) {
    const u4_t qv = *reinterpret_cast<const u4_t*>(qbase + prep_head * kD + 8 * (lane & 15));
#pragma unroll
    for (int i = 0; i < 4; ++i) qbits = max(qbits, max(qv[i] & 0x7FFFu, (qv[i] >> 16) & 0x7FFFu));
  }
  qbits = max(qbits, dpp_u<kQuadSwap1>(qbits));
  qbits = max(qbits, dpp_u<kQuadSwap2>(qbits));
  qbits = max(qbits, dpp_u<kRowHalfMirror>(qbits));
  qbits = max(qbits, dpp_u<kRowMirror>(qbits));     // largest |q| of head lane / 16 (bit pattern)
  const int kq_prep = 12 - half_exponent(qbits);
  int kq_head = 12 - half_exponent(__builtin_amdgcn_readlane(qbits, 0));   // ... of this lane's column's head
  if (head == 1) kq_head = 12 - half_exponent(__builtin_amdgcn_readlane(qbits, 16));
  if (head == 2) kq_head = 12 - half_exponent(__builtin_amdgcn_readlane(qbits, 32));
  if (head == 3) kq_head = 12 - half_exponent(__builtin_amdgcn_readlane(qbits, 48));
  const float ks_head = a.scale_log2 * pow2i(24 - kq_head);   // raw score -> log2 units, but for the block's K exponent
  float qr0 = 0.f, qr1 = 0.f;
  if (prep_head < gq) {
    qr0 = h2f(qbase[prep_head * kD + prep_c0]);
    qr1 = h2f(qbase[prep_head * kD + prep_c1]);
  }
  const float qn0 = qr0 * pow2i(kq_prep) * F::un(prep_i), qn1 = qr1 * pow2i(kq_prep) * F::un(prep_i);

  // ---- residual tokens, part 1: the operands of the scores (16 tokens at a time on the matrix unit)
  const uint16_t* kres = a.k_res + unit * kBlock * kD;
  auto kres_row = [&](int t) { return t == new_slot ? a.k_new + unit * kD : kres + (size_t)t * kD; };
  auto vres_row = [&](int t) { return t == new_slot ? a.v_new + unit * kD : a.v_res + (unit * kBlock + t) * kD; };
  const int nres_groups = (nres + 15) >> 4;
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
  if (new_slot >= 0 && split == 0 && tid < 32) {   // fused step: file the new token for later steps
    const bool is_v = tid >= 16;
    const uint16_t* src = (is_v ? a.v_new : a.k_new) + unit * kD + 8 * (tid & 15);
    uint16_t* dst = const_cast<uint16_t*>(is_v ? a.v_res : a.k_res) + (unit * kBlock + new_slot) * kD + 8 * (tid & 15);
    *reinterpret_cast<u4_t*>(dst) = *reinterpret_cast<const u4_t*>(src);
  }

  Regs r0, r1, r2;
  issue(r0, 0);
  issue(r1, 1);

  // ---- residual tokens, part 2: scores s[t][h] = q_h . k_t * softmax_scale * log2(e)
  if (has_res) {
    for (int grp = wave; grp < nres_groups; grp += kCoopWaves) {
      if (grp != wave) load_res_keys(grp);
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(res_a[j], res_q[j], acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = 16 * grp + 4 * g + r;
        if (t < nres && col < 4) res_s[t][col] = acc[r] * a.scale_log2;
      }
    }
  }

  // ---- running state.  m_run is equal in all lanes of a head in every wave; l, z, x are sums over this
  // lane's own tokens; acc holds O^T of channels 32 wave + 16 T + 4 g + r (column = head) on the scale
  // 2^(kPShift - e_run - 24).
  // xacc = sum_t P'_t * centre code of token t, on the same scale, from the same chain of matrix
  // instructions as acc (so that whatever the unit's accumulation does to a long sum of positive terms,
  // it does to both, and their difference -- the signal, hundreds of times smaller -- keeps its bits).
  float m_run = -INFINITY, l_run = 0.f, z_run = 0.f;
  int e_run = -64;
  f4_t oacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  f4_t xacc = {0.f, 0.f, 0.f, 0.f};
  // Every kFlush blocks the difference moves to osum and both chains start again from zero: the two
  // sums grow with the number of tokens, the signal with its square root.
  constexpr int kFlush = 16;
  f4_t osum[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

  // Q' of a block from its parameters (in r): all four waves, a quarter of the channels each.  Returns the
  // exponent the block's K scales are normalised by (scale * 2^-ek < 1).
  auto prep = [&](const Regs& r) -> int {
    const int ek = half_exponent(wave_max_half_bits(r.kpw)) + 1;
    const float nrm = pow2i(-ek);
    const float s0 = h2f((uint16_t)(r.kp[0] & 0xFFFFu)) * nrm, s1 = h2f((uint16_t)(r.kp[1] & 0xFFFFu)) * nrm;
    const float z0 = h2f((uint16_t)(r.kp[0] >> 16)), z1 = h2f((uint16_t)(r.kp[1] >> 16));
    const float t0 = qn0 * s0, t1 = qn1 * s1;     // exact: 11-bit q times 11-bit scale times powers of two
    const uint16_t h0 = f2h(t0), h1 = f2h(t1);
    const uint16_t l0 = f2h(t0 - h2f(h0)), l1 = f2h(t1 - h2f(h1));
    // entries 2i (run 0) and 2i + 1 (run 1) of slot group prep_sg
    *reinterpret_cast<uint32_t*>(&q_hi[prep_head][8 * prep_sg + 2 * prep_i]) = (uint32_t)h0 | ((uint32_t)h1 << 16);
    *reinterpret_cast<uint32_t*>(&q_lo[prep_head][8 * prep_sg + 2 * prep_i]) = (uint32_t)l0 | ((uint32_t)l1 << 16);
    const float zs = row_sum16(__builtin_fmaf(qr0, z0, qr1 * z1));
    if ((lane & 15) == 0) zpart[prep_head][wave] = zs;
    return ek;
  };

  int ek_next = 0;
  if (cnt > 0) ek_next = prep(r0);
  __syncthreads();   // Q' of the first block (and the residual scores) are in LDS

  auto body = [&](Regs& cur, Regs& nxt, Regs& nxt2, int k) {
    issue(nxt2, k + 2);
    const int ek = ek_next;
    // ---- S^T = K Q'^T for this wave's 32 tokens
    h8_t bq[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      bq[j] = *reinterpret_cast<const h8_t*>(cg & 1 ? &q_lo[head][8 * (4 * g + j)] : &q_hi[head][8 * (4 * g + j)]);
    const f4_t zp = *reinterpret_cast<const f4_t*>(&zpart[head][0]);
    const float zq = ((zp[0] + zp[1]) + (zp[2] + zp[3])) * a.scale_log2;
    f4_t s[2];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(F::dequant(cur.k[T].w, j), bq[j], acc, 0, 0, 0);
      s[T] = acc;
    }
    // high + low partial products meet (even column groups hold the high piece's, odd the low piece's);
    // this lane keeps rows 2 (cg % 2) + {0, 1} of tile cg / 2
    float x0, x1;
    {
      const f4_t u = my_tile ? s[1] : s[0];
      const float a0 = u[0] + dpp_f<kRowShl4>(u[0]), a1 = u[1] + dpp_f<kRowShl4>(u[1]);
      const float b0 = u[2] + dpp_f<kRowShr4>(u[2]), b1 = u[3] + dpp_f<kRowShr4>(u[3]);
      x0 = cg & 1 ? b0 : a0;
      x1 = cg & 1 ? b1 : a1;
    }
    // ---- block maximum per head: over the column groups and lane groups of this wave, then over the waves
    float bm = fmaxf(x0, x1);
    bm = fmaxf(bm, dpp_f<kRowRor4>(bm));
    bm = fmaxf(bm, dpp_f<kRowRor8>(bm));
    bm = fmaxf(bm, __shfl_xor(bm, 16));
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    if (lane < 4) smax[lane][wave] = bm;
    // (meanwhile: this block's V parameters, which do not depend on the maximum)
    const int ev = half_exponent(wave_max_half_bits(cur.vpw));
    const int e_new = max(e_run, ev);
    const float sv0 = h2f((uint16_t)(cur.vp[0] & 0xFFFFu)), zv0 = h2f((uint16_t)(cur.vp[0] >> 16));
    const float sv1 = h2f((uint16_t)(cur.vp[1] & 0xFFFFu)), zv1 = h2f((uint16_t)(cur.vp[1] >> 16));
    // centre code of each token: the code of the value 0, so that what the matrix unit sums is small
    const float c0 = sv0 > 0.f ? rintf(fminf(fmaxf(-zv0 * __builtin_amdgcn_rcpf(sv0), 0.f), F::kQmax)) : 0.f;
    const float c1 = sv1 > 0.f ? rintf(fminf(fmaxf(-zv1 * __builtin_amdgcn_rcpf(sv1), 0.f), F::kQmax)) : 0.f;
    const float pnorm = pow2i(kPShift - e_new);
    const float px0 = sv0 * un0 * pnorm, px1 = sv1 * un1 * pnorm;          // P' = p * px
    const float py0 = __builtin_fmaf(c0, sv0, zv0), py1 = __builtin_fmaf(c1, sv1, zv1);   // value of the centre code
    const uint32_t cpair = (uint32_t)(c0 * iun0) | ((uint32_t)(c1 * iun1) << 16);
    __syncthreads();   // B2: every wave's maximum is in LDS (and every wave is done with Q' of this block)
    const f4_t sm = *reinterpret_cast<const f4_t*>(&smax[head][0]);
    const float bmax = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    const float kS = ks_head * pow2i(ek);   // raw score -> log2 units
    const float m_new = fmaxf(m_run, __builtin_fmaf(bmax, kS, zq));
    const float zoff = zq - m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);          // 0 on the first block
    const float alpha_o = alpha * pow2i(max(e_run - e_new, -126));
    m_run = m_new;
    e_run = e_new;
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x0, kS, zoff));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x1, kS, zoff));
    const uint16_t ph0 = f2h(p0 * px0), ph1 = f2h(p1 * px1);
    *reinterpret_cast<uint32_t*>(&p_s[head][32 * wave + 8 * g + e0]) = (uint32_t)ph0 | ((uint32_t)ph1 << 16);
    l_run = __builtin_fmaf(l_run, alpha, p0 + p1);
    z_run = __builtin_fmaf(z_run, alpha, __builtin_fmaf(p0, py0, p1 * py1));
    if (head == 0) *reinterpret_cast<uint32_t*>(&c_s[32 * wave + 8 * g + e0]) = cpair;
    if (__any(alpha_o != 1.0f)) {
      oacc[0] *= alpha_o;
      oacc[1] *= alpha_o;
      xacc *= alpha_o;
      osum[0] *= alpha_o;
      osum[1] *= alpha_o;
    }
    // Q' of the next block (every wave has read this block's since the barrier above)
    if (k + 1 < cnt) ek_next = prep(nxt);
    __syncthreads();   // B3: P' of the block and Q' of the next one are in LDS
    // ---- O^T += V^T P' for this wave's 32 channels
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const h8_t bp = *reinterpret_cast<const h8_t*>(&p_s[head][32 * g + 8 * j]);
      xacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const h8_t*>(&c_s[32 * g + 8 * j]), bp, xacc, 0, 0, 0);
#pragma unroll
      for (int T = 0; T < 2; ++T)
        oacc[T] = __builtin_amdgcn_mfma_f32_16x16x32_f16(F::dequant(cur.v[T].w, j), bp, oacc[T], 0, 0, 0);
    }
    if ((k % kFlush) == kFlush - 1) {
#pragma unroll
      for (int T = 0; T < 2; ++T) {
        osum[T] += oacc[T] - xacc[0];
        oacc[T] = (f4_t){0.f, 0.f, 0.f, 0.f};
      }
      xacc = (f4_t){0.f, 0.f, 0.f, 0.f};
    }
  };

  for (int k = 0; k < cnt; k += 3) {
    body(r0, r1, r2, k);
    if (k + 1 < cnt) body(r1, r2, r0, k + 1);
    if (k + 2 < cnt) body(r2, r0, r1, k + 2);
  }

  // ---- epilogue: the sums over the lanes of each head, the residual tokens, the partial result
  l_run += dpp_f<kRowRor4>(l_run);  l_run += dpp_f<kRowRor8>(l_run);
  z_run += dpp_f<kRowRor4>(z_run);  z_run += dpp_f<kRowRor8>(z_run);
  l_run += __shfl_xor(l_run, 16);   l_run += __shfl_xor(l_run, 32);
  z_run += __shfl_xor(z_run, 16);   z_run += __shfl_xor(z_run, 32);
  __syncthreads();   // (the last block's LDS reads are done; red is free)
  if (lane < 4) {
    red[0][lane][wave] = l_run;
    red[1][lane][wave] = z_run;
  }
  __syncthreads();
  if (col < 4) {   // column = head
    const f4_t rl = *reinterpret_cast<const f4_t*>(&red[0][col][0]);
    const f4_t rz = *reinterpret_cast<const f4_t*>(&red[1][col][0]);
    float L = (rl[0] + rl[1]) + (rl[2] + rl[3]);
    const float Z = (rz[0] + rz[1]) + (rz[2] + rz[3]);
    float M = m_run;
    // O of this lane's 8 channels, true scale: (acc - xacc) * 2^(24 + e_run - kPShift) + Z
    const float back = cnt > 0 ? pow2i(24 + max(e_run - kPShift, -126)) : 0.f;
    float o[2][4];
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int r = 0; r < 4; ++r) o[T][r] = __builtin_fmaf(osum[T][r] + (oacc[T][r] - xacc[0]), back, Z);
    // the fp16 residual tokens of this workgroup's slice
    if (nres > 0) {
      float M2 = M;
      for (int t = 0; t < nres; ++t) M2 = fmaxf(M2, res_s[t][col]);
      const float f = __builtin_amdgcn_exp2f(M - M2);   // 0 when there were no packed blocks
      L *= f;
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[T][r] *= f;
      M = M2;
      for (int t = 0; t < nres; ++t) {
        const float p = __builtin_amdgcn_exp2f(res_s[t][col] - M);
        L += p;
        const uint16_t* vr = vres_row(rt0 + t) + 32 * wave + 4 * g;
#pragma unroll
        for (int T = 0; T < 2; ++T) {
          const u2_t raw = *reinterpret_cast<const u2_t*>(vr + 16 * T);
          o[T][0] = __builtin_fmaf(p, h2f((uint16_t)(raw[0] & 0xFFFFu)), o[T][0]);
          o[T][1] = __builtin_fmaf(p, h2f((uint16_t)(raw[0] >> 16)), o[T][1]);
          o[T][2] = __builtin_fmaf(p, h2f((uint16_t)(raw[1] & 0xFFFFu)), o[T][2]);
          o[T][3] = __builtin_fmaf(p, h2f((uint16_t)(raw[1] >> 16)), o[T][3]);
        }
      }
    }
    if (col < gq) {
      const size_t row = ((size_t)split * gridDim.z + b) * a.n_q_heads + (size_t)hkv * gq + col;
#pragma unroll
      for (int T = 0; T < 2; ++T) {
        const int c0ch = 32 * wave + 16 * T + 4 * g;
        if (a.out) {   // one split: row == the output row
          store_final_pair(a.out, row * kD + c0ch, a.out_kind, o[T][0], o[T][1], L);
          store_final_pair(a.out, row * kD + c0ch + 2, a.out_kind, o[T][2], o[T][3], L);
        } else {
          *reinterpret_cast<f4_t*>(a.part_o + row * kD + c0ch) = (f4_t){o[T][0], o[T][1], o[T][2], o[T][3]};
        }
      }
      if (!a.out && wave == 0 && g == 0) {
        a.part_ml[row * 2] = M;
        a.part_ml[row * 2 + 1] = L;
      }
    }
  }
}

}  // namespace

bool decode_coop_takes(const bd_cache* c) {
  return (c->format == BD_FMT_INT4 || c->format == BD_FMT_INT2) && c->n_q_heads / c->n_kv_heads <= 4;
}

hipError_t launch_decode_coop(const bd_cache* c, const void* q, int packed_len, int res_len, float softmax_scale,
                              int num_splits, float* part_o, float* part_ml, const void* k_new, const void* v_new,
                              void* out, hipStream_t st) {
  CoopArgs a;
  a.k_codes = (const uint32_t*)c->k_codes;
  a.v_codes = (const uint32_t*)c->v_codes;
  a.k_params = (const uint32_t*)c->k_params;
  a.v_params = (const uint32_t*)c->v_params;
  a.k_res = (const uint16_t*)c->k_res;
  a.v_res = (const uint16_t*)c->v_res;
  a.q = (const uint16_t*)q;
  a.k_new = (const uint16_t*)k_new;
  a.v_new = (const uint16_t*)v_new;
  a.new_slot = k_new ? res_len - 1 : -1;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.out = num_splits == 1 ? out : nullptr;
  a.out_kind = out_kind(c->format, c->out_type);
  a.n_q_heads = c->n_q_heads;
  a.n_kv_heads = c->n_kv_heads;
  a.gq = c->n_q_heads / c->n_kv_heads;
  a.nb = packed_len / kBlock;
  a.nbcap = c->capacity / kBlock;
  a.res_len = res_len;
  a.num_splits = num_splits;
  a.scale_log2 = softmax_scale * kLog2eC;
  dim3 grid(num_splits, c->n_kv_heads, c->batch), block(256);
  if (c->format == BD_FMT_INT4) decode_coop_kernel<4><<<grid, block, 0, st>>>(a);
  else decode_coop_kernel<2><<<grid, block, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace bd
