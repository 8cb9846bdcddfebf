// Bit layouts of the packed int4 / int2 codes as matrix-instruction operands (gfx950), shared by
// the decode kernels.
#pragma once

#include "bd_common.h"
#include "bd_device.h"

namespace bd {
namespace {

// ---- format traits ---------------------------------------------------------------------
// One lane loads WORDS 32-bit words (32 codes) per 16-row tile.  k-step j (of 4) of the tile
// consumes 8 codes as 4 VGPRs; VGPR v holds two codes that arrive multiplied by 1/un(v).
// The B operand must present the other factor in the same order: "slot group" sg = 4*g + j
// (g = lane/16) holds 8 entries, entry e = 2*i + run for the i-th channel of one of two runs
// of 4 consecutive channels.
template <int BITS>
struct Fmt;

template <>
struct Fmt<4> {
  static constexpr int WORDS = 4;
  static constexpr float kQmax = 15.0f;
  // first channel of run `run` (0/1) of slot group sg: word sg, nibbles 0..3 / 4..7
  __device__ static int run_base(int sg, int run) { return 8 * sg + 4 * run; }
  __device__ static constexpr float un(int v) { return (v & 1) ? (1.0f / 16.0f) : 1.0f; }
  __device__ static constexpr float inv_un(int v) { return (v & 1) ? 16.0f : 1.0f; }
  // k-step j = 2*half + jj of the second product contracts the tokens of two S^T tiles of that
  // half: tile_lo(jj) fills the low fp16 half of the P' registers, tile_hi(jj) the high one
  __device__ static constexpr int tile_lo(int jj) { return 2 * jj; }
  __device__ static constexpr int tile_hi(int jj) { return 2 * jj + 1; }
  // groups of up to 4 heads (column group c/4 keeps tiles c/4 and 4 + c/4): kPairShift brings the
  // column group whose tile fills the high half of a P' register next to the one that fills the
  // low half; kStepShift brings the second k-step of a pair to columns 0..3
  static constexpr int kPairShift = kRowShl4, kStepShift = kRowShl8;
  // position of block token t in the k-ordered P' / V operand: lane group t/32, then k-step j,
  // register r, half -- tile T = (t%32)/4 feeds k-step T/2, half T%2
  __device__ static int p_slot(int t) {
    const int T = (t & 31) >> 2, r = t & 3;
    return (t & ~31) + 8 * (T >> 1) + 2 * r + (T & 1);
  }
  // position (8 * slot group + entry) of channel / block token t in that operand order
  __device__ static int operand_pos(int t) { return (t & ~7) + 2 * (t & 3) + ((t >> 2) & 1); }
  __device__ static h8_t dequant(const uint32_t* w, int j) {
    const uint32_t x = w[j], y = x >> 8;
    u4_t r;
    r[0] = x & 0x000F000Fu;   // nibbles 0, 4
    r[1] = x & 0x00F000F0u;   // nibbles 1, 5 (x16)
    r[2] = y & 0x000F000Fu;   // nibbles 2, 6
    r[3] = y & 0x00F000F0u;   // nibbles 3, 7 (x16)
    return __builtin_bit_cast(h8_t, r);
  }
};

template <>
struct Fmt<2> {
  static constexpr int WORDS = 2;
  static constexpr float kQmax = 3.0f;
  // slot group sg = 2*W + jj: word W, crumbs 4*jj + 0..3 (run 0) and 8 + 4*jj + 0..3 (run 1)
  __device__ static int run_base(int sg, int run) { return 16 * (sg >> 1) + 4 * (sg & 1) + 8 * run; }
  __device__ static constexpr float un(int v) { return 1.0f / (float)(1 << (2 * v)); }
  __device__ static constexpr float inv_un(int v) { return (float)(1 << (2 * v)); }
  __device__ static constexpr int tile_lo(int jj) { return jj; }
  __device__ static constexpr int tile_hi(int jj) { return jj + 2; }
  static constexpr int kPairShift = kRowShl8, kStepShift = kRowShl4;
  // tile T = (t%32)/4 feeds k-step 2*(T/4) + T%2, half (T%4)/2
  __device__ static int p_slot(int t) {
    const int T = (t & 31) >> 2, r = t & 3;
    return (t & ~31) + 8 * (2 * (T >> 2) + (T & 1)) + 2 * r + ((T & 3) >> 1);
  }
  __device__ static int operand_pos(int t) {
    return 8 * (2 * (t >> 4) + ((t >> 2) & 1)) + 2 * (t & 3) + ((t >> 3) & 1);
  }
  __device__ static h8_t dequant(const uint32_t* w, int j) {
    const uint32_t x = (j & 1) ? (w[j >> 1] >> 8) : w[j >> 1];
    u4_t r;
    r[0] = x & 0x00030003u;   // crumbs 0, 8      (of the selected byte pair)
    r[1] = x & 0x000C000Cu;   // crumbs 1, 9  (x4)
    r[2] = x & 0x00300030u;   // crumbs 2, 10 (x16)
    r[3] = x & 0x00C000C0u;   // crumbs 3, 11 (x64)
    return __builtin_bit_cast(h8_t, r);
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

}  // namespace
}  // namespace bd
