// Device code shared by the product kernels: code-pair extraction for tiles of
// 256 codes held in registers, the register image of a tile and its loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqr_device.h"

namespace spqr {

// ---------------------------------------------------------------------------
// Pair extraction for 256-code tiles held in registers.
// Returns the bit pattern of two binary16 numbers (1 + q_lo/2^W, 1 + q_hi/2^W):
// one shift puts the two codes on the top mantissa bits of each half-word, one
// v_and_or_b32 masks them and sets the exponent of 1.0.
// ---------------------------------------------------------------------------
struct PairConsts {
  uint32_t mask;     // SGPR: code bits inside both half-words
  uint32_t magic;    // VGPR: 0x3C003C00, binary16 1.0 twice
  uint32_t m0, m1, m2;   // SGPR: single-bit masks of the split pair of a 3-bit triple
};

// Keeps a constant in a scalar / vector register: gfx9 VOP3 encodings take no
// literal and only one scalar operand, so v_and_or_b32 needs (vgpr, sgpr, vgpr).
__device__ __forceinline__ uint32_t in_sgpr(uint32_t v) { asm volatile("" : "+s"(v)); return v; }
__device__ __forceinline__ uint32_t in_vgpr(uint32_t v) { asm volatile("" : "+v"(v)); return v; }

template <int W>
__device__ __forceinline__ PairConsts make_pair_consts() {
  PairConsts k;
  k.mask = in_sgpr(W == 4 ? 0x03C003C0u : 0x03800380u);
  k.magic = in_vgpr(0x3C003C00u);
  k.m0 = in_sgpr(0x00800080u); k.m1 = in_sgpr(0x01000100u); k.m2 = in_sgpr(0x02000200u);
  return k;
}

template <int W>
__device__ __forceinline__ uint32_t pair_f16(const uint32_t* c, int q, const PairConsts& k) {
  if constexpr (W == 4) {
    const uint32_t d = c[q >> 2];
    const int o = 4 * (q & 3);                       // code offset inside each half-word
    const uint32_t t = o < 6 ? (d << (6 - o)) : (d >> (o - 6));
    return (t & k.mask) | k.magic;                   // mantissa bits 9..6
  } else {
    const int t3 = q >> 4, e = q & 15;
    if (e < 15) {
      const uint32_t d = c[3 * t3 + e / 5];
      const int o = 3 * (e % 5);
      const uint32_t t = o < 7 ? (d << (7 - o)) : (d >> (o - 7));
      return (t & k.mask) | k.magic;                 // mantissa bits 9..7
    } else {
      const uint32_t d0 = c[3 * t3], d1 = c[3 * t3 + 1], d2 = c[3 * t3 + 2];
      uint32_t t = ((d0 >> 8) & k.m0) | k.magic;
      t = ((d1 >> 7) & k.m1) | t;
      t = ((d2 >> 6) & k.m2) | t;
      return t;
    }
  }
}

// ---------------------------------------------------------------------------
// Code pairs of the dense loop: one shift serves several pairs.
// A code sitting at bit o <= 6 (3-bit) / o <= 4 (4-bit) of its half-word is already
// inside the binary16 mantissa: masking it in place and OR-ing an exponent gives
//   K + q/2^W   with K = 2^(7-o) (3-bit: 128, 16, 2)  resp. 2^(6-o) (4-bit: 64, 4),
// exactly representable, so only the codes in the upper bits of a half-word need
// a shift, and one shift of the dword (by 9 resp. 8) brings all of them down at
// once.  The price is an offset K that depends on the code's position ("class");
// it is removed per tile with the class sums of the activations (see tile_fma).
//   3-bit: pair e of a triple (e < 15) is code e%5 of dword e/5: codes 0,1,2 are
//          classes 0,1,2, codes 3,4 (after >> 9) classes 0,1; the split pair e = 15
//          is assembled at class 2.
//   4-bit: pair q%4 of a dword: 0,1 are classes 0,1; 2,3 (after >> 8) classes 0,1.
// ---------------------------------------------------------------------------
// SHARED = false keeps one class with K = 1 and a shift per pair (not used by any instance now: tiles of 8 columns,
// 32 accumulators per lane, take the class bookkeeping too since they are built for the larger register budget).
template <int W, bool SHARED> struct CodeClass {
  static constexpr int N = !SHARED ? 1 : (W == 3 ? 3 : 2);
  static constexpr int of_pair(int q) {           // q: pair index inside the tile
    if (!SHARED) return 0;
    if (W == 4) return (q & 3) & 1;
    const int e = q & 15;
    return e == 15 ? 2 : (e % 5) % 3;
  }
  static constexpr float K(int c) {
    return !SHARED ? 1.f : (W == 3 ? (c == 0 ? 128.f : c == 1 ? 16.f : 2.f) : (c == 0 ? 64.f : 4.f));
  }
};
template <int TC> struct SharedShifts { static constexpr bool value = true; };

struct ClassConsts {
  uint32_t mask[3];    // SGPR: code bits of class c inside both half-words
  uint32_t magic[3];   // VGPR: binary16 K(c) twice
  uint32_t m0, m1, m2; // SGPR: single-bit masks of the split pair of a 3-bit triple
};

template <int W>
__device__ __forceinline__ ClassConsts make_class_consts() {
  ClassConsts k;
  if constexpr (W == 3) {
    k.mask[0] = in_sgpr(0x00070007u); k.mask[1] = in_sgpr(0x00380038u); k.mask[2] = in_sgpr(0x01C001C0u);
    k.magic[0] = in_vgpr(0x58005800u); k.magic[1] = in_vgpr(0x4C004C00u); k.magic[2] = in_vgpr(0x40004000u);
    k.m0 = in_sgpr(0x00400040u); k.m1 = in_sgpr(0x00800080u); k.m2 = in_sgpr(0x01000100u);
  } else {
    k.mask[0] = in_sgpr(0x000F000Fu); k.mask[1] = in_sgpr(0x00F000F0u); k.mask[2] = 0;
    k.magic[0] = in_vgpr(0x54005400u); k.magic[1] = in_vgpr(0x44004400u); k.magic[2] = 0;
    k.m0 = k.m1 = k.m2 = 0;
  }
  return k;
}

// The shifted copies of the dwords that hold pair q; refreshed when q enters a
// new triple (3-bit) or dword (4-bit).  All indices are compile-time constants in
// the unrolled loops, so this is three (one) shifts per 16 (4) pairs.
template <int W> struct ShiftedWords { uint32_t s[W == 3 ? 3 : 1]; };

template <int W>
__device__ __forceinline__ void refresh_shifted(ShiftedWords<W>& sw, const uint32_t* c, int q) {
  if constexpr (W == 3) {
    if ((q & 15) == 0) {
      const int t3 = q >> 4;
      sw.s[0] = c[3 * t3] >> 9; sw.s[1] = c[3 * t3 + 1] >> 9; sw.s[2] = c[3 * t3 + 2] >> 9;
    }
  } else {
    if ((q & 3) == 0) sw.s[0] = c[q >> 2] >> 8;
  }
}

// binary16 pair (K + q_lo/2^W, K + q_hi/2^W), K = CodeClass<W>::K(of_pair(q))
template <int W>
__device__ __forceinline__ uint32_t pair_class_f16(const uint32_t* c, const ShiftedWords<W>& sw, int q,
                                                   const ClassConsts& k) {
  if constexpr (W == 4) {
    const int e = q & 3;
    const uint32_t src = e < 2 ? c[q >> 2] : sw.s[0];
    return (src & k.mask[e & 1]) | k.magic[e & 1];
  } else {
    const int t3 = q >> 4, e = q & 15;
    if (e < 15) {
      const int j = e / 5, i = e % 5;
      const uint32_t src = i < 3 ? c[3 * t3 + j] : sw.s[j];
      return (src & k.mask[i % 3]) | k.magic[i % 3];
    } else {                                         // bits 15 / 31 of the three dwords -> bits 6, 7, 8
      uint32_t t = (sw.s[0] & k.m0) | k.magic[2];
      t = ((c[3 * t3 + 1] >> 8) & k.m1) | t;
      t = ((c[3 * t3 + 2] >> 7) & k.m2) | t;
      return t;
    }
  }
}

// The same with the shifts written out (no state carried between pairs; the compiler shares a shifted
// dword between the pairs that are extracted next to each other).
template <int W>
__device__ __forceinline__ uint32_t pair_class_inline(const uint32_t* c, int q, const ClassConsts& k) {
  if constexpr (W == 4) {
    const int e = q & 3;
    const uint32_t d = c[q >> 2], src = e < 2 ? d : (d >> 8);
    return (src & k.mask[e & 1]) | k.magic[e & 1];
  } else {
    const int t3 = q >> 4, e = q & 15;
    if (e < 15) {
      const int j = e / 5, i = e % 5;
      const uint32_t d = c[3 * t3 + j], src = i < 3 ? d : (d >> 9);
      return (src & k.mask[i % 3]) | k.magic[i % 3];
    } else {                                         // bits 15 / 31 of the three dwords -> bits 6, 7, 8
      uint32_t t = ((c[3 * t3] >> 9) & k.m0) | k.magic[2];
      t = ((c[3 * t3 + 1] >> 8) & k.m1) | t;
      t = ((c[3 * t3 + 2] >> 7) & k.m2) | t;
      return t;
    }
  }
}

// ---------------------------------------------------------------------------
// Fused GEMV for tiles of 256 codes (and of 8 x 64 codes, group_axis 1).
//   W     code width (3, 4)
//   TR,TC tile rows / columns, TR*TC == 256 (512)
//   AXIS  0: groups are tile rows (beta2 = TR), 1: groups are tile columns (beta2 = TC)
// Grid: one workgroup per strip of TR rows; blockDim.x = 64 * (waves per workgroup).
// Dynamic LDS: n binary16 values of x (rounded up to 16 bytes).
// ---------------------------------------------------------------------------
//   LV    statistic layout: 1 bilevel, 2 integer zero-point, 3 binary16 statistics per group
template <int W, int TR, int TC, int AXIS, int LV = 1>
struct TileRegs {
  static constexpr int KW = TR * TC * W / 128;
  static constexpr int B2 = AXIS == 0 ? TR : TC;
  static constexpr int NC = 3 * B2 / 16;     // dwords of 3-bit statistic codes (layouts 1 and 2)
  static constexpr int SD = LV == 3 ? B2 : NC + (LV == 2 ? 1 : 2);
  static constexpr int SWF = SD / 4, SR = SD % 4;
  uint32_t c[4 * KW];
  uint32_t s[SD];
};

// STREAM: the tile is read once and not again soon (batch 1): load it past the
// caches' retention (nontemporal).  Batches above 4 come back for the same tiles
// one slice of vectors later and find them in the last-level cache otherwise.
template <bool STREAM, typename V>
__device__ __forceinline__ V load_once(const V* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(p);
  else return *p;
}

template <bool STREAM, int W, int TR, int TC, int AXIS, int LV>
__device__ __forceinline__ void load_tile(TileRegs<W, TR, TC, AXIS, LV>& t, const uint8_t* blk,
                                          int L, int lane) {
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  // statistics first: the tile's work starts with them (loads complete in order)
  const uint8_t* sb = blk + (int64_t)16 * T::KW * L;
#pragma unroll
  for (int k = 0; k < T::SWF; ++k) {
    u32x4 v = load_once<STREAM>(reinterpret_cast<const u32x4*>(sb + ((int64_t)k * L + lane) * 16));
    t.s[4 * k] = v.x; t.s[4 * k + 1] = v.y; t.s[4 * k + 2] = v.z; t.s[4 * k + 3] = v.w;
  }
  const uint8_t* rb = sb + (int64_t)16 * T::SWF * L;
#pragma unroll
  for (int k = 0; k < T::SR; ++k)
    t.s[4 * T::SWF + k] = load_once<STREAM>(reinterpret_cast<const uint32_t*>(rb + ((int64_t)k * L + lane) * 4));
#pragma unroll
  for (int k = 0; k < T::KW; ++k) {
    u32x4 v = load_once<STREAM>(reinterpret_cast<const u32x4*>(blk + ((int64_t)k * L + lane) * 16));
    t.c[4 * k] = v.x; t.c[4 * k + 1] = v.y; t.c[4 * k + 2] = v.z; t.c[4 * k + 3] = v.w;
  }
}

}  // namespace spqr
