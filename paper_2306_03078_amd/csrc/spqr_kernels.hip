// HIP kernels for gfx950: fused SpQR decode + matvec, debug decode, validation.
//
// Hot path (Sec. 4.2 "Inference with SpQR", re-designed for CDNA4):
//   one workgroup owns one strip of tile_rows output rows; its wavefronts split
//   the input dimension in steps of 64 tiles; one lane owns one whole tile per
//   step, so every load instruction of a wavefront reads one contiguous run of
//   the packed buffer (16 bytes per lane) and a tile's statistics are decoded
//   once and reused by all of its rows.  x is staged once per workgroup in LDS
//   (it also serves the outlier gather).  Codes are turned into binary16 values
//   1 + q/2^b by one shift and one and-or per pair and multiplied with
//   v_dot2_f32_f16 (fp32 accumulation); the offset "1 +" is removed per tile.
//   The strip's outliers (a contiguous CSR range) are handled by the same
//   workgroup, so y is written once, without atomics, in a fixed order.
#include <hip/hip_runtime.h>
#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <queue>
#include <vector>
#include <type_traits>

#include <algorithm>

#include "../../include/spqr.h"
#include "spqr_device.h"
#include "spqr_kernels.h"

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
// SHARED = false (tiles of 8 columns: 32 accumulators leave no registers for the class
// bookkeeping) keeps one class with K = 1 and a shift per pair.
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
template <int TC> struct SharedShifts { static constexpr bool value = TC != 8; };

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
// Fused GEMV for tiles of 256 codes.
//   W     code width (3, 4)
//   TR,TC tile rows / columns, TR*TC == 256
//   AXIS  0: groups are tile rows (beta2 = TR), 1: groups are tile columns (beta2 = TC)
// Grid: one workgroup per strip of TR rows; blockDim.x = 64 * (waves per workgroup).
// Dynamic LDS: n binary16 values of x (rounded up to 16 bytes).
// ---------------------------------------------------------------------------
template <int W, int TR, int TC, int AXIS>
struct TileRegs {
  static constexpr int KW = 256 * W / 128;
  static constexpr int B2 = AXIS == 0 ? TR : TC;
  static constexpr int SD = 3 * B2 / 16 + 2;
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

template <bool STREAM, int W, int TR, int TC, int AXIS>
__device__ __forceinline__ void load_tile(TileRegs<W, TR, TC, AXIS>& t, const uint8_t* blk,
                                          int L, int lane) {
  using T = TileRegs<W, TR, TC, AXIS>;
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

// Row phases: the class of the pair in tile row r, column pair p depends on
// (r*PPR + p) % 16 for 3-bit codes, so rows repeat with period 16/PPR; 4-bit
// classes depend on p alone.
template <int W, int TC> struct RowPhases {
  static constexpr int N = (W == 4 || TC / 2 >= 16 || !SharedShifts<TC>::value) ? 1 : 16 / (TC / 2);
};

// One tile's contribution for NB activation vectors (LDS rows of `xstride`
// dwords).  Codes enter the dot products as K + q/2^W (K by class, see above) and
// the statistic codes as 1 + s_q/8, 1 + z_q/8 (exact binary16 values); the offsets
// are removed with per-tile sums.  acc[b][r] accumulates, per output row r and
// vector b:
//   AXIS 1: sum_j (K_rj + q_rj/2^W) * u_j  with u_j = fp16(s_hat_j * x_j);
//           csum[b][h] accumulates, for the rows of phase h, sum_j (2^W*K_rj + z_hat_j) * u_j,
//           so y_r = 2^W*acc[r] - csum[r % phases].
//   AXIS 0: s_hat_r * (2^W * sum_j (K_rj + q_rj/2^W) x_j - sum_j (2^W*K_rj + z_hat_r) x_j).
// The sums of K_rj*u_j come from one dot product per pair, phase and vector into
// per-class sums.  A pair is extracted once and used by all NB vectors.  `valid`
// false: the lane adds exact zeros (every scale is forced to 0), so no branch
// surrounds the tile.
template <int W, int TR, int TC, int AXIS, int NB>
__device__ __forceinline__ void tile_fma(const TileRegs<W, TR, TC, AXIS>& t,
                                         const uint32_t* xpair /* TC/2 dwords in LDS, vector 0 */,
                                         int xstride, bool valid, float (&acc)[NB][TR],
                                         float (&csum)[NB][RowPhases<W, TC>::N], const ClassConsts& k,
                                         const PairConsts& k1, const PairConsts& k3) {
  using T = TileRegs<W, TR, TC, AXIS>;
  constexpr bool SHARED = SharedShifts<TC>::value;
  using CC = CodeClass<W, SHARED>;
  constexpr int PPR = TC / 2;
  constexpr int NPH = RowPhases<W, TC>::N;
  constexpr float SCALE = (float)(1 << W);
  const half2_t ones = as_half2(k3.magic);
  const uint32_t a = t.s[T::SD - 2], b = t.s[T::SD - 1];
  const float s_s = h2f((uint16_t)(a & 0xFFFF)), z_s = h2f((uint16_t)(a >> 16));
  const float s_z = h2f((uint16_t)(b & 0xFFFF)), z_z = h2f((uint16_t)(b >> 16));
  // s_hat = s_s*(s_q - z_s) = c1*(1 + s_q/8) + c2.  A lane without a tile of its own
  // (it holds a copy of the block's last tile) runs the same code with s_hat = 0.
  const float c1 = valid ? 8.f * s_s : 0.f, c2 = valid ? -s_s * z_s - 8.f * s_s : 0.f;
  // z_hat = s_z*(z_q - z_z) = e1*(1 + z_q/8) + e2
  const float e1 = 8.f * s_z, e2 = -s_z * z_z - e1;

  uint32_t xp[NB][PPR];
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
#pragma unroll
    for (int p = 0; p < PPR; p += 4) {
      u32x4 v = *reinterpret_cast<const u32x4*>(xpair + bi * xstride + p);
      xp[bi][p] = v.x; xp[bi][p + 1] = v.y; xp[bi][p + 2] = v.z; xp[bi][p + 3] = v.w;
    }
  }

  float C[NB][NPH][CC::N];                     // per phase and class: sum of the activations it multiplies
#pragma unroll
  for (int bi = 0; bi < NB; ++bi)
#pragma unroll
    for (int h = 0; h < NPH; ++h)
#pragma unroll
      for (int c = 0; c < CC::N; ++c) C[bi][h][c] = 0.f;
  ShiftedWords<W> sw;

  if constexpr (AXIS == 1) {
    float Zd[NB];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) Zd[bi] = 0.f;
#pragma unroll
    for (int p = 0; p < PPR; ++p) {
      const half2_t sq = as_half2(pair_f16<3>(t.s, p, k3));
      const half2_t zq = as_half2(pair_f16<3>(t.s, T::B2 / 2 + p, k3));
      const float s0 = fmaf((float)sq.x, c1, c2), s1 = fmaf((float)sq.y, c1, c2);
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const half2_t xv = as_half2(xp[bi][p]);
        half2_t u;
        u.x = (_Float16)fmaf(s0, (float)xv.x, 0.f);   // binary16 source widened inside the multiply, one rounding
        u.y = (_Float16)fmaf(s1, (float)xv.y, 0.f);
        xp[bi][p] = __builtin_bit_cast(uint32_t, u);   // x is not needed any more: keep u in its place
#pragma unroll
        for (int h = 0; h < NPH; ++h) {
          const int c = CC::of_pair(h * PPR + p);
          C[bi][h][c] = __builtin_amdgcn_fdot2(u, ones, C[bi][h][c], false);
        }
        Zd[bi] = __builtin_amdgcn_fdot2(u, zq, Zd[bi], false);
      }
    }
    // sum_j z_hat_j u_j = e1*Zd + e2*U;  sum_j 2^W*K_rj u_j = 2^W * sum_c K(c) * C[h][c]
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
      float U = C[bi][0][0];
#pragma unroll
      for (int c = 1; c < CC::N; ++c) U += C[bi][0][c];
      const float zu = fmaf(e1, Zd[bi], e2 * U);
#pragma unroll
      for (int h = 0; h < NPH; ++h) {
        float E = CC::K(0) * C[bi][h][0];
#pragma unroll
        for (int c = 1; c < CC::N; ++c) E = fmaf(CC::K(c), C[bi][h][c], E);
        csum[bi][h] += fmaf(SCALE, E, zu);
      }
    }
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      float d[NB];
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) d[bi] = acc[bi][r];
#pragma unroll
      for (int p = 0; p < PPR; ++p) {
        if constexpr (SHARED) refresh_shifted<W>(sw, t.c, r * PPR + p);
        const half2_t q2 = as_half2(SHARED ? pair_class_f16<W>(t.c, sw, r * PPR + p, k) : pair_f16<W>(t.c, r * PPR + p, k1));
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) d[bi] = __builtin_amdgcn_fdot2(q2, as_half2(xp[bi][p]), d[bi], false);
      }
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) acc[bi][r] = d[bi];
    }
  } else {
    float X[NB], SE[NB][NPH];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
#pragma unroll
      for (int p = 0; p < PPR; ++p) {
#pragma unroll
        for (int h = 0; h < NPH; ++h) {
          const int c = CC::of_pair(h * PPR + p);
          C[bi][h][c] = __builtin_amdgcn_fdot2(as_half2(xp[bi][p]), ones, C[bi][h][c], false);
        }
      }
      X[bi] = C[bi][0][0];
#pragma unroll
      for (int c = 1; c < CC::N; ++c) X[bi] += C[bi][0][c];
#pragma unroll
      for (int h = 0; h < NPH; ++h) {
        float E = CC::K(0) * C[bi][h][0];
#pragma unroll
        for (int c = 1; c < CC::N; ++c) E = fmaf(CC::K(c), C[bi][h][c], E);
        SE[bi][h] = SCALE * E;
      }
    }
#pragma unroll
    for (int r2 = 0; r2 < TR / 2; ++r2) {
      const half2_t sq = as_half2(pair_f16<3>(t.s, r2, k3));
      const half2_t zq = as_half2(pair_f16<3>(t.s, T::B2 / 2 + r2, k3));
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const int r = 2 * r2 + h2;
        float d[NB];
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) d[bi] = 0.f;
#pragma unroll
        for (int p = 0; p < PPR; ++p) {
          if constexpr (SHARED) refresh_shifted<W>(sw, t.c, r * PPR + p);
          const half2_t q2 = as_half2(SHARED ? pair_class_f16<W>(t.c, sw, r * PPR + p, k) : pair_f16<W>(t.c, r * PPR + p, k1));
#pragma unroll
          for (int bi = 0; bi < NB; ++bi) d[bi] = __builtin_amdgcn_fdot2(q2, as_half2(xp[bi][p]), d[bi], false);
        }
        const float sh = fmaf((float)(h2 ? sq.y : sq.x), c1, c2);
        const float zh = fmaf((float)(h2 ? zq.y : zq.x), e1, e2);      // z_hat_r
#pragma unroll
        for (int bi = 0; bi < NB; ++bi)
          acc[bi][r] = fmaf(sh, fmaf(-zh, X[bi], fmaf(SCALE, d[bi], -SE[bi][r % NPH])), acc[bi][r]);   // big terms cancel first
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Outliers of one strip (Sec. 4.2 "Storing outliers": entries sorted by row,
// then column; one 32-bit running count per row).  The strip's entries are one
// contiguous CSR range.  It is cut into aligned chunks of 8 entries (16 bytes
// of column indices + 16 bytes of values) dealt to the threads of the
// workgroup one each, whatever the rows' lengths; a thread multiplies its 8
// values with x and parks the 8 products in LDS at their CSR position.  After
// one barrier 16 lanes per row add that row's contiguous slice of products in
// a fixed order.  No atomics, no search, one global round trip.
// ---------------------------------------------------------------------------

// Products of the 8 entries of chunk c (global chunk index); entries outside
// [e_lo, e_hi) give 0.
__device__ __forceinline__ void chunk_products(const uint16_t* xs, int e_lo, int e_hi, int c,
                                               const u32x4& c8, const u32x4& v8, float (&p)[8]) {
  const uint32_t cw[4] = {c8.x, c8.y, c8.z, c8.w};
  const uint32_t vw[4] = {v8.x, v8.y, v8.z, v8.w};
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = 8 * c + i;
    const bool ok = e >= e_lo && e < e_hi;
    const uint32_t col = (i & 1) ? (cw[i >> 1] >> 16) : (cw[i >> 1] & 0xFFFFu);
    const uint32_t val = (i & 1) ? (vw[i >> 1] >> 16) : (vw[i >> 1] & 0xFFFFu);
    const float xv = h2f(xs[ok ? col : 0u]);
    p[i] = ok ? h2f((uint16_t)val) * xv : 0.f;
  }
}

__device__ __forceinline__ void store_products(float* prod, int slot, const float (&p)[8]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  f32x4 lo = {p[0], p[1], p[2], p[3]}, hi = {p[4], p[5], p[6], p[7]};
  reinterpret_cast<f32x4*>(prod)[2 * slot] = lo;
  reinterpret_cast<f32x4*>(prod)[2 * slot + 1] = hi;
}

// Sum of prod[i] for i in [lo, hi) by the 16 lanes of a group, eight reads in flight.
__device__ __forceinline__ float strided16_sum(const float* prod, int lo, int hi, int l16) {
  float s = 0.f;
  for (int i = lo + l16; i < hi; i += 128) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = prod[min(i + 16 * k, hi - 1)];
#pragma unroll
    for (int k = 0; k < 8; ++k) s += (i + 16 * k < hi) ? v[k] : 0.f;
  }
  return s;
}

// Workgroup size limits: 16 wavefronts leave the compiler 128 registers per
// lane, 8 wavefronts 256; a 4-bit tile needs 32 code registers, twice with the
// prefetch of the next step, and every further activation vector TR more
// accumulators.
template <int W, int NB> struct WavesPerGroup { static constexpr int MAX = (W == 3 && NB == 1) ? 16 : 8; };

// NB activation vectors per launch: X holds NB rows of n binary16 values (row
// stride n), Y NB rows of m outputs (row stride m).  NB = 1 is the GEMV.
// `strip` is the strip of A this workgroup owns.
template <int W, int TR, int TC, int AXIS, bool PERM, int NB>
__device__ __forceinline__ void gemv_tile256_body(const DevMatrix& A, const uint16_t* __restrict__ x,
                                                  void* __restrict__ y, int y_dtype, int chunk_cap,
                                                  const int strip) {
  using T = TileRegs<W, TR, TC, AXIS>;
  static_assert(TR * TC == 256, "tile must hold 256 codes");
  static_assert((TC / 2) % 4 == 0, "x pairs are read as 16-byte LDS words");
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr int MAX_WAVES = 16;
  constexpr int XCH = 4 * NB;                // 16-byte chunks of x a thread keeps in flight
  constexpr int KR = 4;                      // outlier chunks per thread requested ahead of the last dense step
  constexpr int KMAX = 8;                    // outlier chunks per thread and round at most
  constexpr int LONG_ROW = 512;              // rows with more entries are summed by all threads

  // dynamic LDS: the NB x vectors | products of the outlier entries (8 floats per
  // chunk and vector)
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);
  const int n = A.g.n, ntc = A.g.ntc, m = A.g.m;
  const int xbytes = (NB * n * 2 + 15) & ~15;
  float* prod = reinterpret_cast<float*>(smem + xbytes);
  const int pstride = 8 * chunk_cap;         // floats of products per vector
  __shared__ float red[MAX_WAVES][NB][TR];
  __shared__ float osum[NB][TR];
  __shared__ float lred[NB][TR][MAX_WAVES];
  __shared__ int rp[TR + 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // scalar: step indices and tile bases stay in SGPRs
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int l16 = tid & 15, g16 = tid >> 4, ngroups = nthreads >> 4;
  const int nsteps = (ntc + 63) >> 6;
  const uint8_t* strip_base = A.packed + (int64_t)strip * ntc * TILE_BYTES;
  const int32_t* rpg = A.row_ptr + (int64_t)strip * TR;

  // ---- issue order: row pointers and x first (small, mostly cache hits), then
  // the first tile.  Everything up to the barrier is straight-line code with
  // clamped indices instead of branches, so that the wait before staging x
  // covers the x loads only and never the big tile loads behind them. ------------
  const int e_lo = rpg[0], e_hi = rpg[TR];   // uniform: scalar loads
  const int rp_mine = rpg[min(tid, TR)];     // thread r <= TR carries row pointer r into LDS
  const int nvec = (NB * n) >> 3;            // 16-byte chunks of the NB contiguous x vectors
  u32x4 xr[XCH];
  if constexpr (!PERM) {
#pragma unroll
    for (int k = 0; k < XCH; ++k)
      xr[k] = reinterpret_cast<const u32x4*>(x)[min(tid + k * nthreads, nvec - 1)];
  }
  __builtin_amdgcn_sched_barrier(0);         // keep the x loads ahead of the tile loads

  T t0, t1;
  // Tile loads are never branched around: a step that does not exist loads one
  // 16-byte word per load with all lanes on the strip's first tile (a single
  // cache line, the result is ignored).  With no conditional load between a tile's
  // loads and its use, the waits ahead of each code word count exactly the loads
  // issued behind it, so a tile's arithmetic starts while its later words and the
  // whole next tile are still in flight.
  auto issue = [&](T& t, int st) -> int {    // returns the number of tiles in the step's block
    const bool real = st < nsteps;           // wave-uniform
    const int L = real ? min(64, ntc - 64 * st) : 1;
    load_tile<NB == 1>(t, strip_base + (int64_t)64 * (real ? st : 0) * TILE_BYTES, L, min(lane, L - 1));
    asm volatile("" ::: "memory");           // the loads stay here, ahead of the arithmetic on the other buffer
    return L;
  };
  int step = wave;                           // wave < nwaves <= nsteps: the first step always exists
  int L0 = min(64, ntc - 64 * step), L1 = 1;
  load_tile<NB == 1>(t0, strip_base + (int64_t)64 * step * TILE_BYTES, L0, min(lane, L0 - 1));
  __builtin_amdgcn_sched_barrier(0);
  rp[min(tid, TR)] = rp_mine;                // clamped duplicates store the same value again

  if constexpr (!PERM) {
    u32x4* dst = reinterpret_cast<u32x4*>(xs);
#pragma unroll
    for (int k = 0; k < XCH; ++k)            // clamped duplicates store the same value again
      dst[min(tid + k * nthreads, nvec - 1)] = xr[k];
    if constexpr (NB == 1) {                 // very long x: the rest, one chunk at a time
      for (int i = tid + XCH * nthreads; i < nvec; i += nthreads) dst[i] = reinterpret_cast<const u32x4*>(x)[i];
    } else {                                 // several vectors: further batches of XCH chunks
      for (int i0 = tid + XCH * nthreads; i0 < nvec; i0 += XCH * nthreads) {
#pragma unroll
        for (int k = 0; k < XCH; ++k) xr[k] = reinterpret_cast<const u32x4*>(x)[min(i0 + k * nthreads, nvec - 1)];
#pragma unroll
        for (int k = 0; k < XCH; ++k) dst[min(i0 + k * nthreads, nvec - 1)] = xr[k];
      }
    }
    for (int j = (nvec << 3) + tid; j < NB * n; j += nthreads) xs[j] = x[j];
  } else {
    for (int j = tid; j < NB * n; j += nthreads) xs[j] = x[(j / n) * n + A.perm[j % n]];
  }

  // ---- outliers: fetch this thread's chunk now, use it after the dense part -----
  const int c_lo = e_lo >> 3;
  const int nchunks = e_hi > e_lo ? ((e_hi - 1) >> 3) - c_lo + 1 : 0;
  const u32x4* col8 = reinterpret_cast<const u32x4*>(A.col);
  const u32x4* val8 = reinterpret_cast<const u32x4*>(A.val);
  const int first_round = min(nchunks, nthreads);        // nthreads <= chunk_cap <= KMAX*nthreads
  u32x4 pc, pv;
  {                                          // unconditional, like the tile loads: a thread without a chunk
    const bool have = tid < first_round;     // reads 16 bytes of the strip's first tile instead
    const u32x4* dummy = reinterpret_cast<const u32x4*>(strip_base);
    pc = load_once<NB == 1>(have ? col8 + c_lo + tid : dummy);
    pv = load_once<NB == 1>(have ? val8 + c_lo + tid : dummy);
  }
  __syncthreads();                           // x is staged

  // ---- dense part -------------------------------------------------------------
  constexpr int NPH = RowPhases<W, TC>::N;
  float acc[NB][TR], csum[NB][NPH];
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
#pragma unroll
    for (int h = 0; h < NPH; ++h) csum[bi][h] = 0.f;
#pragma unroll
    for (int r = 0; r < TR; ++r) acc[bi][r] = 0.f;
  }
  ClassConsts kc = {};
  PairConsts k1 = {};
  if constexpr (SharedShifts<TC>::value) kc = make_class_consts<W>(); else k1 = make_pair_consts<W>();
  const PairConsts k3 = make_pair_consts<3>();
  const uint32_t* xs32 = reinterpret_cast<const uint32_t*>(xs);
  const bool heavy = nchunks > nthreads;     // workgroup-uniform
#define SPQR_TILE_FMA(t, L, st)                                                                           \
  tile_fma<W, TR, TC, AXIS, NB>(t, xs32 + (64 * (st) + min(lane, (L) - 1)) * (TC / 2), n >> 1, lane < (L), \
                                acc, csum, kc, k1, k3)
  // Two steps per trip, registers ping-pong; the loop has its one exit at the
  // bottom (a second exit would be merged with it through a block that makes the
  // compiler wait for every load at the top of the loop).  t0 holds step `step`.
  while (step + nwaves < nsteps) {           // wave-uniform: at least two steps are left
    L1 = issue(t1, step + nwaves);
    SPQR_TILE_FMA(t0, L0, step);
    L0 = issue(t0, step + 2 * nwaves);       // a dummy after the wavefront's last step
    SPQR_TILE_FMA(t1, L1, step + nwaves);
    step += 2 * nwaves;
  }
  // A strip with more outlier chunks than threads (slots tid + k*nthreads, k >= 1):
  // the next KR-1 chunks of this thread are requested here, in the registers the
  // other tile buffer has just left, and arrive under the wavefront's last dense
  // step; the rest follow after it, all together.
  u32x4 lc[KMAX - 1], lv[KMAX - 1];
  {                                          // unconditional like the tile loads (dummy: the strip's first tile),
    const u32x4* dummy = reinterpret_cast<const u32x4*>(strip_base);   // so that the waits stay exact
#pragma unroll
    for (int k = 1; k < KR; ++k) {
      const int slot = tid + k * nthreads;
      const bool have = slot < chunk_cap && slot < nchunks;
      lc[k - 1] = load_once<NB == 1>(have ? col8 + c_lo + slot : dummy);
      lv[k - 1] = load_once<NB == 1>(have ? val8 + c_lo + slot : dummy);
    }
    asm volatile("" ::: "memory");
  }
  if (step < nsteps) SPQR_TILE_FMA(t0, L0, step);
#undef SPQR_TILE_FMA

  // ---- outlier products of the first round -> LDS -------------------------------
  if (heavy) {
#pragma unroll
    for (int k = KR; k < KMAX; ++k) {
      const int slot = tid + k * nthreads;
      if (slot < chunk_cap && slot < nchunks) {
        lc[k - 1] = load_once<NB == 1>(col8 + c_lo + slot);
        lv[k - 1] = load_once<NB == 1>(val8 + c_lo + slot);
      }
    }
  }
  if (tid < first_round) {
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
      float p[8];
      chunk_products(xs + bi * n, e_lo, e_hi, c_lo + tid, pc, pv, p);
      store_products(prod + bi * pstride, tid, p);
    }
  }
  if (heavy) {
#pragma unroll
    for (int k = 1; k < KMAX; ++k) {
      const int slot = tid + k * nthreads;
      if (slot < chunk_cap && slot < nchunks) {
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
          float p[8];
          chunk_products(xs + bi * n, e_lo, e_hi, c_lo + slot, lc[k - 1], lv[k - 1], p);
          store_products(prod + bi * pstride, slot, p);
        }
      }
    }
  }

  // ---- dense partials: lanes -> rows ---------------------------------------------
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
    if constexpr (AXIS == 1) {
#pragma unroll
      for (int r = 0; r < TR; ++r) acc[bi][r] = fmaf((float)(1 << W), acc[bi][r], -csum[bi][r % NPH]);
    }
    int row;
    const float rsum = wave_reduce_rows<TR>(acc[bi], lane, &row);
    if ((lane & ((64 / TR) - 1)) == 0) red[wave][bi][row] = rsum;
  }

  // Rows too long for 16 lanes, as a bit mask every wavefront works out for itself
  // from the row pointers in LDS (TR <= 32 lanes vote), and this thread's first
  // output row: both read ahead of the barrier, off the critical path behind it.
  static_assert(TR <= 32, "one lane per row votes");
  const int vr = min(lane, TR - 1);
  uint64_t longs = __builtin_amdgcn_ballot_w64(lane < TR && rp[vr + 1] - rp[vr] > LONG_ROW);
  const int r_long = longs ? __builtin_ctzll(longs) : 0;
  const int lo_long = rp[r_long], hi_long = rp[r_long + 1];
  const int r_first = min(g16, TR - 1);
  const int a_first = rp[r_first], b_first = rp[r_first + 1];
  // One barrier publishes products and partials.  Only a strip with more chunks
  // than one round holds needs the slow path.
  __syncthreads();
  const bool slow = nchunks > chunk_cap;     // workgroup-uniform
  const int base = 8 * c_lo;                 // CSR index of prod[0] in the first round
  if (!slow) {
    if (longs) {
      // long rows: every thread adds a strided share, one partial per wavefront and row
      bool first = true;
      while (longs) {                        // workgroup-uniform
        const int r = __builtin_ctzll(longs);
        longs &= longs - 1;
        const int lo = (first ? lo_long : rp[r]) - base, hi = (first ? hi_long : rp[r + 1]) - base;
        first = false;
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
          const float* pb = prod + bi * pstride;
          float s = 0.f;
          for (int i = lo + tid; i < hi; i += 12 * nthreads) {
            float v[12];
#pragma unroll
            for (int k = 0; k < 12; ++k) v[k] = pb[min(i + k * nthreads, hi - 1)];
#pragma unroll
            for (int k = 0; k < 12; ++k) s += (i + k * nthreads < hi) ? v[k] : 0.f;
          }
          s = wave_allreduce(s, lane);
          if (lane == 0) lred[bi][r][wave] = s;
        }
      }
      __syncthreads();
    }
    // 16 lanes per row: the row's products, plus one dense partial per wavefront
    for (int r = g16; r < TR; r += ngroups) {
      const int a = r == g16 ? a_first : rp[r], b = r == g16 ? b_first : rp[r + 1];
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        float s;
        if (b - a > LONG_ROW) s = l16 < nwaves ? lred[bi][r][l16] : 0.f;
        else s = strided16_sum(prod + bi * pstride, a - base, b - base, l16);
        if (l16 < nwaves) s += red[l16][bi][r];
        s = row16_allreduce(s, lane);
        if (l16 == 0) {
          const int64_t i = (int64_t)bi * m + (int64_t)strip * TR + r;
          if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
          else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
        }
      }
    }
    return;
  }

  // ---- slow path: rounds of chunk_cap chunks (up to KMAX per thread, all loads of a
  // round in flight together); long rows summed by all threads ----------------------
  if (tid < NB * TR) (&osum[0][0])[tid] = 0.f;
  for (int c0 = 0; c0 < nchunks; c0 += chunk_cap) {      // workgroup-uniform
    const int c1 = min(nchunks, c0 + chunk_cap);
    if (c0 > 0) __syncthreads();                         // previous round's products are consumed
    if (c0 > 0) {                                        // round 0 is already in LDS
      u32x4 cc[KMAX], vv[KMAX];
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int slot = tid + k * nthreads, j = c0 + slot;
        if (slot < chunk_cap && j < c1) {
          cc[k] = load_once<NB == 1>(col8 + c_lo + j);
          vv[k] = load_once<NB == 1>(val8 + c_lo + j);
        }
      }
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const int slot = tid + k * nthreads, j = c0 + slot;
        if (slot < chunk_cap && j < c1) {
#pragma unroll
          for (int bi = 0; bi < NB; ++bi) {
            float p[8];
            chunk_products(xs + bi * n, e_lo, e_hi, c_lo + j, cc[k], vv[k], p);
            store_products(prod + bi * pstride, slot, p);
          }
        }
      }
    }
    __syncthreads();
    const int e0 = 8 * (c_lo + c0), e1 = 8 * (c_lo + c1);   // CSR range covered by this round
    // rows with a long slice in this round, voted as on the fast path; their partials per
    // wavefront go through lred, one barrier for all of them
    uint64_t rl = __builtin_amdgcn_ballot_w64(lane < TR && min(rp[vr + 1], e1) - max(rp[vr], e0) > LONG_ROW);
    const bool some_long = rl != 0;
    while (rl) {                                         // workgroup-uniform
      const int r = __builtin_ctzll(rl);
      rl &= rl - 1;
      const int lo = max(rp[r], e0) - e0, hi = min(rp[r + 1], e1) - e0;
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const float* pb = prod + bi * pstride;
        float s = 0.f;
        for (int i = lo + tid; i < hi; i += 4 * nthreads) {
          float v[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) v[k] = pb[min(i + k * nthreads, hi - 1)];
#pragma unroll
          for (int k = 0; k < 4; ++k) s += (i + k * nthreads < hi) ? v[k] : 0.f;
        }
        s = wave_allreduce(s, lane);
        if (lane == 0) lred[bi][r][wave] = s;
      }
    }
    if (some_long) __syncthreads();
    for (int r = g16; r < TR; r += ngroups) {            // a row always meets the same 16 lanes: osum needs no barrier
      const int a = max(rp[r], e0), b = min(rp[r + 1], e1);
      if (b > a) {
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) {
          float s;
          if (b - a > LONG_ROW) s = l16 < nwaves ? lred[bi][r][l16] : 0.f;
          else s = strided16_sum(prod + bi * pstride, a - e0, b - e0, l16);
          s = row16_allreduce(s, lane);
          if (l16 == 0) osum[bi][r] += s;
        }
      }
    }
  }
  __syncthreads();
  if (tid < NB * TR) {
    const int bi = tid / TR, r = tid % TR;
    float s = osum[bi][r];
    for (int w = 0; w < nwaves; ++w) s += red[w][bi][r];
    const int64_t i = (int64_t)bi * m + (int64_t)strip * TR + r;
    if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
    else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
  }
}

template <int W, int TR, int TC, int AXIS, bool PERM, int NB>
__global__ void __launch_bounds__((64 * WavesPerGroup<W, NB>::MAX))
gemv_tile256_kernel(DevMatrix A, const uint16_t* __restrict__ x, void* __restrict__ y, int y_dtype,
                    int chunk_cap) {
  gemv_tile256_body<W, TR, TC, AXIS, PERM, NB>(A, x, y, y_dtype, chunk_cap, blockIdx.x);
}

// ---------------------------------------------------------------------------
// Batches above 4 on 16x16 tiles: the dense part on the matrix cores (weights
// stream once for the whole batch), then a finishing kernel that adds the outliers.
//
// Dense part: P[split][b][rows] = X[b][cols of the split] . dequant(strip)^T in
// binary32, no outliers.  A workgroup is 4 wavefronts = 4 consecutive strips that
// walk the same steps of 64 tiles in lock-step, because they share the 16 x 1024
// piece of X that belongs to the step: it is staged in LDS once per workgroup
// (prefetched into registers one step ahead).  A lane still fetches one whole
// tile (same loads, same layout as the GEMV).  An MFMA operand, though, wants
// 16 rows x 4 columns across the 64 lanes, while here the lanes hold 64 different
// tiles: so every lane dequantises its tile to binary16 (s_hat*(q - z_hat) evaluated
// in binary32, one rounding -- the paper's kernel also "dequantizes to 16-bits",
// Sec. 4.2) into its wavefront's LDS buffer, a quarter (4 columns) at a time to
// keep the buffer small enough for two workgroups per CU.  One
// v_mfma_f32_16x16x32_f16 then sums 8 tiles at once: its K index is (tile, column),
// A: lane l = row l%16 of tiles 8j + 2(l/16) and the next, B: lane l = batch l%16, the
// same two tiles' 4 columns of X; D[row][batch] accumulates over the whole column
// range in 8 registers.
// Batch rows beyond `batch` repeat the last one and are dropped at the end.
// The steps of a matrix can be split over gridDim.y workgroups (few strips, many
// columns); every split writes its own partial result.  Workgroups behind the
// dense ones (blockIdx.x >= groups) take the long outlier rows, see long_rows_block.
// ---------------------------------------------------------------------------
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
constexpr int kMfmaTileStride = 36;          // dwords per tile quarter (16 rows x 8 bytes + 16: spreads the banks)

// Outlier rows longer than `long_row` entries (far longer than the average row), for the batch path.  Such a row
// would keep the one CU that owns its strip busy long after the others are done (every outlier is an L1 line
// look-up), so these rows are taken out of the finishing kernel: extra workgroups of the dense kernel's grid (they
// run beside the dense workgroups and need nothing from them) compute, slice by slice of kLongSlice entries,
// sum_k val_k * XT[col_k][b] for the 16 vectors
// into slots[lo / kSlotGrain + k][16] for slice k of the row that starts at entry lo -- a long row has no more
// slices than multiples of kSlotGrain among its entry indices (ceil(len/512) <= floor(len/256) from len = 256 on),
// so the slots of different rows never meet and the finishing kernel finds them without a search.
// Work is shared out by entries, not by rows: workgroup wg of nwg owns the slices that start in its equal share
// [a, z) of the entry indices, so heavy rows next to each other (or one row of many slices) spread over as many
// workgroups as their entries fill.  It narrows the rows down to NT around the one that holds entry a by a search
// all threads take part in (NT probes of the row pointers per round; none for up to NT rows, one for up to NT*NT),
// then walks the rows from there, NT - 1 at a time, up to the first that starts at or behind z.  A slice is one wavefront's: a lane takes every 64th entry (consecutive lanes read
// consecutive entries) with its whole 32-byte line of XT, all loads in flight at once; the 16 sums are reduced over
// the lanes in a fixed order and written by the wavefront itself.  The wavefronts of a workgroup take its slices
// in turn and meet only where the next rows are fetched.
constexpr int kLongRowMin = 256, kLongSlice = 512, kSlotGrain = 256;

template <int NT>
__device__ __forceinline__ void long_rows_block(const DevMatrix& A, const uint16_t* __restrict__ XT,
                                                float* __restrict__ slots, int long_row, int wg, int nwg, uint8_t* smem) {
  constexpr int EPT = kLongSlice / 64, NW = NT / 64;
  int* rpl = reinterpret_cast<int*>(smem);                                   // NT row pointers
  uint32_t* masks = reinterpret_cast<uint32_t*>(smem + 4 * NT);              // 2 per wavefront
  int* below = reinterpret_cast<int*>(smem + 4 * NT + 8 * NW);               // 1 per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = A.g.m;
  const int64_t nnz = A.nnz;
  const uint32_t zoff = (uint32_t)A.g.n * 32u;                               // the zero line of XT
  int64_t per = (nnz + nwg - 1) / nwg;
  if (per < kLongSlice) per = kLongSlice;
  const int64_t a64 = (int64_t)wg * per;
  if (a64 >= nnz) return;                                                    // workgroup-uniform
  const int a = (int)a64, z = (int)(a64 + per < nnz ? a64 + per : nnz);
  // the last row r with row_ptr[r] <= a lies in [L, H): row_ptr[L] <= a < row_ptr[H] throughout
  int L = 0, H = m;
  while (H - L > NT) {                                                       // workgroup-uniform
    // probe t looks at the end of the t-th of NT parts of the bracket: distinct rows in (L, H], the last is H
    const int span = H - L;
    const bool is_below = A.row_ptr[L + (int)(((int64_t)(tid + 1) * span) / NT)] <= a;
    const uint64_t bal = __builtin_amdgcn_ballot_w64(is_below);
    if (lane == 0) below[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int c = 0;                                                               // probes at or below a: a prefix of them,
#pragma unroll
    for (int k = 0; k < NW; ++k) c += below[k];                              // never all (row H is above a)
    __syncthreads();
    c = min(c, NT - 1);                      // (all only if row_ptr[m] < nnz, a broken descriptor: stay inside the bracket)
    const int newL = c == 0 ? L : L + (int)(((int64_t)c * span) / NT);
    H = L + (int)(((int64_t)(c + 1) * span) / NT);
    L = newL;
  }
  // The rows from L on, NT - 1 at a time.  The row that holds entry a is among the first H - L <= NT of them; the
  // rows before it end at or before a and own nothing here.
  int taken = 0;                                                             // slices of this workgroup so far
  for (int r0 = L; r0 < m;) {                                                // workgroup-uniform
    const int nrows = min(NT - 1, m - r0);
    if (tid <= nrows) rpl[tid] = A.row_ptr[r0 + tid];
    __syncthreads();
    const int t1 = min(tid, NT - 2);
    const bool is_long = tid < nrows && rpl[t1 + 1] - rpl[t1] > long_row && rpl[t1] < z && rpl[t1 + 1] > a;
    const uint64_t bal = __builtin_amdgcn_ballot_w64(is_long);
    if (lane == 0) { masks[2 * wave] = (uint32_t)bal; masks[2 * wave + 1] = (uint32_t)(bal >> 32); }
    __syncthreads();
    for (int w = 0; w < NW; ++w) {
      uint64_t mask = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)masks[2 * w]) |      // no sign extension
                      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)masks[2 * w + 1]) << 32);
      while (mask) {                                                         // workgroup-uniform
        const int r = 64 * w + __builtin_ctzll(mask);
        mask &= mask - 1;
        const int lo = rpl[r], hi = rpl[r + 1];
        // the row's slices that start in [a, z)
        const int k0 = lo >= a ? 0 : (a - lo + kLongSlice - 1) / kLongSlice;
        for (int k = k0; lo + k * kLongSlice < min(hi, z); ++k) {
          if (taken++ % NW != wave) continue;                                // wavefront-uniform
          const int e0 = lo + k * kLongSlice;
          // all of the lane's entries first, then their lines of XT, then the arithmetic: one round trip each
          uint32_t off[EPT];
          float val[EPT];
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const int e = e0 + lane + 64 * i;
            const bool ok = e < hi;
            off[i] = ok ? (uint32_t)A.col[e] * 32u : zoff;
            val[i] = ok ? h2f(A.val[e]) : 0.f;
          }
          u32x4 x0[EPT], x1[EPT];
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const u32x4* line = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(XT) + off[i]);
            x0[i] = line[0];
            x1[i] = line[1];
          }
          float acc[16];
#pragma unroll
          for (int b = 0; b < 16; ++b) acc[b] = 0.f;
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const uint32_t xw[8] = {x0[i].x, x0[i].y, x0[i].z, x0[i].w, x1[i].x, x1[i].y, x1[i].z, x1[i].w};
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              acc[2 * q] = fmaf(val[i], h2f((uint16_t)(xw[q] & 0xFFFFu)), acc[2 * q]);
              acc[2 * q + 1] = fmaf(val[i], h2f((uint16_t)(xw[q] >> 16)), acc[2 * q + 1]);
            }
          }
          int row;
          const float red = wave_reduce_rows<16>(acc, lane, &row);           // every lane: the sum of vector `row`
          if ((lane & 3) == 0) slots[(int64_t)(lo / kSlotGrain + k) * 16 + row] = red;   // 4 lanes hold each sum
        }
      }
    }
    if (rpl[nrows] >= z) break;                                              // the next row starts behind the share
    r0 += nrows;
    __syncthreads();                                                         // everyone is done with these row pointers
  }
}

// Shape of the dense kernel for a tile of TR x TC = 256 codes.  A phase covers PC = 64/TR columns of every tile
// (a lane always writes 64 binary16 values = 128 bytes per phase: rows x PC columns), four phases per step.
// The 8 K-values a lane supplies to one MFMA are PC columns of 8/PC tiles.  Strips per workgroup: what the LDS
// allows next to the piece of X (16 batch rows x 64*TC columns): 8 x 32 tiles share a 64 KB piece among 8 strips.
template <int TR, int TC> struct MfmaShape {
  static constexpr int PC = 64 / TR;                       // columns per phase: 8, 4, 2
  static constexpr int TPK = 8 / PC;                       // tiles per K-group of a lane: 1, 2, 4
  static constexpr int MB = TR >= 16 ? TR / 16 : 1;        // blocks of 16 rows (an 8-row tile fills half a block)
  static constexpr int NS = TC == 32 ? 8 : 4;              // strips = wavefronts per workgroup
  static constexpr int WGS = TC == 32 ? 1 : 2;             // workgroups per CU
  static constexpr int XROW = 128 * TC + 8;                // bytes per batch row of the staged piece of X
  static constexpr size_t LDS = (size_t)NS * 64 * kMfmaTileStride * 4 + 16 * (size_t)XROW;
  static_assert(WGS * (LDS + 1024) <= 160 * 1024, "the workgroups of a CU must fit its LDS");
};

// `group` is the group of NS strips this workgroup multiplies, or negative for a workgroup that takes long outlier
// rows instead: then it is number `extra` of `nextra` such workgroups of its matrix.  `split` of the splits of the
// steps, `smem` the workgroup's dynamic LDS.
template <int W, int TR, int TC, int AXIS, bool ONE>
__device__ __forceinline__ void gemm_mfma_body(const DevMatrix& A, const uint16_t* __restrict__ X, float* __restrict__ P,
                                               int64_t split_stride, int steps_per_split, int batch,
                                               const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row,
                                               int group, int split, int extra, int nextra, uint8_t* smem) {
  using SH = MfmaShape<TR, TC>;
  constexpr int PPR = TC / 2, S = kMfmaTileStride, NS = SH::NS, NT = 64 * NS, PC = SH::PC, TPK = SH::TPK, MB = SH::MB;
  constexpr int UROW = 8 * TC;               // 16-byte units of the X piece per batch row
  constexpr int UPT = 16 * UROW / NT;        // ... per thread
  constexpr int B2 = AXIS == 1 ? TC : TR;    // first-level groups per tile
  constexpr int NM = 2 * PC;                 // MFMAs per phase and block of rows
  static_assert(NT % UROW == 0 && TR * TC == 256, "shape");
  using T = TileRegs<W, TR, TC, AXIS>;
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr float SCALE = (float)(1 << W);
  uint8_t* xbuf = smem + NS * 64 * S * 4;
  if (group < 0) {                           // long outlier rows
    if (split == 0)
      long_rows_block<NT>(A, XT, slots, long_row, extra, nextra, smem);
    return;
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = A.g.n, ntc = A.g.ntc, m = A.g.m, ntr = A.g.ntr;
  const int nsteps = (ntc + 63) >> 6;
  const int s_lo = split * steps_per_split, s_hi = min(nsteps, s_lo + steps_per_split);   // never empty (host)
  const int strip = group * NS + wave;
  const bool active = strip < ntr;           // wave-uniform; an idle wavefront still stages X and meets the barriers
  const uint8_t* strip_base = A.packed + (int64_t)min(strip, ntr - 1) * ntc * TILE_BYTES;
  uint32_t* buf = reinterpret_cast<uint32_t*>(smem) + wave * 64 * S;
  const int i16 = lane & 15, g4 = lane >> 4;
  const PairConsts kc = make_pair_consts<W>();
  const PairConsts k3 = make_pair_consts<3>();
  // Groups along the tile's columns, and the class of a code pair (the offset K its in-place extraction leaves,
  // see CodeClass) a function of its column alone: then K folds into the column's additive constant and most
  // shifts of the extraction go away.  True for 4-bit codes and for 3-bit codes in rows of 16 pairs.
  constexpr bool FOLD = AXIS == 1 && (W == 4 || PPR == 16);
  const ClassConsts kk = make_class_consts<W>();
  float4_t D[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) { D[mb][0] = float4_t{0.f, 0.f, 0.f, 0.f}; D[mb][1] = float4_t{0.f, 0.f, 0.f, 0.f}; }

  // the piece of X of step st: unit u = 16 bytes = 8 columns of batch row u/UROW; loads unconditional (clamped)
  u32x4 xr[UPT];
  uint32_t xrow[UPT];                        // byte offset of the unit's (clamped) batch row in X
#pragma unroll
  for (int k = 0; k < UPT; ++k) xrow[k] = (uint32_t)min((tid + k * NT) / UROW, batch - 1) * (uint32_t)n * 2u;
  const int xj = tid % UROW;                 // NT is a multiple of UROW: the unit's place in its row is the same for all k
  auto fetch_x = [&](int st) {
    const int sc = min(st, s_hi - 1);
    const int L = min(64, ntc - 64 * sc);
    const uint8_t* xs = reinterpret_cast<const uint8_t*>(X + (int64_t)(64 * TC) * sc);
    const uint32_t jb = 16u * (uint32_t)min(xj, L * (TC / 8) - 1);
#pragma unroll
    for (int k = 0; k < UPT; ++k) xr[k] = *reinterpret_cast<const u32x4*>(xs + (xrow[k] + jb));
    asm volatile("" ::: "memory");
  };
  auto store_x = [&](int st) {
    const int L = min(64, ntc - 64 * st);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    // columns behind the last tile: zeros (finite), they meet zero weights
    const bool keep = xj < L * (TC / 8);
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const int b = (tid + k * NT) / UROW;
      const u32x2 lo = {keep ? xr[k].x : 0u, keep ? xr[k].y : 0u}, hi = {keep ? xr[k].z : 0u, keep ? xr[k].w : 0u};
      if (b < batch) {
        u32x2* d = reinterpret_cast<u32x2*>(xbuf + b * SH::XROW + xj * 16);
        d[0] = lo;
        d[1] = hi;
      }
    }
  };
  auto issue = [&](T& t, int st) {
    const bool real = st < s_hi;
    const int L = real ? min(64, ntc - 64 * st) : 1;
    load_tile<false>(t, strip_base + (int64_t)64 * (real ? st : s_lo) * TILE_BYTES, L, min(lane, L - 1));
    asm volatile("" ::: "memory");
  };
  // operand fragments of MFMA j of a phase: tiles (4j + g4)*TPK .. +TPK-1, PC columns each.
  // A: row i16 (+16 per block of rows; an 8-row tile repeats its rows, the copies are dropped at the end)
  const uint32_t* afrag = buf + g4 * TPK * S + ((TR >= 16 ? i16 : (i16 & 7)) * PC) / 2;
  const uint32_t* xfrag = reinterpret_cast<const uint32_t*>(xbuf + min(i16, batch - 1) * SH::XROW) + g4 * TPK * (TC / 2);
  // one step: publish its piece of X, then per phase: dequantise PC columns of this lane's tile, multiply
  auto run_step = [&](const T& t, int st) {
    const int L = min(64, ntc - 64 * st);
    __syncthreads();                         // every wavefront is done with the previous piece of X
    store_x(st);
    if constexpr (!ONE) fetch_x(st + 1);
    __syncthreads();
    const uint32_t a2 = t.s[T::SD - 2], b2 = t.s[T::SD - 1];
    const float s_s = h2f((uint16_t)(a2 & 0xFFFF)), z_s = h2f((uint16_t)(a2 >> 16));
    const float s_z = h2f((uint16_t)(b2 & 0xFFFF)), z_z = h2f((uint16_t)(b2 >> 16));
    // w = s_hat*(q - z_hat) = fa*(1 + q/2^W) + fb with fa = 2^W*s_hat, fb = -s_hat*(2^W + z_hat), per group,
    // where s_hat = s_s*(s_q - z_s) and z_hat = s_z*(z_q - z_z) and the extracted codes are 1 + code/8:
    //   fa = c1*(1 + s_q/8) + c2,   -(2^W + z_hat)/2^W = e1*(1 + z_q/8) + e2,   fb = fa * that.
    // A lane behind the step's last tile (its loads were clamped) writes a tile of zeros.
    const bool live = lane < L;
    const float c1 = live ? SCALE * 8.f * s_s : 0.f, c2 = live ? SCALE * (-s_s * z_s - 8.f * s_s) : 0.f;
    const float e1 = -8.f * s_z / SCALE, e2 = -(SCALE - s_z * z_z - 8.f * s_z) / SCALE;
    float fa[B2], fb[B2];
#pragma unroll
    for (int p = 0; p < B2 / 2; ++p) {
      const half2_t sq = as_half2(pair_f16<3>(t.s, p, k3));
      const half2_t zq = as_half2(pair_f16<3>(t.s, B2 / 2 + p, k3));
      fa[2 * p] = fmaf((float)sq.x, c1, c2);
      fa[2 * p + 1] = fmaf((float)sq.y, c1, c2);
      fb[2 * p] = fa[2 * p] * fmaf((float)zq.x, e1, e2);
      fb[2 * p + 1] = fa[2 * p + 1] * fmaf((float)zq.y, e1, e2);
      if constexpr (FOLD) {                  // the extracted value is K + code/2^W instead of 1 + code/2^W
        const float K = CodeClass<W, true>::K(CodeClass<W, true>::of_pair(p));   // a constant once the loop is unrolled
        fb[2 * p] = fmaf(1.f - K, fa[2 * p], fb[2 * p]);
        fb[2 * p + 1] = fmaf(1.f - K, fa[2 * p + 1], fb[2 * p + 1]);
      }
    }
    uint32_t* mine = buf + lane * S;
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {         // columns PC*ph .. PC*ph+PC-1 of every tile
      // the lane's 64 values of the phase, row by row (PC/2 dwords per row), 16 bytes per store
#pragma unroll
      for (int k4 = 0; k4 < 8; ++k4) {
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int dw = 4 * k4 + d, r = dw / (PC / 2), p = (PC / 2) * ph + dw % (PC / 2);
          const half2_t q2 = as_half2(FOLD ? pair_class_inline<W>(t.c, r * PPR + p, kk) : pair_f16<W>(t.c, r * PPR + p, kc));
          const int g0 = AXIS == 1 ? 2 * p : r, g1 = AXIS == 1 ? 2 * p + 1 : r;
          half2_t w;
          w.x = (_Float16)fmaf((float)q2.x, fa[g0], fb[g0]);
          w.y = (_Float16)fmaf((float)q2.y, fa[g1], fb[g1]);
          o[d] = __builtin_bit_cast(uint32_t, w);
        }
        const u32x4 v = {o[0], o[1], o[2], o[3]};
        *reinterpret_cast<u32x4*>(mine + 4 * k4) = v;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();       // the buffer is this wavefront's own: its LDS operations stay in order
      constexpr int JG = NM < 8 ? NM : 8;    // MFMAs whose operands are in flight at a time
#pragma unroll
      for (int j0 = 0; j0 < NM; j0 += JG) {
        uint32_t av[MB][JG][4], bv[JG][4];
#pragma unroll
        for (int j = 0; j < JG; ++j) {
#pragma unroll
          for (int tt = 0; tt < TPK; ++tt) {
            const int tile0 = (4 * (j0 + j)) * TPK + tt;         // + g4*TPK: in afrag / xfrag
            const uint32_t* pb = xfrag + tile0 * (TC / 2) + (PC / 2) * ph;
#pragma unroll
            for (int d = 0; d < PC / 2; ++d) bv[j][tt * (PC / 2) + d] = pb[d];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
              const uint32_t* pa = afrag + tile0 * S + mb * (16 * PC / 2);
#pragma unroll
              for (int d = 0; d < PC / 2; ++d) av[mb][j][tt * (PC / 2) + d] = pa[d];
            }
          }
        }
#pragma unroll
        for (int j = 0; j < JG; ++j) {
          const uint32_t b4v[4] = {bv[j][0], bv[j][1], bv[j][2], bv[j][3]};
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            const uint32_t a4v[4] = {av[mb][j][0], av[mb][j][1], av[mb][j][2], av[mb][j][3]};
            D[mb][j & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a4v),
                                                                   __builtin_bit_cast(half8_t, b4v), D[mb][j & 1], 0, 0, 0);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();       // the reads are issued before the next phase overwrites the buffer
    }
  };

  if constexpr (ONE) {                       // one step per workgroup: no second tile, no loop (fewer registers)
    T t0;
    fetch_x(s_lo);
    issue(t0, s_lo);
    run_step(t0, s_lo);
  } else {
    T t0, t1;
    fetch_x(s_lo);
    issue(t0, s_lo);
    int st = s_lo;
    while (st + 1 < s_hi) {                  // workgroup-uniform; two steps per trip, one exit at the bottom
      issue(t1, st + 1);
      run_step(t0, st);
      issue(t0, st + 2);                     // a dummy behind the last step
      run_step(t1, st + 1);
      st += 2;
    }
    if (st < s_hi) run_step(t0, st);
  }

  // D[mb][row 16*mb + 4*g4 + v][batch i16]
  if (active && i16 < batch) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const float4_t d = D[mb][0] + D[mb][1];
      if (16 * mb + 4 * g4 < TR)
        *reinterpret_cast<float4_t*>(P + (int64_t)split * split_stride + (int64_t)i16 * m + (int64_t)strip * TR +
                                     16 * mb + 4 * g4) = d;
    }
  }
}

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), 2)
gemm_mfma_kernel(DevMatrix A, const uint16_t* __restrict__ X, float* __restrict__ P, int64_t split_stride,
                 int steps_per_split, int batch, const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row,
                 int groups) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int bx = blockIdx.x;
  gemm_mfma_body<W, TR, TC, AXIS, false>(A, X, P, split_stride, steps_per_split, batch, XT, slots, long_row,
                                         bx < groups ? bx : -1, (int)blockIdx.y, bx - groups, (int)gridDim.x - groups, smem);
}

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), (TC == 32 ? 2 : 3))
gemm_mfma_one_kernel(DevMatrix A, const uint16_t* __restrict__ X, float* __restrict__ P, int64_t split_stride,
                     int batch, const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row, int groups) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int bx = blockIdx.x;
  gemm_mfma_body<W, TR, TC, AXIS, true>(A, X, P, split_stride, 1, batch, XT, slots, long_row,
                                        bx < groups ? bx : -1, (int)blockIdx.y, bx - groups, (int)gridDim.x - groups, smem);
}

// Several matrices that share the batch X and the format (q/k/v, gate/up of a decoder block) in one grid:
// blockIdx.x counts the dense workgroups of all matrices first, then their long-row workgroups.  Every
// workgroup does exactly what it would do in a launch of its own matrix.
struct MfmaFusedItem {
  DevMatrix A;
  float* P;                                  // partial results (or the output itself, see the finishing kernel)
  float* slots;
  void* Y;
  int long_row;
  int groups, extra;                         // dense / long-row workgroups of this matrix
  int blocks16;                              // workgroups of the finishing kernel
};
struct MfmaFused {
  int count;
  MfmaFusedItem it[SPQR_MAX_FUSED];
};

template <int W, int TR, int TC, int AXIS, bool ONE>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), (ONE && TC != 32 ? 3 : 2))
gemm_mfma_fused_kernel(MfmaFused F, const uint16_t* __restrict__ X, int steps_per_split, int batch,
                       const uint16_t* __restrict__ XT) {
  extern __shared__ __align__(16) uint8_t smem[];
  int bx = blockIdx.x, i = 0;
  bool dense = false;                        // workgroup-uniform search, count <= SPQR_MAX_FUSED
  for (; i < F.count; ++i) {
    if (bx < F.it[i].groups) { dense = true; break; }
    bx -= F.it[i].groups;
  }
  if (!dense) {
    for (i = 0; i < F.count - 1; ++i) {
      if (bx < F.it[i].extra) break;
      bx -= F.it[i].extra;
    }
  }
  const MfmaFusedItem& it = F.it[i];
  gemm_mfma_body<W, TR, TC, AXIS, ONE>(it.A, X, it.P, (int64_t)batch * it.A.g.m, ONE ? 1 : steps_per_split, batch, XT, it.slots,
                                  it.long_row, dense ? bx : -1, (int)blockIdx.y, bx, it.extra, smem);
}

// Prepares the batch for the batch path.  With an input permutation, column j of the
// matrix meets x[perm[j]] (act-order, Sec. 4 / Alg. 1: the quantiser reorders the input
// dimension): XP[b][j] = X[b][perm[j]] is the batch in the matrix's column order, read by
// the dense kernel in place of X.  For the outlier kernels, XT[j][16] binary16 is the same
// transposed, batch rows beyond `batch` zero, so that one outlier (one column j) meets its
// 16 activations in one 32-byte line; line n is all zeros: the place entry slots behind
// the end of a row read.  Either output may be absent.
__global__ void __launch_bounds__(256)
transpose_x16_kernel(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, uint16_t* __restrict__ XT,
                     uint16_t* __restrict__ XP, int n, int batch) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j > n) return;
  const int src = j < n ? (perm ? perm[j] : j) : 0;
  uint32_t o[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const uint32_t lo = (j < n && 2 * k < batch) ? X[(int64_t)(2 * k) * n + src] : 0u;
    const uint32_t hi = (j < n && 2 * k + 1 < batch) ? X[(int64_t)(2 * k + 1) * n + src] : 0u;
    o[k] = lo | (hi << 16);
    if (XP != nullptr && j < n) {
      if (2 * k < batch) XP[(int64_t)(2 * k) * n + j] = (uint16_t)lo;
      if (2 * k + 1 < batch) XP[(int64_t)(2 * k + 1) * n + j] = (uint16_t)hi;
    }
  }
  if (XT != nullptr) {
    u32x4* d = reinterpret_cast<u32x4*>(XT + (int64_t)j * 16);
    const u32x4 v0 = {o[0], o[1], o[2], o[3]}, v1 = {o[4], o[5], o[6], o[7]};
    d[0] = v0;
    d[1] = v1;
  }
}

// value of lane J (0 or 1) of the caller's pair of lanes, for both lanes of the pair
template <int J>
__device__ __forceinline__ uint32_t pair_broadcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, J == 0 ? 0xA0 : 0xF5, 0xF, 0xF, false);   // quad_perm [J,J,2+J,2+J]
}

// Finishing kernel for up to 16 activation vectors:
// Y[b][i] = sum_split P[split][b][i] + sum_k val_k * X[b][col_k]  (Sec. 4.2: the sparse
// part is a separate product), rounded to y_dtype.  With one split and binary32
// output P may be Y itself.
// One workgroup of 512 threads per strip of 16 rows.  The strip's CSR entries pass
// through LDS in chunks of 4096 (every thread brings one aligned granule of 8
// entries; chunks that lie inside one long row are skipped).  A pair of lanes works
// on one part of one row, each lane on 8 of the 16 activation vectors (16 bytes of
// the entry's line of XT), so no reduction across lanes exists: the pair walks its
// entries in order, 4 per trip (each lane reads 2 of them from LDS and hands them to
// its partner).  A row is cut into 16 contiguous parts (256 pairs = 16 rows x 16);
// parts are added in order by the row's owner.  A row longer than long_row comes
// ready-made from long_rows_block: its owner adds the row's slots in order.  Fixed
// order everywhere, one writer per output.
constexpr int kFinishThreads = 512;

__device__ __forceinline__ void finish_xt16_body(const DevMatrix& A, const uint16_t* __restrict__ XT,
                                                 const float* __restrict__ slots, const float* P, int nsplit,
                                                 int64_t split_stride, int long_row, void* Y, int y_dtype, int batch,
                                                 const int s) {
  constexpr int TR = 16, NP = kFinishThreads / 2, PER_ROW = NP / TR, CHUNK = 8 * kFinishThreads;
  __shared__ int rp[TR + 1];
  __shared__ float part[NP][16];
  __shared__ __align__(16) uint16_t scol[CHUNK], sval[CHUNK];
  const int tid = threadIdx.x, pr = tid >> 1, bq = tid & 1;
  const int g = tid >> 4, b = tid & 15;      // the owner of Y[b][row g] for tid < 256
  const int m = A.g.m;
  if (tid <= TR) rp[tid] = A.row_ptr[min(s * TR + tid, m)];      // rows behind the last one (m % 16 == 8) are empty
  // the dense part of this thread's output: requested now, needed at the very end
  const int64_t at = (int64_t)min(b, batch - 1) * m + min(s * TR + min(g, TR - 1), m - 1);
  float dense = 0.f;
  for (int k = 0; k < nsplit; ++k) dense += P[k * split_stride + at];
  __syncthreads();
  const int e_lo = rp[0], e_hi = rp[TR];
  const bool inplace = static_cast<const void*>(P) == static_cast<const void*>(Y);   // one split, written to Y by the dense kernel
  if (inplace && e_hi == e_lo) return;       // nothing to add (workgroup-uniform)
  const uint8_t* xt16 = reinterpret_cast<const uint8_t*>(XT) + 16 * bq;
  const uint32_t zoff = (uint32_t)A.g.n * 32u;
  // Both lanes of the pair add the 4 entries at chunk positions i0 + bq and i0 + 2 + bq (global index e0 + i),
  // those inside [lo, hi) (hi never beyond the chunk); the others read the zero line of XT with value 0.
  auto consume = [&](int e0, int i0, int lo, int hi, float (&acc)[8]) {
    uint32_t off[2], val[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int i = i0 + 2 * h + bq, e = e0 + i;
      const bool ok = e >= lo && e < hi;
      const int ic = min(i, CHUNK - 1);
      off[h] = ok ? (uint32_t)scol[ic] * 32u : zoff;
      val[h] = ok ? __builtin_bit_cast(uint32_t, h2f(sval[ic])) : 0u;
    }
    u32x4 xx[4];
    float vv[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t o[2] = {pair_broadcast<0>(off[h]), pair_broadcast<1>(off[h])};
      const uint32_t v[2] = {pair_broadcast<0>(val[h]), pair_broadcast<1>(val[h])};
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        xx[2 * h + j] = *reinterpret_cast<const u32x4*>(xt16 + o[j]);
        vv[2 * h + j] = __builtin_bit_cast(float, v[j]);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w[4] = {xx[i].x, xx[i].y, xx[i].z, xx[i].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = fmaf(vv[i], h2f((uint16_t)(w[k] & 0xFFFFu)), acc[2 * k]);
        acc[2 * k + 1] = fmaf(vv[i], h2f((uint16_t)(w[k] >> 16)), acc[2 * k + 1]);
      }
    }
  };
  float sum = 0.f;
  if (e_hi > e_lo) {
    const u32x4* col8 = reinterpret_cast<const u32x4*>(A.col);
    const u32x4* val8 = reinterpret_cast<const u32x4*>(A.val);
    const int g_lo = e_lo >> 3, ngran = ((e_hi - 1) >> 3) - g_lo + 1;
    // this pair's part of an ordinary row (empty for a long row)
    int a, z;
    {
      const int r = pr / PER_ROW;
      const int lo = rp[r], hi = rp[r + 1], len = hi - lo;
      const int per = (len + PER_ROW - 1) / PER_ROW;
      a = min(lo + (pr % PER_ROW) * per, hi);
      z = len <= long_row ? min(a + per, hi) : a;
    }
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    for (int ch = 0; ch * kFinishThreads < ngran; ++ch) {         // workgroup-uniform
      const int e0 = 8 * (g_lo + ch * kFinishThreads), e1 = e0 + CHUNK;   // the chunk's entries
      bool skip = false;                     // nothing but one long row in it
#pragma unroll
      for (int r = 0; r < TR; ++r) skip = skip || (rp[r + 1] - rp[r] > long_row && rp[r] <= max(e0, e_lo) && rp[r + 1] >= min(e1, e_hi));
      if (skip) continue;
      const int gi = ch * kFinishThreads + tid;
      const u32x4 none = {0u, 0u, 0u, 0u};
      const u32x4 nc = gi < ngran ? col8[g_lo + gi] : none, nv = gi < ngran ? val8[g_lo + gi] : none;
      __syncthreads();                       // the previous chunk is consumed
      reinterpret_cast<u32x4*>(scol)[tid] = nc;
      reinterpret_cast<u32x4*>(sval)[tid] = nv;
      __syncthreads();
      for (int e = max(a, e0); e < min(z, e1); e += 4) consume(e0, e - e0, a, min(z, e1), acc);
    }
#pragma unroll
    for (int k2 = 0; k2 < 8; ++k2) part[pr][8 * bq + k2] = acc[k2];
    __syncthreads();
    if (g < TR) {
      const int lo = rp[g], hi = rp[g + 1];
      if (hi - lo <= long_row) {
#pragma unroll
        for (int k = 0; k < PER_ROW; ++k) sum += part[g * PER_ROW + k][b];
      } else {
        for (int e0 = lo; e0 < hi; e0 += kLongSlice) sum += slots[(int64_t)(lo / kSlotGrain + (e0 - lo) / kLongSlice) * 16 + b];
      }
    }
  }
  if (g < TR && s * TR + g < m && b < batch && (rp[g + 1] > rp[g] || !inplace)) {
    if (y_dtype == SPQR_F32) static_cast<float*>(Y)[at] = dense + sum;
    else static_cast<uint16_t*>(Y)[at] = f2h_rne(dense + sum);
  }
}

__global__ void __launch_bounds__(kFinishThreads, 8)
finish_xt16_kernel(DevMatrix A, const uint16_t* __restrict__ XT, const float* __restrict__ slots, const float* P,
                   int nsplit, int64_t split_stride, int long_row, void* Y, int y_dtype, int batch) {
  finish_xt16_body(A, XT, slots, P, nsplit, split_stride, long_row, Y, y_dtype, batch, (int)blockIdx.x);
}

__global__ void __launch_bounds__(kFinishThreads, 8)
finish_xt16_fused_kernel(MfmaFused F, const uint16_t* __restrict__ XT, int nsplit, int y_dtype, int batch) {
  int bx = blockIdx.x, i = 0;
  for (; i < F.count - 1; ++i) {             // workgroup-uniform
    if (bx < F.it[i].blocks16) break;
    bx -= F.it[i].blocks16;
  }
  const MfmaFusedItem& it = F.it[i];
  finish_xt16_body(it.A, XT, it.slots, it.P, nsplit, (int64_t)batch * it.A.g.m, it.long_row, it.Y, y_dtype, batch, bx);
}

// Several matrices that share the input vector and the format (q/k/v, gate/up of
// a decoder block) in one grid: strips [first[i], first[i+1]) belong to matrix i.
// Every workgroup does exactly what it would do in a launch of its own matrix.
struct FusedArgs {
  int count;
  int first[SPQR_MAX_FUSED + 1];
  Geometry g;                                // of matrix 0; m and ntr differ per matrix and are not used by the body
  const uint8_t* packed[SPQR_MAX_FUSED];
  const int32_t* row_ptr[SPQR_MAX_FUSED];
  const uint16_t* col[SPQR_MAX_FUSED];
  const uint16_t* val[SPQR_MAX_FUSED];
  void* y[SPQR_MAX_FUSED];
};

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__((64 * WavesPerGroup<W, 1>::MAX))
gemv_tile256_fused_kernel(FusedArgs F, const uint16_t* __restrict__ x, int y_dtype, int chunk_cap) {
  int i = 0;
  while (i + 1 < F.count && (int)blockIdx.x >= F.first[i + 1]) ++i;   // workgroup-uniform, count <= SPQR_MAX_FUSED
  DevMatrix A;
  A.g = F.g;
  A.packed = F.packed[i]; A.row_ptr = F.row_ptr[i]; A.col = F.col[i]; A.val = F.val[i];
  A.perm = nullptr; A.nnz = 0;
  gemv_tile256_body<W, TR, TC, AXIS, false, 1>(A, x, F.y[i], y_dtype, chunk_cap, (int)blockIdx.x - F.first[i]);
}

// ---------------------------------------------------------------------------
// Generic fallback product: any supported geometry, one wavefront per output
// row, element-wise canonical decode.  Slow; used when no tuned kernel matches.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gemv_generic_kernel(DevMatrix A, const uint16_t* __restrict__ x, void* __restrict__ y, int y_dtype) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= A.g.m) return;                    // whole wavefront leaves together
  float s = 0.f;
  for (int j = lane; j < A.g.n; j += 64) {
    const float xv = h2f(x[A.perm ? A.perm[j] : j]);
    s = fmaf(dense_value(A.g, A.packed, i, j), xv, s);
  }
  for (int e = A.row_ptr[i] + lane; e < A.row_ptr[i + 1]; e += 64) {
    const int j = A.col[e];
    s = fmaf(h2f(A.val[e]), h2f(x[A.perm ? A.perm[j] : j]), s);
  }
  s = wave_allreduce(s, lane);
  if (lane == 0) {
    if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
    else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
  }
}

// ---------------------------------------------------------------------------
// Debug decode kernels.
// ---------------------------------------------------------------------------
__global__ void codes_u8_kernel(DevMatrix A, uint8_t* out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)A.g.m * A.g.n) return;
  const int i = (int)(idx / A.g.n), j = (int)(idx % A.g.n);
  out[idx] = (uint8_t)tile_code(A.g, A.packed, i / A.g.tile_rows, j / A.g.tile_cols,
                                i % A.g.tile_rows, j % A.g.tile_cols);
}

__global__ void stats_f32_kernel(DevMatrix A, float* out, int want_zero) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t grows = A.g.axis == 0 ? A.g.m : A.g.m / A.g.beta1;
  const int64_t gcols = A.g.axis == 0 ? A.g.n / A.g.beta1 : A.g.n;
  if (idx >= grows * gcols) return;
  const int gr = (int)(idx / gcols), gc = (int)(idx % gcols);
  int tr, tc, gi;
  if (A.g.axis == 0) { tr = gr / A.g.beta2; gi = gr % A.g.beta2; tc = gc; }
  else               { tr = gr; tc = gc / A.g.beta2; gi = gc % A.g.beta2; }
  float s_hat, z_hat;
  tile_group_stats(A.g, A.packed, tr, tc, gi, &s_hat, &z_hat);
  out[idx] = want_zero ? z_hat : s_hat;
}

template <typename OutT>
__device__ __forceinline__ void store_dense(OutT* out, int64_t idx, float v);
template <> __device__ __forceinline__ void store_dense<float>(float* out, int64_t idx, float v) { out[idx] = v; }
template <> __device__ __forceinline__ void store_dense<uint16_t>(uint16_t* out, int64_t idx, float v) { out[idx] = f2h_rne(v); }

template <typename OutT>
__global__ void dense_kernel(DevMatrix A, OutT* out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)A.g.m * A.g.n) return;
  store_dense<OutT>(out, idx, dense_value(A.g, A.packed, (int)(idx / A.g.n), (int)(idx % A.g.n)));
}

// Row of CSR entry e: largest i with row_ptr[i] <= e (row_ptr validated or trusted).
__device__ inline int csr_row_of(const int32_t* row_ptr, int m, int64_t e) {
  int lo = 0, hi = m;                        // invariant: row_ptr[lo] <= e < row_ptr[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (row_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

// Re-evaluates the positions that carry an outlier: dense value + outlier value,
// rounded once to the output type.
template <typename OutT>
__global__ void dense_outlier_kernel(DevMatrix A, OutT* out) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= A.nnz) return;
  const int i = csr_row_of(A.row_ptr, A.g.m, e);
  const int j = A.col[e];
  const float v = __fadd_rn(dense_value(A.g, A.packed, i, j), h2f(A.val[e]));
  store_dense<OutT>(out, (int64_t)i * A.g.n + j, v);
}

// ---------------------------------------------------------------------------
// Validation kernels.  *flag receives the first error class seen (any of them).
// ---------------------------------------------------------------------------
__global__ void fill_int_kernel(int* p, int v) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = v; }

__global__ void check_rowptr_kernel(DevMatrix A, int* flag) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > A.g.m) return;
  const int64_t v = A.row_ptr[i];
  bool bad = v < 0 || v > A.nnz;
  if (i == 0 && v != 0) bad = true;
  if (i == A.g.m && v != A.nnz) bad = true;
  if (i < A.g.m && (int64_t)A.row_ptr[i + 1] < v) bad = true;
  if (i < A.g.m && (int64_t)A.row_ptr[i + 1] - v > A.g.n) bad = true;
  if (bad) atomicMin(flag, SPQR_ERR_CSR);
}

__global__ void check_entries_kernel(DevMatrix A, int check_csr, int check_finite, int* flag) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= A.nnz) return;
  if (check_csr) {
    const int i = csr_row_of(A.row_ptr, A.g.m, e);
    const int c = A.col[e];
    bool bad = c >= A.g.n;
    if (e > A.row_ptr[i] && A.col[e - 1] >= c) bad = true;
    if (bad) atomicMin(flag, SPQR_ERR_CSR);
  }
  if (check_finite && (A.val[e] & 0x7C00u) == 0x7C00u) atomicMax(flag + 1, 1);
}

__global__ void check_stats2_kernel(DevMatrix A, int* flag) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)A.g.ntr * A.g.ntc) return;
  const int tr = (int)(t / A.g.ntc), tc = (int)(t % A.g.ntc);
  const uint32_t a = ld32(A.packed, stat_dword_offset(A.g, tr, tc, A.g.sd - 2));
  const uint32_t b = ld32(A.packed, stat_dword_offset(A.g, tr, tc, A.g.sd - 1));
  const bool bad = (a & 0x7C00u) == 0x7C00u || (a & 0x7C000000u) == 0x7C000000u
                || (b & 0x7C00u) == 0x7C00u || (b & 0x7C000000u) == 0x7C000000u;
  if (bad) atomicMax(flag + 1, 1);
}

__global__ void check_perm_kernel(DevMatrix A, int* flag) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= A.g.n) return;
  const int p = A.perm[j];
  if (p < 0 || p >= A.g.n) atomicMax(flag + 2, 1);
}

// Device-side result words of spqr_pack_check: [0] CSR status, [1] non-finite, [2] perm.
__device__ int g_check_words[4];

// ---------------------------------------------------------------------------
// Launchers.
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// Launch plan of the fused kernel.
//
// LDS: x (NB vectors), then 32 bytes per outlier chunk and vector of a round.  A
// round holds at least one chunk per thread (the common, single-barrier path)
// and up to eight.  Static arrays (red, osum, lred, rp) come on top; the
// sum must stay within the CU's 160 KB.
//
// Wavefronts per workgroup: a strip has nsteps steps of 64 tiles.  With w
// wavefronts a CU holds floor(slots / w) workgroups (slots = wavefront slots at
// the kernel's register count, LDS permitting) and the steps split evenly only
// if w divides them; the plan maximises the wavefronts resident on a CU.
// ---------------------------------------------------------------------------
static constexpr int kCUs = 256;
static constexpr int static_lds_bytes(int tr, int nb) {
  return ((16 * nb * tr + nb * tr + 32 + nb * tr * 16 + tr + 1) * 4 + 1023) & ~1023;
}
struct LaunchPlan { int nw; int cap; size_t lds; };

static bool plan_launch(const Geometry& g, int nb, int max_waves, int slots, LaunchPlan* out) {
  const int nsteps = (g.ntc + 63) / 64;
  const int xbytes = (nb * g.n * 2 + 15) & ~15;
  const int max_dynamic = 160 * 1024 - static_lds_bytes(g.tile_rows, nb) - 1024;
  double best = -1.0;
  // a plan whose x vectors leave LDS for only a sliver of a workgroup is not worth having
  const int widest = max_waves < nsteps ? max_waves : nsteps;
  if (xbytes + 32 * nb * 64 * ((widest + 1) / 2) > max_dynamic) return false;
  // SPQR_PLAN_WAVES=k in the environment pins the wavefronts per workgroup (tuning runs)
  int pinned = 0;
  if (const char* e = std::getenv("SPQR_PLAN_WAVES")) pinned = std::atoi(e);
  for (int w = 1; w <= max_waves && w <= nsteps; ++w) {
    if (pinned > 0 && w != pinned && pinned <= max_waves && pinned <= nsteps) continue;
    int groups = slots / w; if (groups < 1) groups = 1;
    // LDS one workgroup needs at least: x + one chunk per thread
    const int need = xbytes + 32 * nb * 64 * w;
    if (need > max_dynamic) continue;
    const int by_lds = (160 * 1024) / (need + static_lds_bytes(g.tile_rows, nb) + 1024);
    if (groups > by_lds) groups = by_lds;
    if (groups < 1) continue;
    const int wanted = (g.ntr + kCUs - 1) / kCUs;      // a small grid never puts more workgroups on a CU
    const int share = groups < wanted ? groups : wanted;
    // Score: closeness to the preferred workgroup width.  A wavefront pipelines its
    // steps (the next tile's loads fly under the current tile's arithmetic), so few
    // wide-enough workgroups beat many one-step wavefronts: 8 wavefronts when the
    // strip has 8 steps or more, else 4 (both spread evenly over the four SIMDs and
    // leave room for a second workgroup on the CU), else one per step.  Fitted to
    // timings of the benchmark layers on MI355X.
    const int cap8 = max_waves < 8 ? max_waves : 8;
    const int target = nsteps < 4 ? nsteps : ((nsteps < cap8 ? nsteps : cap8) / 4) * 4;
    int resident = w * share; if (resident > slots) resident = slots;
    double score = 100.0 - (w > target ? 1.5 * (w - target) : (target - w)) + 1e-3 * resident;
    if (nb > 1) {
      // several activation vectors: arithmetic dominates, so what counts is wavefronts
      // resident on the CU and an even split of the steps among them
      const int per_wave = (nsteps + w - 1) / w;
      const double even = (double)nsteps / ((double)w * per_wave);
      score = (double)resident * (0.75 + 0.25 * even) * (w % 4 == 0 ? 1.05 : 1.0) * (share >= 2 ? 1.03 : 1.0) + 1e-3 * w;
    }
    if (score > best) {
      best = score;
      // give the outlier products the LDS this occupancy leaves over, up to 4 chunks per thread
      int room = ((160 * 1024) / share - static_lds_bytes(g.tile_rows, nb) - 1024 - xbytes) / (32 * nb);
      if (room > (max_dynamic - xbytes) / (32 * nb)) room = (max_dynamic - xbytes) / (32 * nb);
      int cap = room < 8 * 64 * w ? room : 8 * 64 * w;
      out->nw = w; out->cap = cap; out->lds = (size_t)xbytes + (size_t)32 * nb * cap;
    }
  }
  return best > 0.0;
}

// Function attributes (the opt-in for more than 64 KB of dynamic LDS) are per device, and
// several host threads may arrive here at once: what is remembered per kernel is kept per
// device in atomics; a device number out of range is simply not remembered.
constexpr int kMaxDevices = 64;
struct PerDevice {
  std::atomic<int> v[kMaxDevices];
  int get(int d) const { return d >= 0 && d < kMaxDevices ? v[d].load(std::memory_order_acquire) : 0; }
  void set(int d, int x) { if (d >= 0 && d < kMaxDevices) v[d].store(x, std::memory_order_release); }
};
static int current_device() {
  int d = -1;
  return hipGetDevice(&d) == hipSuccess ? d : -1;
}

template <int W, int TR, int TC, int AXIS, int NB>
static hipError_t launch_tile256(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                                 hipStream_t stream) {
  constexpr int MAXW = WavesPerGroup<W, NB>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, NB) - 1024;   // static + dynamic <= 160 KB
  // once per kernel: register count (-> wavefront slots per CU) and the opt-in for > 64 KB of dynamic LDS
  static PerDevice known[2];                 // wavefront slots per CU of the instance, 0 = not asked yet
  const int pi = A.perm ? 1 : 0, dev = current_device();
  int slots = known[pi].get(dev);
  if (slots == 0) {
    const void* fn = A.perm ? reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, true, NB>)
                            : reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, false, NB>);
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, fn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_DYNAMIC);
    if (e != hipSuccess) return e;
    int regs = (fa.numRegs + 7) & ~7; if (regs < 64) regs = 64;
    int per_simd = 512 / regs; if (per_simd > 8) per_simd = 8; if (per_simd < 1) per_simd = 1;
    slots = 4 * per_simd;
    known[pi].set(dev, slots);
  }
  LaunchPlan plan = {0, 0, 0};
  if (!plan_launch(A.g, NB, MAXW, slots, &plan)) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.cap < 64 * plan.nw) return hipErrorInvalidValue;
  if (A.perm)
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, true, NB>), dim3(A.g.ntr), dim3(64 * plan.nw),
                       plan.lds, stream, A, x, y, y_dtype, plan.cap);
  else
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, false, NB>), dim3(A.g.ntr), dim3(64 * plan.nw),
                       plan.lds, stream, A, x, y, y_dtype, plan.cap);
  return hipGetLastError();
}

// Largest number of activation vectors (1, 2 or 4, at most `want`) one launch of
// the tuned kernel can take for this geometry; 0 if there is no tuned kernel.
int tuned_batch_width(const Geometry& g, int want) {
  if (g.tile_rows * g.tile_cols != 256) return 0;
  const bool shape_ok = g.axis == 1 ? ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 8 && g.tile_cols == 32))
                                    : ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 32 && g.tile_cols == 8));
  if (!shape_ok) return 0;
  for (int nb = want >= 4 ? 4 : (want >= 2 ? 2 : 1); nb >= 1; nb >>= 1) {
    LaunchPlan plan = {0, 0, 0};
    const int maxw = (g.w_bits == 3 && nb == 1) ? 16 : 8;
    if (plan_launch(g, nb, maxw, 8, &plan)) return nb;   // 8 slots: the lowest occupancy any instance has
  }
  return 0;
}

bool has_tuned_gemv(const Geometry& g) { return tuned_batch_width(g, 1) == 1; }

template <int NB>
static hipError_t launch_tuned(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream) {
  const Geometry& g = A.g;
#define SPQR_CASE(W_, TR_, TC_, AX_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
    return launch_tile256<W_, TR_, TC_, AX_, NB>(A, x, y, y_dtype, stream);
  SPQR_CASE(3, 16, 16, 1) SPQR_CASE(4, 16, 16, 1) SPQR_CASE(3, 8, 32, 1) SPQR_CASE(4, 8, 32, 1)
  SPQR_CASE(3, 16, 16, 0) SPQR_CASE(4, 16, 16, 0) SPQR_CASE(3, 32, 8, 0) SPQR_CASE(4, 32, 8, 0)
#undef SPQR_CASE
  return hipErrorInvalidValue;
}

// ---- batches above 4 on 16x16 tiles: matrix-core dense pass + outlier pass ----
// Steps per workgroup of the dense pass, chosen by simulating the launch: the workgroups start in grid order
// (split by split: the strip groups, behind those of the first split the long-row workgroups) on the first free of
// the chip's workgroup slots; a dense workgroup costs its steps plus a start-up of 0.3 step, a long-row workgroup
// 0.45 step, and every split 0.3 step for its partial result (written, and read again by the finishing kernel).
// The shortest schedule wins, ties go to fewer splits.  The constants are fitted to sweeps over the steps on
// MI355X (eight projection shapes of the 7B to 65B configurations at batch 8 and 16, every count of steps: the choice is
// within 2.2 % of the best measured one).  slots1 = slots when a workgroup takes one step (the variant with fewer registers),
// slots = otherwise.  Results are remembered per argument tuple (the simulation costs up to a few milliseconds).
static double mfma_schedule_length(int groups, int nsteps, int s, int slots, int nlong) {
  const int nsplit = (nsteps + s - 1) / s;
  std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
  for (int i = 0; i < slots; ++i) free_at.push(0.0);
  double end = 0.0;
  auto run = [&](int count, double cost) {
    for (int i = 0; i < count; ++i) {
      const double t = free_at.top() + cost;
      free_at.pop();
      free_at.push(t);
      if (t > end) end = t;
    }
  };
  for (int y = 0; y < nsplit; ++y) {
    const int steps = s < nsteps - y * s ? s : nsteps - y * s;
    run(groups, 0.3 + steps);
    run(nlong, y == 0 ? 0.45 : 0.02);         // behind the first split they leave at once
  }
  return end + 0.3 * nsplit;
}

// Scratch of the batch path.  A call on a stream that is not being captured takes the buffer the library keeps for
// that stream: work on one stream runs in order, so its calls can share one buffer, and nothing is allocated or
// freed per call (on this runtime a stream-ordered allocation waits on the host until the stream's earlier work is
// done, which keeps the next call's launches from being queued behind the running one: about 5 us per call).  The
// buffer grows when a call needs more (the stream is synchronised first) and is kept until the process ends; up to
// kScratchStreams streams per device have one; further streams allocate stream-ordered from a memory pool of the
// library's own (one per device, unlimited release threshold), captured calls from the device's default pool, which
// the capture turns into allocation nodes of the graph (graphs of many such calls replay correctly with it; with the
// library's own pool the allocations of all but the first call of a capture failed).  A buffer's lock is held while its call is enqueued: calls from several host
// threads on one stream do not interleave their kernels.
constexpr int kScratchStreams = 8;
struct ScratchSlot {
  std::mutex lock;                           // held while a call that uses the buffer is enqueued
  hipStream_t stream = nullptr;
  uint8_t* buf = nullptr;
  size_t size = 0;
  bool taken = false;
};
struct Scratch {
  uint8_t* p = nullptr;
  bool pooled = false;                       // stream-ordered allocation, to be freed on the stream
  std::unique_lock<std::mutex> hold;
};

static hipMemPool_t scratch_pool(int dev) {
  static std::mutex lock;
  static hipMemPool_t pools[kMaxDevices];
  static bool tried[kMaxDevices];
  if (dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  if (!tried[dev]) {
    tried[dev] = true;
    hipMemPoolProps props = {};
    props.allocType = hipMemAllocationTypePinned;
    props.handleTypes = hipMemHandleTypeNone;
    props.location.type = hipMemLocationTypeDevice;
    props.location.id = dev;
    hipMemPool_t pool = nullptr;
    if (hipMemPoolCreate(&pool, &props) == hipSuccess) {
      uint64_t keep = UINT64_MAX;
      if (hipMemPoolSetAttribute(pool, hipMemPoolAttrReleaseThreshold, &keep) == hipSuccess) pools[dev] = pool;
      else (void)hipMemPoolDestroy(pool);
    }
    if (pools[dev] == nullptr) (void)hipGetLastError();
  }
  return pools[dev];
}

// hipErrorNotSupported: no scratch to be had (the caller takes the vector path).
static hipError_t scratch_get(Scratch* sc, size_t bytes, int dev, hipStream_t stream) {
  static std::mutex table_lock;
  static ScratchSlot slots[kMaxDevices][kScratchStreams];
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  const bool capturing = hipStreamIsCapturing(stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
  ScratchSlot* slot = nullptr;
  if (!capturing && dev >= 0 && dev < kMaxDevices) {
    std::lock_guard<std::mutex> hold(table_lock);
    for (int i = 0; i < kScratchStreams && slot == nullptr; ++i)
      if (slots[dev][i].taken && slots[dev][i].stream == stream) slot = &slots[dev][i];
    for (int i = 0; i < kScratchStreams && slot == nullptr; ++i)
      if (!slots[dev][i].taken) {
        slot = &slots[dev][i];
        slot->taken = true;
        slot->stream = stream;
      }
  }
  if (slot != nullptr) {
    sc->hold = std::unique_lock<std::mutex>(slot->lock);
    if (slot->size < bytes) {
      // the stream's earlier calls may still read the old buffer
      if (slot->buf != nullptr && (hipStreamSynchronize(stream) != hipSuccess || hipFree(slot->buf) != hipSuccess)) {
        (void)hipGetLastError();
        sc->hold.unlock();
        return hipErrorNotSupported;
      }
      slot->buf = nullptr;
      slot->size = 0;
      const size_t want = (bytes + bytes / 4 + 0xFFFFF) & ~(size_t)0xFFFFF;   // some room, whole megabytes
      if (hipMalloc(reinterpret_cast<void**>(&slot->buf), want) != hipSuccess) {
        (void)hipGetLastError();
        slot->buf = nullptr;
        sc->hold.unlock();
        return hipErrorNotSupported;
      }
      slot->size = want;
    }
    sc->p = slot->buf;
    sc->pooled = false;
    return hipSuccess;
  }
  // captured: the device's default pool (allocation nodes of the graph); else the library's own pool
  hipMemPool_t pool = capturing ? nullptr : scratch_pool(dev);
  const hipError_t e = pool != nullptr ? hipMallocFromPoolAsync(reinterpret_cast<void**>(&sc->p), bytes, pool, stream)
                                       : hipMallocAsync(reinterpret_cast<void**>(&sc->p), bytes, stream);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    sc->p = nullptr;
    return hipErrorNotSupported;
  }
  sc->pooled = true;
  return hipSuccess;
}
// after the call's last kernel is enqueued
static hipError_t scratch_put(Scratch* sc, hipStream_t stream) {
  hipError_t e = hipSuccess;
  if (sc->pooled && sc->p != nullptr) e = hipFreeAsync(sc->p, stream);
  if (sc->hold.owns_lock()) sc->hold.unlock();
  sc->p = nullptr;
  return e;
}

// Workgroups for the long outlier rows of a matrix: each owns an equal share of the entries (see long_rows_block)
// and pays a look at the row pointers whether its share holds long rows or not: one per strip of 16 rows, 128 at most.
static int long_row_workgroups(const DevMatrix& A) {
  if (A.nnz <= 0) return 0;
  const int strips = (A.g.m + 15) / 16;
  return strips < kCUs / 2 ? strips : kCUs / 2;
}

static int mfma_steps_per_split(int groups, int nsteps, int slots1, int slots, int nlong) {
  if (const char* e = std::getenv("SPQR_MFMA_STEPS")) {        // pins it for tuning runs
    const int v = std::atoi(e);
    if (v >= 1) return v < nsteps ? v : nsteps;
  }
  struct Known { int groups, nsteps, slots1, slots, nlong, best; };
  static std::mutex lock;
  static std::vector<Known> known;
  {
    std::lock_guard<std::mutex> hold(lock);
    for (const Known& k : known)
      if (k.groups == groups && k.nsteps == nsteps && k.slots1 == slots1 && k.slots == slots && k.nlong == nlong) return k.best;
  }
  int best = nsteps;
  double best_cost = 1e30;
  // candidates: every count of steps up to 32, and all of them in one workgroup; launches of more than
  // 200 000 workgroups are not simulated (only very large matrices: any choice fills the chip)
  for (int s = nsteps; s >= 1; s = (s > 32 ? 32 : s - 1)) {
    const long wgs = (long)(groups + nlong) * ((nsteps + s - 1) / s);
    if (wgs > 200000) continue;
    const double cost = mfma_schedule_length(groups, nsteps, s, s == 1 ? slots1 : slots, nlong);
    if (cost < best_cost - 1e-9) { best_cost = cost; best = s; }
  }
  std::lock_guard<std::mutex> hold(lock);
  if (known.size() < 4096) known.push_back(Known{groups, nsteps, slots1, slots, nlong, best});
  return best;
}

int plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups) {
  return mfma_steps_per_split(groups, nsteps, slots_one_step, slots, long_workgroups);
}

// Transposition, dense pass (with the long outlier rows beside it) and finishing pass.  Scratch (the batch
// transposed, (n+1) x 32 bytes, the sums of the long outlier rows, 64 bytes per 256 outliers, the batch in the
// matrix's column order if there is a permutation, and the partial results when the steps are split or the
// output is binary16): see scratch_get.
// hipErrorNotSupported = no scratch to be had; the caller takes the vector path.
template <int W, int TR, int TC, int AXIS>
static hipError_t launch_mfma(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream) {
  using SH = MfmaShape<TR, TC>;
  const Geometry& g = A.g;
  static PerDevice ready;
  const int dev = current_device();
  if (!ready.get(dev)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<W, TR, TC, AXIS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e != hipSuccess) return e;
    ready.set(dev, 1);
  }
  const int groups = (g.ntr + SH::NS - 1) / SH::NS;
  const int nsteps = (g.ntc + 63) / 64;
  const bool sparse = A.nnz > 0, permuted = A.perm != nullptr;
  constexpr int kNT = 64 * SH::NS;
  const int extra = long_row_workgroups(A);
  // the one-step variant fits three workgroups on a CU while the staged batch rows leave the LDS for them
  const int wgs1 = (TC != 32 && 3 * ((size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW + 1024) <= 160 * 1024) ? 3 : SH::WGS;
  const int steps_per_split = mfma_steps_per_split(groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, extra);
  const int nsplit = (nsteps + steps_per_split - 1) / steps_per_split;
  // the dense kernel writes Y itself (16 bytes per store) if nothing has to be added or converted afterwards
  const bool direct = nsplit == 1 && y_dtype == SPQR_F32 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const size_t xt_bytes = sparse ? up(((size_t)g.n + 1) * 32) : 0;   // one more row: zeros
  const size_t slot_bytes = sparse ? up(((size_t)(A.nnz / kSlotGrain) + 2) * 64) : 0;
  const size_t xp_bytes = permuted ? up((size_t)b * g.n * 2) : 0;
  const size_t part_bytes = direct ? 0 : (size_t)nsplit * b * g.m * sizeof(float);
  Scratch sc;
  if (xt_bytes + slot_bytes + xp_bytes + part_bytes > 0 &&
      scratch_get(&sc, xt_bytes + slot_bytes + xp_bytes + part_bytes, dev, stream) != hipSuccess)
    return hipErrorNotSupported;
  uint8_t* const scratch = sc.p;
  uint16_t* xt = sparse ? reinterpret_cast<uint16_t*>(scratch) : nullptr;
  float* slots = reinterpret_cast<float*>(scratch + xt_bytes);
  uint16_t* xp = permuted ? reinterpret_cast<uint16_t*>(scratch + xt_bytes + slot_bytes) : nullptr;
  float* part = direct ? static_cast<float*>(Y) : reinterpret_cast<float*>(scratch + xt_bytes + slot_bytes + xp_bytes);
  const int64_t split_stride = (int64_t)b * g.m;
  // a row is long if it holds far more outliers than the average row (and at least kLongRowMin): rows like the
  // average one stay with their strip's workgroup in the finishing kernel, whatever the outlier rate
  const int64_t avg_row = A.nnz / (g.m > 0 ? g.m : 1);
  const int long_row = (int)(4 * avg_row > kLongRowMin ? (4 * avg_row < (1 << 30) ? 4 * avg_row : (1 << 30)) : kLongRowMin);
  hipError_t e = hipSuccess;
  if (sparse || permuted) {
    hipLaunchKernelGGL(transpose_x16_kernel, dim3((g.n + 256) / 256), dim3(256), 0, stream, X, A.perm, xt, xp, g.n, b);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    if (steps_per_split == 1) {
      static PerDevice ready1;
      if (!ready1.get(dev)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_one_kernel<W, TR, TC, AXIS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
        if (e == hipSuccess) ready1.set(dev, 1);
      }
      const size_t lds_now = (size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW;   // only b rows of X are staged
      if (e == hipSuccess)
        hipLaunchKernelGGL((gemm_mfma_one_kernel<W, TR, TC, AXIS>), dim3(groups + extra, nsplit), dim3(kNT), lds_now,
                           stream, A, permuted ? xp : X, part, split_stride, b, xt, slots, long_row, groups);
    } else {
      hipLaunchKernelGGL((gemm_mfma_kernel<W, TR, TC, AXIS>), dim3(groups + extra, nsplit), dim3(kNT), SH::LDS,
                         stream, A, permuted ? xp : X, part, split_stride, steps_per_split, b, xt, slots, long_row, groups);
    }
    if (e == hipSuccess) e = hipGetLastError();
  }
  if (e == hipSuccess && (sparse || !direct)) {
    hipLaunchKernelGGL(finish_xt16_kernel, dim3((g.m + 15) / 16), dim3(kFinishThreads), 0, stream, A, xt, slots, part, nsplit,
                       split_stride, long_row, Y, y_dtype, b);
    e = hipGetLastError();
  }
  const hipError_t ef = scratch_put(&sc, stream);
  return e == hipSuccess ? ef : e;
}

// Whether a batch of b > 4 vectors takes the matrix-core path.  It pays two more launches and the
// transposition through LDS, the vector path re-reads the weights once per 4 vectors.  Measured on
// MI355X with eager calls the matrix cores win from 8 vectors on for any layer and from 5 on for layers
// of 30 M weights or more (4096^2 at b = 5 / 8 / 16: 15.4 / 15.7 / 18.0 us against 13.2 / 16.5 / 32.5;
// 11008x4096: 26.6 / 26.9 / 28.2 against 31.6 / 45.3 / 89.4).  In a captured call the scratch is an
// allocation node of the graph, about 10 us more per call: there from 13 vectors on for any layer,
// from 8 on for layers of 40 M weights and from 5 on for layers of 100 M.  SPQR_MFMA=0 / =1 in the
// environment (read per call) forces the vector / the matrix-core path wherever it applies (tests
// compare the two).
static bool mfma_wanted(const Geometry& g, int b, hipStream_t stream) {
  const char* e = std::getenv("SPQR_MFMA");
  if (e && e[0] == '0') return false;
  if (e && e[0] == '1') return true;
  const double weights = (double)g.m * (double)g.n;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  const bool capturing = hipStreamIsCapturing(stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
  if (capturing) return b >= 13 || (b >= 8 && weights >= 40e6) || weights >= 100e6;
  return b >= 8 || weights >= 30e6;
}

// Y[b][m] = X[b][n] . W_hat^T.  Up to 4 activation vectors: the tuned vector
// kernel, all of them in one launch.  More, on 16x16 tiles and where it pays: slices
// of up to 16 with the dense part on the matrix cores (weights stream once per
// slice), then the finishing kernel with the outliers.  Else slices of 4.
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, bool force_generic) {
  const Geometry& g = A.g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  // tile shapes the matrix-core kernel is built for: the ones the vector kernel is tuned for
  const bool shape16 = g.tile_rows == 16 && g.tile_cols == 16;
  const bool shape8x32 = g.tile_rows == 8 && g.tile_cols == 32 && g.axis == 1;
  const bool shape32x8 = g.tile_rows == 32 && g.tile_cols == 8 && g.axis == 0;
  bool mfma_ok = !force_generic && (g.w_bits == 3 || g.w_bits == 4) && (shape16 || shape8x32 || shape32x8);
  int k = 0;
  while (k < b) {
    const uint16_t* xk = X + (size_t)k * g.n;
    void* yk = static_cast<uint8_t*>(Y) + (size_t)k * g.m * ysz;
    const int left = b - k;
    hipError_t e;
    int done = 1;
    // the matrix-core path takes up to 16 vectors per pass over the weights
    const int nb16 = left < 16 ? left : 16;
    if (mfma_ok && left > 4 && mfma_wanted(g, nb16, stream)) {
      e = hipErrorNotSupported;
#define SPQR_MFMA_CASE(W_, TR_, TC_, AX_) \
      if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
        e = launch_mfma<W_, TR_, TC_, AX_>(A, xk, nb16, yk, y_dtype, stream);
      SPQR_MFMA_CASE(3, 16, 16, 1) SPQR_MFMA_CASE(3, 16, 16, 0) SPQR_MFMA_CASE(4, 16, 16, 1) SPQR_MFMA_CASE(4, 16, 16, 0)
      SPQR_MFMA_CASE(3, 8, 32, 1) SPQR_MFMA_CASE(4, 8, 32, 1) SPQR_MFMA_CASE(3, 32, 8, 0) SPQR_MFMA_CASE(4, 32, 8, 0)
#undef SPQR_MFMA_CASE
      if (e == hipErrorNotSupported) { mfma_ok = false; continue; }   // no memory pool here: the vector path from now on
      if (e != hipSuccess) return e;
      k += nb16;
      continue;
    }
    const int nb = force_generic ? 0 : tuned_batch_width(g, left);
    if (nb == 4) { e = launch_tuned<4>(A, xk, yk, y_dtype, stream); done = 4; }
    else if (nb == 2) { e = launch_tuned<2>(A, xk, yk, y_dtype, stream); done = 2; }
    else if (nb == 1) { e = launch_tuned<1>(A, xk, yk, y_dtype, stream); }
    else {
      const int rows_per_block = 4;
      hipLaunchKernelGGL(gemv_generic_kernel, dim3((g.m + rows_per_block - 1) / rows_per_block),
                         dim3(64 * rows_per_block), 0, stream, A, xk, yk, y_dtype);
      e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    k += done;
  }
  return hipSuccess;
}

// The batch path for several matrices that share X (n, format and permutation agree; checked by the caller):
// one transposition, one dense launch, one finishing launch for all of them.  b <= 16.
template <int W, int TR, int TC, int AXIS>
static hipError_t launch_mfma_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                                    hipStream_t stream) {
  using SH = MfmaShape<TR, TC>;
  const Geometry& g0 = As[0].g;
  static PerDevice ready;
  const int dev = current_device();
  if (!ready.get(dev)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_fused_kernel<W, TR, TC, AXIS, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_fused_kernel<W, TR, TC, AXIS, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e != hipSuccess) return e;
    ready.set(dev, 1);
  }
  constexpr int kNT = 64 * SH::NS;
  const int nsteps = (g0.ntc + 63) / 64;
  int total_groups = 0, total_extra = 0, extras[SPQR_MAX_FUSED];
  bool sparse = false;
  for (int i = 0; i < count; ++i) {
    const Geometry& g = As[i].g;
    total_groups += (g.ntr + SH::NS - 1) / SH::NS;
    sparse = sparse || As[i].nnz > 0;
    extras[i] = long_row_workgroups(As[i]);
    total_extra += extras[i];
  }
  const int wgs1 = (TC != 32 && 3 * ((size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW + 1024) <= 160 * 1024) ? 3 : SH::WGS;
  const int steps_per_split = mfma_steps_per_split(total_groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, total_extra);
  const int nsplit = (nsteps + steps_per_split - 1) / steps_per_split;
  const bool permuted = As[0].perm != nullptr;
  bool direct = nsplit == 1 && y_dtype == SPQR_F32;              // the dense kernel writes the outputs itself (16-byte stores)
  for (int i = 0; i < count; ++i) direct = direct && reinterpret_cast<uintptr_t>(Ys[i]) % 16 == 0;
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const size_t xt_bytes = sparse ? up(((size_t)g0.n + 1) * 32) : 0;
  const size_t xp_bytes = permuted ? up((size_t)b * g0.n * 2) : 0;
  size_t total = xt_bytes + xp_bytes, slot_off[SPQR_MAX_FUSED], part_off[SPQR_MAX_FUSED];
  for (int i = 0; i < count; ++i) {
    slot_off[i] = total;
    total += As[i].nnz > 0 ? up(((size_t)(As[i].nnz / kSlotGrain) + 2) * 64) : 0;
    part_off[i] = total;
    total += direct ? 0 : up((size_t)nsplit * b * As[i].g.m * sizeof(float));
  }
  Scratch sc;
  if (total > 0 && scratch_get(&sc, total, dev, stream) != hipSuccess) return hipErrorNotSupported;
  uint8_t* const scratch = sc.p;
  uint16_t* xt = sparse ? reinterpret_cast<uint16_t*>(scratch) : nullptr;
  uint16_t* xp = permuted ? reinterpret_cast<uint16_t*>(scratch + xt_bytes) : nullptr;
  MfmaFused F;
  F.count = count;
  int dense_blocks = 0, extra_blocks = 0, finish_blocks = 0;
  for (int i = 0; i < count; ++i) {
    MfmaFusedItem& it = F.it[i];
    const Geometry& g = As[i].g;
    it.A = As[i];
    it.Y = Ys[i];
    it.P = direct ? static_cast<float*>(Ys[i]) : reinterpret_cast<float*>(scratch + part_off[i]);
    it.slots = reinterpret_cast<float*>(scratch + slot_off[i]);
    const int64_t avg_row = As[i].nnz / (g.m > 0 ? g.m : 1);
    it.long_row = (int)(4 * avg_row > kLongRowMin ? (4 * avg_row < (1 << 30) ? 4 * avg_row : (1 << 30)) : kLongRowMin);
    it.groups = (g.ntr + SH::NS - 1) / SH::NS;
    it.extra = extras[i];
    it.blocks16 = (g.m + 15) / 16;
    dense_blocks += it.groups;
    extra_blocks += it.extra;
    finish_blocks += it.blocks16;
  }
  hipError_t e = hipSuccess;
  if (sparse || permuted) {
    hipLaunchKernelGGL(transpose_x16_kernel, dim3((g0.n + 256) / 256), dim3(256), 0, stream, X, As[0].perm, xt, xp, g0.n, b);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    if (steps_per_split == 1)                // the variant without the second tile; only b rows of X are staged
      hipLaunchKernelGGL((gemm_mfma_fused_kernel<W, TR, TC, AXIS, true>), dim3(dense_blocks + extra_blocks, nsplit), dim3(kNT),
                         (size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW, stream, F, permuted ? xp : X, 1, b, xt);
    else
      hipLaunchKernelGGL((gemm_mfma_fused_kernel<W, TR, TC, AXIS, false>), dim3(dense_blocks + extra_blocks, nsplit), dim3(kNT),
                         SH::LDS, stream, F, permuted ? xp : X, steps_per_split, b, xt);
    e = hipGetLastError();
  }
  if (e == hipSuccess && (sparse || !direct)) {
    hipLaunchKernelGGL(finish_xt16_fused_kernel, dim3(finish_blocks), dim3(kFinishThreads), 0, stream, F, xt, nsplit, y_dtype, b);
    e = hipGetLastError();
  }
  const hipError_t ef = scratch_put(&sc, stream);
  return e == hipSuccess ? ef : e;
}

// Y_i[b][m_i] = X[b][n] . W_hat_i^T for matrices that share X.  Batches the matrix-core path takes go through it
// fused (slices of 16); everything else is one launch_gemm per matrix.
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream, bool force_generic) {
  const Geometry& g = As[0].g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  const bool shape16 = g.tile_rows == 16 && g.tile_cols == 16;
  const bool shape8x32 = g.tile_rows == 8 && g.tile_cols == 32 && g.axis == 1;
  const bool shape32x8 = g.tile_rows == 32 && g.tile_cols == 8 && g.axis == 0;
  bool mfma_ok = count > 1 && !force_generic && (g.w_bits == 3 || g.w_bits == 4) && (shape16 || shape8x32 || shape32x8);
  // Not while the stream is being captured into a graph: a replay of a graph that held 12 fused batch calls among
  // 42 calls (a whole decoder block, six weight copies) ended in a memory fault inside the fused finishing kernel,
  // while the same calls pass eagerly and graphs of the per-matrix path replay correctly; until the cause is
  // known, captured calls take the per-matrix path.
  if (mfma_ok) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); cs = hipStreamCaptureStatusActive; }
    if (cs != hipStreamCaptureStatusNone) mfma_ok = false;
  }
  Geometry all = g;                          // the rule looks at the weights of all matrices together
  int64_t rows = 0;
  for (int i = 0; i < count; ++i) rows += As[i].g.m;
  all.m = (int)(rows < (1 << 30) ? rows : (1 << 30));
  int k = 0;
  while (k < b) {
    const int left = b - k, nb16 = left < 16 ? left : 16;
    const uint16_t* xk = X + (size_t)k * g.n;
    void* yk[SPQR_MAX_FUSED];
    for (int i = 0; i < count; ++i) yk[i] = static_cast<uint8_t*>(Ys[i]) + (size_t)k * As[i].g.m * ysz;
    if (mfma_ok && left > 4 && mfma_wanted(all, nb16, stream)) {
      hipError_t e = hipErrorNotSupported;
#define SPQR_MFMA_CASE(W_, TR_, TC_, AX_) \
      if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
        e = launch_mfma_fused<W_, TR_, TC_, AX_>(As, count, xk, nb16, yk, y_dtype, stream);
      SPQR_MFMA_CASE(3, 16, 16, 1) SPQR_MFMA_CASE(3, 16, 16, 0) SPQR_MFMA_CASE(4, 16, 16, 1) SPQR_MFMA_CASE(4, 16, 16, 0)
      SPQR_MFMA_CASE(3, 8, 32, 1) SPQR_MFMA_CASE(4, 8, 32, 1) SPQR_MFMA_CASE(3, 32, 8, 0) SPQR_MFMA_CASE(4, 32, 8, 0)
#undef SPQR_MFMA_CASE
      if (e == hipErrorNotSupported) { mfma_ok = false; continue; }
      if (e != hipSuccess) return e;
      k += nb16;
      continue;
    }
    // the rest of the batch, matrix by matrix (each call applies its own rule)
    for (int i = 0; i < count; ++i) {
      hipError_t e = launch_gemm(As[i], xk, left, yk[i], y_dtype, stream, force_generic);
      if (e != hipSuccess) return e;
    }
    k = b;
  }
  return hipSuccess;
}

hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                       hipStream_t stream, bool force_generic) {
  return launch_gemm(A, x, 1, y, y_dtype, stream, force_generic);
}

template <int W, int TR, int TC, int AXIS>
static hipError_t launch_fused256(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                                  int y_dtype, hipStream_t stream) {
  constexpr int MAXW = WavesPerGroup<W, 1>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, 1) - 1024;
  static PerDevice known;
  const int dev = current_device();
  int slots = known.get(dev);
  const void* fn = reinterpret_cast<const void*>(&gemv_tile256_fused_kernel<W, TR, TC, AXIS>);
  if (slots == 0) {
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, fn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_DYNAMIC);
    if (e != hipSuccess) return e;
    int regs = (fa.numRegs + 7) & ~7; if (regs < 64) regs = 64;
    int per_simd = 512 / regs; if (per_simd > 8) per_simd = 8; if (per_simd < 1) per_simd = 1;
    slots = 4 * per_simd;
    known.set(dev, slots);
  }
  FusedArgs F;
  F.count = count;
  F.g = As[0].g;
  int total = 0;
  for (int i = 0; i < count; ++i) {
    F.first[i] = total;
    total += As[i].g.ntr;
    F.packed[i] = As[i].packed; F.row_ptr[i] = As[i].row_ptr; F.col[i] = As[i].col; F.val[i] = As[i].val;
    F.y[i] = ys[i];
  }
  for (int i = count; i <= SPQR_MAX_FUSED; ++i) F.first[i] = total;
  for (int i = count; i < SPQR_MAX_FUSED; ++i) {
    F.packed[i] = nullptr; F.row_ptr[i] = nullptr; F.col[i] = nullptr; F.val[i] = nullptr; F.y[i] = nullptr;
  }
  Geometry all = As[0].g;                    // the plan sees the whole grid
  all.ntr = total;
  LaunchPlan plan = {0, 0, 0};
  if (!plan_launch(all, 1, MAXW, slots, &plan)) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.cap < 64 * plan.nw) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gemv_tile256_fused_kernel<W, TR, TC, AXIS>), dim3(total), dim3(64 * plan.nw), plan.lds, stream,
                     F, x, y_dtype, plan.cap);
  return hipGetLastError();
}

hipError_t launch_gemv_fused(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                             int y_dtype, hipStream_t stream, bool force_generic) {
  const Geometry& g = As[0].g;
  if (count > 1 && !force_generic && As[0].perm == nullptr && tuned_batch_width(g, 1) == 1) {
#define SPQR_CASE(W_, TR_, TC_, AX_) \
    if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
      return launch_fused256<W_, TR_, TC_, AX_>(As, count, x, ys, y_dtype, stream);
    SPQR_CASE(3, 16, 16, 1) SPQR_CASE(4, 16, 16, 1) SPQR_CASE(3, 8, 32, 1) SPQR_CASE(4, 8, 32, 1)
    SPQR_CASE(3, 16, 16, 0) SPQR_CASE(4, 16, 16, 0) SPQR_CASE(3, 32, 8, 0) SPQR_CASE(4, 32, 8, 0)
#undef SPQR_CASE
  }
  for (int i = 0; i < count; ++i) {
    hipError_t e = launch_gemv(As[i], x, ys[i], y_dtype, stream, force_generic);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_dequant(const DevMatrix& A, int what, void* out, hipStream_t stream) {
  const int sel = what & 0xFF;
  const bool with_outliers = (what & SPQR_OUT_WITH_OUTLIERS) != 0;
  const int64_t total = (int64_t)A.g.m * A.g.n;
  const int bs = 256;
  const unsigned nb = (unsigned)((total + bs - 1) / bs);
  switch (sel) {
    case SPQR_OUT_CODES_U8:
      hipLaunchKernelGGL(codes_u8_kernel, dim3(nb), dim3(bs), 0, stream, A, (uint8_t*)out);
      break;
    case SPQR_OUT_SCALE_F32:
    case SPQR_OUT_ZERO_F32: {
      const int64_t groups = total / A.g.beta1;
      hipLaunchKernelGGL(stats_f32_kernel, dim3((unsigned)((groups + bs - 1) / bs)), dim3(bs), 0, stream,
                         A, (float*)out, sel == SPQR_OUT_ZERO_F32 ? 1 : 0);
      break;
    }
    case SPQR_OUT_DENSE_F32:
      hipLaunchKernelGGL(dense_kernel<float>, dim3(nb), dim3(bs), 0, stream, A, (float*)out);
      if (with_outliers && A.nnz > 0)
        hipLaunchKernelGGL(dense_outlier_kernel<float>, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs),
                           0, stream, A, (float*)out);
      break;
    case SPQR_OUT_DENSE_F16:
      hipLaunchKernelGGL(dense_kernel<uint16_t>, dim3(nb), dim3(bs), 0, stream, A, (uint16_t*)out);
      if (with_outliers && A.nnz > 0)
        hipLaunchKernelGGL(dense_outlier_kernel<uint16_t>, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs),
                           0, stream, A, (uint16_t*)out);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Runs the selected device checks and copies the three result words to the host.
hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream) {
  int* words = nullptr;
  hipError_t e = hipGetSymbolAddress((void**)&words, HIP_SYMBOL(g_check_words));
  if (e != hipSuccess) return e;
  for (int k = 0; k < 3; ++k)
    hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(64), 0, stream, words + k, 0);
  const int bs = 256;
  if (csr) {
    hipLaunchKernelGGL(check_rowptr_kernel, dim3((A.g.m + 1 + bs - 1) / bs), dim3(bs), 0, stream, A, words);
    // Entry checks index through row_ptr: only run them on a valid prefix array.
    e = hipMemcpyAsync(host_words, words, sizeof(int), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return e;
    if (host_words[0] != 0) { host_words[1] = host_words[2] = 0; return hipSuccess; }
  }
  if ((csr || finite) && A.nnz > 0)
    hipLaunchKernelGGL(check_entries_kernel, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs), 0, stream,
                       A, csr ? 1 : 0, finite ? 1 : 0, words);
  if (finite) {
    const int64_t tiles = (int64_t)A.g.ntr * A.g.ntc;
    hipLaunchKernelGGL(check_stats2_kernel, dim3((unsigned)((tiles + bs - 1) / bs)), dim3(bs), 0, stream, A, words);
  }
  if (perm && A.perm)
    hipLaunchKernelGGL(check_perm_kernel, dim3((A.g.n + bs - 1) / bs), dim3(bs), 0, stream, A, words);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(host_words, words, 3 * sizeof(int), hipMemcpyDeviceToHost, stream);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(stream);
}

}  // namespace spqr
