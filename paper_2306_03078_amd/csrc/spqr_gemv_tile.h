// The fused decode + matvec kernel for tiles of 256 codes (Sec. 4.2 "Inference
// with SpQR", re-designed for CDNA4): device code only; launchers in spqr_gemv.hip.
//
//   one workgroup owns one strip of tile_rows output rows; its wavefronts split
//   the input dimension in steps of 64 tiles; one lane owns one whole tile per
//   step, so every load instruction of a wavefront reads one contiguous run of
//   the packed buffer (16 bytes per lane) and a tile's statistics are decoded
//   once and reused by all of its rows.  x is staged once per workgroup in LDS
//   (it also serves the outlier gather).  Codes are turned into binary16 values
//   K + q/2^b by one and-or per pair and multiplied with v_dot2_f32_f16 (fp32
//   accumulation); the offset K is removed per tile.  The strip's outliers (a
//   contiguous CSR range) are handled by the same workgroup, so y is written
//   once, without atomics, in a fixed order.
#pragma once
#include "../../include/spqr.h"
#include "spqr_tile.h"

namespace spqr {

// Row phases: the class of the pair in tile row r, column pair p depends on
// (r*PPR + p) % 16 for 3-bit codes, so rows repeat with period 16/PPR; 4-bit
// classes depend on p alone.
template <int W, int TC> struct RowPhases {
  static constexpr int N = (W == 4 || TC / 2 >= 16 || !SharedShifts<TC>::value) ? 1 : 16 / (TC / 2);
};

// Row dot products on the matrix cores.  The vector ALU is what bounds a launch much larger than the chip, and half
// of a tile's instructions are the v_dot2 of its code pairs.  v_mfma_f32_4x4x4_16b_f16 works on 16 independent
// blocks of 4 lanes: D_b[i][j] = sum_k A_b[i][k] * B_b[k][j], lane 4b + i supplying row i of A (4 binary16 values)
// and lane 4b + j column j of B.  With a lane's two extracted code pairs as its A values and the matching two pairs of
// u as its B values, the diagonal element D_b[l % 4][l % 4] is the lane's own dot product over four columns (the
// other twelve products of a block pair one lane's codes with another lane's activations and are ignored); it sits
// in register l % 4 of the lane's four result registers, whichever way the block's result is laid out.  One
// instruction replaces two v_dot2 and runs beside the vector ALU; a tile row keeps four accumulators instead of one.
#ifndef SPQR_ROW_DOTS_MFMA
#define SPQR_ROW_DOTS_MFMA 1
#endif
template <int W, int TR, int TC, int AXIS, int NB, int LV> struct RowDotsOnMatrixCores {
  static constexpr bool value = SPQR_ROW_DOTS_MFMA && W == 3 && TR == 8 && TC == 32 && AXIS == 1 && NB == 1 && LV == 1;
};
// Instances built for workgroups of at most 8 wavefronts (up to 168 registers at three wavefronts per SIMD): those with
// four accumulators per row, and strips of 32 rows (32 accumulators plus the class bookkeeping: 143 registers; under
// the 128 of a 16-wavefront workgroup they spilled, and 22016x8192 took 28.1 instead of 25.3 us).
template <int W, int TR, int TC, int AXIS, int NB, int LV> struct LargeRegisterBudget {
  static constexpr bool value = RowDotsOnMatrixCores<W, TR, TC, AXIS, NB, LV>::value || TR >= 32;
};
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

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
// (fp16(s0 * x.lo), fp16(s1 * x.hi)): the binary16 halves of xpair are widened inside the multiply and each
// product is rounded once, straight into its half of the result (two instructions per pair).
__device__ __forceinline__ uint32_t scaled_pair_f16(float s0, float s1, uint32_t xpair) {
  uint32_t u;
  asm("v_fma_mixlo_f16 %0, %1, %3, 0 op_sel_hi:[0,1,0]\n\t"
      "v_fma_mixhi_f16 %0, %2, %3, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]"
      : "=&v"(u) : "v"(s0), "v"(s1), "v"(xpair));
  return u;
}

// High halves of two dwords as one pair: (a >> 16) | (b & 0xFFFF0000).
__device__ __forceinline__ uint32_t high_halves(uint32_t a, uint32_t b) {
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// A tile wider than 32 columns (8 x 64, group_axis 1: Sec. 5's beta2 = 64) is worked off in column halves: TC is the
// width of the view, TCF the tile's, H the half; a half has whole 3-bit triples per row (TC / 2 = 16 pairs), so
// classes, phases and shifted words are those of an 8 x 32 tile.
// MF: the row dot products go to the matrix cores and accumulate in accm (four registers per row, the lane's own
// sum in register lane % 4); acc is then left alone.
template <int W, int TR, int TC, int AXIS, int NB, int LV, int TCF = TC, int H = 0, bool MF = false>
__device__ __forceinline__ void tile_fma(const TileRegs<W, TR, TCF, AXIS, LV>& t,
                                         const uint32_t* xpair /* TC/2 dwords in LDS, vector 0 */,
                                         int xstride, bool valid, float (&acc)[NB][TR], f32x4 (&accm)[MF ? TR : 1],
                                         float (&csum)[NB][RowPhases<W, TC>::N], const ClassConsts& k,
                                         const PairConsts& k1, const PairConsts& k3) {
  using T = TileRegs<W, TR, TCF, AXIS, LV>;
  static_assert(TCF == TC || (AXIS == 1 && TC == 32 && TCF == 2 * TC && H < 2), "column halves of an 8 x 64 tile");
  constexpr bool SHARED = SharedShifts<TC>::value;
  using CC = CodeClass<W, SHARED>;
  constexpr int PPR = TC / 2;                // pairs per row of the view
  constexpr int PPRF = TCF / 2;              // pairs per row of the tile
  constexpr int P0 = H * PPR;                // first pair of the view inside a row, first group pair of the view
  constexpr int NPH = RowPhases<W, TC>::N;
  constexpr float SCALE = (float)(1 << W);
  constexpr bool CODES = LV != 3;            // first-level statistics are 3-bit codes
  const half2_t ones = as_half2(k3.magic);
  // Second-level statistics: layout 1 holds both pairs, layout 2 (integer zero-point: z_hat = z_q) the scales'
  // pair only, which is layout 1 with s_z = 1, z_z = 0; layout 3 has binary16 (s_hat, z_hat) per group instead.
  const uint32_t a = CODES ? t.s[T::NC] : 0u;
  const float s_s = h2f((uint16_t)(a & 0xFFFF)), z_s = h2f((uint16_t)(a >> 16));
  float s_z = 1.f, z_z = 0.f;
  if constexpr (LV == 1) {
    const uint32_t b = t.s[T::NC + 1];
    s_z = h2f((uint16_t)(b & 0xFFFF)); z_z = h2f((uint16_t)(b >> 16));
  }
  // s_hat = s_s*(s_q - z_s) = c1*(1 + s_q/8) + c2.  A lane without a tile of its own
  // (it holds a copy of the block's last tile) runs the same code with s_hat = 0.
  // (Layout 3: s_hat = c1 * s with c1 = 1 or 0.)
  const float c1 = valid ? (CODES ? 8.f * s_s : 1.f) : 0.f, c2 = valid ? -s_s * z_s - 8.f * s_s : 0.f;
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
    // The statistic codes are 3-bit pairs in the weight codes' format.  With 3-bit weights (and shared shifts) they
    // are extracted the same way, in place, as K + code/8 with K by the pair's class: the scale's offset goes into the
    // additive constant of its class (c2k), the zero's offset leaves with the class sums the weight codes need
    // anyway, because pair PPR + p of the zero codes has the class of weight pair p in phase ZPH.
    constexpr bool STATS_IN_PLACE = W == 3 && SHARED && CODES;
    constexpr int ZPH = NPH == 1 ? 0 : 1;
    static_assert(!STATS_IN_PLACE || (PPR % 16 == 0 && NPH == 1) || (PPR == 8 && NPH == 2), "class of a zero-code pair");
    float c2k[3] = {c2, c2, c2};
    ShiftedWords<3> sws, swz;
    if constexpr (STATS_IN_PLACE) {
      using C3 = CodeClass<3, true>;
#pragma unroll
      for (int c = 0; c < 3; ++c) c2k[c] = valid ? fmaf(-8.f * (C3::K(c) - 1.f), s_s, -s_s * z_s - 8.f * s_s) : 0.f;
#pragma unroll
      for (int j = 0; j < 3; ++j) {           // the triples that hold the view's scale and zero codes
        sws.s[j] = t.s[3 * (P0 / 16) + j] >> 9;
        swz.s[j] = t.s[3 * ((T::B2 / 2 + P0) / 16) + j] >> 9;
      }
    }
    float Zd[NB];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) Zd[bi] = 0.f;
#pragma unroll
    for (int p = 0; p < PPR; ++p) {
      half2_t zq;
      float s0, s1;
      if constexpr (CODES) {
        const half2_t sq = as_half2(STATS_IN_PLACE ? pair_class_f16<3>(t.s, sws, P0 + p, k) : pair_f16<3>(t.s, P0 + p, k3));
        zq = as_half2(STATS_IN_PLACE ? pair_class_f16<3>(t.s, swz, T::B2 / 2 + P0 + p, k)
                                     : pair_f16<3>(t.s, T::B2 / 2 + P0 + p, k3));
        const float c2p = STATS_IN_PLACE ? c2k[CodeClass<3, true>::of_pair(p)] : c2;
        s0 = fmaf((float)sq.x, c1, c2p); s1 = fmaf((float)sq.y, c1, c2p);
      } else {                               // dword j of the statistics: s_hat_j | z_hat_j << 16
        const uint32_t d0 = t.s[2 * (P0 + p)], d1 = t.s[2 * (P0 + p) + 1];
        s0 = c1 * h2f((uint16_t)(d0 & 0xFFFF)); s1 = c1 * h2f((uint16_t)(d1 & 0xFFFF));
        zq = as_half2(high_halves(d0, d1));
      }
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        const half2_t u = as_half2(scaled_pair_f16(s0, s1, xp[bi][p]));
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
      float E[NPH];
#pragma unroll
      for (int h = 0; h < NPH; ++h) {
        E[h] = CC::K(0) * C[bi][h][0];
#pragma unroll
        for (int c = 1; c < CC::N; ++c) E[h] = fmaf(CC::K(c), C[bi][h][c], E[h]);
      }
      // zero codes extracted in place carry their class offsets: sum_j (K - 1) u_j = E[ZPH] - U
      const float zd = STATS_IN_PLACE ? Zd[bi] - E[ZPH] + U : Zd[bi];
      const float zu = CODES ? fmaf(e1, zd, e2 * U) : zd;          // layout 3: zq held z_hat itself
#pragma unroll
      for (int h = 0; h < NPH; ++h) csum[bi][h] += fmaf(SCALE, E[h], zu);
    }
    if constexpr (MF) {
      static_assert(NB == 1 && SHARED && PPR % 2 == 0, "two code pairs per matrix instruction");
#pragma unroll
      for (int r = 0; r < TR; ++r) {
        f32x4 d = accm[r];
#pragma unroll
        for (int p = 0; p < PPR; p += 2) {
          const int q = r * PPRF + P0 + p;
          refresh_shifted<W>(sw, t.c, q);
          const uint32_t qa = pair_class_f16<W>(t.c, sw, q, k);
          refresh_shifted<W>(sw, t.c, q + 1);
          const uint32_t qb = pair_class_f16<W>(t.c, sw, q + 1, k);
          typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
          const u32x2 a2 = {qa, qb}, b2 = {xp[0][p], xp[0][p + 1]};
          d = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, a2), __builtin_bit_cast(half4_t, b2), d, 0, 0, 0);
        }
        accm[r] = d;
      }
    } else {
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      float d[NB];
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) d[bi] = acc[bi][r];
#pragma unroll
      for (int p = 0; p < PPR; ++p) {
        const int q = r * PPRF + P0 + p;     // pair of the tile
        if constexpr (SHARED) refresh_shifted<W>(sw, t.c, q);
        const half2_t q2 = as_half2(SHARED ? pair_class_f16<W>(t.c, sw, q, k) : pair_f16<W>(t.c, q, k1));
#pragma unroll
        for (int bi = 0; bi < NB; ++bi) d[bi] = __builtin_amdgcn_fdot2(q2, as_half2(xp[bi][p]), d[bi], false);
      }
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) acc[bi][r] = d[bi];
    }
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
      half2_t sq, zq;
      if constexpr (CODES) {
        sq = as_half2(pair_f16<3>(t.s, r2, k3));
        zq = as_half2(pair_f16<3>(t.s, T::B2 / 2 + r2, k3));
      } else {                               // dword r of the statistics: s_hat_r | z_hat_r << 16
        sq = as_half2(__builtin_amdgcn_perm(t.s[2 * r2 + 1], t.s[2 * r2], 0x05040100u));   // the two low halves
        zq = as_half2(high_halves(t.s[2 * r2], t.s[2 * r2 + 1]));
      }
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
        const float sh = CODES ? fmaf((float)(h2 ? sq.y : sq.x), c1, c2) : c1 * (float)(h2 ? sq.y : sq.x);
        const float zh = CODES ? fmaf((float)(h2 ? zq.y : zq.x), e1, e2) : (float)(h2 ? zq.y : zq.x);   // z_hat_r
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

// Products of the 8 entries of one chunk.  A chunk at the edge of the workgroup's CSR range also holds entries
// of its neighbours' rows (or, behind the matrix's last entry, whatever follows in the granule): their
// products are parked like the others and never read, because the row sums only walk [row_ptr[r],
// row_ptr[r+1]) of the workgroup's own rows; a column index is clamped to n - 1 so that the read of x stays
// inside the staged vector whatever the entry holds.
__device__ __forceinline__ void chunk_products(const uint16_t* xs, uint32_t last_col,
                                               const u32x4& c8, const u32x4& v8, float (&p)[8]) {
  const uint32_t cw[4] = {c8.x, c8.y, c8.z, c8.w};
  const uint32_t vw[4] = {v8.x, v8.y, v8.z, v8.w};
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t col = (i & 1) ? (cw[i >> 1] >> 16) : (cw[i >> 1] & 0xFFFFu);
    const half2_t v2 = as_half2(vw[i >> 1]);
    const _Float16 xv = __builtin_bit_cast(_Float16, xs[min(col, last_col)]);
    p[i] = fmaf((float)((i & 1) ? v2.y : v2.x), (float)xv, 0.f);   // both binary16 sources widened inside the multiply
  }
}

__device__ __forceinline__ void store_products(float* prod, int slot, const float (&p)[8]) {
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
// Layout 3 keeps beta2 statistic dwords per tile instead of 8: it needs the 256.
// So does a tile of 512 codes (48 code registers per buffer).
// And so do the four accumulators per row of the instances whose row dot products run on the matrix cores (MF).
template <int W, int NB, int LV = 1, int CODES = 256, bool MF = false> struct WavesPerGroup {
  static constexpr int MAX = (W == 3 && NB == 1 && LV != 3 && CODES == 256 && !MF) ? 16 : 8;
};

// NB activation vectors per launch: X holds NB rows of n binary16 values (row
// stride n), Y NB rows of m outputs (row stride m).  NB = 1 is the GEMV.
// The workgroup owns the R consecutive strips from `first_strip` on (those that
// exist): R * TR <= RowsPerGroup rows, one contiguous CSR range.  Its wavefronts
// are dealt to the strips P each (the host makes the workgroup R * P wavefronts,
// R <= 8, and P <= steps of a strip); wavefront `part` of a strip takes the steps part,
// part + P, ...  One staging of x and one epilogue serve all R strips, and a
// wavefront that has several steps keeps the next tile's loads in flight under
// the current tile's arithmetic.
template <int TR, int NB> struct RowsPerGroup { static constexpr int MAX = NB == 1 ? 64 : TR; };

template <int W, int TR, int TC, int AXIS, bool PERM, int NB, int LV>
__device__ __forceinline__ void gemv_tile256_body(const DevMatrix& A, const uint16_t* __restrict__ x,
                                                  void* __restrict__ y, int y_dtype, int chunk_cap,
                                                  const int first_strip, const int R, const int P,
                                                  const bool shared_lds = false, const int spare_cap = 0) {
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  static_assert(TR * TC == 256 || (TR == 8 && TC == 64 && AXIS == 1), "tiles of 256 codes, or 8 x 64");
  static_assert((TC / 2) % 4 == 0, "x pairs are read as 16-byte LDS words");
  constexpr int TCV = TR * TC == 256 ? TC : TC / 2;      // columns tile_fma takes at a time
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr int MAX_WAVES = 16;
  constexpr int XCH = 4 * NB;                // 16-byte chunks of x a thread keeps in flight
  constexpr int KR = 4;                      // outlier chunks per thread requested ahead of the last dense step
  constexpr int KMAX = 8;                    // outlier chunks per thread and round at most
  constexpr int LONG_ROW = 512;              // rows with more entries are summed by all threads
  constexpr int ROWS_MAX = RowsPerGroup<TR, NB>::MAX;
  static_assert(ROWS_MAX <= 64 && ROWS_MAX % TR == 0, "one lane per row votes on long rows");

  // dynamic LDS: the NB x vectors | products of the outlier entries (8 floats per
  // chunk and vector).  shared_lds (one vector, no permutation; a launch whose LDS was sized for narrower matrices):
  // the products take the place of x once every wavefront is done with it -- they wait in registers for one more
  // barrier -- and a strip with more chunks than that holds goes through rounds of the `spare_cap` chunks that the
  // LDS behind x holds (x stays where it is), or, if that is less than a chunk per thread or would take more than two
  // rounds, through rounds of the whole LDS with x read from global memory.
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);
  const int n = A.g.n, ntc = A.g.ntc, m = A.g.m;
  const int xbytes = (NB * n * 2 + 15) & ~15;
  const bool alias = NB == 1 && !PERM && shared_lds;     // workgroup-uniform
  float* prod = reinterpret_cast<float*>(smem + (alias ? 0 : xbytes));
  const int pstride = 8 * chunk_cap;         // floats of products per vector
  __shared__ float red[MAX_WAVES][NB][TR];
  __shared__ float osum[NB][ROWS_MAX];
  __shared__ float lred[NB][ROWS_MAX][MAX_WAVES];
  __shared__ int rp[ROWS_MAX + 1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // scalar: step indices and tile bases stay in SGPRs
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int l16 = tid & 15, g16 = tid >> 4, ngroups = nthreads >> 4;
  const int nsteps = (ntc + 63) >> 6;
  // strip of this wavefront inside the workgroup, without a division: wave < R * P, R <= 8 (scalar compares)
  int sw = 0;
#pragma unroll
  for (int k = 1; k < 8; ++k) sw += (wave >= k * P) ? 1 : 0;
  const int part = wave - sw * P;
  const bool live = first_strip + sw < A.g.ntr;                  // wave-uniform; false: a strip behind the last one
  const int strip = min(first_strip + sw, A.g.ntr - 1);          // (the wavefront then adds zeros of the last strip)
  const int row0 = first_strip * TR;
  const int ROWS = min(R * TR, m - row0);    // rows of this workgroup
  const uint8_t* strip_base = A.packed + (int64_t)strip * ntc * TILE_BYTES;
  const int32_t* rpg = A.row_ptr + row0;

  // ---- issue order: row pointers and x first (small, mostly cache hits), then
  // the first tile.  Everything up to the barrier is straight-line code with
  // clamped indices instead of branches, so that the wait before staging x
  // covers the x loads only and never the big tile loads behind them. ------------
  const int e_lo = rpg[0], e_hi = rpg[ROWS]; // uniform: scalar loads
  const int rp_mine = rpg[min(tid, ROWS)];   // thread r <= ROWS carries row pointer r into LDS (ROWS < 64 R <= threads)
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
  int step = part;                           // part < P <= nsteps: the first step always exists
  int L0 = min(64, ntc - 64 * step), L1 = 1;
  load_tile<NB == 1>(t0, strip_base + (int64_t)64 * step * TILE_BYTES, L0, min(lane, L0 - 1));
  __builtin_amdgcn_sched_barrier(0);
  rp[min(tid, ROWS)] = rp_mine;              // clamped duplicates store the same value again

  if constexpr (!PERM) {
    u32x4* dst = reinterpret_cast<u32x4*>(xs);
#pragma unroll
    for (int k = 0; k < XCH; ++k)            // clamped duplicates store the same value again
      dst[min(tid + k * nthreads, nvec - 1)] = xr[k];
    // a long x (or several vectors): further batches of XCH chunks, the loads of a batch in flight together
    for (int i0 = tid + XCH * nthreads; i0 < nvec; i0 += XCH * nthreads) {
#pragma unroll
      for (int k = 0; k < XCH; ++k) xr[k] = reinterpret_cast<const u32x4*>(x)[min(i0 + k * nthreads, nvec - 1)];
#pragma unroll
      for (int k = 0; k < XCH; ++k) dst[min(i0 + k * nthreads, nvec - 1)] = xr[k];
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
  constexpr int NPH = RowPhases<W, TCV>::N;
  constexpr bool MF = RowDotsOnMatrixCores<W, TR, TC, AXIS, NB, LV>::value;
  float acc[NB][TR], csum[NB][NPH];
  f32x4 accm[MF ? TR : 1];
#pragma unroll
  for (int r = 0; r < (MF ? TR : 1); ++r) accm[r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int bi = 0; bi < NB; ++bi) {
#pragma unroll
    for (int h = 0; h < NPH; ++h) csum[bi][h] = 0.f;
#pragma unroll
    for (int r = 0; r < TR; ++r) acc[bi][r] = 0.f;
  }
  ClassConsts kc = {};
  PairConsts k1 = {};
  if constexpr (SharedShifts<TCV>::value) kc = make_class_consts<W>(); else k1 = make_pair_consts<W>();
  const PairConsts k3 = make_pair_consts<3>();
  const uint32_t* xs32 = reinterpret_cast<const uint32_t*>(xs);
  const bool heavy = nchunks > nthreads;     // workgroup-uniform
#define SPQR_TILE_FMA(t, L, st)                                                                            \
  do {                                                                                                     \
    const uint32_t* xt_ = xs32 + (64 * (st) + min(lane, (L) - 1)) * (TC / 2);                              \
    const bool valid_ = live && lane < (L);                                                                \
    tile_fma<W, TR, TCV, AXIS, NB, LV, TC, 0, MF>(t, xt_, n >> 1, valid_, acc, accm, csum, kc, k1, k3);             \
    if constexpr (TCV != TC)                                                                                         \
      tile_fma<W, TR, TCV, AXIS, NB, LV, TC, 1, MF>(t, xt_ + TCV / 2, n >> 1, valid_, acc, accm, csum, kc, k1, k3); \
  } while (0)
  // Two steps per trip, registers ping-pong; the loop has its one exit at the
  // bottom (a second exit would be merged with it through a block that makes the
  // compiler wait for every load at the top of the loop).  t0 holds step `step`.
  while (step + P < nsteps) {                // wave-uniform: at least two steps are left
    L1 = issue(t1, step + P);
    SPQR_TILE_FMA(t0, L0, step);
    L0 = issue(t0, step + 2 * P);            // a dummy after the wavefront's last step
    SPQR_TILE_FMA(t1, L1, step + P);
    step += 2 * P;
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
  const bool slow = nchunks > chunk_cap;     // workgroup-uniform: more chunks than one round holds
  if (!alias) {
    if (tid < first_round) {
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        float p[8];
        chunk_products(xs + bi * n, (uint32_t)(n - 1), pc, pv, p);
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
            chunk_products(xs + bi * n, (uint32_t)(n - 1), lc[k - 1], lv[k - 1], p);
            store_products(prod + bi * pstride, slot, p);
          }
        }
      }
    }
  }

  // ---- dense partials: lanes -> rows ---------------------------------------------
  if constexpr (MF) {                        // the lane's own sums out of the matrix cores' result registers
    const int t4 = lane & 3;
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      const f32x4 d = accm[r];
      acc[0][r] = t4 == 0 ? d.x : (t4 == 1 ? d.y : (t4 == 2 ? d.z : d.w));
    }
  }
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

  if constexpr (NB == 1 && !PERM) {
    if (alias && !slow) {
      // the products of a chunk in the registers of its columns and values, parked once x is no longer read
      auto in_place = [&](u32x4& c8, u32x4& v8) {
        float p[8];
        chunk_products(xs, (uint32_t)(n - 1), c8, v8, p);
        c8 = u32x4{__float_as_uint(p[0]), __float_as_uint(p[1]), __float_as_uint(p[2]), __float_as_uint(p[3])};
        v8 = u32x4{__float_as_uint(p[4]), __float_as_uint(p[5]), __float_as_uint(p[6]), __float_as_uint(p[7])};
      };
      if (tid < first_round) in_place(pc, pv);
      if (heavy) {
#pragma unroll
        for (int k = 1; k < KMAX; ++k) {
          const int slot = tid + k * nthreads;
          if (slot < chunk_cap && slot < nchunks) in_place(lc[k - 1], lv[k - 1]);
        }
      }
      __syncthreads();                       // every wavefront has left x behind
      u32x4* park = reinterpret_cast<u32x4*>(prod);
      if (tid < first_round) { park[2 * tid] = pc; park[2 * tid + 1] = pv; }
      if (heavy) {
#pragma unroll
        for (int k = 1; k < KMAX; ++k) {
          const int slot = tid + k * nthreads;
          if (slot < chunk_cap && slot < nchunks) { park[2 * slot] = lc[k - 1]; park[2 * slot + 1] = lv[k - 1]; }
        }
      }
    }
  }

  // Rows too long for 16 lanes, as a bit mask every wavefront works out for itself
  // from the row pointers in LDS (TR <= 32 lanes vote), and this thread's first
  // output row: both read ahead of the barrier, off the critical path behind it.
  const int vr = min(lane, ROWS - 1);
  uint64_t longs = __builtin_amdgcn_ballot_w64(lane < ROWS && rp[vr + 1] - rp[vr] > LONG_ROW);
  const int r_long = longs ? __builtin_ctzll(longs) : 0;
  const int lo_long = rp[r_long], hi_long = rp[r_long + 1];
  const int r_first = min(g16, ROWS - 1);
  const int a_first = rp[r_first], b_first = rp[r_first + 1];
  // One barrier publishes products and partials.  Only a strip with more chunks
  // than one round holds needs the slow path.
  __syncthreads();
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
    for (int r = g16; r < ROWS; r += ngroups) {
      const int a = r == g16 ? a_first : rp[r], b = r == g16 ? b_first : rp[r + 1];
      const int w0 = (r / TR) * P, rr = r % TR;        // the row's strip: its wavefronts, the row inside it
#pragma unroll
      for (int bi = 0; bi < NB; ++bi) {
        float s;
        if (b - a > LONG_ROW) s = l16 < nwaves ? lred[bi][r][l16] : 0.f;
        else s = strided16_sum(prod + bi * pstride, a - base, b - base, l16);
        if (l16 < P) s += red[w0 + l16][bi][rr];
        s = row16_allreduce(s, lane);
        if (l16 == 0) {
          const int64_t i = (int64_t)bi * m + row0 + r;
          if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
          else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
        }
      }
    }
    return;
  }

  // ---- slow path: rounds of chunk_cap chunks (up to KMAX per thread, all loads of a
  // round in flight together); long rows summed by all threads ----------------------
  // more than two such rounds: rounds of the whole LDS with x from global memory are fewer and faster (a workgroup
  // with two full rows of 11008 outliers: the 7B-shaped block 34.4 -> 32.8 us)
  const bool x_global = alias && (spare_cap < nthreads || nchunks > 2 * spare_cap);   // workgroup-uniform
  if (alias && !x_global) {                              // x stays, the rounds use what is left behind it
    prod = reinterpret_cast<float*>(smem + xbytes);
    chunk_cap = spare_cap;
  }
  for (int i = tid; i < NB * ROWS_MAX; i += nthreads) (&osum[0][0])[i] = 0.f;
  for (int c0 = 0; c0 < nchunks; c0 += chunk_cap) {      // workgroup-uniform
    const int c1 = min(nchunks, c0 + chunk_cap);
    if (c0 > 0) __syncthreads();                         // previous round's products are consumed
    if (c0 > 0 || alias) {                               // round 0 is already in LDS (unless x was in its place)
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
            if (x_global) chunk_products(x, (uint32_t)(n - 1), cc[k], vv[k], p);  // x in LDS is being overwritten
            else chunk_products(xs + bi * n, (uint32_t)(n - 1), cc[k], vv[k], p);
            store_products(prod + bi * pstride, slot, p);
          }
        }
      }
    }
    __syncthreads();
    const int e0 = 8 * (c_lo + c0), e1 = 8 * (c_lo + c1);   // CSR range covered by this round
    // rows with a long slice in this round, voted as on the fast path; their partials per
    // wavefront go through lred, one barrier for all of them
    uint64_t rl = __builtin_amdgcn_ballot_w64(lane < ROWS && min(rp[vr + 1], e1) - max(rp[vr], e0) > LONG_ROW);
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
    for (int r = g16; r < ROWS; r += ngroups) {          // a row always meets the same 16 lanes: osum needs no barrier
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
  for (int o = tid; o < NB * ROWS; o += nthreads) {
    const int bi = o / ROWS, r = o % ROWS;
    float s = osum[bi][r];
    for (int w = 0; w < P; ++w) s += red[(r / TR) * P + w][bi][r % TR];
    const int64_t i = (int64_t)bi * m + row0 + r;
    if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
    else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
  }
}

template <int W, int TR, int TC, int AXIS, bool PERM, int NB, int LV = 1>
__global__ void __launch_bounds__((64 * WavesPerGroup<W, NB, LV, TR * TC, LargeRegisterBudget<W, TR, TC, AXIS, NB, LV>::value>::MAX))
gemv_tile256_kernel(DevMatrix A, const uint16_t* __restrict__ x, void* __restrict__ y, int y_dtype,
                    int chunk_cap, int strips_per_group, int waves_per_strip) {
  gemv_tile256_body<W, TR, TC, AXIS, PERM, NB, LV>(A, x, y, y_dtype, chunk_cap, blockIdx.x * strips_per_group,
                                               strips_per_group, waves_per_strip);
}

// Several matrices of one format (the q/k/v or gate/up projections of a decoder block, or all
// projections of a block) in one grid: workgroups [first[i], first[i+1]) belong to matrix i, each
// with its own input vector and its own plan.  A workgroup of a matrix as wide as the launch's
// LDS was sized for does exactly what it would do in a launch of its own matrix.
struct FusedArgs {
  int count;
  int first[SPQR_MAX_FUSED + 1];
  Geometry g;                                // of matrix 0; m, ntr, n and ntc are set per matrix below
  int m[SPQR_MAX_FUSED];
  int n[SPQR_MAX_FUSED];
  int R[SPQR_MAX_FUSED], P[SPQR_MAX_FUSED];  // strips per workgroup, wavefronts per strip (R * P = the launch's wavefronts)
  int cap[SPQR_MAX_FUSED];                   // outlier chunks of a round
  int shared_lds[SPQR_MAX_FUSED];            // 1: the products take the place of x (a matrix wider than the launch's LDS was sized for)
  int spare_cap[SPQR_MAX_FUSED];             // chunks the LDS behind x holds then
  const uint8_t* packed[SPQR_MAX_FUSED];
  const int32_t* row_ptr[SPQR_MAX_FUSED];
  const uint16_t* col[SPQR_MAX_FUSED];
  const uint16_t* val[SPQR_MAX_FUSED];
  const uint16_t* x[SPQR_MAX_FUSED];
  void* y[SPQR_MAX_FUSED];
};

template <int W, int TR, int TC, int AXIS, int LV = 1>
__global__ void __launch_bounds__((64 * WavesPerGroup<W, 1, LV, TR * TC, LargeRegisterBudget<W, TR, TC, AXIS, 1, LV>::value>::MAX))
gemv_tile256_fused_kernel(FusedArgs F, int y_dtype) {
  int i = 0;
  while (i + 1 < F.count && (int)blockIdx.x >= F.first[i + 1]) ++i;   // workgroup-uniform, count <= SPQR_MAX_FUSED
  DevMatrix A;
  A.g = F.g;
  A.g.m = F.m[i]; A.g.ntr = F.m[i] / TR;
  A.g.n = F.n[i]; A.g.ntc = F.n[i] / TC;
  A.packed = F.packed[i]; A.row_ptr = F.row_ptr[i]; A.col = F.col[i]; A.val = F.val[i];
  A.perm = nullptr; A.nnz = 0;
  const int R = F.R[i];
  gemv_tile256_body<W, TR, TC, AXIS, false, 1, LV>(A, F.x[i], F.y[i], y_dtype, F.cap[i],
                                               ((int)blockIdx.x - F.first[i]) * R, R, F.P[i], F.shared_lds[i] != 0, F.spare_cap[i]);
}

}  // namespace spqr
