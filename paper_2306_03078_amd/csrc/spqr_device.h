// Device-side helpers shared by the kernels: cross-lane exchange on a 64-wide
// wavefront, fp16 bit tricks, and generic (slow) accessors into layout V1.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqr_layout.h"

namespace spqr {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct DevMatrix {
  Geometry g;
  const uint8_t* packed;
  const int32_t* row_ptr;
  const uint16_t* col;
  const uint16_t* val;
  const int32_t* perm;
  int64_t nnz;
  int32_t max_row_nnz;            // hint for the launch plan: longest outlier row, 0 = unknown
};

__device__ __forceinline__ float h2f(uint16_t bits) {
  return (float)__builtin_bit_cast(_Float16, bits);
}
__device__ __forceinline__ uint16_t f2h_rne(float v) {
  return __builtin_bit_cast(uint16_t, (_Float16)v);   // v_cvt_f16_f32: round to nearest even
}
__device__ __forceinline__ half2_t as_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }

// ---- lane exchange ---------------------------------------------------------
// DPP controls (GCN3+/CDNA): quad_perm = sel0 | sel1<<2 | sel2<<4 | sel3<<6,
// row_ror:n = 0x120 + n, row_mirror = 0x140, row_half_mirror = 0x141.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true);
  return __builtin_bit_cast(float, r);
}
// Value of lane (lane ^ 16) inside each group of 32 lanes: ds_swizzle, bit mode
// (and_mask 0x1f, or_mask 0, xor_mask 0x10).
__device__ __forceinline__ float swizzle_xor16(float v) {
  int r = __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (0x10 << 10) | 0x1F);
  return __builtin_bit_cast(float, r);
}
// Value of lane (lane ^ 32).
__device__ __forceinline__ float bperm_xor32(float v, int lane) {
  int r = __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v));
  return __builtin_bit_cast(float, r);
}

// Partner exchange used by the reduction stages.  Stage s pairs every lane with
// a partner that differs in lane bit (5 - s) and agrees in all higher bits:
//   s=0: lane^32   s=1: lane^16   s=2: 15-lane (row mirror)   s=3: 7-lane (half mirror)
//   s=4: lane^3 (quad reverse)    s=5: lane^1
template <int S>
__device__ __forceinline__ float stage_partner(float v, int lane) {
  if constexpr (S == 0) return bperm_xor32(v, lane);
  else if constexpr (S == 1) return swizzle_xor16(v);
  else if constexpr (S == 2) return dpp_f32<0x140>(v);
  else if constexpr (S == 3) return dpp_f32<0x141>(v);
  else if constexpr (S == 4) return dpp_f32<0x1B>(v);    // quad_perm [3,2,1,0]
  else return dpp_f32<0xB1>(v);                          // quad_perm [1,0,3,2]
}

template <int S, int END>
__device__ __forceinline__ float allreduce_stages(float v, int lane) {
  if constexpr (S < END) {
    v += stage_partner<S>(v, lane);
    return allreduce_stages<S + 1, END>(v, lane);
  } else {
    return v;
  }
}
// Sum over all 64 lanes, result in every lane.
__device__ __forceinline__ float wave_allreduce(float v, int lane) {
  return allreduce_stages<0, 6>(v, lane);
}
// Sum over each aligned group of 16 lanes, result in every lane of the group.
__device__ __forceinline__ float row16_allreduce(float v, int lane) {
  return allreduce_stages<2, 6>(v, lane);
}

// Reduce R per-lane values (R = 8, 16 or 32, one per output row) over the 64
// lanes.  Stage s halves the number of values a lane still carries: the lane
// keeps the half selected by its bit (5 - s) and hands the other half to its
// partner.  After log2(R) stages every lane holds one row's sum over a subset
// of lanes; the remaining stages finish it.  Returns the sum of row `row`.
template <int R, int S, int N>
__device__ __forceinline__ void scatter_stages(float (&v)[R], int lane) {
  if constexpr (N > 1) {
    constexpr int H = N / 2;
    const bool up = (lane >> (5 - S)) & 1;
#pragma unroll
    for (int i = 0; i < H; ++i) {
      float send = up ? v[i] : v[i + H];
      float keep = up ? v[i + H] : v[i];
      v[i] = keep + stage_partner<S>(send, lane);
    }
    scatter_stages<R, S + 1, H>(v, lane);
  }
}
template <int R>
__device__ __forceinline__ float wave_reduce_rows(float (&v)[R], int lane, int* row) {
  constexpr int NST = R == 8 ? 3 : (R == 16 ? 4 : 5);
  static_assert(R == 8 || R == 16 || R == 32, "row count per tile");
  scatter_stages<R, 0, R>(v, lane);
  float r = allreduce_stages<NST, 6>(v[0], lane);
  int idx = 0;
#pragma unroll
  for (int s = 0; s < NST; ++s) idx |= ((lane >> (5 - s)) & 1) << (NST - 1 - s);
  *row = idx;
  return r;
}

// ---- generic accessors (debug decode, validation, fallback product) --------
__device__ __forceinline__ uint32_t ld32(const uint8_t* base, int64_t off) {
  return *reinterpret_cast<const uint32_t*>(base + off);
}

// The b_w-bit code of tile-local (r, c) of tile (tr, tc).
__device__ inline uint32_t tile_code(const Geometry& g, const uint8_t* packed,
                                     int tr, int tc, int r, int c) {
  const int q = r * (g.tile_cols >> 1) + (c >> 1);
  const int hi = (c & 1) * 16;
  PairLoc p = pair_loc(g.w_bits, q);
  if (!p.split) {
    uint32_t d = ld32(packed, code_dword_offset(g, tr, tc, p.dword));
    return (d >> (p.shift + hi)) & ((1u << g.w_bits) - 1u);
  }
  uint32_t v = 0;
  for (int i = 0; i < 3; ++i) {
    uint32_t d = ld32(packed, code_dword_offset(g, tr, tc, p.dword + i));
    v |= ((d >> (15 + hi)) & 1u) << i;
  }
  return v;
}

// Statistic code number idx (0 <= idx < 2*beta2: scales first, then zeros).
__device__ inline uint32_t tile_stat_code(const Geometry& g, const uint8_t* packed,
                                          int tr, int tc, int idx) {
  const int hi = (idx & 1) * 16;
  PairLoc p = pair_loc(3, idx >> 1);
  if (!p.split) {
    uint32_t d = ld32(packed, stat_dword_offset(g, tr, tc, p.dword));
    return (d >> (p.shift + hi)) & 7u;
  }
  uint32_t v = 0;
  for (int i = 0; i < 3; ++i) {
    uint32_t d = ld32(packed, stat_dword_offset(g, tr, tc, p.dword + i));
    v |= ((d >> (15 + hi)) & 1u) << i;
  }
  return v;
}

// Canonical binary32 statistics of group `gi` of a tile: widen, subtract,
// multiply, each rounded once (Alg. 1 dequantize applied to the statistic codes).
// Integer zero-point (Sec. 5, "round zero"): z_hat is the code.  16-bit statistics
// (Sec. 5): dword gi holds s | z << 16 as binary16, widened exactly.
__device__ inline void tile_group_stats(const Geometry& g, const uint8_t* packed,
                                        int tr, int tc, int gi, float* s_hat, float* z_hat) {
  if (g.layout == kStats16) {
    const uint32_t d = ld32(packed, stat_dword_offset(g, tr, tc, gi));
    *s_hat = h2f((uint16_t)(d & 0xFFFF));
    *z_hat = h2f((uint16_t)(d >> 16));
    return;
  }
  const int nc = 3 * g.beta2 / 16;             // dwords of statistic codes
  const uint32_t a = ld32(packed, stat_dword_offset(g, tr, tc, nc));
  const float s_s = h2f((uint16_t)(a & 0xFFFF)), z_s = h2f((uint16_t)(a >> 16));
  const float sq = (float)tile_stat_code(g, packed, tr, tc, gi);
  const float zq = (float)tile_stat_code(g, packed, tr, tc, g.beta2 + gi);
  *s_hat = __fmul_rn(s_s, __fsub_rn(sq, z_s));
  if (g.layout == kRoundZero) { *z_hat = zq; return; }
  const uint32_t b = ld32(packed, stat_dword_offset(g, tr, tc, nc + 1));
  const float s_z = h2f((uint16_t)(b & 0xFFFF)), z_z = h2f((uint16_t)(b >> 16));
  *z_hat = __fmul_rn(s_z, __fsub_rn(zq, z_z));
}

// Canonical binary32 dense value of W_hat[i, j] without outliers.
__device__ inline float dense_value(const Geometry& g, const uint8_t* packed, int i, int j) {
  const int tr = i / g.tile_rows, r = i % g.tile_rows;
  const int tc = j / g.tile_cols, c = j % g.tile_cols;
  float s_hat, z_hat;
  tile_group_stats(g, packed, tr, tc, g.axis == 0 ? r : c, &s_hat, &z_hat);
  const float q = (float)tile_code(g, packed, tr, tc, r, c);
  return __fmul_rn(s_hat, __fsub_rn(q, z_hat));
}

}  // namespace spqr
