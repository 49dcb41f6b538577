// The SpQR quantiser's column sweep (Alg. 1, lines 4-20, with its subroutines outliers(), error(),
// fit_statistics(), fit_quantizer(), quantize(), dequantize()) and the gathering of the outlier set.
//
// Every floating-point step is ONE rounded binary64 operation, in the order the algorithm states, so the integer
// results do not depend on how the work is spread over the machine: no fused multiply-add (contraction is off
// for this file), true divisions, sums from left to right.
//
// Rows are independent except for the second level of the statistics, which joins beta2 consecutive rows of a
// column block: a lane owns a row, a workgroup 64 consecutive rows, and the lanes of a tile exchange the
// minima / maxima of their statistics with cross-lane shuffles.  The workgroup's wavefronts all hold the same 64
// rows: each computes the block's statistics, codes and errors for itself (identical inputs, identical results:
// nothing has to be exchanged), they share out the leave-one-out tests of the block's columns and the columns
// right of the block that receive the error feedback (line 16, the O(m n^2) part).  The working copy of W is
// column-major, so a wavefront's access to a column is one contiguous run.
#pragma clang fp contract(off)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

#include "../../include/spqr_encode.h"

namespace spqr_enc {

#ifndef SPQR_SWEEP_WAVES
#define SPQR_SWEEP_WAVES 16
#endif
#ifndef SPQR_SWEEP_PREFETCH
#define SPQR_SWEEP_PREFETCH 0       // a chunk ahead in registers: pays with 8 wavefronts per workgroup, not with 16 (4 per SIMD hide the loads)
#endif
constexpr int kWaves = SPQR_SWEEP_WAVES;     // wavefronts per workgroup of the sweep
constexpr int kRows = 64;                    // rows per workgroup: one per lane

// binary64 -> binary16, round to nearest even, in one rounding (integer arithmetic on the bit pattern).
__device__ __forceinline__ uint16_t f64_to_f16_bits(double x) {
  const uint64_t b = __builtin_bit_cast(uint64_t, x);
  const uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
  const int e = (int)((b >> 52) & 0x7FF);
  const uint64_t mant = b & 0xFFFFFFFFFFFFFull;
  if (e == 0x7FF) return sign | (mant ? 0x7E00u : 0x7C00u);
  const int E = e - 1023;
  if (E > 15) return sign | 0x7C00u;
  if (E >= -14) {
    uint32_t h = (uint32_t)((E + 15) << 10) | (uint32_t)(mant >> 42);
    const uint64_t rem = mant & ((1ull << 42) - 1), half = 1ull << 41;
    if (rem > half || (rem == half && (h & 1u))) ++h;          // a carry runs into the exponent, up to infinity
    return sign | (uint16_t)h;
  }
  if (e == 0) return sign;                                     // binary64 subnormals are far below 2^-25
  int shift = 42 + (-14 - E);
  if (shift > 63) return sign;
  const uint64_t full = mant | (1ull << 52);
  uint32_t h = (uint32_t)(full >> shift);
  const uint64_t rem = full & ((1ull << shift) - 1), half = 1ull << (shift - 1);
  if (rem > half || (rem == half && (h & 1u))) ++h;
  return sign | (uint16_t)h;
}

__device__ __forceinline__ double f16_bits_to_f64(uint16_t h) {
  return (double)__builtin_bit_cast(_Float16, h);              // widening is exact
}

// Alg. 1 quantize with the clamp to the code range.
__device__ __forceinline__ double quantize(double v, double s, double z, double top) {
  const double q = floor(v / s + z + 0.5);
  return fmin(fmax(q, 0.0), top);
}

// Alg. 1 fit_quantizer from a group's minimum and maximum.
__device__ __forceinline__ void fit_from_range(double lo, double hi, double levels, double* s, double* z) {
  double sc = (hi - lo) / levels;
  if (sc == 0.0) sc = 1.0;
  *s = sc;
  *z = -lo / sc;
}

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)b, mask, 64);
  const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(b >> 32), mask, 64);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// One first-level statistic through the second level (Alg. 1 fit_statistics, lines 4-10): the beta2 lanes of a tile
// fit a quantiser to their values, round its two parameters to binary16, and every lane gets its code and the
// de-quantised statistic.
__device__ __forceinline__ void second_level(double v, int beta2, double levels, double* hat, uint8_t* code,
                                             uint16_t* s2_bits, uint16_t* z2_bits) {
  double lo = v, hi = v;
  for (int off = 1; off < beta2; off <<= 1) {
    lo = fmin(lo, shfl_xor_f64(lo, off));
    hi = fmax(hi, shfl_xor_f64(hi, off));
  }
  double s2, z2;
  fit_from_range(lo, hi, levels, &s2, &z2);
  uint16_t sb = f64_to_f16_bits(s2);
  double s2h = f16_bits_to_f64(sb);
  if (s2h == 0.0) { s2h = 1.0; sb = 0x3C00u; z2 = -lo; }
  const uint16_t zb = f64_to_f16_bits(z2);
  const double z2h = f16_bits_to_f64(zb);
  const double c = quantize(v, s2h, z2h, levels);
  *hat = s2h * (c - z2h);
  *code = (uint8_t)c;
  *s2_bits = sb; *z2_bits = zb;
}

struct SweepArgs {
  const double* U;       // H^ic [n][n]
  double* Wt;            // working copy, column-major: Wt[j * m + i]
  int m, n, beta2;
  double w_top, s_top, z_top;   // 2^bits - 1
  double tau;
  spqr_quantized_t out;
};

constexpr int kSuper = 64;                   // columns whose error feedback to the far columns is applied in one pass

// LDS of the sweep (dynamic: more than 64 KB).
template <int B1> struct SweepLds {
  static constexpr int CB = B1 >= 8 ? 8 : 4;             // columns per chunk of the feedback
  double esb[kSuper][kRows];                             // errors E of the current super-block's columns
  double utile[kWaves][kSuper][CB];                      // per wavefront: the piece of H^ic of its current chunk
  double wbs[B1][kRows];                                 // the block's columns
  double ublk[B1][B1];                                   // the block's corner of H^ic
  uint32_t omask[kWaves][kRows];
  uint8_t qs[kRows][B1], ms[kRows][B1];
  uint16_t vs[kRows][B1];
};

// Line 14 / line 16 for the columns [k_begin, k_end): W[:, k] -= E[:, j] * H^ic[urow0 + j, k] for j = 0 .. rows - 1, in
// that order, one product and one difference at a time.  esrc[j][lane] is E of column urow0 + j.  Chunks of CB
// columns are dealt to the wavefronts; a chunk's columns of W and its rows x CB piece of H^ic are requested one
// chunk ahead; the piece passes through a corner of LDS that belongs to the wavefront, from where every lane reads
// the same numbers (broadcast reads).  (k_end - k_begin) is a multiple of CB.
template <int CB>
__device__ __forceinline__ void feedback(double* __restrict__ Wt, const double* __restrict__ U, int m, int n, int rrow,
                                         bool live, int lane, int wave, int urow0, int rows, int k_begin, int k_end,
                                         const double (*esrc)[kRows], double (*ut)[CB]) {
  constexpr int PER = kSuper * CB / 64;                  // values of the largest piece per lane
  const uint32_t roff = (uint32_t)rrow * 8u;             // a column's address = its uniform base + this 32-bit offset
  const int cells = rows * CB;
  int k0 = k_begin + CB * wave;
  if (k0 >= k_end) return;                               // wave-uniform
  double cur[CB], nxt[CB], ucur[PER], unxt[PER];
#pragma unroll
  for (int q = 0; q < CB; ++q) cur[q] = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(Wt + (size_t)(k0 + q) * m) + roff);
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    const int idx = min(lane + 64 * p, cells - 1);
    ucur[p] = U[(size_t)(urow0 + idx / CB) * n + k0 + idx % CB];
  }
  for (; k0 < k_end; k0 += CB * kWaves) {                // wave-uniform
    const int k1 = k0 + CB * kWaves < k_end ? k0 + CB * kWaves : k0;   // behind the last chunk: the same one again, unused
    if (SPQR_SWEEP_PREFETCH) {
#pragma unroll
    for (int q = 0; q < CB; ++q) nxt[q] = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(Wt + (size_t)(k1 + q) * m) + roff);
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int idx = min(lane + 64 * p, cells - 1);
      unxt[p] = U[(size_t)(urow0 + idx / CB) * n + k1 + idx % CB];
    }
    }
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int idx = lane + 64 * p;
      if (idx < cells) ut[idx / CB][idx % CB] = ucur[p];
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll 2
    for (int j = 0; j < rows; ++j) {
      const double ej = esrc[j][lane];
#pragma unroll
      for (int q = 0; q < CB; q += 2) {
        typedef double f64x2 __attribute__((ext_vector_type(2)));
        const f64x2 uu = *reinterpret_cast<const f64x2*>(&ut[j][q]);
        cur[q] = cur[q] - ej * uu.x;
        cur[q + 1] = cur[q + 1] - ej * uu.y;
      }
    }
    __builtin_amdgcn_wave_barrier();
    if (live) {
#pragma unroll
      for (int q = 0; q < CB; ++q) *reinterpret_cast<double*>(reinterpret_cast<char*>(Wt + (size_t)(k0 + q) * m) + roff) = cur[q];
    }
    if (SPQR_SWEEP_PREFETCH) {
#pragma unroll
      for (int q = 0; q < CB; ++q) cur[q] = nxt[q];
#pragma unroll
      for (int p = 0; p < PER; ++p) ucur[p] = unxt[p];
    } else if (k1 != k0) {
#pragma unroll
      for (int q = 0; q < CB; ++q) cur[q] = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(Wt + (size_t)(k1 + q) * m) + roff);
#pragma unroll
      for (int p = 0; p < PER; ++p) {
        const int idx = min(lane + 64 * p, cells - 1);
        ucur[p] = U[(size_t)(urow0 + idx / CB) * n + k1 + idx % CB];
      }
    }
  }
}

template <int B1>
__global__ void __launch_bounds__(64 * kWaves) sweep_kernel(SweepArgs a) {
  using Lds = SweepLds<B1>;
  constexpr int CB = Lds::CB;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  Lds& S = *reinterpret_cast<Lds*>(smem);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = a.m, n = a.n;
  const int row = blockIdx.x * kRows + lane;
  const bool live = row < m;                 // a tile is all live or all dead: m is a multiple of beta2, beta2 divides 64
  const int rrow = live ? row : m - 1;       // dead lanes shadow the last row and write nothing
  const int ng = n / B1;
  const double* __restrict__ U = a.U;
  double* __restrict__ Wt = a.Wt;

  // Super-blocks of kSuper columns: inside one, a block's errors reach the super-block's remaining columns at once
  // (they are needed next); the columns right of the super-block receive all of its errors in one pass afterwards,
  // column by column in the same order j = 0, 1, ... - the same operations on every weight as updating after every
  // block, with 1 / (kSuper / B1) of the traffic over the working copy.
  for (int sb = 0; sb < n; sb += kSuper) {
    const int sbw = min(kSuper, n - sb);
    for (int i = sb; i < sb + sbw; i += B1) {
      const int g = i / B1;
      // the block's B1 x B1 corner of H^ic (rows i.., columns i..) for everybody, and its columns of W
      for (int idx = threadIdx.x; idx < B1 * B1; idx += 64 * kWaves)
        S.ublk[idx / B1][idx % B1] = U[(size_t)(i + idx / B1) * n + i + idx % B1];
      if (wave == 0) {
        double wb[B1];
#pragma unroll
        for (int c = 0; c < B1; ++c) wb[c] = Wt[(size_t)(i + c) * m + rrow];
#pragma unroll
        for (int c = 0; c < B1; ++c) S.wbs[c][lane] = wb[c];
      }
      __syncthreads();

      // ---- outliers(): this wavefront's share of the leave-one-out tests (line 8).  The loops over the group stay
      // rolled: a division is a dozen instructions, and sixteen of them side by side cost more registers than a lane
      // has. ----
      uint32_t mine = 0;
      if (a.tau < INFINITY) {
        auto group_error = [&](int x) -> double {        // summed error of the group without column x (-1: all columns)
          double lo = INFINITY, hi = -INFINITY;
#pragma unroll 4
          for (int c = 0; c < B1; ++c) {
            const double v = S.wbs[c][lane];
            if (c != x) { lo = fmin(lo, v); hi = fmax(hi, v); }
          }
          double s, z;
          fit_from_range(lo, hi, a.w_top, &s, &z);
          double t = 0.0;
#pragma unroll 2
          for (int c = 0; c < B1; ++c) {
            if (c != x) {
              const double v = S.wbs[c][lane];
              const double e = (v - s * (quantize(v, s, z, a.w_top) - z)) / S.ublk[c][c];
              t = t + e * e;
            }
          }
          return t;
        };
        const double base = group_error(-1);
        for (int x = wave; x < B1; x += kWaves)          // candidate column x (wave-uniform)
          if ((base - group_error(x)) > a.tau) mine |= 1u << x;
      }
      S.omask[wave][lane] = mine;
      __syncthreads();

      // ---- fit_statistics() (line 9) and lines 10-15 by the first wavefront alone: the block's columns are taken
      // one after the other, each depending on the one before, so there is nothing to share out; the loops stay
      // rolled over the copy of the block in LDS, which now belongs to this wavefront (the others are past their
      // tests).  The errors go to LDS for everybody's feedback passes. ----
      if (wave == 0) {
        uint32_t om = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) om |= S.omask[w][lane];
        double s_hat, z_hat;
        uint8_t sq, zq;
        uint16_t ssb, zsb, szb, zzb;
        {
          double lo = INFINITY, hi = -INFINITY;
#pragma unroll 4
          for (int c = 0; c < B1; ++c) {
            const double v = S.wbs[c][lane];
            if (!((om >> c) & 1u)) { lo = fmin(lo, v); hi = fmax(hi, v); }
          }
          if (lo > hi) { lo = 0.0; hi = 0.0; }   // nothing left
          double s1, z1;
          fit_from_range(lo, hi, a.w_top, &s1, &z1);
          second_level(s1, a.beta2, a.s_top, &s_hat, &sq, &ssb, &zsb);
          second_level(z1, a.beta2, a.z_top, &z_hat, &zq, &szb, &zzb);
        }
#pragma unroll 1
        for (int c = 0; c < B1; ++c) {
          const bool is_out = (om >> c) & 1u;
          const double v = S.wbs[c][lane];
          const double q = quantize(v, s_hat, z_hat, a.w_top);
          const double wq = s_hat * (q - z_hat);
          const double ec = (v - wq) / S.ublk[c][c] * (is_out ? 0.0 : 1.0);
          S.esb[i - sb + c][lane] = ec;
#pragma unroll 4
          for (int k = c; k < B1; ++k) S.wbs[k][lane] = S.wbs[k][lane] - ec * S.ublk[c][k];     // line 14, inside the block
          S.qs[lane][c] = (uint8_t)q;
          S.ms[lane][c] = is_out ? 1 : 0;
          S.vs[lane][c] = is_out ? f64_to_f16_bits(S.wbs[c][lane] - wq) : (uint16_t)0;
        }
        if (live) {
          const size_t at = (size_t)row * n + i;
#pragma unroll
          for (int k = 0; k < B1 / 4; ++k) {
            reinterpret_cast<uint32_t*>(a.out.Q + at)[k] = reinterpret_cast<const uint32_t*>(S.qs[lane])[k];
            reinterpret_cast<uint32_t*>(a.out.outlier_mask + at)[k] = reinterpret_cast<const uint32_t*>(S.ms[lane])[k];
          }
#pragma unroll
          for (int k = 0; k < B1 / 2; ++k)
            reinterpret_cast<uint32_t*>(a.out.outlier_val + at)[k] = reinterpret_cast<const uint32_t*>(S.vs[lane])[k];
          a.out.s_q[(size_t)row * ng + g] = sq;
          a.out.z_q[(size_t)row * ng + g] = zq;
          if ((row % a.beta2) == 0) {
            const size_t t = (size_t)(row / a.beta2) * ng + g;
            a.out.s_s[t] = ssb; a.out.z_s[t] = zsb; a.out.s_z[t] = szb; a.out.z_z[t] = zzb;
          }
#pragma unroll 4
          for (int c = 0; c < B1; ++c) Wt[(size_t)(i + c) * m + row] = S.wbs[c][lane];
        }
      }
      __syncthreads();
      // ---- line 16 for the rest of the super-block ----
      feedback<CB>(Wt, U, m, n, rrow, live, lane, wave, i, B1, i + B1, sb + sbw, S.esb + (i - sb), S.utile[wave]);
      __syncthreads();       // the next block's columns are complete; wbs, ublk, omask are free again
    }
    // ---- line 16 for everything right of the super-block: all of its errors in one pass ----
    feedback<CB>(Wt, U, m, n, rrow, live, lane, wave, sb, sbw, sb + sbw, n, S.esb, S.utile[wave]);
    __syncthreads();
  }
}

// W[m][n] row-major <-> Wt[n][m] column-major, through a 32 x 32 LDS tile.
__global__ void __launch_bounds__(256) transpose_kernel(const double* __restrict__ src, double* __restrict__ dst,
                                                       int rows, int cols) {   // src[rows][cols] -> dst[cols][rows]
  __shared__ double tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  for (int k = ty; k < 32; k += 8) {
    const int r = r0 + k, c = c0 + tx;
    tile[k][tx] = (r < rows && c < cols) ? src[(size_t)r * cols + c] : 0.0;
  }
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int c = c0 + k, r = r0 + tx;
    if (r < rows && c < cols) dst[(size_t)c * rows + r] = tile[tx][k];
  }
}

// Outliers per row, then the exclusive prefix (one workgroup: m is at most a few tens of thousands).
__global__ void __launch_bounds__(256) count_rows_kernel(const uint8_t* __restrict__ mask, int m, int n,
                                                        int32_t* __restrict__ counts) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= m) return;
  const uint32_t* p = reinterpret_cast<const uint32_t*>(mask + (size_t)row * n);
  int c = 0;
  for (int k = lane; k < n / 4; k += 64) c += __popc(p[k] & 0x01010101u);
  for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
  if (lane == 0) counts[row + 1] = c;
}

__global__ void __launch_bounds__(1024) prefix_kernel(int32_t* __restrict__ row_ptr, int m) {   // in place on [1, m]
  __shared__ int part[1024];
  const int t = threadIdx.x;
  const int per = (m + 1023) / 1024;
  const int lo = min(m, t * per), hi = min(m, lo + per);
  int s = 0;
  for (int r = lo; r < hi; ++r) s += row_ptr[r + 1];
  part[t] = s;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int v = t >= off ? part[t - off] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int run = t ? part[t - 1] : 0;
  if (t == 0) row_ptr[0] = 0;
  for (int r = lo; r < hi; ++r) { run += row_ptr[r + 1]; row_ptr[r + 1] = run; }
}

// Alg. 1 gather_outlier_matrix: one wavefront per row, entries in column order.
__global__ void __launch_bounds__(256) gather_kernel(const uint8_t* __restrict__ mask, const uint16_t* __restrict__ dense,
                                                    const int32_t* __restrict__ row_ptr, int m, int n,
                                                    uint16_t* __restrict__ col, uint16_t* __restrict__ val) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= m) return;
  int at = row_ptr[row];
  for (int c0 = 0; c0 < n; c0 += 64) {
    const int c = c0 + lane;
    const bool is = c < n && mask[(size_t)row * n + c] != 0;
    const uint64_t vote = __ballot(is);
    if (is) {
      const int k = at + __popcll(vote & ((1ull << lane) - 1));
      col[k] = (uint16_t)c;
      val[k] = dense[(size_t)row * n + c];
    }
    at += __popcll(vote);
  }
}

// The sweep's LDS exceeds the 64 KB a kernel gets without asking: the opt-in is per device and is asked for on every
// call (a cheap host call; nothing is remembered, so nothing has to be guarded between threads).
template <int B1>
hipError_t launch_sweep(dim3 grid, dim3 block, hipStream_t st, const SweepArgs& a) {
  const int lds = (int)sizeof(SweepLds<B1>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sweep_kernel<B1>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sweep_kernel<B1>, grid, block, lds, st, a);
  return hipGetLastError();
}

}  // namespace spqr_enc

extern "C" {

size_t spqr_quantize_workspace_bytes(int32_t m, int32_t n) {
  if (m < 1 || n < 1) return 0;
  return ((size_t)m * n * sizeof(double) + 255) & ~(size_t)255;
}

int spqr_quantize(const double* W, const double* Hic, int32_t m, int32_t n, int32_t w_bits, int32_t s_bits,
                  int32_t z_bits, int32_t beta1, int32_t beta2, double tau, const spqr_quantized_t* out,
                  void* workspace, size_t workspace_bytes, void* stream) {
  using namespace spqr_enc;
  if (!W || !Hic || !out || !workspace) return SPQR_ERR_NULL;
  if (!out->Q || !out->s_q || !out->z_q || !out->s_s || !out->z_s || !out->s_z || !out->z_z || !out->outlier_mask ||
      !out->outlier_val || !out->row_ptr)
    return SPQR_ERR_NULL;
  if (w_bits < 2 || w_bits > 8 || s_bits < 1 || s_bits > 8 || z_bits < 1 || z_bits > 8) return SPQR_ERR_PARAM;
  if (beta1 != 4 && beta1 != 8 && beta1 != 16 && beta1 != 32) return SPQR_ERR_PARAM;
  if (beta2 < 2 || beta2 > 64 || (beta2 & (beta2 - 1)) != 0) return SPQR_ERR_PARAM;
  if (tau != tau) return SPQR_ERR_PARAM;
  if (m < 1 || n < 1 || m % beta2 != 0 || n % beta1 != 0) return SPQR_ERR_SHAPE;
  if (workspace_bytes < spqr_quantize_workspace_bytes(m, n)) return SPQR_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(W) % 8 != 0 ||
      reinterpret_cast<uintptr_t>(Hic) % 8 != 0 || reinterpret_cast<uintptr_t>(out->Q) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(out->outlier_mask) % 4 != 0 || reinterpret_cast<uintptr_t>(out->outlier_val) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(out->row_ptr) % 4 != 0 || reinterpret_cast<uintptr_t>(out->W_final) % 8 != 0)
    return SPQR_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  SweepArgs a;
  a.U = Hic; a.Wt = static_cast<double*>(workspace);
  a.m = m; a.n = n; a.beta2 = beta2;
  a.w_top = (double)((1 << w_bits) - 1); a.s_top = (double)((1 << s_bits) - 1); a.z_top = (double)((1 << z_bits) - 1);
  a.tau = tau;
  a.out = *out;
  const dim3 tgrid((n + 31) / 32, (m + 31) / 32);
  hipLaunchKernelGGL(transpose_kernel, tgrid, dim3(256), 0, st, W, a.Wt, m, n);
  const dim3 grid((m + kRows - 1) / kRows), block(64 * kWaves);
  hipError_t e = hipSuccess;
  switch (beta1) {
    case 4: e = launch_sweep<4>(grid, block, st, a); break;
    case 8: e = launch_sweep<8>(grid, block, st, a); break;
    case 16: e = launch_sweep<16>(grid, block, st, a); break;
    default: e = launch_sweep<32>(grid, block, st, a); break;
  }
  if (e != hipSuccess) return SPQR_ERR_HIP;
  if (out->W_final) {
    const dim3 bgrid((m + 31) / 32, (n + 31) / 32);
    hipLaunchKernelGGL(transpose_kernel, bgrid, dim3(256), 0, st, a.Wt, out->W_final, n, m);
  }
  hipLaunchKernelGGL(count_rows_kernel, dim3((m + 3) / 4), dim3(256), 0, st, out->outlier_mask, m, n, out->row_ptr);
  hipLaunchKernelGGL(prefix_kernel, dim3(1), dim3(1024), 0, st, out->row_ptr, m);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

int spqr_gather_outliers(const uint8_t* outlier_mask, const uint16_t* outlier_val, const int32_t* row_ptr,
                         int32_t m, int32_t n, uint16_t* col_idx, uint16_t* val, void* stream) {
  using namespace spqr_enc;
  if (!outlier_mask || !outlier_val || !row_ptr || !col_idx || !val) return SPQR_ERR_NULL;
  if (m < 1 || n < 1 || n > 65536) return SPQR_ERR_SHAPE;
  hipLaunchKernelGGL(gather_kernel, dim3((m + 3) / 4), dim3(256), 0, static_cast<hipStream_t>(stream), outlier_mask,
                     outlier_val, row_ptr, m, n, col_idx, val);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

}  // extern "C"
