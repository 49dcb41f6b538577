// Lines 2 and 3 of Alg. 1 (SpQRQuantize): H = 2 X X^T and H^ic = Cholesky((H + lambda I)^-1), binary64.
//
// The factor the sweep needs is the upper triangular U with U^T U = (H + lambda I)^-1.  With A = H + lambda I
// and J the index reversal, a lower Cholesky factor L of J A J gives A = R R^T with R = J L J upper triangular,
// so A^-1 = R^-T R^-1 and U = R^-1 = J L^-1 J: one Cholesky factorisation and one triangular inverse, both in the
// reversed index space, no product of two triangular matrices and no second factorisation.
//
//   init      L <- lower triangle of J A J, padded with an identity to a multiple of 64
//   per block column k (64 wide): potrf of the diagonal block and its inverse (one workgroup, in LDS);
//             the panel below times that inverse (transposed); the trailing lower triangle minus panel x panel^T
//   trtri     X = L^-1 by doubling: with L = [[A, 0], [C, B]], L^-1 = [[A^-1, 0], [-B^-1 C A^-1, B^-1]].  Level s joins
//             neighbouring diagonal blocks of 64 * 2^s: two launches of 64 x 64 tile products per level (T = C A^-1,
//             then -B^-1 T written over C), every tile of every pair in parallel.  The inverse ends up where L was
//             (strictly lower blocks) plus the diagonal blocks' inverses from the potrf step.
//   final     U[i][j] = X[n-1-i][n-1-j] for j >= i
//
// MI355X runs binary64 fused multiply-adds on the vector ALU at the rate of its binary64 matrix instructions, so
// the products are plain register-tiled FMAs fed from LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/spqr_encode.h"

namespace spqr_fac {

constexpr int NB = 64;                       // block size of the factorisation
constexpr int KC = 16;                       // depth of one LDS stage of a tile product
constexpr int LP = NB + 4;                   // padded row of a staged operand (rows stay 32-byte aligned)

// acc[r][c] += sum_{k < K} fa(ty*4 + r, k) * fb(tx + 16*c, k): a 64 x 64 tile by 256 threads; a thread's four columns
// are 16 apart, so that the lanes of a wavefront read consecutive words of a staged row (no bank conflicts).
template <class FA, class FB>
__device__ __forceinline__ void tile_nt(double (&acc)[4][4], int K, FA fa, FB fb, double (*As)[LP],
                                        double (*Bs)[LP]) {
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  for (int k0 = 0; k0 < K; k0 += KC) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = t + 256 * q, ii = idx >> 4, kk = idx & 15;
      As[kk][ii] = fa(ii, k0 + kk);
      Bs[kk][ii] = fb(ii, k0 + kk);
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      double av[4], bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) { av[r] = As[kk][ty * 4 + r]; bv[r] = Bs[kk][tx + 16 * r]; }
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fma(av[r], bv[c], acc[r][c]);
    }
    __syncthreads();
  }
}

// acc[r][c] += sum_{kb <= k < ke} fa(ty*4 + r, k) * fb(k, tx + 16*c): the second operand given by rows (k, j).
template <class FA, class FB>
__device__ __forceinline__ void tile_nn(double (&acc)[4][4], int kb, int ke, FA fa, FB fb, double (*As)[LP],
                                        double (*Bs)[LP]) {
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  for (int k0 = kb; k0 < ke; k0 += KC) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int idx = t + 256 * q;
      As[idx & 15][idx >> 4] = fa(idx >> 4, k0 + (idx & 15));      // consecutive threads: consecutive k of one row
      Bs[idx >> 6][idx & 63] = fb(k0 + (idx >> 6), idx & 63);      // consecutive threads: consecutive j of one row k
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      double av[4], bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) { av[r] = As[kk][ty * 4 + r]; bv[r] = Bs[kk][tx + 16 * r]; }
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fma(av[r], bv[c], acc[r][c]);
    }
    __syncthreads();
  }
}

// H = 2 X X^T, tiles on and above the diagonal, mirrored.
__global__ void __launch_bounds__(256) hessian_kernel(const double* __restrict__ X, int n, int d, double* __restrict__ H) {
  __shared__ __attribute__((aligned(32))) double As[KC][LP], Bs[KC][LP];
  const int bi = blockIdx.y, bj = blockIdx.x;
  if (bj < bi) return;
  const int i0 = bi * NB, j0 = bj * NB;
  double acc[4][4] = {};
  auto fa = [&](int i, int k) { return (i0 + i < n && k < d) ? X[(size_t)(i0 + i) * d + k] : 0.0; };
  auto fb = [&](int j, int k) { return (j0 + j < n && k < d) ? X[(size_t)(j0 + j) * d + k] : 0.0; };
  tile_nt(acc, d, fa, fb, As, Bs);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int i = i0 + ty * 4 + r, j = j0 + tx + 16 * c;
      if (i < n && j < n) {
        const double v = 2.0 * acc[r][c];
        H[(size_t)i * n + j] = v;
        if (bi != bj) H[(size_t)j * n + i] = v;
      }
    }
}

__global__ void __launch_bounds__(256) init_reversed_kernel(const double* __restrict__ H, int n, int np, double lambda,
                                                           double* __restrict__ L) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)np * np) return;
  const int a = (int)(idx / np), b = (int)(idx % np);
  double v = 0.0;
  if (b <= a) {
    if (a < n) v = H[(size_t)(n - 1 - a) * n + (n - 1 - b)] + (a == b ? lambda : 0.0);   // lower triangle of J A J
    else v = a == b ? 1.0 : 0.0;
  }
  L[idx] = v;
}

// A lane's double as every lane sees it (v_readlane: the source lane is uniform).
__device__ __forceinline__ double readlane_f64(double v, int src) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, src);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), src);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Diagonal block kb: Cholesky factor in place, its inverse to Dinv[kb].  One wavefront, a lane per row, the row in
// registers: the 64 steps depend on each other, so there is nothing for more wavefronts to do but wait at barriers.
// Column j of the factor reaches the other rows through v_readlane (lane k holds L[k][j]), not through memory.
__global__ void __launch_bounds__(64) potrf_diag_kernel(double* __restrict__ L, int np, int kb, double* __restrict__ Dinv) {
  __shared__ double D[NB][NB + 1];
  const int lane = threadIdx.x;
  double* blk = L + (size_t)kb * NB * np + (size_t)kb * NB;
  double r[NB];                              // row `lane` of the block
  for (int idx = lane; idx < NB * NB; idx += 64) D[idx >> 6][idx & 63] = blk[(size_t)(idx >> 6) * np + (idx & 63)];   // coalesced
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int k = 0; k < NB; ++k) r[k] = D[lane][k];
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const double djj = sqrt(readlane_f64(r[j], j));
    const double lij = r[j] / djj;           // L[lane][j] for lane > j
    r[j] = lane == j ? djj : lij;
#pragma unroll
    for (int k = j + 1; k < NB; ++k) r[k] = fma(-lij, readlane_f64(lij, k), r[k]);   // meaningful for k <= lane
  }
#pragma unroll
  for (int k = 0; k < NB; ++k) {
    D[lane][k] = k <= lane ? r[k] : 0.0;
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  for (int idx = lane; idx < NB * NB; idx += 64) blk[(size_t)(idx >> 6) * np + (idx & 63)] = D[idx >> 6][idx & 63];
  // inverse of the lower triangular block: column `lane`, kept in registers while it is built (the factor is read
  // from LDS, every lane the same element); two running sums halve the chain of dependent additions
  double* inv = Dinv + (size_t)kb * NB * NB;
  {
    const int c = lane;
    double v[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int k = 0; k + 1 < i; k += 2) { s0 = fma(D[i][k], v[k], s0); s1 = fma(D[i][k + 1], v[k + 1], s1); }
      if (i & 1) s0 = fma(D[i][i - 1], v[i - 1], s0);
      const double dii = D[i][i];
      v[i] = i < c ? 0.0 : (i == c ? 1.0 / dii : -(s0 + s1) / dii);    // v[k] = 0 above the diagonal of the inverse
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) inv[i * NB + c] = v[i];
  }
}

// Panel below diagonal block kb: A[ib, kb] <- A[ib, kb] . inv(L_kk)^T
__global__ void __launch_bounds__(256) trsm_panel_kernel(double* __restrict__ L, int np, int kb, const double* __restrict__ Dinv) {
  __shared__ __attribute__((aligned(32))) double As[KC][LP], Bs[KC][LP];
  const int ib = kb + 1 + blockIdx.x;
  double* blk = L + (size_t)ib * NB * np + (size_t)kb * NB;
  const double* inv = Dinv + (size_t)kb * NB * NB;
  double acc[4][4] = {};
  auto fa = [&](int r, int k) { return blk[(size_t)r * np + k]; };
  auto fb = [&](int c, int k) { return inv[c * NB + k]; };
  tile_nt(acc, NB, fa, fb, As, Bs);          // every read of the block is done when tile_nt returns
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) blk[(size_t)(ty * 4 + r) * np + tx + 16 * c] = acc[r][c];
}

// Trailing update: A[ib, jb] -= P_ib . P_jb^T for kb < jb <= ib.
__global__ void __launch_bounds__(256) syrk_kernel(double* __restrict__ L, int np, int kb) {
  __shared__ __attribute__((aligned(32))) double As[KC][LP], Bs[KC][LP];
  const int ib = kb + 1 + blockIdx.y, jb = kb + 1 + blockIdx.x;
  if (jb > ib) return;
  const double* pi = L + (size_t)ib * NB * np + (size_t)kb * NB;
  const double* pj = L + (size_t)jb * NB * np + (size_t)kb * NB;
  double acc[4][4] = {};
  auto fa = [&](int r, int k) { return pi[(size_t)r * np + k]; };
  auto fb = [&](int c, int k) { return pj[(size_t)c * np + k]; };
  tile_nt(acc, NB, fa, fb, As, Bs);
  double* blk = L + (size_t)ib * NB * np + (size_t)jb * NB;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) blk[(size_t)(ty * 4 + r) * np + tx + 16 * c] -= acc[r][c];
}

// Element (r, c), r >= c, of the inverse as far as it is built: the diagonal 64-blocks live in Dinv, the blocks
// below them where L was.
__device__ __forceinline__ double inverse_at(const double* __restrict__ L, const double* __restrict__ Dinv, int np,
                                             int r, int c) {
  const int rb = r >> 6, cb = c >> 6;
  if (rb == cb) return Dinv[(size_t)rb * NB * NB + (r & 63) * NB + (c & 63)];
  return rb > cb ? L[(size_t)r * np + c] : 0.0;
}

// Level with diagonal blocks of `b` rows: pair p joins A = [2pb, 2pb + b) and B = [2pb + b, min(2pb + 2b, np)).
// Step 1: T = C . A^-1 into `T` (at C's place);  C = L[B rows, A columns].
__global__ void __launch_bounds__(256) trtri_step1_kernel(const double* __restrict__ L, const double* __restrict__ Dinv,
                                                         int np, int b, double* __restrict__ T) {
  __shared__ __attribute__((aligned(32))) double As[KC][LP], Bs[KC][LP];
  const int a0 = 2 * b * blockIdx.z, b0 = a0 + b;
  const int i0 = b0 + blockIdx.y * NB, j0 = blockIdx.x * NB;        // tile: rows i0.. (in B), columns a0 + j0.. (in A)
  if (i0 >= np) return;                                              // B is shorter than b, or missing
  double acc[4][4] = {};
  auto fa = [&](int i, int k) { return L[(size_t)(i0 + i) * np + a0 + k]; };
  auto fb = [&](int k, int j) { return inverse_at(L, Dinv, np, a0 + k, a0 + j0 + j); };
  tile_nn(acc, j0, b, fa, fb, As, Bs);                               // A^-1 is lower triangular: rows k >= j0 only
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) T[(size_t)(i0 + ty * 4 + r) * np + a0 + j0 + tx + 16 * c] = acc[r][c];
}

// Step 2: -B^-1 . T over C.
__global__ void __launch_bounds__(256) trtri_step2_kernel(double* __restrict__ L, const double* __restrict__ Dinv, int np,
                                                         int b, const double* __restrict__ T) {
  __shared__ __attribute__((aligned(32))) double As[KC][LP], Bs[KC][LP];
  const int a0 = 2 * b * blockIdx.z, b0 = a0 + b;
  const int i0 = blockIdx.y * NB, j0 = blockIdx.x * NB;              // tile: rows b0 + i0.., columns a0 + j0..
  if (b0 + i0 >= np) return;
  double acc[4][4] = {};
  // B^-1 (lower triangular, rows / columns relative to b0): its blocks left of the diagonal were written by the
  // lower levels, which are complete; this level writes blocks of C only
  auto fa = [&](int i, int k) { return inverse_at(L, Dinv, np, b0 + i0 + i, b0 + k); };
  auto fb = [&](int k, int j) { return T[(size_t)(b0 + k) * np + a0 + j0 + j]; };
  tile_nn(acc, 0, i0 + NB, fa, fb, As, Bs);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) L[(size_t)(b0 + i0 + ty * 4 + r) * np + a0 + j0 + tx + 16 * c] = -acc[r][c];
}

__global__ void __launch_bounds__(256) unreverse_kernel(const double* __restrict__ L, const double* __restrict__ Dinv, int n,
                                                       int np, double* __restrict__ U) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)n * n) return;
  const int i = (int)(idx / n), j = (int)(idx % n);
  U[idx] = j >= i ? inverse_at(L, Dinv, np, n - 1 - i, n - 1 - j) : 0.0;
}

}  // namespace spqr_fac

extern "C" {

int spqr_hessian(const double* X, int32_t n, int32_t d, double* H, void* stream) {
  using namespace spqr_fac;
  if (!X || !H) return SPQR_ERR_NULL;
  if (n < 1 || d < 1) return SPQR_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(X) % 8 != 0 || reinterpret_cast<uintptr_t>(H) % 8 != 0) return SPQR_ERR_ALIGN;
  const int nb = (n + NB - 1) / NB;
  hipLaunchKernelGGL(hessian_kernel, dim3(nb, nb), dim3(256), 0, static_cast<hipStream_t>(stream), X, n, d, H);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

size_t spqr_inverse_cholesky_workspace_bytes(int32_t n) {
  if (n < 1) return 0;
  const size_t np = ((size_t)n + spqr_fac::NB - 1) / spqr_fac::NB * spqr_fac::NB;
  return (2 * np * np + np * spqr_fac::NB) * sizeof(double);
}

int spqr_inverse_cholesky(const double* H, int32_t n, double lambda, double* Hic, void* workspace,
                          size_t workspace_bytes, void* stream) {
  using namespace spqr_fac;
  if (!H || !Hic || !workspace) return SPQR_ERR_NULL;
  if (n < 1) return SPQR_ERR_SHAPE;
  if (lambda != lambda) return SPQR_ERR_PARAM;
  if (workspace_bytes < spqr_inverse_cholesky_workspace_bytes(n)) return SPQR_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(H) % 8 != 0 ||
      reinterpret_cast<uintptr_t>(Hic) % 8 != 0)
    return SPQR_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int np = (n + NB - 1) / NB * NB, nb = np / NB;
  double* L = static_cast<double*>(workspace);
  double* X = L + (size_t)np * np;
  double* Dinv = X + (size_t)np * np;
  const unsigned cells = (unsigned)(((size_t)np * np + 255) / 256);
  hipLaunchKernelGGL(init_reversed_kernel, dim3(cells), dim3(256), 0, st, H, n, np, lambda, L);
  for (int kb = 0; kb < nb; ++kb) {
    hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(64), 0, st, L, np, kb, Dinv);
    const int rest = nb - kb - 1;
    if (rest > 0) {
      hipLaunchKernelGGL(trsm_panel_kernel, dim3(rest), dim3(256), 0, st, L, np, kb, Dinv);
      hipLaunchKernelGGL(syrk_kernel, dim3(rest, rest), dim3(256), 0, st, L, np, kb);
    }
  }
  for (int b = NB; b < np; b *= 2) {
    const int tiles = b / NB, pairs = (np + 2 * b - 1) / (2 * b);
    hipLaunchKernelGGL(trtri_step1_kernel, dim3(tiles, tiles, pairs), dim3(256), 0, st, L, Dinv, np, b, X);
    hipLaunchKernelGGL(trtri_step2_kernel, dim3(tiles, tiles, pairs), dim3(256), 0, st, L, Dinv, np, b, X);
  }
  hipLaunchKernelGGL(unreverse_kernel, dim3((unsigned)(((size_t)n * n + 255) / 256)), dim3(256), 0, st, L, Dinv, n, np, Hic);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

}  // extern "C"
