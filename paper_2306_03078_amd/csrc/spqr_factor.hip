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
//   trtri     X = L^-1 by block forward substitution, one workgroup per slice of 16 columns of X (columns of an
//             inverse are independent), using the diagonal blocks' inverses
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

// acc[r][c] += sum_{k < K} fa(ty*4 + r, k) * fb(tx*4 + c, k): a 64 x 64 tile by 256 threads.
template <class FA, class FB>
__device__ __forceinline__ void tile_nt(double (&acc)[4][4], int K, FA fa, FB fb, double (*As)[NB + 1],
                                        double (*Bs)[NB + 1]) {
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
      for (int r = 0; r < 4; ++r) { av[r] = As[kk][ty * 4 + r]; bv[r] = Bs[kk][tx * 4 + r]; }
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
  __shared__ double As[KC][NB + 1], Bs[KC][NB + 1];
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
      const int i = i0 + ty * 4 + r, j = j0 + tx * 4 + c;
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

// Diagonal block kb: Cholesky factor in place, its inverse to Dinv[kb].
__global__ void __launch_bounds__(256) potrf_diag_kernel(double* __restrict__ L, int np, int kb, double* __restrict__ Dinv) {
  __shared__ double D[NB][NB], V[NB][NB];   // 64 KB: the static limit, so no padding
  const int t = threadIdx.x;
  double* blk = L + (size_t)kb * NB * np + (size_t)kb * NB;
  for (int idx = t; idx < NB * NB; idx += 256) D[idx >> 6][idx & 63] = blk[(size_t)(idx >> 6) * np + (idx & 63)];
  __syncthreads();
  for (int j = 0; j < NB; ++j) {
    if (t == 0) D[j][j] = sqrt(D[j][j]);
    __syncthreads();
    if (t > j && t < NB) D[t][j] = D[t][j] / D[j][j];
    __syncthreads();
    // trailing update of the lower triangle: rows i > j, columns j < k <= i
    const int rem = NB - 1 - j;
    for (int idx = t; idx < rem * rem; idx += 256) {
      const int i = j + 1 + idx / rem, k = j + 1 + idx % rem;
      if (k <= i) D[i][k] = fma(-D[i][j], D[k][j], D[i][k]);
    }
    __syncthreads();
  }
  // inverse of the lower triangular block, one column per thread
  if (t < NB) {
    const int c = t;
    for (int i = 0; i < c; ++i) V[i][c] = 0.0;
    V[c][c] = 1.0 / D[c][c];
    for (int i = c + 1; i < NB; ++i) {
      double s = 0.0;
      for (int k = c; k < i; ++k) s = fma(D[i][k], V[k][c], s);
      V[i][c] = -s / D[i][i];
    }
  }
  __syncthreads();
  double* inv = Dinv + (size_t)kb * NB * NB;
  for (int idx = t; idx < NB * NB; idx += 256) {
    const int i = idx >> 6, k = idx & 63;
    blk[(size_t)i * np + k] = k <= i ? D[i][k] : 0.0;
    inv[idx] = V[i][k];
  }
}

// Panel below diagonal block kb: A[ib, kb] <- A[ib, kb] . inv(L_kk)^T
__global__ void __launch_bounds__(256) trsm_panel_kernel(double* __restrict__ L, int np, int kb, const double* __restrict__ Dinv) {
  __shared__ double As[KC][NB + 1], Bs[KC][NB + 1];
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
    for (int c = 0; c < 4; ++c) blk[(size_t)(ty * 4 + r) * np + tx * 4 + c] = acc[r][c];
}

// Trailing update: A[ib, jb] -= P_ib . P_jb^T for kb < jb <= ib.
__global__ void __launch_bounds__(256) syrk_kernel(double* __restrict__ L, int np, int kb) {
  __shared__ double As[KC][NB + 1], Bs[KC][NB + 1];
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
    for (int c = 0; c < 4; ++c) blk[(size_t)(ty * 4 + r) * np + tx * 4 + c] -= acc[r][c];
}

// X = L^-1, 16 columns per workgroup: X[kb] = inv(L_kk) (its 16 columns); for ib > kb:
// X[ib] = -inv(L_ii) . sum_{kb <= jb < ib} L[ib, jb] . X[jb].
__global__ void __launch_bounds__(256) trtri_kernel(const double* __restrict__ L, int np, const double* __restrict__ Dinv,
                                                   double* __restrict__ X) {
  __shared__ double Ls[NB][NB + 1], Xs[NB][17], Ss[NB][17];
  const int t = threadIdx.x;
  const int c0 = blockIdx.x * 16, kb = c0 / NB, nb = np / NB;
  const int r = t >> 2, cq = (t & 3) * 4;
  // rows above the diagonal block are zero
  for (int idx = t; idx < kb * NB * 16; idx += 256) X[(size_t)(idx >> 4) * np + c0 + (idx & 15)] = 0.0;
  {
    const double* inv = Dinv + (size_t)kb * NB * NB;
    for (int idx = t; idx < NB * 16; idx += 256) {
      const int i = idx >> 4, c = idx & 15;
      X[(size_t)(kb * NB + i) * np + c0 + c] = inv[i * NB + (c0 - kb * NB) + c];
    }
  }
  __syncthreads();
  for (int ib = kb + 1; ib < nb; ++ib) {
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    for (int jb = kb; jb < ib; ++jb) {
      const double* lb = L + (size_t)ib * NB * np + (size_t)jb * NB;
      for (int idx = t; idx < NB * NB; idx += 256) Ls[idx >> 6][idx & 63] = lb[(size_t)(idx >> 6) * np + (idx & 63)];
      for (int idx = t; idx < NB * 16; idx += 256) Xs[idx >> 4][idx & 15] = X[(size_t)(jb * NB + (idx >> 4)) * np + c0 + (idx & 15)];
      __syncthreads();
#pragma unroll 8
      for (int k = 0; k < NB; ++k) {
        const double l = Ls[r][k];
#pragma unroll
        for (int c = 0; c < 4; ++c) s[c] = fma(l, Xs[k][cq + c], s[c]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) Ss[r][cq + c] = s[c];
    const double* inv = Dinv + (size_t)ib * NB * NB;
    for (int idx = t; idx < NB * NB; idx += 256) Ls[idx >> 6][idx & 63] = inv[idx];
    __syncthreads();
    double o[4] = {0.0, 0.0, 0.0, 0.0};
    for (int k = 0; k <= r; ++k) {
      const double l = Ls[r][k];
#pragma unroll
      for (int c = 0; c < 4; ++c) o[c] = fma(l, Ss[k][cq + c], o[c]);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) X[(size_t)(ib * NB + r) * np + c0 + cq + c] = -o[c];
    __syncthreads();       // this block row of X is read back as X[jb] from the next ib on
  }
}

__global__ void __launch_bounds__(256) unreverse_kernel(const double* __restrict__ X, int n, int np, double* __restrict__ U) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)n * n) return;
  const int i = (int)(idx / n), j = (int)(idx % n);
  U[idx] = j >= i ? X[(size_t)(n - 1 - i) * np + (n - 1 - j)] : 0.0;
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
    hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(256), 0, st, L, np, kb, Dinv);
    const int rest = nb - kb - 1;
    if (rest > 0) {
      hipLaunchKernelGGL(trsm_panel_kernel, dim3(rest), dim3(256), 0, st, L, np, kb, Dinv);
      hipLaunchKernelGGL(syrk_kernel, dim3(rest, rest), dim3(256), 0, st, L, np, kb);
    }
  }
  hipLaunchKernelGGL(trtri_kernel, dim3(np / 16), dim3(256), 0, st, L, np, Dinv, X);
  hipLaunchKernelGGL(unreverse_kernel, dim3((unsigned)(((size_t)n * n + 255) / 256)), dim3(256), 0, st, X, n, np, Hic);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

}  // extern "C"
