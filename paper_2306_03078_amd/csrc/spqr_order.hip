// The activation-order heuristic around the quantiser (App. B: permutation_order act_order; Sec. 5 ablations): the
// input columns are processed in the order of decreasing Hessian diagonal.  perm[j] = the original column that is
// processed (and stored) as column j; ties go to the smaller index, so the order is a pure function of diag(H).
//
// Sort: a bitonic network over (key, index) pairs in global memory, one launch per compare-exchange step (n is at
// most 65536: 136 short launches at worst, 78 for n = 4096), padded to a power of two with keys of minus infinity.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

#include "../../include/spqr_encode.h"

namespace spqr_ord {

__global__ void __launch_bounds__(256) init_keys_kernel(const double* __restrict__ H, int n, int np2, double* __restrict__ key,
                                                       int32_t* __restrict__ idx) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= np2) return;
  key[i] = i < n ? H[(size_t)i * n + i] : -INFINITY;
  idx[i] = i;
}

// (ka, ia) comes before (kb, ib): larger key first, equal keys by index.
__device__ __forceinline__ bool before(double ka, int ia, double kb, int ib) { return ka > kb || (ka == kb && ia < ib); }

__global__ void __launch_bounds__(256) bitonic_step_kernel(double* __restrict__ key, int32_t* __restrict__ idx, int np2, int k, int j) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= np2) return;
  const int l = i ^ j;
  if (l <= i) return;
  const double ki = key[i], kl = key[l];
  const int ii = idx[i], il = idx[l];
  const bool up = (i & k) == 0;              // this pair is put in order (up) or in reverse order
  const bool swap = up ? before(kl, il, ki, ii) : before(ki, ii, kl, il);
  if (swap) { key[i] = kl; key[l] = ki; idx[i] = il; idx[l] = ii; }
}

__global__ void __launch_bounds__(256) permute_columns_kernel(const double* __restrict__ W, int m, int n, const int32_t* __restrict__ perm,
                                                             double* __restrict__ out) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)m * n) return;
  const int i = (int)(t / n), j = (int)(t % n);
  out[t] = W[(size_t)i * n + perm[j]];
}

__global__ void __launch_bounds__(256) permute_symmetric_kernel(const double* __restrict__ H, int n, const int32_t* __restrict__ perm,
                                                               double* __restrict__ out) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)n * n) return;
  const int i = (int)(t / n), j = (int)(t % n);
  out[t] = H[(size_t)perm[i] * n + perm[j]];
}

static int pow2_at_least(int n) { int p = 1; while (p < n) p <<= 1; return p; }

}  // namespace spqr_ord

extern "C" {

size_t spqr_act_order_workspace_bytes(int32_t n) {
  if (n < 1) return 0;
  const size_t p = (size_t)spqr_ord::pow2_at_least(n);
  return p * (sizeof(double) + sizeof(int32_t));
}

int spqr_act_order(const double* H, int32_t n, int32_t* perm, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace spqr_ord;
  if (!H || !perm || !workspace) return SPQR_ERR_NULL;
  if (n < 1 || n > 65536) return SPQR_ERR_SHAPE;
  if (workspace_bytes < spqr_act_order_workspace_bytes(n)) return SPQR_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || reinterpret_cast<uintptr_t>(H) % 8 != 0 ||
      reinterpret_cast<uintptr_t>(perm) % 4 != 0)
    return SPQR_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int np2 = pow2_at_least(n);
  double* key = static_cast<double*>(workspace);
  int32_t* idx = reinterpret_cast<int32_t*>(key + np2);
  const dim3 grid((np2 + 255) / 256), block(256);
  hipLaunchKernelGGL(init_keys_kernel, grid, block, 0, st, H, n, np2, key, idx);
  for (int k = 2; k <= np2; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) hipLaunchKernelGGL(bitonic_step_kernel, grid, block, 0, st, key, idx, np2, k, j);
  if (hipMemcpyAsync(perm, idx, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, st) != hipSuccess) return SPQR_ERR_HIP;
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

int spqr_permute_columns(const double* W, int32_t m, int32_t n, const int32_t* perm, double* W_out, void* stream) {
  using namespace spqr_ord;
  if (!W || !perm || !W_out) return SPQR_ERR_NULL;
  if (m < 1 || n < 1) return SPQR_ERR_SHAPE;
  if (W == W_out) return SPQR_ERR_PARAM;
  const size_t cells = (size_t)m * n;
  hipLaunchKernelGGL(permute_columns_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     W, m, n, perm, W_out);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

int spqr_permute_symmetric(const double* H, int32_t n, const int32_t* perm, double* H_out, void* stream) {
  using namespace spqr_ord;
  if (!H || !perm || !H_out) return SPQR_ERR_NULL;
  if (n < 1) return SPQR_ERR_SHAPE;
  if (H == H_out) return SPQR_ERR_PARAM;
  const size_t cells = (size_t)n * n;
  hipLaunchKernelGGL(permute_symmetric_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     H, n, perm, H_out);
  return hipGetLastError() == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

}  // extern "C"
