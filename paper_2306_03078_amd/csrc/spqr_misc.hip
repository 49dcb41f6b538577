// Generic fallback product, debug decode and validation kernels with their launchers.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_device.h"
#include "spqr_kernels.h"

namespace spqr {

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
  // the dwords that hold binary16 numbers: the second-level ones behind the codes, or all of them
  const int first = A.g.layout == kStats16 ? 0 : 3 * A.g.beta2 / 16;
  bool bad = false;
  for (int d = first; d < A.g.sd; ++d) {
    const uint32_t a = ld32(A.packed, stat_dword_offset(A.g, tr, tc, d));
    bad = bad || (a & 0x7C00u) == 0x7C00u || (a & 0x7C000000u) == 0x7C000000u;
  }
  if (bad) atomicMax(flag + 1, 1);
}

__global__ void check_perm_kernel(DevMatrix A, int* flag) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= A.g.n) return;
  const int p = A.perm[j];
  if (p < 0 || p >= A.g.n) atomicMax(flag + 2, 1);
}

hipError_t launch_generic(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream) {
  const int rows_per_block = 4;
  hipLaunchKernelGGL(gemv_generic_kernel, dim3((A.g.m + rows_per_block - 1) / rows_per_block),
                     dim3(64 * rows_per_block), 0, stream, A, x, y, y_dtype);
  return hipGetLastError();
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

// Runs the selected device checks and copies the three result words ([0] CSR status, [1] non-finite, [2] perm)
// to the host.  The words live in 16 bytes of device memory allocated for this call alone, so that calls on
// different streams never share them; the call synchronises anyway.
static hipError_t run_checks_on(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                                int* words, hipStream_t stream) {
  hipError_t e = hipSuccess;
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

hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream) {
  int* words = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&words), 4 * sizeof(int));
  if (e != hipSuccess) return e;
  e = run_checks_on(A, csr, finite, perm, host_words, words, stream);
  if (e != hipSuccess) (void)hipStreamSynchronize(stream);      // nothing of this call may still use the words
  const hipError_t ef = hipFree(words);
  return e != hipSuccess ? e : ef;
}

}  // namespace spqr
