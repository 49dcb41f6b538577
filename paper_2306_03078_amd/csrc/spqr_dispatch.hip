// Which kernels a product call takes: host logic only.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_kernels.h"

namespace spqr {

// Y[b][m] = X[b][n] . W_hat^T.  Up to 4 activation vectors: the tuned vector
// kernel, all of them in one launch.  More, on 16x16 tiles and where it pays: slices
// of up to 16 with the dense part on the matrix cores (weights stream once per
// slice), then the finishing kernel with the outliers.  Else slices of 4.
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, bool force_generic) {
  const Geometry& g = A.g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  bool mfma_ok = !force_generic && mfma_has_instance(g);
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
      e = launch_mfma(A, xk, nb16, yk, y_dtype, stream);
      if (e == hipErrorNotSupported) { mfma_ok = false; continue; }   // no memory pool here: the vector path from now on
      if (e != hipSuccess) return e;
      k += nb16;
      continue;
    }
    const int nb = force_generic ? 0 : tuned_batch_width(g, left);
    if (nb >= 1) { e = launch_tuned(A, xk, nb, yk, y_dtype, stream); done = nb; }
    else e = launch_generic(A, xk, yk, y_dtype, stream);
    if (e != hipSuccess) return e;
    k += done;
  }
  return hipSuccess;
}

// Y_i[b][m_i] = X[b][n] . W_hat_i^T for matrices that share X.  Batches the matrix-core path takes go through it
// fused (slices of 16); everything else is one launch_gemm per matrix.
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream, bool force_generic) {
  const Geometry& g = As[0].g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  bool mfma_ok = count > 1 && !force_generic && mfma_has_instance(g);
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
      hipError_t e = launch_mfma_fused(As, count, xk, nb16, yk, y_dtype, stream);
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

}  // namespace spqr
