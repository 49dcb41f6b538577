// Which kernels a product call takes: host logic only.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_kernels.h"

namespace spqr {

// Process-wide switches for tuning runs and tests (spqr_set_option); all zero in production.
static std::atomic<int> g_options[SPQR_OPT_COUNT_];
int option(int which) {
  return which >= 0 && which < SPQR_OPT_COUNT_ ? g_options[which].load(std::memory_order_relaxed) : 0;
}
bool set_option(int which, int value) {
  if (which < 0 || which >= SPQR_OPT_COUNT_) return false;
  g_options[which].store(value, std::memory_order_relaxed);
  return true;
}

// Smallest batch the matrix-core path is considered for (below it the vector kernel's 2- and 4-vector forms win
// or tie on every layer measured).
static constexpr int kMfmaMinBatch = 4;

// Y[b][m] = X[b][n] . W_hat^T.  Up to 4 activation vectors: the tuned vector kernel, all of them in one launch
// (4 vectors on a large layer: the matrix cores, see mfma_wanted).  More, where a matrix-core instance exists and
// it pays: slices of up to 16 with the dense part on the matrix cores (weights stream once per slice), then the
// finishing kernel with the outliers.  Else slices of 4.
// ws.from_caller: scratch comes from the caller; nothing is allocated, freed or waited for, the choice of path
// never depends on the stream's state, and a workspace that is too small is hipErrorOutOfMemory.
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, const Workspace& ws) {
  const Geometry& g = A.g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  const bool force_generic = option(SPQR_OPT_FORCE_GENERIC) != 0;
  bool mfma_ok = !force_generic && mfma_has_instance(g);
  const bool alloc_nodes = mfma_ok && !ws.from_caller && b >= kMfmaMinBatch && stream_is_capturing(stream);
  // A large batch: one dense binary16 copy of the matrix in scratch, one matrix-core multiply for all vectors.
  if (!force_generic && prefill_has_instance(g) && prefill_wanted(A, b) &&
      reinterpret_cast<uintptr_t>(Y) % 16 == 0) {
    const hipError_t e = launch_prefill_scratch(A, X, b, Y, y_dtype, stream, ws);
    if (e != hipErrorNotSupported) return e;   // no scratch of that size: the slices below
  }
  int k = 0;
  while (k < b) {
    const uint16_t* xk = X + (size_t)k * g.n;
    void* yk = static_cast<uint8_t*>(Y) + (size_t)k * g.m * ysz;
    const int left = b - k;
    hipError_t e;
    int done = 1;
    // the matrix-core path takes up to 16 vectors per pass over the weights
    const int nb16 = left < 16 ? left : 16;
    if (mfma_ok && left >= kMfmaMinBatch && mfma_wanted(g, nb16, alloc_nodes)) {
      e = launch_mfma(A, xk, nb16, yk, y_dtype, stream, ws);
      if (e == hipErrorNotSupported) { mfma_ok = false; continue; }   // no scratch to be had: the vector path from now on
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

// Whether launch_gemm_fused takes the fused matrix-core launches for a slice of nb vectors.
static bool fused_mfma_wanted(const DevMatrix* As, int count, int nb, bool alloc_nodes) {
  Geometry all = As[0].g;                    // the rule looks at the weights of all matrices together
  int64_t rows = 0;
  for (int i = 0; i < count; ++i) rows += As[i].g.m;
  all.m = (int)(rows < (1 << 30) ? rows : (1 << 30));
  return nb >= kMfmaMinBatch && mfma_wanted(all, nb, alloc_nodes);
}

// Y_i[b][m_i] = X[b][n] . W_hat_i^T for matrices that share X.  Batches the matrix-core path takes go through it
// fused (slices of 16); everything else is one launch_gemm per matrix.
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream, const Workspace& ws) {
  const Geometry& g = As[0].g;
  const size_t ysz = y_dtype == SPQR_F32 ? 4 : 2;
  const bool force_generic = option(SPQR_OPT_FORCE_GENERIC) != 0;
  bool mfma_ok = count > 1 && !force_generic && mfma_has_instance(g);
  // Not while the stream is being captured into a graph: a replay of a graph that held 12 fused batch calls among
  // 42 calls (a whole decoder block, six weight copies) ended in a memory fault inside the fused finishing kernel,
  // while the same calls pass eagerly and graphs of the per-matrix path replay correctly; until the cause is
  // known, captured calls take the per-matrix path.
  const bool capturing = mfma_ok && b >= kMfmaMinBatch && stream_is_capturing(stream);
  if (capturing) mfma_ok = false;
  // a large batch: every matrix through its dense copy (launch_gemm falls back to the slices where it cannot)
  bool dense = !force_generic && prefill_has_instance(g);
  for (int i = 0; i < count && dense; ++i) dense = prefill_wanted(As[i], b);
  if (dense) mfma_ok = false;
  int k = 0;
  while (k < b) {
    const int left = b - k, nb16 = left < 16 ? left : 16;
    const uint16_t* xk = X + (size_t)k * g.n;
    void* yk[SPQR_MAX_FUSED];
    for (int i = 0; i < count; ++i) yk[i] = static_cast<uint8_t*>(Ys[i]) + (size_t)k * As[i].g.m * ysz;
    if (mfma_ok && fused_mfma_wanted(As, count, nb16, false)) {
      hipError_t e = launch_mfma_fused(As, count, xk, nb16, yk, y_dtype, stream, ws);
      if (e == hipErrorNotSupported) { mfma_ok = false; continue; }
      if (e != hipSuccess) return e;
      k += nb16;
      continue;
    }
    // the rest of the batch, matrix by matrix (each call applies its own rule)
    for (int i = 0; i < count; ++i) {
      hipError_t e = launch_gemm(As[i], xk, left, yk[i], y_dtype, stream, ws);
      if (e != hipSuccess) return e;
    }
    k = b;
  }
  return hipSuccess;
}

// Device scratch a product of these matrices with a batch of b needs at most when the caller brings it
// (0: the call takes kernels that need none).  One matrix: launch_gemm; several: launch_gemm_fused, which may
// fall back to one launch_gemm per matrix, so the bound covers both.
size_t workspace_bound(const DevMatrix* As, int count, int b, bool with_dense_copy) {
  if (option(SPQR_OPT_FORCE_GENERIC) != 0) return 0;
  size_t worst = 0;
  // a large batch: the dense copy of one matrix at a time (a smaller workspace sends the call to the slices of 16)
  if (with_dense_copy && prefill_has_instance(As[0].g))
    for (int i = 0; i < count; ++i) {
      if (!prefill_wanted(As[i], b)) continue;
      const size_t need = prefill_workspace_bytes(As[i], b);
      if (need > worst) worst = need;
    }
  if (!mfma_has_instance(As[0].g) || b < kMfmaMinBatch) return worst;
  // slices of 16, then the rest: the needs of min(b, 16) vectors and of the last slice bound all of them
  const int sizes[2] = {b < 16 ? b : 16, b % 16};
  for (int si = 0; si < 2; ++si) {
    const int nb = sizes[si];
    if (nb < kMfmaMinBatch) continue;
    const bool fused = count > 1 && fused_mfma_wanted(As, count, nb, false);
    bool any_single = false;
    for (int i = 0; i < count; ++i) any_single = any_single || mfma_wanted(As[i].g, nb, false);
    if (!fused && !any_single) continue;
    const size_t need = mfma_workspace_bound(As, count, nb, fused);
    if (need > worst) worst = need;
  }
  return worst;
}

hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream) {
  Workspace none;
  return launch_gemm(A, x, 1, y, y_dtype, stream, none);
}

}  // namespace spqr
