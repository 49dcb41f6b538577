// Internal interfaces between the library's translation units (launchers are host functions).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "../../include/spqr.h"
#include "spqr_device.h"

namespace spqr {

constexpr int kCUs = 256;                    // compute units of an MI355X

// Function attributes (the opt-in for more than 64 KB of dynamic LDS) are per device, and
// several host threads may arrive at a launcher at once: what is remembered per kernel is kept
// per device in atomics; a device number out of range is simply not remembered.
constexpr int kMaxDevices = 64;
struct PerDevice {
  std::atomic<int> v[kMaxDevices];
  int get(int d) const { return d >= 0 && d < kMaxDevices ? v[d].load(std::memory_order_acquire) : 0; }
  void set(int d, int x) { if (d >= 0 && d < kMaxDevices) v[d].store(x, std::memory_order_release); }
};
inline int current_device() {
  int d = -1;
  return hipGetDevice(&d) == hipSuccess ? d : -1;
}

// Where a call's device scratch comes from.  from_caller: [p, p + bytes), 256-byte aligned, brought by the caller
// (or the library's static array): the call allocates nothing, frees nothing and waits for nothing.  Otherwise the
// library's own scratch, kept per stream (see spqr_mfma.hip).
struct Workspace {
  bool from_caller = false;
  uint8_t* p = nullptr;
  size_t bytes = 0;
};

// ---- spqr_dispatch.hip: what the C ABI calls ----
int option(int which);                       // SPQR_OPT_* switches, 0 unless spqr_set_option changed them
bool set_option(int which, int value);
hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream);
// hipErrorOutOfMemory: the caller's workspace is too small (never with library scratch).
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, const Workspace& ws);
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys,
                             int y_dtype, hipStream_t stream, const Workspace& ws);
size_t workspace_bound(const DevMatrix* As, int count, int b, bool with_dense_copy = true);

// ---- spqr_gemv.hip: the vector kernel ----
// Largest number of activation vectors (1, 2 or 4, at most `want`) one launch of the tuned kernel takes for this
// geometry; 0 if there is no tuned kernel.
int tuned_batch_width(const Geometry& g, int want);
bool has_tuned_gemv(const Geometry& g);
// One launch of the tuned kernel for nb = 1, 2 or 4 vectors (a width tuned_batch_width() returned).
hipError_t launch_tuned(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream);
// `count` matrices sharing x and the format, one launch when a tuned kernel exists and no
// permutation is set, else one launch each.
hipError_t launch_gemv_fused(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                             int y_dtype, hipStream_t stream);
// The same with one input vector per matrix (the matrices agree in n and format).
hipError_t launch_gemv_grouped(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys,
                               int y_dtype, hipStream_t stream);

// ---- spqr_mfma.hip: the matrix-core path for batches of 4 to 16 ----
// Whether the path exists for this geometry / is worth taking for a batch of b vectors (alloc_nodes: the scratch
// would be allocation nodes of a graph under capture).
bool mfma_has_instance(const Geometry& g);
bool mfma_wanted(const Geometry& g, int b, bool alloc_nodes);
bool stream_is_capturing(hipStream_t stream);
// hipErrorNotSupported: no library scratch to be had, the caller takes the vector path; hipErrorOutOfMemory: the
// caller's workspace is too small.  b <= 16.
hipError_t launch_mfma(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                       const Workspace& ws);
hipError_t launch_mfma_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream, const Workspace& ws);
// Upper bound of the scratch of such a call: one matrix at a time and, if `fused`, all of them in one launch set.
size_t mfma_workspace_bound(const DevMatrix* As, int count, int b, bool fused);
// The library's static device array as a workspace (callers that cannot allocate); its size is
// SPQR_STATIC_SCRATCH_BYTES.
hipError_t static_workspace(Workspace* ws);
// Steps of 64 tiles per workgroup of the batch path's dense launch (host arithmetic only, see the definition).
int plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups);

// Large batches through a dense binary16 copy of the matrix (spqr_prefill.hip) on the library's scratch or the
// caller's workspace.  hipErrorNotSupported: no scratch of that size to be had (or the stream is being captured
// and the library would have to allocate it): the caller takes the slices of 16.
hipError_t launch_prefill_scratch(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                                  const Workspace& ws);

// ---- spqr_prefill.hip: large batches ----
bool prefill_has_instance(const Geometry& g);
bool prefill_wanted(const DevMatrix& A, int b);
size_t prefill_workspace_bytes(const DevMatrix& A, int b);
// `scratch`: prefill_workspace_bytes(A, b) bytes, 256-byte aligned; Y 16-byte aligned.
hipError_t launch_prefill(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                          uint8_t* scratch);

// ---- spqr_misc.hip: fallback product, debug decode, validation ----
hipError_t launch_generic(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_dequant(const DevMatrix& A, int what, void* out, hipStream_t stream);
hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream);

}  // namespace spqr
