// Internal interfaces between the library's translation units (launchers are host functions).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

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

// ---- spqr_dispatch.hip: what the C ABI calls ----
hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                       hipStream_t stream, bool force_generic);
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, bool force_generic);
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys,
                             int y_dtype, hipStream_t stream, bool force_generic);

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
                             int y_dtype, hipStream_t stream, bool force_generic);

// ---- spqr_mfma.hip: the matrix-core path for batches above 4 ----
// Whether the path exists for this geometry / is worth taking for a batch of b vectors on this stream.
bool mfma_has_instance(const Geometry& g);
bool mfma_wanted(const Geometry& g, int b, hipStream_t stream);
// hipErrorNotSupported: no scratch to be had; the caller takes the vector path.  b <= 16.
hipError_t launch_mfma(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream);
hipError_t launch_mfma_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream);
// Steps of 64 tiles per workgroup of the batch path's dense launch (host arithmetic only, see the definition).
int plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups);

// ---- spqr_misc.hip: fallback product, debug decode, validation ----
hipError_t launch_generic(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_dequant(const DevMatrix& A, int what, void* out, hipStream_t stream);
hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream);

}  // namespace spqr
