// Host-callable launchers implemented in spqr_kernels.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "spqr_device.h"

namespace spqr {

bool has_tuned_gemv(const Geometry& g);
hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                       hipStream_t stream, bool force_generic);
hipError_t launch_gemm(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype,
                       hipStream_t stream, bool force_generic);
// `count` matrices sharing x and the format, one launch when a tuned kernel exists and no
// permutation is set, else one launch each.
hipError_t launch_gemv_fused(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                             int y_dtype, hipStream_t stream, bool force_generic);
hipError_t launch_gemm_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys,
                             int y_dtype, hipStream_t stream, bool force_generic);
hipError_t launch_dequant(const DevMatrix& A, int what, void* out, hipStream_t stream);
hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream);

// Steps of 64 tiles per workgroup of the batch path's dense launch (host arithmetic only, see the definition).
int plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups);

}  // namespace spqr
