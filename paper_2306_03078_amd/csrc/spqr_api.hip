// C ABI entry points: descriptor validation and dispatch to the kernels.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "../../include/spqr.h"
#include "spqr_kernels.h"
#include "spqr_gemv_inst.h"
#include "spqr_test_hooks.h"

namespace {

// O(1) checks shared by every device entry point.
int to_device_matrix(const spqr_matrix_t* A, spqr::DevMatrix* D) {
  if (!A) return SPQR_ERR_NULL;
  if (A->max_row_nnz < 0) return SPQR_ERR_PARAM;
  int rc = spqr::make_geometry(A->layout_version, A->m, A->n, A->w_bits, A->s_bits, A->z_bits, A->beta1, A->beta2,
                               A->group_axis, &D->g);
  if (rc) return rc;
  if (!A->packed || !A->row_ptr) return SPQR_ERR_NULL;
  if (A->nnz < 0 || A->nnz > (int64_t)A->m * A->n || A->nnz > 0x7FFFFFFFll) return SPQR_ERR_SIZE;
  if (A->nnz > 0 && (!A->col_idx || !A->out_val)) return SPQR_ERR_NULL;
  if (A->packed_bytes != (int64_t)D->g.ntr * D->g.ntc * D->g.tile_bytes) return SPQR_ERR_SIZE;
  if (reinterpret_cast<uintptr_t>(A->packed) % 16 != 0) return SPQR_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(A->row_ptr) % 4 != 0) return SPQR_ERR_ALIGN;
  // the kernels read the outlier arrays in aligned 16-byte granules
  if (reinterpret_cast<uintptr_t>(A->col_idx) % 16 != 0) return SPQR_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(A->out_val) % 16 != 0) return SPQR_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(A->perm) % 4 != 0) return SPQR_ERR_ALIGN;
  D->packed = static_cast<const uint8_t*>(A->packed);
  D->row_ptr = A->row_ptr;
  D->col = A->col_idx;
  D->val = A->out_val;
  D->perm = A->perm;
  D->nnz = A->nnz;
  D->max_row_nnz = A->max_row_nnz;
  return SPQR_OK;
}

int hip_status(hipError_t e) {
  if (e == hipSuccess) return SPQR_OK;
  if (e == hipErrorOutOfMemory) return SPQR_ERR_WORKSPACE;   // the launchers' signal for a workspace that is too small
  return SPQR_ERR_HIP;
}

// Checks shared by the batch entry points, the descriptors first; fills D[0..count).
int check_batch_call(const spqr_matrix_t* const* A, int count, const uint16_t* X_f16, int b, void* const* Y,
                     int y_dtype, spqr::DevMatrix* D) {
  if (!A) return SPQR_ERR_NULL;
  if (count < 1 || count > SPQR_MAX_FUSED) return SPQR_ERR_PARAM;
  for (int i = 0; i < count; ++i) {
    int rc = to_device_matrix(A[i], &D[i]);
    if (rc) return rc;
  }
  if (!Y || !X_f16) return SPQR_ERR_NULL;
  if (b < 1 || b > SPQR_MAX_BATCH) return SPQR_ERR_BATCH;
  if (y_dtype != SPQR_F32 && y_dtype != SPQR_F16) return SPQR_ERR_DTYPE;
  if (reinterpret_cast<uintptr_t>(X_f16) % 16 != 0) return SPQR_ERR_ALIGN;
  for (int i = 0; i < count; ++i) {
    if (!Y[i]) return SPQR_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(Y[i]) % (y_dtype == SPQR_F32 ? 4 : 2) != 0) return SPQR_ERR_ALIGN;
    const spqr_matrix_t *a = A[i], *a0 = A[0];
    if (a->n != a0->n || a->w_bits != a0->w_bits || a->s_bits != a0->s_bits || a->z_bits != a0->z_bits ||
        a->beta1 != a0->beta1 || a->beta2 != a0->beta2 || a->group_axis != a0->group_axis ||
        a->layout_version != a0->layout_version || a->perm != a0->perm)
      return SPQR_ERR_PARAM;
  }
  return SPQR_OK;
}

int caller_workspace(void* workspace, int64_t workspace_bytes, spqr::Workspace* ws) {
  if (workspace_bytes < 0) return SPQR_ERR_SIZE;
  if (workspace_bytes > 0 && !workspace) return SPQR_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return SPQR_ERR_ALIGN;
  ws->from_caller = true;
  ws->p = static_cast<uint8_t*>(workspace);
  ws->bytes = static_cast<size_t>(workspace_bytes);
  return SPQR_OK;
}

}  // namespace

extern "C" int spqr_pack_check(const spqr_matrix_t* A, uint32_t flags, void* stream) {
  spqr::DevMatrix D;
  int rc = to_device_matrix(A, &D);
  if (rc) return rc;
  if ((flags & ~(SPQR_CHECK_CSR | SPQR_CHECK_NONFINITE | SPQR_CHECK_PERM)) != 0) return SPQR_ERR_PARAM;
  if (flags == 0) return SPQR_OK;
  int words[3] = {0, 0, 0};
  hipError_t e = spqr::run_checks(D, flags & SPQR_CHECK_CSR, flags & SPQR_CHECK_NONFINITE,
                                  flags & SPQR_CHECK_PERM, words, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return SPQR_ERR_HIP;
  if (words[0] != 0) return SPQR_ERR_CSR;
  if (words[2] != 0) return SPQR_ERR_PARAM;
  if (words[1] != 0) return SPQR_ERR_NONFINITE;
  return SPQR_OK;
}

extern "C" int spqr_set_option(int option, int value) {
  bool ok = true;
  switch (option) {
    case SPQR_OPT_BATCH_PATH: ok = value >= SPQR_BATCH_PATH_AUTO && value <= SPQR_BATCH_PATH_DENSE; break;
    case SPQR_OPT_FORCE_GENERIC: ok = value == 0 || value == 1; break;
    case SPQR_OPT_BATCH_STEPS: ok = value >= 0; break;
    case SPQR_OPT_DENSE_ROWS: ok = value == 0 || value == 64 || value == 128; break;
    case SPQR_OPT_GEMV_PLAN: ok = value >= 0 && value < 16 * 17; break;
    default: ok = false;
  }
  return ok && spqr::set_option(option, value) ? SPQR_OK : SPQR_ERR_PARAM;
}

extern "C" int spqr_gemm_smallbatch(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y,
                                    int y_dtype, void* stream) {
  spqr::DevMatrix D;
  int rc = check_batch_call(&A, 1, X_f16, b, &Y, y_dtype, &D);
  if (rc) return rc;
  spqr::Workspace library;
  return hip_status(spqr::launch_gemm(D, X_f16, b, Y, y_dtype, static_cast<hipStream_t>(stream), library));
}

extern "C" int spqr_gemv(const spqr_matrix_t* A, const uint16_t* x_f16, void* y, int y_dtype,
                         void* stream) {
  return spqr_gemm_smallbatch(A, x_f16, 1, y, y_dtype, stream);
}

extern "C" int64_t spqr_workspace_bytes(const spqr_matrix_t* const* A, int count, int b) {
  if (!A) return SPQR_ERR_NULL;
  if (count < 1 || count > SPQR_MAX_FUSED) return SPQR_ERR_PARAM;
  if (b < 1 || b > SPQR_MAX_BATCH) return SPQR_ERR_BATCH;
  spqr::DevMatrix D[SPQR_MAX_FUSED];
  for (int i = 0; i < count; ++i) {
    if (!A[i]) return SPQR_ERR_NULL;
    int rc = to_device_matrix(A[i], &D[i]);
    if (rc) return rc;
    if (A[i]->n != A[0]->n || A[i]->w_bits != A[0]->w_bits || A[i]->beta1 != A[0]->beta1 || A[i]->beta2 != A[0]->beta2 ||
        A[i]->group_axis != A[0]->group_axis || A[i]->perm != A[0]->perm)
      return SPQR_ERR_PARAM;
  }
  return static_cast<int64_t>(spqr::workspace_bound(D, count, b));
}

extern "C" int spqr_gemm_smallbatch_ws(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y, int y_dtype,
                                       void* workspace, int64_t workspace_bytes, void* stream) {
  spqr::DevMatrix D;
  int rc = check_batch_call(&A, 1, X_f16, b, &Y, y_dtype, &D);
  if (rc) return rc;
  spqr::Workspace ws;
  rc = caller_workspace(workspace, workspace_bytes, &ws);
  if (rc) return rc;
  return hip_status(spqr::launch_gemm(D, X_f16, b, Y, y_dtype, static_cast<hipStream_t>(stream), ws));
}

extern "C" int spqr_gemm_fused_ws(const spqr_matrix_t* const* A, int count, const uint16_t* X_f16, int b,
                                  void* const* Y, int y_dtype, void* workspace, int64_t workspace_bytes,
                                  void* stream) {
  spqr::DevMatrix D[SPQR_MAX_FUSED];
  int rc = check_batch_call(A, count, X_f16, b, Y, y_dtype, D);
  if (rc) return rc;
  spqr::Workspace ws;
  rc = caller_workspace(workspace, workspace_bytes, &ws);
  if (rc) return rc;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  return hip_status(b == 1 ? spqr::launch_gemv_fused(D, count, X_f16, Y, y_dtype, st)
                           : spqr::launch_gemm_fused(D, count, X_f16, b, Y, y_dtype, st, ws));
}

extern "C" int spqr_gemv_fused(const spqr_matrix_t* const* A, int count, const uint16_t* x_f16,
                               void* const* y, int y_dtype, void* stream) {
  spqr::DevMatrix D[SPQR_MAX_FUSED];
  int rc = check_batch_call(A, count, x_f16, 1, y, y_dtype, D);
  if (rc) return rc;
  return hip_status(spqr::launch_gemv_fused(D, count, x_f16, y, y_dtype, static_cast<hipStream_t>(stream)));
}

extern "C" int spqr_gemv_grouped(const spqr_matrix_t* const* A, int count, const uint16_t* const* x_f16,
                                 void* const* y, int y_dtype, void* stream) {
  if (!A || !y || !x_f16) return SPQR_ERR_NULL;
  if (count < 1 || count > SPQR_MAX_GROUPED) return SPQR_ERR_PARAM;
  if (y_dtype != SPQR_F32 && y_dtype != SPQR_F16) return SPQR_ERR_DTYPE;
  spqr::DevMatrix D[SPQR_MAX_GROUPED];
  for (int i = 0; i < count; ++i) {
    if (!A[i] || !y[i] || !x_f16[i]) return SPQR_ERR_NULL;
    int rc = to_device_matrix(A[i], &D[i]);
    if (rc) return rc;
    if (reinterpret_cast<uintptr_t>(x_f16[i]) % 16 != 0) return SPQR_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(y[i]) % (y_dtype == SPQR_F32 ? 4 : 2) != 0) return SPQR_ERR_ALIGN;
  }
  // matrices that agree in format (and have no permutation) go together, up to SPQR_MAX_FUSED at a time, in the
  // order given; the launcher sorts them by input width
  bool done[SPQR_MAX_GROUPED] = {};
  const hipStream_t st = static_cast<hipStream_t>(stream);
  for (int i = 0; i < count; ++i) {
    if (done[i]) continue;
    spqr::DevMatrix G[SPQR_MAX_FUSED];
    const uint16_t* xs[SPQR_MAX_FUSED];
    void* ys[SPQR_MAX_FUSED];
    int k = 0;
    for (int j = i; j < count && k < SPQR_MAX_FUSED; ++j) {
      const spqr_matrix_t *a = A[j], *a0 = A[i];
      const bool same = a->w_bits == a0->w_bits && a->beta1 == a0->beta1 && a->beta2 == a0->beta2 &&
                        a->group_axis == a0->group_axis && a->layout_version == a0->layout_version &&
                        a->perm == nullptr && a0->perm == nullptr;
      if (done[j] || (j != i && !same)) continue;
      G[k] = D[j]; xs[k] = x_f16[j]; ys[k] = y[j]; ++k;
      done[j] = true;
    }
    const hipError_t e = spqr::launch_gemv_grouped(G, k, xs, ys, y_dtype, st);
    if (e != hipSuccess) return SPQR_ERR_HIP;
  }
  return SPQR_OK;
}

extern "C" int spqr_gemm_fused(const spqr_matrix_t* const* A, int count, const uint16_t* X_f16, int b,
                               void* const* Y, int y_dtype, void* stream) {
  spqr::DevMatrix D[SPQR_MAX_FUSED];
  int rc = check_batch_call(A, count, X_f16, b, Y, y_dtype, D);
  if (rc) return rc;
  const hipStream_t st = static_cast<hipStream_t>(stream);
  spqr::Workspace library;
  return hip_status(b == 1 ? spqr::launch_gemv_fused(D, count, X_f16, Y, y_dtype, st)
                           : spqr::launch_gemm_fused(D, count, X_f16, b, Y, y_dtype, st, library));
}

extern "C" int spqr_gemm_smallbatch_noalloc(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y,
                                            int y_dtype, void* stream) {
  spqr::DevMatrix D;
  int rc = check_batch_call(&A, 1, X_f16, b, &Y, y_dtype, &D);
  if (rc) return rc;
  // sizes beyond the static array are refused before anything is launched
  if (spqr::workspace_bound(&D, 1, b, false) > (size_t)SPQR_STATIC_SCRATCH_BYTES) return SPQR_ERR_WORKSPACE;
  spqr::Workspace ws;
  if (spqr::static_workspace(&ws) != hipSuccess) return SPQR_ERR_HIP;
  return hip_status(spqr::launch_gemm(D, X_f16, b, Y, y_dtype, static_cast<hipStream_t>(stream), ws));
}

extern "C" int spqr_dequant_dense(const spqr_matrix_t* A, int what, void* out, void* stream) {
  spqr::DevMatrix D;
  int rc = to_device_matrix(A, &D);
  if (rc) return rc;
  if (!out) return SPQR_ERR_NULL;
  const int sel = what & 0xFF;
  if ((what & ~(0xFF | SPQR_OUT_WITH_OUTLIERS)) != 0 || sel > SPQR_OUT_DENSE_F16) return SPQR_ERR_DTYPE;
  if ((what & SPQR_OUT_WITH_OUTLIERS) && sel != SPQR_OUT_DENSE_F32 && sel != SPQR_OUT_DENSE_F16)
    return SPQR_ERR_DTYPE;
  hipError_t e = spqr::launch_dequant(D, what, out, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPQR_OK : SPQR_ERR_HIP;
}

extern "C" int spqr_plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups) {
  if (groups < 1 || nsteps < 1 || slots_one_step < 1 || slots < 1 || long_workgroups < 0) return SPQR_ERR_PARAM;
  return spqr::plan_batch_steps(groups, nsteps, slots_one_step, slots, long_workgroups);
}

extern "C" int spqr_plan_grouped(int count, const int32_t* m, const int32_t* n, const int32_t* max_row_nnz,
                                 const int64_t* nnz, int w_bits, int beta1, int beta2, int group_axis, int layout_version,
                                 int max_waves, int slots, int row_dots_on_matrix_cores, int32_t* entries,
                                 int32_t* wavefronts, int64_t* lds_bytes) {
  if (!m || !n || !max_row_nnz || !nnz || !entries || !wavefronts || !lds_bytes) return SPQR_ERR_NULL;
  if (count < 1 || count > SPQR_MAX_FUSED || max_waves < 1 || max_waves > 16 || slots < 1 || slots > 32) return SPQR_ERR_PARAM;
  spqr::DevMatrix D[SPQR_MAX_FUSED];
  const int sbits = layout_version == spqr::kStats16 ? 16 : 3;
  for (int i = 0; i < count; ++i) {
    if (max_row_nnz[i] < 0 || nnz[i] < 0) return SPQR_ERR_PARAM;
    const int rc = spqr::make_geometry(layout_version, m[i], n[i], w_bits, sbits, sbits, beta1, beta2, group_axis, &D[i].g);
    if (rc) return rc;
    D[i].packed = nullptr; D[i].row_ptr = nullptr; D[i].col = nullptr; D[i].val = nullptr; D[i].perm = nullptr;
    D[i].nnz = nnz[i]; D[i].max_row_nnz = max_row_nnz[i];
  }
  spqr::GroupedPlan gp;
  if (!spqr::plan_grouped(D, count, max_waves, slots, row_dots_on_matrix_cores != 0, &gp)) return SPQR_ERR_PARAM;
  for (int j = 0; j < gp.count; ++j) {
    const spqr::GroupedEntry& e = gp.e[j];
    int32_t* o = entries + 7 * j;
    o[0] = e.index; o[1] = e.R; o[2] = e.P; o[3] = e.cap; o[4] = e.shared; o[5] = e.spare_cap;
    o[6] = (D[e.index].g.ntr + e.R - 1) / e.R;
  }
  *wavefronts = gp.nw;
  *lds_bytes = (int64_t)gp.lds;
  return gp.count;
}
