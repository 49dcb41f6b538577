// Launch templates of the fused decode + matvec kernel and the macro that instantiates them for one statistic
// layout: each layout's instances are a translation unit of their own (spqr_gemv_l1/l2/l3.hip), compiled side by
// side.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_gemv_tile.h"
#include "spqr_kernels.h"

namespace spqr {

// Static LDS of the kernel (red, osum, lred, rp), rounded up; it and the dynamic part must stay within the
// CU's 160 KB.
static constexpr int static_lds_bytes(int tr, int nb) {
  const int rows = nb == 1 ? 64 : tr;        // RowsPerGroup<TR, NB>::MAX
  return ((16 * nb * tr + nb * rows + 32 + nb * rows * 16 + rows + 1) * 4 + 1023) & ~1023;
}
// lds: dynamic LDS of the launch; lds_room: the most it could be without costing a resident workgroup
struct LaunchPlan { int P; int R; int cap; size_t lds; size_t lds_room; };


// spqr_gemv.hip
bool plan_launch(const Geometry& g, int nb, int max_waves, int slots, LaunchPlan* out, int max_row_nnz = 0, bool mf = false);
hipError_t kernel_slots(const void* fn, int max_dynamic, PerDevice* known, int* slots);
// A grouped launch: table entry k is matrix e[k].index with its plan (R strips per workgroup, P wavefronts per strip),
// the chunks of a round of outlier products, whether those take the place of x (`shared`) and, if so, the chunks
// the LDS behind x holds; nw = R * P wavefronts per workgroup, lds = the launch's dynamic LDS.
struct GroupedEntry { int index, R, P, cap, shared, spare_cap; };
struct GroupedPlan { int count; GroupedEntry e[SPQR_MAX_FUSED]; int nw; size_t lds; };
bool plan_grouped(const DevMatrix* As, int count, int max_waves, int slots, bool mf, GroupedPlan* out);
// one pair per statistic layout (spqr_gemv_l1/l2/l3.hip), one for the 8 x 64 tiles of layout 1 (spqr_gemv_l1w.hip)
hipError_t launch_tuned_l1(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_tuned_l2(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_tuned_l3(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_tuned_l1w(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream);
hipError_t launch_fused_l1w(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys, int y_dtype,
                            hipStream_t stream, uint32_t* taken);
hipError_t launch_fused_l1(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys, int y_dtype,
                            hipStream_t stream, uint32_t* taken);
hipError_t launch_fused_l2(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys, int y_dtype,
                            hipStream_t stream, uint32_t* taken);
hipError_t launch_fused_l3(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys, int y_dtype,
                            hipStream_t stream, uint32_t* taken);

template <int W, int TR, int TC, int AXIS, int NB, int LV>
static hipError_t launch_tile256(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                                 hipStream_t stream) {
  constexpr int MAXW = WavesPerGroup<W, NB, LV, TR * TC, LargeRegisterBudget<W, TR, TC, AXIS, NB, LV>::value>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, NB) - 1024;   // static + dynamic <= 160 KB
  static PerDevice known[2];                 // wavefront slots per CU of the instance, 0 = not asked yet
  const void* fn = A.perm ? reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, true, NB, LV>)
                          : reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, false, NB, LV>);
  int slots = 0;
  hipError_t e = kernel_slots(fn, MAX_DYNAMIC, &known[A.perm ? 1 : 0], &slots);
  if (e != hipSuccess) return e;
  LaunchPlan plan = {0, 0, 0, 0, 0};
  if (!plan_launch(A.g, NB, MAXW, slots, &plan, A.max_row_nnz, RowDotsOnMatrixCores<W, TR, TC, AXIS, NB, LV>::value)) return hipErrorInvalidValue;
  const int nw = plan.P * plan.R;
  // what the kernel assumes of its launch and of the tile's size: checked here, on the host
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  if (A.g.kw != T::KW || A.g.sd != T::SD || A.g.layout != LV) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.cap < 64 * nw || nw > MAXW || plan.R * TR > RowsPerGroup<TR, NB>::MAX ||
      plan.P > (A.g.ntc + 63) / 64 || plan.P < 1 || plan.R < 1 || plan.R > 8)
    return hipErrorInvalidValue;
  const dim3 grid((A.g.ntr + plan.R - 1) / plan.R), block(64 * nw);
  if (A.perm)
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, true, NB, LV>), grid, block, plan.lds, stream, A, x, y,
                       y_dtype, plan.cap, plan.R, plan.P);
  else
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, false, NB, LV>), grid, block, plan.lds, stream, A, x, y,
                       y_dtype, plan.cap, plan.R, plan.P);
  return hipGetLastError();
}

// One launch for matrices of one format.  Those of the width of As[0] (the caller puts them first) size the launch:
// its plan and its dynamic LDS.  Which of the others ride along, and how, is plan_grouped()'s decision (spqr_gemv.hip).
// Bit i of `taken` is set for every matrix launched.
template <int W, int TR, int TC, int AXIS, int LV>
static hipError_t launch_fused256(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys,
                                  int y_dtype, hipStream_t stream, uint32_t* taken) {
  constexpr int MAXW = WavesPerGroup<W, 1, LV, TR * TC, LargeRegisterBudget<W, TR, TC, AXIS, 1, LV>::value>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, 1) - 1024;
  static PerDevice known;
  int slots = 0;
  *taken = 0;
  if (count < 1 || count > SPQR_MAX_FUSED) return hipErrorInvalidValue;
  hipError_t e = kernel_slots(reinterpret_cast<const void*>(&gemv_tile256_fused_kernel<W, TR, TC, AXIS, LV>), MAX_DYNAMIC,
                              &known, &slots);
  if (e != hipSuccess) return e;
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  const Geometry& g0 = As[0].g;
  if (g0.kw != T::KW || g0.sd != T::SD || g0.layout != LV || g0.tile_rows != TR || g0.tile_cols != TC) return hipErrorInvalidValue;
  GroupedPlan gp;
  if (!plan_grouped(As, count, MAXW, slots, RowDotsOnMatrixCores<W, TR, TC, AXIS, 1, LV>::value, &gp)) return hipErrorInvalidValue;
  // what the kernel assumes of its launch: checked here, on the host
  const int nw = gp.nw;
  if (gp.count < 1 || gp.count > SPQR_MAX_FUSED || gp.lds > (size_t)MAX_DYNAMIC || nw < 1 || nw > MAXW) return hipErrorInvalidValue;
  FusedArgs F;
  F.g = g0;
  int total = 0;                             // workgroups
  for (int k = 0; k < gp.count; ++k) {
    const GroupedEntry& en = gp.e[k];
    if (en.index < 0 || en.index >= count) return hipErrorInvalidValue;
    const DevMatrix& A = As[en.index];
    const Geometry& g = A.g;
    const size_t xbytes = ((size_t)g.n * 2 + 15) & ~(size_t)15;
    if (en.R < 1 || en.R > 8 || en.P < 1 || en.R * en.P != nw || en.R * TR > RowsPerGroup<TR, 1>::MAX || en.P > (g.ntc + 63) / 64 ||
        en.cap < 64 * nw || en.cap > 8 * 64 * nw || g.kw != T::KW || g.sd != T::SD || g.layout != LV || xbytes > gp.lds ||
        (size_t)32 * en.cap + (en.shared ? 0 : xbytes) > gp.lds || (en.shared && xbytes + (size_t)32 * en.spare_cap > gp.lds))
      return hipErrorInvalidValue;
    F.first[k] = total;
    total += (g.ntr + en.R - 1) / en.R;
    F.m[k] = g.m; F.n[k] = g.n;
    F.R[k] = en.R; F.P[k] = en.P; F.cap[k] = en.cap; F.shared_lds[k] = en.shared; F.spare_cap[k] = en.spare_cap;
    F.packed[k] = A.packed; F.row_ptr[k] = A.row_ptr; F.col[k] = A.col; F.val[k] = A.val;
    F.x[k] = xs[en.index];
    F.y[k] = ys[en.index];
    *taken |= 1u << en.index;
  }
  F.count = gp.count;
  for (int i = gp.count; i <= SPQR_MAX_FUSED; ++i) F.first[i] = total;
  for (int i = gp.count; i < SPQR_MAX_FUSED; ++i) {
    F.m[i] = 0; F.n[i] = 0; F.R[i] = 1; F.P[i] = 1; F.cap[i] = 0; F.shared_lds[i] = 0; F.spare_cap[i] = 0;
    F.packed[i] = nullptr; F.row_ptr[i] = nullptr; F.col[i] = nullptr; F.val[i] = nullptr; F.x[i] = nullptr; F.y[i] = nullptr;
  }
  hipLaunchKernelGGL((gemv_tile256_fused_kernel<W, TR, TC, AXIS, LV>), dim3(total), dim3(64 * nw), gp.lds, stream, F, y_dtype);
  return hipGetLastError();
}

// Defines launch_tuned_<NAME> and launch_fused_<NAME> for the tile shapes in CASES (a list of
// CASE(w_bits, tile_rows, tile_cols, group_axis, layout)) and the vector counts NBS (SPQR_NB_124 or SPQR_NB_1).
#define SPQR_NB_124(NBCASE) NBCASE(1) NBCASE(2) NBCASE(4)
#define SPQR_NB_1(NBCASE) NBCASE(1)
#define SPQR_DEFINE_GEMV_UNIT(NAME, LV, CASES, NBS)                                                                  \
  template <int NB>                                                                                                \
  static hipError_t launch_tuned_nb_(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,                  \
                                     hipStream_t stream) {                                                         \
    const Geometry& g = A.g;                                                                                       \
    CASES(SPQR_TUNED_CASE_, LV)                                                                                    \
    return hipErrorInvalidValue;                                                                                   \
  }                                                                                                                \
  hipError_t launch_tuned_##NAME(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype,               \
                                hipStream_t stream) {                                                              \
    NBS(SPQR_NB_CASE_)                                                                                             \
    return hipErrorInvalidValue;                                                                                   \
  }                                                                                                                \
  hipError_t launch_fused_##NAME(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys,        \
                                int y_dtype, hipStream_t stream, uint32_t* taken) {                                \
    const Geometry& g = As[0].g;                                                                                   \
    CASES(SPQR_FUSED_CASE_, LV)                                                                                    \
    return hipErrorInvalidValue;                                                                                   \
  }
#define SPQR_TUNED_CASE_(W_, TR_, TC_, AX_, LV_)                                              \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_)            \
    return launch_tile256<W_, TR_, TC_, AX_, NB, LV_>(A, x, y, y_dtype, stream);
#define SPQR_FUSED_CASE_(W_, TR_, TC_, AX_, LV_)                                              \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_)            \
    return launch_fused256<W_, TR_, TC_, AX_, LV_>(As, count, xs, ys, y_dtype, stream, taken);
#define SPQR_NB_CASE_(NB_) if (nb == NB_) return launch_tuned_nb_<NB_>(A, x, y, y_dtype, stream);

// The tile shapes with a tuned kernel (tuned_batch_width() in spqr_gemv.hip lists the same).
#define SPQR_GEMV_SHAPES(CASE, LV)                                                          \
  CASE(3, 16, 16, 1, LV) CASE(4, 16, 16, 1, LV) CASE(3, 8, 32, 1, LV) CASE(4, 8, 32, 1, LV) \
  CASE(3, 16, 16, 0, LV) CASE(4, 16, 16, 0, LV) CASE(3, 32, 8, 0, LV) CASE(4, 32, 8, 0, LV)
// beta1 = 8, beta2 = 64 (the size-matched setting of Sec. 5), 3-bit, group_axis 1
#define SPQR_GEMV_WIDE_SHAPES(CASE, LV) CASE(3, 8, 64, 1, LV)

}  // namespace spqr
