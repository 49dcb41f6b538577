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
// its plan and its dynamic LDS.  A matrix of another width rides along if that LDS serves it too: a narrower one
// with the same plan (its x leaves the products more room), a wider one with two wavefronts per strip and the
// outlier products in the place of x (see the kernel), provided the caller's hint on the longest outlier row says
// that a workgroup's chunks then fit one round.  Bit i of `taken` is set for every matrix launched.
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
  const int n0 = As[0].g.n;
  Geometry all = As[0].g;                    // the plan sees the strips of all matrices of the base width
  all.ntr = 0;
  int longest = 0;                           // the longest outlier row any of them is said to have
  for (int i = 0; i < count; ++i) {
    if (As[i].g.n != n0) continue;
    all.ntr += As[i].g.ntr;
    if (As[i].max_row_nnz > longest) longest = As[i].max_row_nnz;
  }
  LaunchPlan plan = {0, 0, 0, 0, 0};
  if (!plan_launch(all, 1, MAXW, slots, &plan, longest, RowDotsOnMatrixCores<W, TR, TC, AXIS, 1, LV>::value)) return hipErrorInvalidValue;
  const int nw = plan.P * plan.R;
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  if (all.kw != T::KW || all.sd != T::SD || all.layout != LV) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.lds_room > (size_t)MAX_DYNAMIC || plan.lds_room < plan.lds || plan.cap < 64 * nw ||
      nw > MAXW || plan.R * TR > RowsPerGroup<TR, 1>::MAX || plan.P > (all.ntc + 63) / 64 || plan.P < 1 || plan.R < 1 || plan.R > 8)
    return hipErrorInvalidValue;
  FusedArgs F;
  F.g = As[0].g;
  size_t lds = plan.lds;
  int total = 0, k = 0;                      // workgroups, table entries
  // The wider matrices come first in the grid: their wavefronts have the most steps, and the launch ends when its
  // last workgroup does (65B block: 80.5 against 81.5 us with them last).
  for (int pass = 0; pass < 2; ++pass)
  for (int i = 0; i < count; ++i) {
    const Geometry& g = As[i].g;
    if ((g.n > n0) != (pass == 0)) continue;
    const int nsteps = (g.ntc + 63) / 64;
    const size_t xbytes = ((size_t)g.n * 2 + 15) & ~(size_t)15;
    int R = plan.R, P = plan.P, cap = plan.cap, shared = 0;
    size_t need = plan.lds;
    if (g.n < n0) {                          // its x is shorter: the same plan, the products get the difference
      if (P > nsteps) continue;
      cap = (int)((plan.lds - xbytes) / 32);
      if (cap > 8 * 64 * nw) cap = 8 * 64 * nw;
    } else if (g.n > n0) {                   // its x is longer: the products wait and take its place
      if (nw % 2 != 0 || nsteps < 2 || (nw / 2) * TR > RowsPerGroup<TR, 1>::MAX || nw / 2 > 8) continue;
      P = 2; R = nw / 2;
      need = xbytes > plan.lds ? xbytes : plan.lds;
      if (need > plan.lds_room) continue;
      cap = (int)(need / 32);
      if (cap > 8 * 64 * nw) cap = 8 * 64 * nw;
      // A workgroup's R * TR rows: at most that many longest rows, in chunks of 8 entries, plus the two ragged
      // ends.  Where a few rows are long (full rows), the matrix takes one strip per workgroup with all wavefronts
      // on it (half the rows and half the steps per wavefront for the workgroup that owns such a row), and those
      // workgroups go through rounds (see the kernel) -- as long as the average workgroup has room to spare and
      // the launch is long enough for them, the first of the grid, to end before the others do (steps of 64 tiles
      // per wavefront slot of the chip: LLaMA-33B block, rows of up to 17920 outliers, 8.9 steps per slot: 69.0 ->
      // 60.0 us; LLaMA-7B block, 8 full rows of 11008 of which two in one strip, 2.3: 30.0 -> 29.2 us, with the
      // full rows in 8 strips 28.7 -> 23.4 us; gate, up and down of that block alone, 1.3: 24.7 -> 27.2 us).
      if (As[i].max_row_nnz <= 0 && As[i].nnz != 0) continue;   // no hint (a matrix without outliers needs none)
      if ((int64_t)R * TR * As[i].max_row_nnz / 8 + 2 > cap) {
        const int64_t spare = ((int64_t)plan.lds_room - (int64_t)xbytes) / 32;
        if (nsteps >= nw) { P = nw; R = 1; }
        const int64_t typical = (int64_t)((double)As[i].nnz / g.m * R * TR / 8.0 * 1.5) + 2;
        const double steps_per_slot = (double)all.ntr * ((all.ntc + 63) / 64) / ((double)slots * kCUs);
        if (spare < 64 * nw || typical > cap || steps_per_slot < 2.0) continue;
        need = plan.lds_room;                // all the LDS this residency has
        cap = (int)(need / 32);
        if (cap > 8 * 64 * nw) cap = 8 * 64 * nw;
      }
      shared = 1;
    }
    if (cap < 64 * nw || g.kw != T::KW || g.sd != T::SD || g.layout != LV) continue;
    if (need > lds) lds = need;
    F.first[k] = total;
    total += (g.ntr + R - 1) / R;
    F.m[k] = g.m; F.n[k] = g.n;
    F.R[k] = R; F.P[k] = P; F.cap[k] = cap; F.shared_lds[k] = shared; F.spare_cap[k] = 0;
    F.packed[k] = As[i].packed; F.row_ptr[k] = As[i].row_ptr; F.col[k] = As[i].col; F.val[k] = As[i].val;
    F.x[k] = xs[i];
    F.y[k] = ys[i];
    *taken |= 1u << i;
    ++k;
  }
  F.count = k;
  for (int i = 0; i < k; ++i) {              // the LDS behind x, now that the launch's size is known
    const int64_t spare = ((int64_t)lds - (((int64_t)F.n[i] * 2 + 15) & ~(int64_t)15)) / 32;
    if (F.shared_lds[i]) F.spare_cap[i] = spare < 0 ? 0 : (spare > F.cap[i] ? F.cap[i] : (int)spare);
  }
  for (int i = k; i <= SPQR_MAX_FUSED; ++i) F.first[i] = total;
  for (int i = k; i < SPQR_MAX_FUSED; ++i) {
    F.m[i] = 0; F.n[i] = 0; F.R[i] = 1; F.P[i] = 1; F.cap[i] = 0; F.shared_lds[i] = 0; F.spare_cap[i] = 0;
    F.packed[i] = nullptr; F.row_ptr[i] = nullptr; F.col[i] = nullptr; F.val[i] = nullptr; F.x[i] = nullptr; F.y[i] = nullptr;
  }
  if (lds > (size_t)MAX_DYNAMIC || k < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gemv_tile256_fused_kernel<W, TR, TC, AXIS, LV>), dim3(total), dim3(64 * nw), lds, stream, F, y_dtype);
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
