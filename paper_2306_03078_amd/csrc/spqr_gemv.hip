// Launchers of the fused decode + matvec kernel (spqr_gemv_tile.h): launch plan, instances, one launch
// for several matrices that share the input vector.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_gemv_tile.h"
#include "spqr_kernels.h"

namespace spqr {

// ---------------------------------------------------------------------------
// Launch plan of the fused kernel.
//
// LDS: x (NB vectors), then 32 bytes per outlier chunk and vector of a round.  A
// round holds at least one chunk per thread (the common, single-barrier path)
// and up to eight.  Static arrays (red, osum, lred, rp) come on top; the
// sum must stay within the CU's 160 KB.
//
// Wavefronts per workgroup: a strip has nsteps steps of 64 tiles.  With w
// wavefronts a CU holds floor(slots / w) workgroups (slots = wavefront slots at
// the kernel's register count, LDS permitting) and the steps split evenly only
// if w divides them; the plan maximises the wavefronts resident on a CU.
// ---------------------------------------------------------------------------
static constexpr int static_lds_bytes(int tr, int nb) {
  return ((16 * nb * tr + nb * tr + 32 + nb * tr * 16 + tr + 1) * 4 + 1023) & ~1023;
}
struct LaunchPlan { int nw; int cap; size_t lds; };

static bool plan_launch(const Geometry& g, int nb, int max_waves, int slots, LaunchPlan* out) {
  const int nsteps = (g.ntc + 63) / 64;
  const int xbytes = (nb * g.n * 2 + 15) & ~15;
  const int max_dynamic = 160 * 1024 - static_lds_bytes(g.tile_rows, nb) - 1024;
  double best = -1.0;
  // a plan whose x vectors leave LDS for only a sliver of a workgroup is not worth having
  const int widest = max_waves < nsteps ? max_waves : nsteps;
  if (xbytes + 32 * nb * 64 * ((widest + 1) / 2) > max_dynamic) return false;
  // SPQR_PLAN_WAVES=k in the environment pins the wavefronts per workgroup (tuning runs)
  int pinned = 0;
  if (const char* e = std::getenv("SPQR_PLAN_WAVES")) pinned = std::atoi(e);
  for (int w = 1; w <= max_waves && w <= nsteps; ++w) {
    if (pinned > 0 && w != pinned && pinned <= max_waves && pinned <= nsteps) continue;
    int groups = slots / w; if (groups < 1) groups = 1;
    // LDS one workgroup needs at least: x + one chunk per thread
    const int need = xbytes + 32 * nb * 64 * w;
    if (need > max_dynamic) continue;
    const int by_lds = (160 * 1024) / (need + static_lds_bytes(g.tile_rows, nb) + 1024);
    if (groups > by_lds) groups = by_lds;
    if (groups < 1) continue;
    const int wanted = (g.ntr + kCUs - 1) / kCUs;      // a small grid never puts more workgroups on a CU
    const int share = groups < wanted ? groups : wanted;
    // Score: closeness to the preferred workgroup width.  A wavefront pipelines its
    // steps (the next tile's loads fly under the current tile's arithmetic), so few
    // wide-enough workgroups beat many one-step wavefronts: 8 wavefronts when the
    // strip has 8 steps or more, else 4 (both spread evenly over the four SIMDs and
    // leave room for a second workgroup on the CU), else one per step.  Fitted to
    // timings of the benchmark layers on MI355X.
    const int cap8 = max_waves < 8 ? max_waves : 8;
    const int target = nsteps < 4 ? nsteps : ((nsteps < cap8 ? nsteps : cap8) / 4) * 4;
    int resident = w * share; if (resident > slots) resident = slots;
    double score = 100.0 - (w > target ? 1.5 * (w - target) : (target - w)) + 1e-3 * resident;
    if (nb > 1) {
      // several activation vectors: arithmetic dominates, so what counts is wavefronts
      // resident on the CU and an even split of the steps among them
      const int per_wave = (nsteps + w - 1) / w;
      const double even = (double)nsteps / ((double)w * per_wave);
      score = (double)resident * (0.75 + 0.25 * even) * (w % 4 == 0 ? 1.05 : 1.0) * (share >= 2 ? 1.03 : 1.0) + 1e-3 * w;
    }
    if (score > best) {
      best = score;
      // give the outlier products the LDS this occupancy leaves over, up to 4 chunks per thread
      int room = ((160 * 1024) / share - static_lds_bytes(g.tile_rows, nb) - 1024 - xbytes) / (32 * nb);
      if (room > (max_dynamic - xbytes) / (32 * nb)) room = (max_dynamic - xbytes) / (32 * nb);
      int cap = room < 8 * 64 * w ? room : 8 * 64 * w;
      out->nw = w; out->cap = cap; out->lds = (size_t)xbytes + (size_t)32 * nb * cap;
    }
  }
  return best > 0.0;
}

template <int W, int TR, int TC, int AXIS, int NB>
static hipError_t launch_tile256(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                                 hipStream_t stream) {
  constexpr int MAXW = WavesPerGroup<W, NB>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, NB) - 1024;   // static + dynamic <= 160 KB
  // once per kernel: register count (-> wavefront slots per CU) and the opt-in for > 64 KB of dynamic LDS
  static PerDevice known[2];                 // wavefront slots per CU of the instance, 0 = not asked yet
  const int pi = A.perm ? 1 : 0, dev = current_device();
  int slots = known[pi].get(dev);
  if (slots == 0) {
    const void* fn = A.perm ? reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, true, NB>)
                            : reinterpret_cast<const void*>(&gemv_tile256_kernel<W, TR, TC, AXIS, false, NB>);
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, fn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_DYNAMIC);
    if (e != hipSuccess) return e;
    int regs = (fa.numRegs + 7) & ~7; if (regs < 64) regs = 64;
    int per_simd = 512 / regs; if (per_simd > 8) per_simd = 8; if (per_simd < 1) per_simd = 1;
    slots = 4 * per_simd;
    known[pi].set(dev, slots);
  }
  LaunchPlan plan = {0, 0, 0};
  if (!plan_launch(A.g, NB, MAXW, slots, &plan)) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.cap < 64 * plan.nw) return hipErrorInvalidValue;
  if (A.perm)
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, true, NB>), dim3(A.g.ntr), dim3(64 * plan.nw),
                       plan.lds, stream, A, x, y, y_dtype, plan.cap);
  else
    hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS, false, NB>), dim3(A.g.ntr), dim3(64 * plan.nw),
                       plan.lds, stream, A, x, y, y_dtype, plan.cap);
  return hipGetLastError();
}

// Largest number of activation vectors (1, 2 or 4, at most `want`) one launch of
// the tuned kernel can take for this geometry; 0 if there is no tuned kernel.
int tuned_batch_width(const Geometry& g, int want) {
  if (g.tile_rows * g.tile_cols != 256) return 0;
  const bool shape_ok = g.axis == 1 ? ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 8 && g.tile_cols == 32))
                                    : ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 32 && g.tile_cols == 8));
  if (!shape_ok) return 0;
  for (int nb = want >= 4 ? 4 : (want >= 2 ? 2 : 1); nb >= 1; nb >>= 1) {
    LaunchPlan plan = {0, 0, 0};
    const int maxw = (g.w_bits == 3 && nb == 1) ? 16 : 8;
    if (plan_launch(g, nb, maxw, 8, &plan)) return nb;   // 8 slots: the lowest occupancy any instance has
  }
  return 0;
}

bool has_tuned_gemv(const Geometry& g) { return tuned_batch_width(g, 1) == 1; }

template <int NB>
static hipError_t launch_tuned_nb(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype, hipStream_t stream) {
  const Geometry& g = A.g;
#define SPQR_CASE(W_, TR_, TC_, AX_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
    return launch_tile256<W_, TR_, TC_, AX_, NB>(A, x, y, y_dtype, stream);
  SPQR_CASE(3, 16, 16, 1) SPQR_CASE(4, 16, 16, 1) SPQR_CASE(3, 8, 32, 1) SPQR_CASE(4, 8, 32, 1)
  SPQR_CASE(3, 16, 16, 0) SPQR_CASE(4, 16, 16, 0) SPQR_CASE(3, 32, 8, 0) SPQR_CASE(4, 32, 8, 0)
#undef SPQR_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_tuned(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream) {
  if (nb == 4) return launch_tuned_nb<4>(A, x, y, y_dtype, stream);
  if (nb == 2) return launch_tuned_nb<2>(A, x, y, y_dtype, stream);
  if (nb == 1) return launch_tuned_nb<1>(A, x, y, y_dtype, stream);
  return hipErrorInvalidValue;
}

template <int W, int TR, int TC, int AXIS>
static hipError_t launch_fused256(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                                  int y_dtype, hipStream_t stream) {
  constexpr int MAXW = WavesPerGroup<W, 1>::MAX;
  constexpr int MAX_DYNAMIC = 160 * 1024 - static_lds_bytes(TR, 1) - 1024;
  static PerDevice known;
  const int dev = current_device();
  int slots = known.get(dev);
  const void* fn = reinterpret_cast<const void*>(&gemv_tile256_fused_kernel<W, TR, TC, AXIS>);
  if (slots == 0) {
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, fn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_DYNAMIC);
    if (e != hipSuccess) return e;
    int regs = (fa.numRegs + 7) & ~7; if (regs < 64) regs = 64;
    int per_simd = 512 / regs; if (per_simd > 8) per_simd = 8; if (per_simd < 1) per_simd = 1;
    slots = 4 * per_simd;
    known.set(dev, slots);
  }
  FusedArgs F;
  F.count = count;
  F.g = As[0].g;
  int total = 0;
  for (int i = 0; i < count; ++i) {
    F.first[i] = total;
    total += As[i].g.ntr;
    F.packed[i] = As[i].packed; F.row_ptr[i] = As[i].row_ptr; F.col[i] = As[i].col; F.val[i] = As[i].val;
    F.y[i] = ys[i];
  }
  for (int i = count; i <= SPQR_MAX_FUSED; ++i) F.first[i] = total;
  for (int i = count; i < SPQR_MAX_FUSED; ++i) {
    F.packed[i] = nullptr; F.row_ptr[i] = nullptr; F.col[i] = nullptr; F.val[i] = nullptr; F.y[i] = nullptr;
  }
  Geometry all = As[0].g;                    // the plan sees the whole grid
  all.ntr = total;
  LaunchPlan plan = {0, 0, 0};
  if (!plan_launch(all, 1, MAXW, slots, &plan)) return hipErrorInvalidValue;
  if (plan.lds > (size_t)MAX_DYNAMIC || plan.cap < 64 * plan.nw) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gemv_tile256_fused_kernel<W, TR, TC, AXIS>), dim3(total), dim3(64 * plan.nw), plan.lds, stream,
                     F, x, y_dtype, plan.cap);
  return hipGetLastError();
}

hipError_t launch_gemv_fused(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                             int y_dtype, hipStream_t stream, bool force_generic) {
  const Geometry& g = As[0].g;
  if (count > 1 && !force_generic && As[0].perm == nullptr && tuned_batch_width(g, 1) == 1) {
#define SPQR_CASE(W_, TR_, TC_, AX_) \
    if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
      return launch_fused256<W_, TR_, TC_, AX_>(As, count, x, ys, y_dtype, stream);
    SPQR_CASE(3, 16, 16, 1) SPQR_CASE(4, 16, 16, 1) SPQR_CASE(3, 8, 32, 1) SPQR_CASE(4, 8, 32, 1)
    SPQR_CASE(3, 16, 16, 0) SPQR_CASE(4, 16, 16, 0) SPQR_CASE(3, 32, 8, 0) SPQR_CASE(4, 32, 8, 0)
#undef SPQR_CASE
  }
  for (int i = 0; i < count; ++i) {
    hipError_t e = launch_gemv(As[i], x, ys[i], y_dtype, stream, force_generic);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace spqr
