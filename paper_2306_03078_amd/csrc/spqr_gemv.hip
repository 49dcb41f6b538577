// Host side of the fused decode + matvec kernel (spqr_gemv_tile.h): launch plan and the choice of the instance
// (the instances themselves: spqr_gemv_l1/l2/l3.hip); one launch for several matrices of one format.
#include "spqr_gemv_inst.h"

namespace spqr {

// ---------------------------------------------------------------------------
// Launch plan of the fused kernel.
//
// A workgroup owns R consecutive strips and has R * P wavefronts, P per strip (a strip has nsteps steps of 64
// tiles; wavefront `part` of a strip takes the steps part, part + P, ...).
//
// LDS: x (NB vectors), then 32 bytes per outlier chunk and vector of a round.  A round holds at least one chunk
// per thread (the common, single-barrier path) and up to eight.  Static arrays (red, osum, lred, rp) come on
// top; the sum must stay within the CU's 160 KB.
// ---------------------------------------------------------------------------
bool plan_launch(const Geometry& g, int nb, int max_waves, int slots, LaunchPlan* out, int max_row_nnz, bool mf) {
  const int nsteps = (g.ntc + 63) / 64;
  const int xbytes = (nb * g.n * 2 + 15) & ~15;
  const int fixed = static_lds_bytes(g.tile_rows, nb) + 1024;
  const int max_dynamic = 160 * 1024 - fixed;
  const int rmax = nb == 1 ? 64 / g.tile_rows : 1;
  // a plan whose x vectors leave LDS for only a sliver of a workgroup is not worth having
  const int widest = max_waves < nsteps ? max_waves : nsteps;
  if (xbytes + 32 * nb * 64 * ((widest + 1) / 2) > max_dynamic) return false;
  int P = 0, R = 1;
  if (const int pin = option(SPQR_OPT_GEMV_PLAN); pin > 0 && nb == 1) {   // tuning runs: 16 * P + R
    const int pin_p = pin >> 4, pin_r = pin & 15;
    P = pin_p < 1 ? 1 : (pin_p < nsteps ? pin_p : nsteps);
    R = pin_r < 1 ? 1 : (pin_r > rmax ? rmax : pin_r);
    while (R > 1 && R * P > max_waves) --R;
    if (P > max_waves) P = max_waves;
  } else if (nb == 1) {
    // Wavefronts per strip and strips per workgroup, fitted to sweeps of (P, R) over the benchmark layers on
    // MI355X (both tile shapes of either orientation, 3- and 4-bit).  Workgroups of four wavefronts, one step
    // each, win wherever a strip has up to 8 steps: many small workgroups in every phase of their life keep
    // both the memory pipeline and the vector ALUs fed (wider workgroups lose 10-60 % there).  Longer strips
    // (the `down` projections: 11-18 steps): two strips per workgroup with two wavefronts each, so that every
    // wavefront has several steps with the next tile in flight under the current one (-12 % on 8192x22016,
    // -22 % on 6656x17920 against eight one-or-two-step wavefronts), as long as that still leaves more
    // workgroups than compute units; else eight wavefronts on one strip.
    // A launch with far more work than the chip holds at once (a large matrix, or several in one grid: four
    // steps or more per wavefront slot) is bound by vector-ALU issue rather than by how fast it fills and drains
    // the chip: there two wavefronts per strip, two steps each, save the per-wavefront overhead of every second
    // step (-7 % at 4 steps per slot, -13 to -18 % at 6 to 9).
    const double steps_per_slot = (double)g.ntr * nsteps / (16.0 * kCUs);
    // Instances whose row dot products run on the matrix cores (mf) hold three wavefronts per SIMD and are less
    // bound by vector-ALU issue: one wavefront per strip with all of its steps, four strips per workgroup, wins on
    // the large launches (six projections of a 65B block in one grid: 65.4 against 67.3 us with two two-step
    // wavefronts per strip) and on long strips with at least a workgroup per compute unit (8192x22016: 23.0 against
    // 23.6); a single 22016x8192 takes two two-step wavefronts (23.7 against 25.4 with four one-step ones).
    // Strips of 32 rows (beta2 = 32 along the rows: 32 accumulators per lane, two strips per workgroup at most): four
    // wavefronts on one strip whatever its length (22016x8192: 28.1 against 33.2 us for two strips of two wavefronts,
    // 8192x22016: 25.4 against 26.0 for eight wavefronts, six 65B projections in one grid: 81.1 against 82.6-85.8).
    // Tiles of 8 x 64 (a step covers 4096 columns, so strips are short): two strips of two wavefronts (22016x8192: 23.8
    // against 26.0 us for one strip of two, 8192^2: 10.4 against 12.2, 8192x22016: 24.6 against 28.1 for four on one strip).
    if (g.tile_rows == 8 && g.tile_cols == 64 && nsteps >= 2 && max_waves >= 4 && max_row_nnz <= 16000) { P = 2; R = 2; }
    else if (g.tile_rows >= 32 && nsteps >= 4 && max_waves >= 4 && max_row_nnz <= 16000) { P = 4; R = 1; }
    else if (mf && rmax >= 4 && max_waves >= 4 && max_row_nnz <= 16000 &&
        ((nsteps <= 8 && nsteps >= 4 && steps_per_slot >= 3.5) || (nsteps > 8 && g.ntr >= 4 * kCUs))) { P = 1; R = 4; }
    else if (mf && rmax >= 2 && nsteps <= 8 && nsteps >= 4 && steps_per_slot >= 2.0) { P = 2; R = 2; }
    else if (nsteps <= 8 && !(nsteps >= 4 && steps_per_slot >= 3.5 && rmax >= 2)) { P = nsteps < 4 ? nsteps : 4; R = 1; }
    // A row of very many outliers (the caller's hint) makes its strip's workgroup the last to finish: if the row
    // does not fit the one round of 8 chunks per thread that four wavefronts hold in LDS (16384 entries), eight
    // wavefronts take it in one (6656x17920 with Zipf row counts, rows of up to 17920 entries: 21.4 against
    // 26.4 us; rows that fit, e.g. 11008 entries in 4096x11008, are slower with eight: 11.9 against 9.9).
    else if (nsteps > 8 && max_row_nnz > 16000 && rmax >= 2 && max_waves >= 8) { P = 4; R = 2; }
    else if (nsteps <= 8 || (g.ntr >= 400 && rmax >= 2)) { P = 2; R = 2; }
    else { P = max_waves < 8 ? max_waves : 8; R = 1; }
  } else {
    // several activation vectors (one strip per workgroup): four wavefronts per strip, as for one vector -- swept
    // over 1..8 wavefronts on eight benchmark layers at 2 and 4 vectors: four is best or tied on every one (against
    // a rule that maximised the resident wavefronts: 6656x6656 at 2 vectors 16.4 -> 11.5 us, 17920x6656 at 4 vectors
    // 51.5 -> 44.7, 8192x22016 at 2 vectors 44.3 -> 39.3; many small workgroups in every phase of their life again).
    // A very long outlier row (the caller's hint) is summed by all threads of its workgroup: eight wavefronts then
    // (full rows of 11008 entries, 4096x11008 at 2 / 4 vectors: 18.2 / 36.3 against 20.8 / 40.4 us with four; rows
    // of 17920 entries, 6656x17920: 39.8 against 41.9; rows of up to 6656 entries are faster with four: 17.0
    // against 18.0 on 6656x6656, 30.0 against 39.6 on 17920x6656).
    (void)slots;
    const int want = max_row_nnz > 8192 ? 8 : 4;
    P = nsteps < want ? nsteps : want;
    if (P > max_waves) P = max_waves;
  }
  // the widest plan that fits the LDS: x + one chunk per thread
  while (P > 1 && xbytes + 32 * nb * 64 * R * P > max_dynamic) { if (R > 1) --R; else --P; }
  const int w = R * P;
  const int need = xbytes + 32 * nb * 64 * w;
  if (need > max_dynamic) return false;
  int groups = slots / w; if (groups < 1) groups = 1;
  const int by_lds = (160 * 1024) / (need + fixed);
  if (groups > by_lds) groups = by_lds;
  if (groups < 1) groups = 1;
  const int ngroups = (g.ntr + R - 1) / R;
  const int wanted = (ngroups + kCUs - 1) / kCUs;
  const int share = groups < wanted ? groups : wanted;
  // give the outlier products the LDS this occupancy leaves over, up to 8 chunks per thread
  int room = ((160 * 1024) / share - fixed - xbytes) / (32 * nb);
  if (room > (max_dynamic - xbytes) / (32 * nb)) room = (max_dynamic - xbytes) / (32 * nb);
  const int cap = room < 8 * 64 * w ? room : 8 * 64 * w;
  out->P = P; out->R = R; out->cap = cap; out->lds = (size_t)xbytes + (size_t)32 * nb * cap;
  out->lds_room = (size_t)xbytes + (size_t)32 * nb * room;
  return true;
}

// ---------------------------------------------------------------------------
// Plan of one grouped launch (host arithmetic only).  The matrices of the width of As[0] (the caller puts them
// first) size the launch: its plan and its dynamic LDS.  A matrix of another width rides along if that LDS serves it
// too: a narrower one with the same plan (its x leaves the products more room), a wider one with the outlier
// products in the place of x (see the kernel), provided the caller's hint on the longest outlier row says that a
// workgroup's chunks then fit one round -- or, failing that, that only a few workgroups are that heavy and the
// launch is long enough to cover them.  Matrices that do not fit are left out (the caller launches them next).
// ---------------------------------------------------------------------------
bool plan_grouped(const DevMatrix* As, int count, int max_waves, int slots, bool mf, GroupedPlan* out) {
  out->count = 0; out->nw = 0; out->lds = 0;
  if (count < 1 || count > SPQR_MAX_FUSED) return false;
  const Geometry& g0 = As[0].g;
  const int TR = g0.tile_rows, n0 = g0.n;
  const int rows_max = 64;                   // RowsPerGroup<TR, 1>::MAX
  const size_t max_dynamic = 160 * 1024 - static_lds_bytes(TR, 1) - 1024;
  Geometry all = g0;                         // the plan sees the strips of all matrices of the base width
  all.ntr = 0;
  int longest = 0;                           // the longest outlier row any of them is said to have
  for (int i = 0; i < count; ++i) {
    if (As[i].g.n != n0) continue;
    all.ntr += As[i].g.ntr;
    if (As[i].max_row_nnz > longest) longest = As[i].max_row_nnz;
  }
  LaunchPlan plan = {0, 0, 0, 0, 0};
  if (!plan_launch(all, 1, max_waves, slots, &plan, longest, mf)) return false;
  const int nw = plan.P * plan.R;
  if (plan.lds > max_dynamic || plan.lds_room > max_dynamic || plan.lds_room < plan.lds || plan.cap < 64 * nw ||
      nw > max_waves || plan.R * TR > rows_max || plan.P > (all.ntc + 63) / 64 || plan.P < 1 || plan.R < 1 || plan.R > 8)
    return false;
  size_t lds = plan.lds;
  int k = 0;
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
      if (nw % 2 != 0 || nsteps < 2 || (nw / 2) * TR > rows_max || nw / 2 > 8) continue;
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
    if (cap < 64 * nw || g.kw != g0.kw || g.sd != g0.sd || g.layout != g0.layout || g.tile_rows != g0.tile_rows ||
        g.tile_cols != g0.tile_cols)
      continue;
    if (need > lds) lds = need;
    out->e[k] = GroupedEntry{i, R, P, cap, shared, 0};
    ++k;
  }
  if (k < 1 || lds > max_dynamic) return false;
  for (int j = 0; j < k; ++j) {              // the LDS behind x, now that the launch's size is known
    GroupedEntry& en = out->e[j];
    const int64_t spare = ((int64_t)lds - (((int64_t)As[en.index].g.n * 2 + 15) & ~(int64_t)15)) / 32;
    if (en.shared) en.spare_cap = spare < 0 ? 0 : (spare > en.cap ? en.cap : (int)spare);
  }
  out->count = k; out->nw = nw; out->lds = lds;
  return true;
}

// Wavefront slots per CU of a kernel (from its register count), asked once per device; also opts the kernel in
// for more than 64 KB of dynamic LDS.
hipError_t kernel_slots(const void* fn, int max_dynamic, PerDevice* known, int* slots) {
  const int dev = current_device();
  *slots = known->get(dev);
  if (*slots != 0) return hipSuccess;
  hipFuncAttributes fa;
  hipError_t e = hipFuncGetAttributes(&fa, fn);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, max_dynamic);
  if (e != hipSuccess) return e;
  int regs = (fa.numRegs + 7) & ~7; if (regs < 64) regs = 64;
  int per_simd = 512 / regs; if (per_simd > 8) per_simd = 8; if (per_simd < 1) per_simd = 1;
  *slots = 4 * per_simd;
  known->set(dev, *slots);
  return hipSuccess;
}

// Largest number of activation vectors (1, 2 or 4, at most `want`) one launch of
// the tuned kernel can take for this geometry; 0 if there is no tuned kernel.
static bool wide_tile(const Geometry& g) {   // 8 x 64, 3-bit, group_axis 1, bilevel: its own instance, one vector per launch
  return g.tile_rows == 8 && g.tile_cols == 64 && g.axis == 1 && g.w_bits == 3 && g.layout == kBilevel;
}

int tuned_batch_width(const Geometry& g, int want) {
  const bool wide = wide_tile(g);
  if (g.tile_rows * g.tile_cols != 256 && !wide) return 0;
  const bool shape_ok = wide || (g.axis == 1 ? ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 8 && g.tile_cols == 32))
                                             : ((g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 32 && g.tile_cols == 8)));
  if (!shape_ok) return 0;
  if (g.layout != kBilevel || wide) want = 1;  // built for one vector per launch
  for (int nb = want >= 4 ? 4 : (want >= 2 ? 2 : 1); nb >= 1; nb >>= 1) {
    LaunchPlan plan = {0, 0, 0, 0};
    const bool mf = RowDotsOnMatrixCores<3, 8, 32, 1, 1, 1>::value && g.w_bits == 3 && g.tile_rows == 8 &&
                    g.tile_cols == 32 && g.axis == 1 && nb == 1 && g.layout == kBilevel;
    const int maxw = (g.w_bits == 3 && nb == 1 && g.layout != kStats16 && !wide && !mf && g.tile_rows < 32) ? 16 : 8;   // WavesPerGroup
    if (plan_launch(g, nb, maxw, 8, &plan)) return nb;   // 8 slots: the lowest occupancy any instance has
  }
  return 0;
}

bool has_tuned_gemv(const Geometry& g) { return tuned_batch_width(g, 1) == 1; }

hipError_t launch_tuned(const DevMatrix& A, const uint16_t* x, int nb, void* y, int y_dtype, hipStream_t stream) {
  if (wide_tile(A.g)) return launch_tuned_l1w(A, x, nb, y, y_dtype, stream);
  if (A.g.layout == kBilevel) return launch_tuned_l1(A, x, nb, y, y_dtype, stream);
  if (A.g.layout == kRoundZero) return launch_tuned_l2(A, x, nb, y, y_dtype, stream);
  return launch_tuned_l3(A, x, nb, y, y_dtype, stream);
}

// Matrices of one format, each with its own input vector: one launch when a tuned kernel exists and no
// permutation is set, else one launch each.  Input widths may differ: the width with the most strips sizes the
// launch, and the launcher says which of the other matrices it could take along (`taken`); the rest go round again.
hipError_t launch_gemv_grouped(const DevMatrix* As, int count, const uint16_t* const* xs, void* const* ys,
                               int y_dtype, hipStream_t stream) {
  if (count > 1 && count <= SPQR_MAX_FUSED && option(SPQR_OPT_FORCE_GENERIC) == 0) {
    bool perm = false;
    for (int i = 0; i < count; ++i) perm = perm || As[i].perm != nullptr;
    // the base width: most strips; its matrices first
    int base = 0; int64_t best = -1;
    for (int i = 0; i < count; ++i) {
      int64_t strips = 0;
      for (int j = 0; j < count; ++j) if (As[j].g.n == As[i].g.n) strips += As[j].g.ntr;
      if (strips > best) { best = strips; base = i; }
    }
    const Geometry& g = As[base].g;
    if (!perm && tuned_batch_width(g, 1) == 1) {
      DevMatrix G[SPQR_MAX_FUSED]; const uint16_t* gx[SPQR_MAX_FUSED]; void* gy[SPQR_MAX_FUSED];
      int k = 0;
      for (int pass = 0; pass < 2; ++pass)
        for (int i = 0; i < count; ++i)
          if ((As[i].g.n == As[base].g.n) == (pass == 0)) { G[k] = As[i]; gx[k] = xs[i]; gy[k] = ys[i]; ++k; }
      uint32_t taken = 0;
      hipError_t e;
      if (wide_tile(g)) e = launch_fused_l1w(G, count, gx, gy, y_dtype, stream, &taken);
      else if (g.layout == kBilevel) e = launch_fused_l1(G, count, gx, gy, y_dtype, stream, &taken);
      else if (g.layout == kRoundZero) e = launch_fused_l2(G, count, gx, gy, y_dtype, stream, &taken);
      else e = launch_fused_l3(G, count, gx, gy, y_dtype, stream, &taken);
      if (e != hipSuccess) return e;
      k = 0;                                 // what the launch left behind (never a matrix of the base width)
      for (int i = 0; i < count; ++i)
        if (!(taken >> i & 1)) { G[k] = G[i]; gx[k] = gx[i]; gy[k] = gy[i]; ++k; }
      return k > 0 ? launch_gemv_grouped(G, k, gx, gy, y_dtype, stream) : hipSuccess;
    }
  }
  for (int i = 0; i < count; ++i) {
    hipError_t e = launch_gemv(As[i], xs[i], ys[i], y_dtype, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_gemv_fused(const DevMatrix* As, int count, const uint16_t* x, void* const* ys,
                             int y_dtype, hipStream_t stream) {
  const uint16_t* xs[SPQR_MAX_FUSED];
  for (int i = 0; i < count && i < SPQR_MAX_FUSED; ++i) xs[i] = x;
  return launch_gemv_grouped(As, count, xs, ys, y_dtype, stream);
}

}  // namespace spqr
