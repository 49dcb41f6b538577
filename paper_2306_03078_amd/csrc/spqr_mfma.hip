// Batches above 4 vectors: dense part on the matrix cores, outliers in a finishing kernel; launchers,
// launch plan and scratch of that path.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <queue>
#include <vector>

#include "../../include/spqr.h"
#include "spqr_tile.h"
#include "spqr_kernels.h"

namespace spqr {

// ---------------------------------------------------------------------------
// Batches above 4 on 16x16 tiles: the dense part on the matrix cores (weights
// stream once for the whole batch), then a finishing kernel that adds the outliers.
//
// Dense part: P[split][b][rows] = X[b][cols of the split] . dequant(strip)^T in
// binary32, no outliers.  A workgroup is 4 wavefronts = 4 consecutive strips that
// walk the same steps of 64 tiles in lock-step, because they share the 16 x 1024
// piece of X that belongs to the step: it is staged in LDS once per workgroup
// (prefetched into registers one step ahead).  A lane still fetches one whole
// tile (same loads, same layout as the GEMV).  An MFMA operand, though, wants
// 16 rows x 4 columns across the 64 lanes, while here the lanes hold 64 different
// tiles: so every lane dequantises its tile to binary16 (s_hat*(q - z_hat) evaluated
// in binary32, one rounding -- the kernel of Sec. 4.2 multiplies 16-bit weights
// as well) into its wavefront's LDS buffer, a quarter (4 columns) at a time to
// keep the buffer small enough for two workgroups per CU.  One
// v_mfma_f32_16x16x32_f16 then sums 8 tiles at once: its K index is (tile, column),
// A: lane l = row l%16 of tiles 8j + 2(l/16) and the next, B: lane l = batch l%16, the
// same two tiles' 4 columns of X; D[row][batch] accumulates over the whole column
// range in 8 registers.
// Batch rows beyond `batch` repeat the last one and are dropped at the end.
// The steps of a matrix can be split over gridDim.y workgroups (few strips, many
// columns); every split writes its own partial result.  Workgroups behind the
// dense ones (blockIdx.x >= groups) take the long outlier rows, see long_rows_block.
// ---------------------------------------------------------------------------
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
constexpr int kMfmaTileStride = 36;          // dwords per tile quarter (16 rows x 8 bytes + 16: spreads the banks)

// Outlier rows longer than `long_row` entries (far longer than the average row), for the batch path.  Such a row
// would keep the one CU that owns its strip busy long after the others are done (every outlier is an L1 line
// look-up), so these rows are taken out of the finishing kernel: extra workgroups of the dense kernel's grid (they
// run beside the dense workgroups and need nothing from them) compute, slice by slice of kLongSlice entries,
// sum_k val_k * XT[col_k][b] for the 16 vectors
// into slots[lo / kSlotGrain + k][16] for slice k of the row that starts at entry lo -- a long row has no more
// slices than multiples of kSlotGrain among its entry indices (ceil(len/512) <= floor(len/256) from len = 256 on),
// so the slots of different rows never meet and the finishing kernel finds them without a search.
// Work is shared out by entries, not by rows: workgroup wg of nwg owns the slices that start in its equal share
// [a, z) of the entry indices, so heavy rows next to each other (or one row of many slices) spread over as many
// workgroups as their entries fill.  It narrows the rows down to NT around the one that holds entry a by a search
// all threads take part in (NT probes of the row pointers per round; none for up to NT rows, one for up to NT*NT),
// then walks the rows from there, NT - 1 at a time, up to the first that starts at or behind z.  A slice is one wavefront's: a lane takes every 64th entry (consecutive lanes read
// consecutive entries) with its whole 32-byte line of XT, all loads in flight at once; the 16 sums are reduced over
// the lanes in a fixed order and written by the wavefront itself.  The wavefronts of a workgroup take its slices
// in turn and meet only where the next rows are fetched.
constexpr int kLongRowMin = 256, kLongSlice = 512, kSlotGrain = 256;

template <int NT>
__device__ __forceinline__ void long_rows_block(const DevMatrix& A, const uint16_t* __restrict__ XT,
                                                float* __restrict__ slots, int long_row, int wg, int nwg, uint8_t* smem) {
  constexpr int EPT = kLongSlice / 64, NW = NT / 64;
  int* rpl = reinterpret_cast<int*>(smem);                                   // NT row pointers
  uint32_t* masks = reinterpret_cast<uint32_t*>(smem + 4 * NT);              // 2 per wavefront
  int* below = reinterpret_cast<int*>(smem + 4 * NT + 8 * NW);               // 1 per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = A.g.m;
  const int64_t nnz = A.nnz;
  const uint32_t zoff = (uint32_t)A.g.n * 32u;                               // the zero line of XT
  int64_t per = (nnz + nwg - 1) / nwg;
  if (per < kLongSlice) per = kLongSlice;
  const int64_t a64 = (int64_t)wg * per;
  if (a64 >= nnz) return;                                                    // workgroup-uniform
  const int a = (int)a64, z = (int)(a64 + per < nnz ? a64 + per : nnz);
  // the last row r with row_ptr[r] <= a lies in [L, H): row_ptr[L] <= a < row_ptr[H] throughout
  int L = 0, H = m;
  while (H - L > NT) {                                                       // workgroup-uniform
    // probe t looks at the end of the t-th of NT parts of the bracket: distinct rows in (L, H], the last is H
    const int span = H - L;
    const bool is_below = A.row_ptr[L + (int)(((int64_t)(tid + 1) * span) / NT)] <= a;
    const uint64_t bal = __builtin_amdgcn_ballot_w64(is_below);
    if (lane == 0) below[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int c = 0;                                                               // probes at or below a: a prefix of them,
#pragma unroll
    for (int k = 0; k < NW; ++k) c += below[k];                              // never all (row H is above a)
    __syncthreads();
    c = min(c, NT - 1);                      // (all only if row_ptr[m] < nnz, a broken descriptor: stay inside the bracket)
    const int newL = c == 0 ? L : L + (int)(((int64_t)c * span) / NT);
    H = L + (int)(((int64_t)(c + 1) * span) / NT);
    L = newL;
  }
  // The rows from L on, NT - 1 at a time.  The row that holds entry a is among the first H - L <= NT of them; the
  // rows before it end at or before a and own nothing here.
  int taken = 0;                                                             // slices of this workgroup so far
  for (int r0 = L; r0 < m;) {                                                // workgroup-uniform
    const int nrows = min(NT - 1, m - r0);
    if (tid <= nrows) rpl[tid] = A.row_ptr[r0 + tid];
    __syncthreads();
    const int t1 = min(tid, NT - 2);
    const bool is_long = tid < nrows && rpl[t1 + 1] - rpl[t1] > long_row && rpl[t1] < z && rpl[t1 + 1] > a;
    const uint64_t bal = __builtin_amdgcn_ballot_w64(is_long);
    if (lane == 0) { masks[2 * wave] = (uint32_t)bal; masks[2 * wave + 1] = (uint32_t)(bal >> 32); }
    __syncthreads();
    for (int w = 0; w < NW; ++w) {
      uint64_t mask = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)masks[2 * w]) |      // no sign extension
                      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)masks[2 * w + 1]) << 32);
      while (mask) {                                                         // workgroup-uniform
        const int r = 64 * w + __builtin_ctzll(mask);
        mask &= mask - 1;
        const int lo = rpl[r], hi = rpl[r + 1];
        // the row's slices that start in [a, z)
        const int k0 = lo >= a ? 0 : (a - lo + kLongSlice - 1) / kLongSlice;
        for (int k = k0; lo + k * kLongSlice < min(hi, z); ++k) {
          if (taken++ % NW != wave) continue;                                // wavefront-uniform
          const int e0 = lo + k * kLongSlice;
          // all of the lane's entries first, then their lines of XT, then the arithmetic: one round trip each
          uint32_t off[EPT];
          float val[EPT];
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const int e = e0 + lane + 64 * i;
            const bool ok = e < hi;
            off[i] = ok ? (uint32_t)A.col[e] * 32u : zoff;
            val[i] = ok ? h2f(A.val[e]) : 0.f;
          }
          u32x4 x0[EPT], x1[EPT];
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const u32x4* line = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(XT) + off[i]);
            x0[i] = line[0];
            x1[i] = line[1];
          }
          float acc[16];
#pragma unroll
          for (int b = 0; b < 16; ++b) acc[b] = 0.f;
#pragma unroll
          for (int i = 0; i < EPT; ++i) {
            const uint32_t xw[8] = {x0[i].x, x0[i].y, x0[i].z, x0[i].w, x1[i].x, x1[i].y, x1[i].z, x1[i].w};
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              acc[2 * q] = fmaf(val[i], h2f((uint16_t)(xw[q] & 0xFFFFu)), acc[2 * q]);
              acc[2 * q + 1] = fmaf(val[i], h2f((uint16_t)(xw[q] >> 16)), acc[2 * q + 1]);
            }
          }
          int row;
          const float red = wave_reduce_rows<16>(acc, lane, &row);           // every lane: the sum of vector `row`
          if ((lane & 3) == 0) slots[(int64_t)(lo / kSlotGrain + k) * 16 + row] = red;   // 4 lanes hold each sum
        }
      }
    }
    if (rpl[nrows] >= z) break;                                              // the next row starts behind the share
    r0 += nrows;
    __syncthreads();                                                         // everyone is done with these row pointers
  }
}

// Shape of the dense kernel for a tile of TR x TC = 256 codes.  A phase covers PC = 64/TR columns of every tile
// (a lane always writes 64 binary16 values = 128 bytes per phase: rows x PC columns), four phases per step.
// The 8 K-values a lane supplies to one MFMA are PC columns of 8/PC tiles.  Strips per workgroup: what the LDS
// allows next to the piece of X (16 batch rows x 64*TC columns): 8 x 32 tiles share a 64 KB piece among 8 strips.
template <int TR, int TC> struct MfmaShape {
  static constexpr int PC = 64 / TR;                       // columns per phase: 8, 4, 2
  static constexpr int TPK = 8 / PC;                       // tiles per K-group of a lane: 1, 2, 4
  static constexpr int MB = TR >= 16 ? TR / 16 : 1;        // blocks of 16 rows (an 8-row tile fills half a block)
  static constexpr int NS = TC == 32 ? 8 : 4;              // strips = wavefronts per workgroup
  static constexpr int WGS = TC == 32 ? 1 : 2;             // workgroups per CU
  static constexpr int XROW = 128 * TC + 8;                // bytes per batch row of the staged piece of X
  static constexpr size_t LDS = (size_t)NS * 64 * kMfmaTileStride * 4 + 16 * (size_t)XROW;
  static_assert(WGS * (LDS + 1024) <= 160 * 1024, "the workgroups of a CU must fit its LDS");
};

// `group` is the group of NS strips this workgroup multiplies, or negative for a workgroup that takes long outlier
// rows instead: then it is number `extra` of `nextra` such workgroups of its matrix.  `split` of the splits of the
// steps, `smem` the workgroup's dynamic LDS.
template <int W, int TR, int TC, int AXIS, bool ONE>
__device__ __forceinline__ void gemm_mfma_body(const DevMatrix& A, const uint16_t* __restrict__ X, float* __restrict__ P,
                                               int64_t split_stride, int steps_per_split, int batch,
                                               const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row,
                                               int group, int split, int extra, int nextra, uint8_t* smem) {
  using SH = MfmaShape<TR, TC>;
  constexpr int PPR = TC / 2, S = kMfmaTileStride, NS = SH::NS, NT = 64 * NS, PC = SH::PC, TPK = SH::TPK, MB = SH::MB;
  constexpr int UROW = 8 * TC;               // 16-byte units of the X piece per batch row
  constexpr int UPT = 16 * UROW / NT;        // ... per thread
  constexpr int B2 = AXIS == 1 ? TC : TR;    // first-level groups per tile
  constexpr int NM = 2 * PC;                 // MFMAs per phase and block of rows
  static_assert(NT % UROW == 0 && TR * TC == 256, "shape");
  using T = TileRegs<W, TR, TC, AXIS>;
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr float SCALE = (float)(1 << W);
  uint8_t* xbuf = smem + NS * 64 * S * 4;
  if (group < 0) {                           // long outlier rows
    if (split == 0)
      long_rows_block<NT>(A, XT, slots, long_row, extra, nextra, smem);
    return;
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = A.g.n, ntc = A.g.ntc, m = A.g.m, ntr = A.g.ntr;
  const int nsteps = (ntc + 63) >> 6;
  const int s_lo = split * steps_per_split, s_hi = min(nsteps, s_lo + steps_per_split);   // never empty (host)
  const int strip = group * NS + wave;
  const bool active = strip < ntr;           // wave-uniform; an idle wavefront still stages X and meets the barriers
  const uint8_t* strip_base = A.packed + (int64_t)min(strip, ntr - 1) * ntc * TILE_BYTES;
  uint32_t* buf = reinterpret_cast<uint32_t*>(smem) + wave * 64 * S;
  const int i16 = lane & 15, g4 = lane >> 4;
  const PairConsts kc = make_pair_consts<W>();
  const PairConsts k3 = make_pair_consts<3>();
  // Groups along the tile's columns, and the class of a code pair (the offset K its in-place extraction leaves,
  // see CodeClass) a function of its column alone: then K folds into the column's additive constant and most
  // shifts of the extraction go away.  True for 4-bit codes and for 3-bit codes in rows of 16 pairs.
  constexpr bool FOLD = AXIS == 1 && (W == 4 || PPR == 16);
  const ClassConsts kk = make_class_consts<W>();
  float4_t D[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) { D[mb][0] = float4_t{0.f, 0.f, 0.f, 0.f}; D[mb][1] = float4_t{0.f, 0.f, 0.f, 0.f}; }

  // the piece of X of step st: unit u = 16 bytes = 8 columns of batch row u/UROW; loads unconditional (clamped)
  u32x4 xr[UPT];
  uint32_t xrow[UPT];                        // byte offset of the unit's (clamped) batch row in X
#pragma unroll
  for (int k = 0; k < UPT; ++k) xrow[k] = (uint32_t)min((tid + k * NT) / UROW, batch - 1) * (uint32_t)n * 2u;
  const int xj = tid % UROW;                 // NT is a multiple of UROW: the unit's place in its row is the same for all k
  auto fetch_x = [&](int st) {
    const int sc = min(st, s_hi - 1);
    const int L = min(64, ntc - 64 * sc);
    const uint8_t* xs = reinterpret_cast<const uint8_t*>(X + (int64_t)(64 * TC) * sc);
    const uint32_t jb = 16u * (uint32_t)min(xj, L * (TC / 8) - 1);
#pragma unroll
    for (int k = 0; k < UPT; ++k) xr[k] = *reinterpret_cast<const u32x4*>(xs + (xrow[k] + jb));
    asm volatile("" ::: "memory");
  };
  auto store_x = [&](int st) {
    const int L = min(64, ntc - 64 * st);
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    // columns behind the last tile: zeros (finite), they meet zero weights
    const bool keep = xj < L * (TC / 8);
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const int b = (tid + k * NT) / UROW;
      const u32x2 lo = {keep ? xr[k].x : 0u, keep ? xr[k].y : 0u}, hi = {keep ? xr[k].z : 0u, keep ? xr[k].w : 0u};
      if (b < batch) {
        u32x2* d = reinterpret_cast<u32x2*>(xbuf + b * SH::XROW + xj * 16);
        d[0] = lo;
        d[1] = hi;
      }
    }
  };
  auto issue = [&](T& t, int st) {
    const bool real = st < s_hi;
    const int L = real ? min(64, ntc - 64 * st) : 1;
    load_tile<false>(t, strip_base + (int64_t)64 * (real ? st : s_lo) * TILE_BYTES, L, min(lane, L - 1));
    asm volatile("" ::: "memory");
  };
  // operand fragments of MFMA j of a phase: tiles (4j + g4)*TPK .. +TPK-1, PC columns each.
  // A: row i16 (+16 per block of rows; an 8-row tile repeats its rows, the copies are dropped at the end)
  const uint32_t* afrag = buf + g4 * TPK * S + ((TR >= 16 ? i16 : (i16 & 7)) * PC) / 2;
  const uint32_t* xfrag = reinterpret_cast<const uint32_t*>(xbuf + min(i16, batch - 1) * SH::XROW) + g4 * TPK * (TC / 2);
  // one step: publish its piece of X, then per phase: dequantise PC columns of this lane's tile, multiply
  auto run_step = [&](const T& t, int st) {
    const int L = min(64, ntc - 64 * st);
    __syncthreads();                         // every wavefront is done with the previous piece of X
    store_x(st);
    if constexpr (!ONE) fetch_x(st + 1);
    __syncthreads();
    const uint32_t a2 = t.s[T::SD - 2], b2 = t.s[T::SD - 1];
    const float s_s = h2f((uint16_t)(a2 & 0xFFFF)), z_s = h2f((uint16_t)(a2 >> 16));
    const float s_z = h2f((uint16_t)(b2 & 0xFFFF)), z_z = h2f((uint16_t)(b2 >> 16));
    // w = s_hat*(q - z_hat) = fa*(1 + q/2^W) + fb with fa = 2^W*s_hat, fb = -s_hat*(2^W + z_hat), per group,
    // where s_hat = s_s*(s_q - z_s) and z_hat = s_z*(z_q - z_z) and the extracted codes are 1 + code/8:
    //   fa = c1*(1 + s_q/8) + c2,   -(2^W + z_hat)/2^W = e1*(1 + z_q/8) + e2,   fb = fa * that.
    // A lane behind the step's last tile (its loads were clamped) writes a tile of zeros.
    const bool live = lane < L;
    const float c1 = live ? SCALE * 8.f * s_s : 0.f, c2 = live ? SCALE * (-s_s * z_s - 8.f * s_s) : 0.f;
    const float e1 = -8.f * s_z / SCALE, e2 = -(SCALE - s_z * z_z - 8.f * s_z) / SCALE;
    float fa[B2], fb[B2];
#pragma unroll
    for (int p = 0; p < B2 / 2; ++p) {
      const half2_t sq = as_half2(pair_f16<3>(t.s, p, k3));
      const half2_t zq = as_half2(pair_f16<3>(t.s, B2 / 2 + p, k3));
      fa[2 * p] = fmaf((float)sq.x, c1, c2);
      fa[2 * p + 1] = fmaf((float)sq.y, c1, c2);
      fb[2 * p] = fa[2 * p] * fmaf((float)zq.x, e1, e2);
      fb[2 * p + 1] = fa[2 * p + 1] * fmaf((float)zq.y, e1, e2);
      if constexpr (FOLD) {                  // the extracted value is K + code/2^W instead of 1 + code/2^W
        const float K = CodeClass<W, true>::K(CodeClass<W, true>::of_pair(p));   // a constant once the loop is unrolled
        fb[2 * p] = fmaf(1.f - K, fa[2 * p], fb[2 * p]);
        fb[2 * p + 1] = fmaf(1.f - K, fa[2 * p + 1], fb[2 * p + 1]);
      }
    }
    uint32_t* mine = buf + lane * S;
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {         // columns PC*ph .. PC*ph+PC-1 of every tile
      // the lane's 64 values of the phase, row by row (PC/2 dwords per row), 16 bytes per store
#pragma unroll
      for (int k4 = 0; k4 < 8; ++k4) {
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int dw = 4 * k4 + d, r = dw / (PC / 2), p = (PC / 2) * ph + dw % (PC / 2);
          const half2_t q2 = as_half2(FOLD ? pair_class_inline<W>(t.c, r * PPR + p, kk) : pair_f16<W>(t.c, r * PPR + p, kc));
          const int g0 = AXIS == 1 ? 2 * p : r, g1 = AXIS == 1 ? 2 * p + 1 : r;
          half2_t w;
          w.x = (_Float16)fmaf((float)q2.x, fa[g0], fb[g0]);
          w.y = (_Float16)fmaf((float)q2.y, fa[g1], fb[g1]);
          o[d] = __builtin_bit_cast(uint32_t, w);
        }
        const u32x4 v = {o[0], o[1], o[2], o[3]};
        *reinterpret_cast<u32x4*>(mine + 4 * k4) = v;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();       // the buffer is this wavefront's own: its LDS operations stay in order
      constexpr int JG = NM < 8 ? NM : 8;    // MFMAs whose operands are in flight at a time
#pragma unroll
      for (int j0 = 0; j0 < NM; j0 += JG) {
        uint32_t av[MB][JG][4], bv[JG][4];
#pragma unroll
        for (int j = 0; j < JG; ++j) {
#pragma unroll
          for (int tt = 0; tt < TPK; ++tt) {
            const int tile0 = (4 * (j0 + j)) * TPK + tt;         // + g4*TPK: in afrag / xfrag
            const uint32_t* pb = xfrag + tile0 * (TC / 2) + (PC / 2) * ph;
#pragma unroll
            for (int d = 0; d < PC / 2; ++d) bv[j][tt * (PC / 2) + d] = pb[d];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
              const uint32_t* pa = afrag + tile0 * S + mb * (16 * PC / 2);
#pragma unroll
              for (int d = 0; d < PC / 2; ++d) av[mb][j][tt * (PC / 2) + d] = pa[d];
            }
          }
        }
#pragma unroll
        for (int j = 0; j < JG; ++j) {
          const uint32_t b4v[4] = {bv[j][0], bv[j][1], bv[j][2], bv[j][3]};
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            const uint32_t a4v[4] = {av[mb][j][0], av[mb][j][1], av[mb][j][2], av[mb][j][3]};
            D[mb][j & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a4v),
                                                                   __builtin_bit_cast(half8_t, b4v), D[mb][j & 1], 0, 0, 0);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();       // the reads are issued before the next phase overwrites the buffer
    }
  };

  if constexpr (ONE) {                       // one step per workgroup: no second tile, no loop (fewer registers)
    T t0;
    fetch_x(s_lo);
    issue(t0, s_lo);
    run_step(t0, s_lo);
  } else {
    T t0, t1;
    fetch_x(s_lo);
    issue(t0, s_lo);
    int st = s_lo;
    while (st + 1 < s_hi) {                  // workgroup-uniform; two steps per trip, one exit at the bottom
      issue(t1, st + 1);
      run_step(t0, st);
      issue(t0, st + 2);                     // a dummy behind the last step
      run_step(t1, st + 1);
      st += 2;
    }
    if (st < s_hi) run_step(t0, st);
  }

  // D[mb][row 16*mb + 4*g4 + v][batch i16]
  if (active && i16 < batch) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const float4_t d = D[mb][0] + D[mb][1];
      if (16 * mb + 4 * g4 < TR)
        *reinterpret_cast<float4_t*>(P + (int64_t)split * split_stride + (int64_t)i16 * m + (int64_t)strip * TR +
                                     16 * mb + 4 * g4) = d;
    }
  }
}

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), 2)
gemm_mfma_kernel(DevMatrix A, const uint16_t* __restrict__ X, float* __restrict__ P, int64_t split_stride,
                 int steps_per_split, int batch, const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row,
                 int groups) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int bx = blockIdx.x;
  gemm_mfma_body<W, TR, TC, AXIS, false>(A, X, P, split_stride, steps_per_split, batch, XT, slots, long_row,
                                         bx < groups ? bx : -1, (int)blockIdx.y, bx - groups, (int)gridDim.x - groups, smem);
}

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), (TC == 32 ? 2 : 3))
gemm_mfma_one_kernel(DevMatrix A, const uint16_t* __restrict__ X, float* __restrict__ P, int64_t split_stride,
                     int batch, const uint16_t* __restrict__ XT, float* __restrict__ slots, int long_row, int groups) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int bx = blockIdx.x;
  gemm_mfma_body<W, TR, TC, AXIS, true>(A, X, P, split_stride, 1, batch, XT, slots, long_row,
                                        bx < groups ? bx : -1, (int)blockIdx.y, bx - groups, (int)gridDim.x - groups, smem);
}

// Several matrices that share the batch X and the format (q/k/v, gate/up of a decoder block) in one grid:
// blockIdx.x counts the dense workgroups of all matrices first, then their long-row workgroups.  Every
// workgroup does exactly what it would do in a launch of its own matrix.
struct MfmaFusedItem {
  DevMatrix A;
  float* P;                                  // partial results (or the output itself, see the finishing kernel)
  float* slots;
  void* Y;
  int long_row;
  int groups, extra;                         // dense / long-row workgroups of this matrix
  int blocks16;                              // workgroups of the finishing kernel
};
struct MfmaFused {
  int count;
  MfmaFusedItem it[SPQR_MAX_FUSED];
};

template <int W, int TR, int TC, int AXIS, bool ONE>
__global__ void __launch_bounds__((64 * MfmaShape<TR, TC>::NS), (ONE && TC != 32 ? 3 : 2))
gemm_mfma_fused_kernel(MfmaFused F, const uint16_t* __restrict__ X, int steps_per_split, int batch,
                       const uint16_t* __restrict__ XT) {
  extern __shared__ __align__(16) uint8_t smem[];
  int bx = blockIdx.x, i = 0;
  bool dense = false;                        // workgroup-uniform search, count <= SPQR_MAX_FUSED
  for (; i < F.count; ++i) {
    if (bx < F.it[i].groups) { dense = true; break; }
    bx -= F.it[i].groups;
  }
  if (!dense) {
    for (i = 0; i < F.count - 1; ++i) {
      if (bx < F.it[i].extra) break;
      bx -= F.it[i].extra;
    }
  }
  const MfmaFusedItem& it = F.it[i];
  gemm_mfma_body<W, TR, TC, AXIS, ONE>(it.A, X, it.P, (int64_t)batch * it.A.g.m, ONE ? 1 : steps_per_split, batch, XT, it.slots,
                                  it.long_row, dense ? bx : -1, (int)blockIdx.y, bx, it.extra, smem);
}

// Prepares the batch for the batch path.  With an input permutation, column j of the
// matrix meets x[perm[j]] (act-order, Sec. 4 / Alg. 1: the quantiser reorders the input
// dimension): XP[b][j] = X[b][perm[j]] is the batch in the matrix's column order, read by
// the dense kernel in place of X.  For the outlier kernels, XT[j][16] binary16 is the same
// transposed, batch rows beyond `batch` zero, so that one outlier (one column j) meets its
// 16 activations in one 32-byte line; line n is all zeros: the place entry slots behind
// the end of a row read.  Either output may be absent.
__global__ void __launch_bounds__(256)
transpose_x16_kernel(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, uint16_t* __restrict__ XT,
                     uint16_t* __restrict__ XP, int n, int batch) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j > n) return;
  const int src = j < n ? (perm ? perm[j] : j) : 0;
  uint32_t o[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const uint32_t lo = (j < n && 2 * k < batch) ? X[(int64_t)(2 * k) * n + src] : 0u;
    const uint32_t hi = (j < n && 2 * k + 1 < batch) ? X[(int64_t)(2 * k + 1) * n + src] : 0u;
    o[k] = lo | (hi << 16);
    if (XP != nullptr && j < n) {
      if (2 * k < batch) XP[(int64_t)(2 * k) * n + j] = (uint16_t)lo;
      if (2 * k + 1 < batch) XP[(int64_t)(2 * k + 1) * n + j] = (uint16_t)hi;
    }
  }
  if (XT != nullptr) {
    u32x4* d = reinterpret_cast<u32x4*>(XT + (int64_t)j * 16);
    const u32x4 v0 = {o[0], o[1], o[2], o[3]}, v1 = {o[4], o[5], o[6], o[7]};
    d[0] = v0;
    d[1] = v1;
  }
}

// value of lane J (0 or 1) of the caller's pair of lanes, for both lanes of the pair
template <int J>
__device__ __forceinline__ uint32_t pair_broadcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, J == 0 ? 0xA0 : 0xF5, 0xF, 0xF, false);   // quad_perm [J,J,2+J,2+J]
}

// Finishing kernel for up to 16 activation vectors:
// Y[b][i] = sum_split P[split][b][i] + sum_k val_k * X[b][col_k]  (Sec. 4.2: the sparse
// part is a separate product), rounded to y_dtype.  With one split and binary32
// output P may be Y itself.
// One workgroup of 512 threads per strip of 16 rows.  The strip's CSR entries pass
// through LDS in chunks of 4096 (every thread brings one aligned granule of 8
// entries; chunks that lie inside one long row are skipped).  A pair of lanes works
// on one part of one row, each lane on 8 of the 16 activation vectors (16 bytes of
// the entry's line of XT), so no reduction across lanes exists: the pair walks its
// entries in order, 4 per trip (each lane reads 2 of them from LDS and hands them to
// its partner).  A row is cut into 16 contiguous parts (256 pairs = 16 rows x 16);
// parts are added in order by the row's owner.  A row longer than long_row comes
// ready-made from long_rows_block: its owner adds the row's slots in order.  Fixed
// order everywhere, one writer per output.
constexpr int kFinishThreads = 512;

__device__ __forceinline__ void finish_xt16_body(const DevMatrix& A, const uint16_t* __restrict__ XT,
                                                 const float* __restrict__ slots, const float* P, int nsplit,
                                                 int64_t split_stride, int long_row, void* Y, int y_dtype, int batch,
                                                 const int s) {
  constexpr int TR = 16, NP = kFinishThreads / 2, PER_ROW = NP / TR, CHUNK = 8 * kFinishThreads;
  __shared__ int rp[TR + 1];
  __shared__ float part[NP][16];
  __shared__ __align__(16) uint16_t scol[CHUNK], sval[CHUNK];
  const int tid = threadIdx.x, pr = tid >> 1, bq = tid & 1;
  const int g = tid >> 4, b = tid & 15;      // the owner of Y[b][row g] for tid < 256
  const int m = A.g.m;
  if (tid <= TR) rp[tid] = A.row_ptr[min(s * TR + tid, m)];      // rows behind the last one (m % 16 == 8) are empty
  // the dense part of this thread's output: requested now, needed at the very end
  const int64_t at = (int64_t)min(b, batch - 1) * m + min(s * TR + min(g, TR - 1), m - 1);
  float dense = 0.f;
  for (int k = 0; k < nsplit; ++k) dense += P[k * split_stride + at];
  __syncthreads();
  const int e_lo = rp[0], e_hi = rp[TR];
  const bool inplace = static_cast<const void*>(P) == static_cast<const void*>(Y);   // one split, written to Y by the dense kernel
  if (inplace && e_hi == e_lo) return;       // nothing to add (workgroup-uniform)
  const uint8_t* xt16 = reinterpret_cast<const uint8_t*>(XT) + 16 * bq;
  const uint32_t zoff = (uint32_t)A.g.n * 32u;
  // Both lanes of the pair add the 4 entries at chunk positions i0 + bq and i0 + 2 + bq (global index e0 + i),
  // those inside [lo, hi) (hi never beyond the chunk); the others read the zero line of XT with value 0.
  auto consume = [&](int e0, int i0, int lo, int hi, float (&acc)[8]) {
    uint32_t off[2], val[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int i = i0 + 2 * h + bq, e = e0 + i;
      const bool ok = e >= lo && e < hi;
      const int ic = min(i, CHUNK - 1);
      off[h] = ok ? (uint32_t)scol[ic] * 32u : zoff;
      val[h] = ok ? __builtin_bit_cast(uint32_t, h2f(sval[ic])) : 0u;
    }
    u32x4 xx[4];
    float vv[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t o[2] = {pair_broadcast<0>(off[h]), pair_broadcast<1>(off[h])};
      const uint32_t v[2] = {pair_broadcast<0>(val[h]), pair_broadcast<1>(val[h])};
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        xx[2 * h + j] = *reinterpret_cast<const u32x4*>(xt16 + o[j]);
        vv[2 * h + j] = __builtin_bit_cast(float, v[j]);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w[4] = {xx[i].x, xx[i].y, xx[i].z, xx[i].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = fmaf(vv[i], h2f((uint16_t)(w[k] & 0xFFFFu)), acc[2 * k]);
        acc[2 * k + 1] = fmaf(vv[i], h2f((uint16_t)(w[k] >> 16)), acc[2 * k + 1]);
      }
    }
  };
  float sum = 0.f;
  if (e_hi > e_lo) {
    const u32x4* col8 = reinterpret_cast<const u32x4*>(A.col);
    const u32x4* val8 = reinterpret_cast<const u32x4*>(A.val);
    const int g_lo = e_lo >> 3, ngran = ((e_hi - 1) >> 3) - g_lo + 1;
    // this pair's part of an ordinary row (empty for a long row)
    int a, z;
    {
      const int r = pr / PER_ROW;
      const int lo = rp[r], hi = rp[r + 1], len = hi - lo;
      const int per = (len + PER_ROW - 1) / PER_ROW;
      a = min(lo + (pr % PER_ROW) * per, hi);
      z = len <= long_row ? min(a + per, hi) : a;
    }
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    for (int ch = 0; ch * kFinishThreads < ngran; ++ch) {         // workgroup-uniform
      const int e0 = 8 * (g_lo + ch * kFinishThreads), e1 = e0 + CHUNK;   // the chunk's entries
      bool skip = false;                     // nothing but one long row in it
#pragma unroll
      for (int r = 0; r < TR; ++r) skip = skip || (rp[r + 1] - rp[r] > long_row && rp[r] <= max(e0, e_lo) && rp[r + 1] >= min(e1, e_hi));
      if (skip) continue;
      const int gi = ch * kFinishThreads + tid;
      const u32x4 none = {0u, 0u, 0u, 0u};
      const u32x4 nc = gi < ngran ? col8[g_lo + gi] : none, nv = gi < ngran ? val8[g_lo + gi] : none;
      __syncthreads();                       // the previous chunk is consumed
      reinterpret_cast<u32x4*>(scol)[tid] = nc;
      reinterpret_cast<u32x4*>(sval)[tid] = nv;
      __syncthreads();
      for (int e = max(a, e0); e < min(z, e1); e += 4) consume(e0, e - e0, a, min(z, e1), acc);
    }
#pragma unroll
    for (int k2 = 0; k2 < 8; ++k2) part[pr][8 * bq + k2] = acc[k2];
    __syncthreads();
    if (g < TR) {
      const int lo = rp[g], hi = rp[g + 1];
      if (hi - lo <= long_row) {
#pragma unroll
        for (int k = 0; k < PER_ROW; ++k) sum += part[g * PER_ROW + k][b];
      } else {
        for (int e0 = lo; e0 < hi; e0 += kLongSlice) sum += slots[(int64_t)(lo / kSlotGrain + (e0 - lo) / kLongSlice) * 16 + b];
      }
    }
  }
  if (g < TR && s * TR + g < m && b < batch && (rp[g + 1] > rp[g] || !inplace)) {
    if (y_dtype == SPQR_F32) static_cast<float*>(Y)[at] = dense + sum;
    else static_cast<uint16_t*>(Y)[at] = f2h_rne(dense + sum);
  }
}

__global__ void __launch_bounds__(kFinishThreads, 8)
finish_xt16_kernel(DevMatrix A, const uint16_t* __restrict__ XT, const float* __restrict__ slots, const float* P,
                   int nsplit, int64_t split_stride, int long_row, void* Y, int y_dtype, int batch) {
  finish_xt16_body(A, XT, slots, P, nsplit, split_stride, long_row, Y, y_dtype, batch, (int)blockIdx.x);
}

__global__ void __launch_bounds__(kFinishThreads, 8)
finish_xt16_fused_kernel(MfmaFused F, const uint16_t* __restrict__ XT, int nsplit, int y_dtype, int batch) {
  int bx = blockIdx.x, i = 0;
  for (; i < F.count - 1; ++i) {             // workgroup-uniform
    if (bx < F.it[i].blocks16) break;
    bx -= F.it[i].blocks16;
  }
  const MfmaFusedItem& it = F.it[i];
  finish_xt16_body(it.A, XT, it.slots, it.P, nsplit, (int64_t)batch * it.A.g.m, it.long_row, it.Y, y_dtype, batch, bx);
}

// ---- batches above 4 on 16x16 tiles: matrix-core dense pass + outlier pass ----
// Steps per workgroup of the dense pass, chosen by simulating the launch: the workgroups start in grid order
// (split by split: the strip groups, behind those of the first split the long-row workgroups) on the first free of
// the chip's workgroup slots; a dense workgroup costs its steps plus a start-up of 0.3 step, a long-row workgroup
// 0.45 step, and every split 0.3 step for its partial result (written, and read again by the finishing kernel).
// The shortest schedule wins, ties go to fewer splits.  The constants are fitted to sweeps over the steps on
// MI355X (eight projection shapes of the 7B to 65B configurations at batch 8 and 16, every count of steps: the choice is
// within 2.2 % of the best measured one).  slots1 = slots when a workgroup takes one step (the variant with fewer registers),
// slots = otherwise.  Results are remembered per argument tuple (the simulation costs up to a few milliseconds).
static double mfma_schedule_length(int groups, int nsteps, int s, int slots, int nlong) {
  const int nsplit = (nsteps + s - 1) / s;
  std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
  for (int i = 0; i < slots; ++i) free_at.push(0.0);
  double end = 0.0;
  auto run = [&](int count, double cost) {
    for (int i = 0; i < count; ++i) {
      const double t = free_at.top() + cost;
      free_at.pop();
      free_at.push(t);
      if (t > end) end = t;
    }
  };
  for (int y = 0; y < nsplit; ++y) {
    const int steps = s < nsteps - y * s ? s : nsteps - y * s;
    run(groups, 0.3 + steps);
    run(nlong, y == 0 ? 0.45 : 0.02);         // behind the first split they leave at once
  }
  return end + 0.3 * nsplit;
}

// Scratch of the batch path.  A call on a stream that is not being captured takes the buffer the library keeps for
// that stream: work on one stream runs in order, so its calls can share one buffer, and nothing is allocated or
// freed per call (on this runtime a stream-ordered allocation waits on the host until the stream's earlier work is
// done, which keeps the next call's launches from being queued behind the running one: about 5 us per call).  The
// buffer grows when a call needs more (the stream is synchronised first) and is kept until the process ends; up to
// kScratchStreams streams per device have one; further streams allocate stream-ordered from a memory pool of the
// library's own (one per device, unlimited release threshold), captured calls from the device's default pool, which
// the capture turns into allocation nodes of the graph (graphs of many such calls replay correctly with it; with the
// library's own pool the allocations of all but the first call of a capture failed).  A buffer's lock is held while its call is enqueued: calls from several host
// threads on one stream do not interleave their kernels.
constexpr int kScratchStreams = 8;
struct ScratchSlot {
  std::mutex lock;                           // held while a call that uses the buffer is enqueued
  hipStream_t stream = nullptr;
  uint8_t* buf = nullptr;
  size_t size = 0;
  bool taken = false;
};
struct Scratch {
  uint8_t* p = nullptr;
  bool pooled = false;                       // stream-ordered allocation, to be freed on the stream
  std::unique_lock<std::mutex> hold;
};

static hipMemPool_t scratch_pool(int dev) {
  static std::mutex lock;
  static hipMemPool_t pools[kMaxDevices];
  static bool tried[kMaxDevices];
  if (dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  if (!tried[dev]) {
    tried[dev] = true;
    hipMemPoolProps props = {};
    props.allocType = hipMemAllocationTypePinned;
    props.handleTypes = hipMemHandleTypeNone;
    props.location.type = hipMemLocationTypeDevice;
    props.location.id = dev;
    hipMemPool_t pool = nullptr;
    if (hipMemPoolCreate(&pool, &props) == hipSuccess) {
      uint64_t keep = UINT64_MAX;
      if (hipMemPoolSetAttribute(pool, hipMemPoolAttrReleaseThreshold, &keep) == hipSuccess) pools[dev] = pool;
      else (void)hipMemPoolDestroy(pool);
    }
    if (pools[dev] == nullptr) (void)hipGetLastError();
  }
  return pools[dev];
}

// hipErrorNotSupported: no scratch to be had (the caller takes the vector path).
static hipError_t scratch_get(Scratch* sc, size_t bytes, int dev, hipStream_t stream, bool allow_stream_ordered = true) {
  static std::mutex table_lock;
  static ScratchSlot slots[kMaxDevices][kScratchStreams];
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  const bool capturing = hipStreamIsCapturing(stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
  ScratchSlot* slot = nullptr;
  if (!capturing && dev >= 0 && dev < kMaxDevices) {
    std::lock_guard<std::mutex> hold(table_lock);
    for (int i = 0; i < kScratchStreams && slot == nullptr; ++i)
      if (slots[dev][i].taken && slots[dev][i].stream == stream) slot = &slots[dev][i];
    for (int i = 0; i < kScratchStreams && slot == nullptr; ++i)
      if (!slots[dev][i].taken) {
        slot = &slots[dev][i];
        slot->taken = true;
        slot->stream = stream;
      }
  }
  if (slot != nullptr) {
    sc->hold = std::unique_lock<std::mutex>(slot->lock);
    if (slot->size < bytes) {
      // the stream's earlier calls may still read the old buffer
      if (slot->buf != nullptr && (hipStreamSynchronize(stream) != hipSuccess || hipFree(slot->buf) != hipSuccess)) {
        (void)hipGetLastError();
        sc->hold.unlock();
        return hipErrorNotSupported;
      }
      slot->buf = nullptr;
      slot->size = 0;
      const size_t want = (bytes + bytes / 4 + 0xFFFFF) & ~(size_t)0xFFFFF;   // some room, whole megabytes
      if (hipMalloc(reinterpret_cast<void**>(&slot->buf), want) != hipSuccess) {
        (void)hipGetLastError();
        slot->buf = nullptr;
        sc->hold.unlock();
        return hipErrorNotSupported;
      }
      slot->size = want;
    }
    sc->p = slot->buf;
    sc->pooled = false;
    return hipSuccess;
  }
  // The fused launch set never runs on a stream-ordered allocation: that is the kind of scratch the one memory
  // fault seen on this path had (a captured graph of fused calls, cause unknown); its caller falls back to one
  // call per matrix.
  if (!allow_stream_ordered) return hipErrorNotSupported;
  // captured: the device's default pool (allocation nodes of the graph); else the library's own pool
  hipMemPool_t pool = capturing ? nullptr : scratch_pool(dev);
  const hipError_t e = pool != nullptr ? hipMallocFromPoolAsync(reinterpret_cast<void**>(&sc->p), bytes, pool, stream)
                                       : hipMallocAsync(reinterpret_cast<void**>(&sc->p), bytes, stream);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    sc->p = nullptr;
    return hipErrorNotSupported;
  }
  sc->pooled = true;
  return hipSuccess;
}
// after the call's last kernel is enqueued
static hipError_t scratch_put(Scratch* sc, hipStream_t stream) {
  hipError_t e = hipSuccess;
  if (sc->pooled && sc->p != nullptr) e = hipFreeAsync(sc->p, stream);
  if (sc->hold.owns_lock()) sc->hold.unlock();
  sc->p = nullptr;
  return e;
}

// Workgroups for the long outlier rows of a matrix: each owns an equal share of the entries (see long_rows_block)
// and pays a look at the row pointers whether its share holds long rows or not: one per strip of 16 rows, 128 at most.
static int long_row_workgroups(const DevMatrix& A) {
  if (A.nnz <= 0) return 0;
  const int strips = (A.g.m + 15) / 16;
  return strips < kCUs / 2 ? strips : kCUs / 2;
}

static int mfma_steps_per_split(int groups, int nsteps, int slots1, int slots, int nlong) {
  if (const int v = option(SPQR_OPT_BATCH_STEPS); v >= 1) return v < nsteps ? v : nsteps;   // pinned (tuning, tests)
  struct Known { int groups, nsteps, slots1, slots, nlong, best; };
  static std::mutex lock;
  static std::vector<Known> known;
  {
    std::lock_guard<std::mutex> hold(lock);
    for (const Known& k : known)
      if (k.groups == groups && k.nsteps == nsteps && k.slots1 == slots1 && k.slots == slots && k.nlong == nlong) return k.best;
  }
  int best = nsteps;
  double best_cost = 1e30;
  // candidates: every count of steps up to 32, and all of them in one workgroup; launches of more than
  // 200 000 workgroups are not simulated (only very large matrices: any choice fills the chip)
  for (int s = nsteps; s >= 1; s = (s > 32 ? 32 : s - 1)) {
    const long wgs = (long)(groups + nlong) * ((nsteps + s - 1) / s);
    if (wgs > 200000) continue;
    const double cost = mfma_schedule_length(groups, nsteps, s, s == 1 ? slots1 : slots, nlong);
    if (cost < best_cost - 1e-9) { best_cost = cost; best = s; }
  }
  std::lock_guard<std::mutex> hold(lock);
  if (known.size() < 4096) known.push_back(Known{groups, nsteps, slots1, slots, nlong, best});
  return best;
}

int plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups) {
  return mfma_steps_per_split(groups, nsteps, slots_one_step, slots, long_workgroups);
}

// Transposition, dense pass (with the long outlier rows beside it) and finishing pass.  Scratch (the batch
// transposed, (n+1) x 32 bytes, the sums of the long outlier rows, 64 bytes per 256 outliers, the batch in the
// matrix's column order if there is a permutation, and the partial results when the steps are split or the
// output is binary16): see scratch_get.
// hipErrorNotSupported = no scratch to be had; the caller takes the vector path.
template <int W, int TR, int TC, int AXIS>
static hipError_t launch_mfma_t(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                                const Workspace& ws) {
  using SH = MfmaShape<TR, TC>;
  const Geometry& g = A.g;
  static PerDevice ready;
  const int dev = current_device();
  if (!ready.get(dev)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<W, TR, TC, AXIS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e != hipSuccess) return e;
    ready.set(dev, 1);
  }
  const int groups = (g.ntr + SH::NS - 1) / SH::NS;
  const int nsteps = (g.ntc + 63) / 64;
  const bool sparse = A.nnz > 0, permuted = A.perm != nullptr;
  constexpr int kNT = 64 * SH::NS;
  const int extra = long_row_workgroups(A);
  // the one-step variant fits three workgroups on a CU while the staged batch rows leave the LDS for them
  const int wgs1 = (TC != 32 && 3 * ((size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW + 1024) <= 160 * 1024) ? 3 : SH::WGS;
  const int steps_per_split = mfma_steps_per_split(groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, extra);
  const int nsplit = (nsteps + steps_per_split - 1) / steps_per_split;
  // the dense kernel writes Y itself (16 bytes per store) if nothing has to be added or converted afterwards
  const bool direct = nsplit == 1 && y_dtype == SPQR_F32 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const size_t xt_bytes = sparse ? up(((size_t)g.n + 1) * 32) : 0;   // one more row: zeros
  const size_t slot_bytes = sparse ? up(((size_t)(A.nnz / kSlotGrain) + 2) * 64) : 0;
  const size_t xp_bytes = permuted ? up((size_t)b * g.n * 2) : 0;
  const size_t part_bytes = direct ? 0 : (size_t)nsplit * b * g.m * sizeof(float);
  Scratch sc;
  uint8_t* scratch = nullptr;
  if (const size_t need = xt_bytes + slot_bytes + xp_bytes + part_bytes; need > 0) {
    if (ws.from_caller) {                    // nothing is allocated, freed or waited for
      if (ws.p == nullptr || ws.bytes < need) return hipErrorOutOfMemory;
      scratch = ws.p;
    } else {
      if (scratch_get(&sc, need, dev, stream) != hipSuccess) return hipErrorNotSupported;
      scratch = sc.p;
    }
  }
  uint16_t* xt = sparse ? reinterpret_cast<uint16_t*>(scratch) : nullptr;
  float* slots = reinterpret_cast<float*>(scratch + xt_bytes);
  uint16_t* xp = permuted ? reinterpret_cast<uint16_t*>(scratch + xt_bytes + slot_bytes) : nullptr;
  float* part = direct ? static_cast<float*>(Y) : reinterpret_cast<float*>(scratch + xt_bytes + slot_bytes + xp_bytes);
  const int64_t split_stride = (int64_t)b * g.m;
  // a row is long if it holds far more outliers than the average row (and at least kLongRowMin): rows like the
  // average one stay with their strip's workgroup in the finishing kernel, whatever the outlier rate
  const int64_t avg_row = A.nnz / (g.m > 0 ? g.m : 1);
  const int long_row = (int)(4 * avg_row > kLongRowMin ? (4 * avg_row < (1 << 30) ? 4 * avg_row : (1 << 30)) : kLongRowMin);
  hipError_t e = hipSuccess;
  if (sparse || permuted) {
    hipLaunchKernelGGL(transpose_x16_kernel, dim3((g.n + 256) / 256), dim3(256), 0, stream, X, A.perm, xt, xp, g.n, b);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    if (steps_per_split == 1) {
      static PerDevice ready1;
      if (!ready1.get(dev)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_one_kernel<W, TR, TC, AXIS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
        if (e == hipSuccess) ready1.set(dev, 1);
      }
      const size_t lds_now = (size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW;   // only b rows of X are staged
      if (e == hipSuccess)
        hipLaunchKernelGGL((gemm_mfma_one_kernel<W, TR, TC, AXIS>), dim3(groups + extra, nsplit), dim3(kNT), lds_now,
                           stream, A, permuted ? xp : X, part, split_stride, b, xt, slots, long_row, groups);
    } else {
      hipLaunchKernelGGL((gemm_mfma_kernel<W, TR, TC, AXIS>), dim3(groups + extra, nsplit), dim3(kNT), SH::LDS,
                         stream, A, permuted ? xp : X, part, split_stride, steps_per_split, b, xt, slots, long_row, groups);
    }
    if (e == hipSuccess) e = hipGetLastError();
  }
  if (e == hipSuccess && (sparse || !direct)) {
    hipLaunchKernelGGL(finish_xt16_kernel, dim3((g.m + 15) / 16), dim3(kFinishThreads), 0, stream, A, xt, slots, part, nsplit,
                       split_stride, long_row, Y, y_dtype, b);
    e = hipGetLastError();
  }
  const hipError_t ef = scratch_put(&sc, stream);
  return e == hipSuccess ? ef : e;
}

// Whether a batch of b > 4 vectors takes the matrix-core path.  It pays two more launches and the
// transposition through LDS, the vector path re-reads the weights once per 4 vectors.  Measured on
// MI355X with eager calls (a sweep of b = 2..16 over the layers of the 7B, 33B and 65B shapes, both paths forced)
// the matrix cores win from 7 vectors on for any layer (4096^2 at b = 5 / 6 / 7 / 8: 19.9 / 20.0 / 20.0 / 20.1 us
// against 17.4 / 19.6 / 25.2 / 23.8) and from 4 on for layers of 30 M weights or more (17920x6656 at b = 4:
// about 52 us against 61; layers of 45 M weights are break-even at 4).  `alloc_nodes`: the call's scratch would be
// allocation nodes of a graph under capture (library-owned scratch on a capturing stream), about 10 us more
// per call: then from 13 vectors on for any layer, from 8 on for layers of 40 M weights and from 5 on for
// layers of 100 M.  The option SPQR_OPT_BATCH_PATH forces one or the other wherever both apply (tests
// compare the two).
bool mfma_wanted(const Geometry& g, int b, bool alloc_nodes) {
  const int forced = option(SPQR_OPT_BATCH_PATH);
  if (forced == SPQR_BATCH_PATH_VECTOR) return false;
  if (forced == SPQR_BATCH_PATH_MATRIX) return true;   // (_DENSE: the rule below, for calls the dense copy cannot take)
  const double weights = (double)g.m * (double)g.n;
  if (alloc_nodes) return b >= 13 || (b >= 8 && weights >= 40e6) || weights >= 100e6;
  return b >= 7 || weights >= 30e6;
}

bool stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); return true; }
  return cs != hipStreamCaptureStatusNone;
}

template <int W, int TR, int TC, int AXIS>
static hipError_t launch_mfma_fused_t(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                                      hipStream_t stream, const Workspace& ws) {
  using SH = MfmaShape<TR, TC>;
  const Geometry& g0 = As[0].g;
  static PerDevice ready;
  const int dev = current_device();
  if (!ready.get(dev)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_fused_kernel<W, TR, TC, AXIS, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_fused_kernel<W, TR, TC, AXIS, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SH::LDS);
    if (e != hipSuccess) return e;
    ready.set(dev, 1);
  }
  constexpr int kNT = 64 * SH::NS;
  const int nsteps = (g0.ntc + 63) / 64;
  int total_groups = 0, total_extra = 0, extras[SPQR_MAX_FUSED];
  bool sparse = false;
  for (int i = 0; i < count; ++i) {
    const Geometry& g = As[i].g;
    total_groups += (g.ntr + SH::NS - 1) / SH::NS;
    sparse = sparse || As[i].nnz > 0;
    extras[i] = long_row_workgroups(As[i]);
    total_extra += extras[i];
  }
  const int wgs1 = (TC != 32 && 3 * ((size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW + 1024) <= 160 * 1024) ? 3 : SH::WGS;
  const int steps_per_split = mfma_steps_per_split(total_groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, total_extra);
  const int nsplit = (nsteps + steps_per_split - 1) / steps_per_split;
  const bool permuted = As[0].perm != nullptr;
  bool direct = nsplit == 1 && y_dtype == SPQR_F32;              // the dense kernel writes the outputs itself (16-byte stores)
  for (int i = 0; i < count; ++i) direct = direct && reinterpret_cast<uintptr_t>(Ys[i]) % 16 == 0;
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const size_t xt_bytes = sparse ? up(((size_t)g0.n + 1) * 32) : 0;
  const size_t xp_bytes = permuted ? up((size_t)b * g0.n * 2) : 0;
  size_t total = xt_bytes + xp_bytes, slot_off[SPQR_MAX_FUSED], part_off[SPQR_MAX_FUSED];
  for (int i = 0; i < count; ++i) {
    slot_off[i] = total;
    total += As[i].nnz > 0 ? up(((size_t)(As[i].nnz / kSlotGrain) + 2) * 64) : 0;
    part_off[i] = total;
    total += direct ? 0 : up((size_t)nsplit * b * As[i].g.m * sizeof(float));
  }
  Scratch sc;
  uint8_t* scratch = nullptr;
  if (total > 0) {
    if (ws.from_caller) {
      if (ws.p == nullptr || ws.bytes < total) return hipErrorOutOfMemory;
      scratch = ws.p;
    } else {
      if (scratch_get(&sc, total, dev, stream, false) != hipSuccess) return hipErrorNotSupported;
      scratch = sc.p;
    }
  }
  uint16_t* xt = sparse ? reinterpret_cast<uint16_t*>(scratch) : nullptr;
  uint16_t* xp = permuted ? reinterpret_cast<uint16_t*>(scratch + xt_bytes) : nullptr;
  MfmaFused F;
  F.count = count;
  int dense_blocks = 0, extra_blocks = 0, finish_blocks = 0;
  for (int i = 0; i < count; ++i) {
    MfmaFusedItem& it = F.it[i];
    const Geometry& g = As[i].g;
    it.A = As[i];
    it.Y = Ys[i];
    it.P = direct ? static_cast<float*>(Ys[i]) : reinterpret_cast<float*>(scratch + part_off[i]);
    it.slots = reinterpret_cast<float*>(scratch + slot_off[i]);
    const int64_t avg_row = As[i].nnz / (g.m > 0 ? g.m : 1);
    it.long_row = (int)(4 * avg_row > kLongRowMin ? (4 * avg_row < (1 << 30) ? 4 * avg_row : (1 << 30)) : kLongRowMin);
    it.groups = (g.ntr + SH::NS - 1) / SH::NS;
    it.extra = extras[i];
    it.blocks16 = (g.m + 15) / 16;
    dense_blocks += it.groups;
    extra_blocks += it.extra;
    finish_blocks += it.blocks16;
  }
  hipError_t e = hipSuccess;
  if (sparse || permuted) {
    hipLaunchKernelGGL(transpose_x16_kernel, dim3((g0.n + 256) / 256), dim3(256), 0, stream, X, As[0].perm, xt, xp, g0.n, b);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    if (steps_per_split == 1)                // the variant without the second tile; only b rows of X are staged
      hipLaunchKernelGGL((gemm_mfma_fused_kernel<W, TR, TC, AXIS, true>), dim3(dense_blocks + extra_blocks, nsplit), dim3(kNT),
                         (size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW, stream, F, permuted ? xp : X, 1, b, xt);
    else
      hipLaunchKernelGGL((gemm_mfma_fused_kernel<W, TR, TC, AXIS, false>), dim3(dense_blocks + extra_blocks, nsplit), dim3(kNT),
                         SH::LDS, stream, F, permuted ? xp : X, steps_per_split, b, xt);
    e = hipGetLastError();
  }
  if (e == hipSuccess && (sparse || !direct)) {
    hipLaunchKernelGGL(finish_xt16_fused_kernel, dim3(finish_blocks), dim3(kFinishThreads), 0, stream, F, xt, nsplit, y_dtype, b);
    e = hipGetLastError();
  }
  const hipError_t ef = scratch_put(&sc, stream);
  return e == hipSuccess ? ef : e;
}


#define SPQR_MFMA_INSTANCES(CASE) \
  CASE(3, 16, 16, 1) CASE(3, 16, 16, 0) CASE(4, 16, 16, 1) CASE(4, 16, 16, 0) \
  CASE(3, 8, 32, 1) CASE(4, 8, 32, 1) CASE(3, 32, 8, 0) CASE(4, 32, 8, 0)

// Upper bound of the scratch a batch of b <= 16 vectors needs on this path (the launchers need less when the dense
// kernel can write the output itself): for one matrix alone, and for `count` matrices in one fused launch set.
template <int TR, int TC>
static size_t mfma_scratch_bound(const DevMatrix* As, int count, int b, bool fused) {
  using SH = MfmaShape<TR, TC>;
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const Geometry& g0 = As[0].g;
  const int nsteps = (g0.ntc + 63) / 64;
  const int wgs1 = (TC != 32 && 3 * ((size_t)SH::NS * 64 * kMfmaTileStride * 4 + (size_t)b * SH::XROW + 1024) <= 160 * 1024) ? 3 : SH::WGS;
  int total_groups = 0, total_extra = 0;
  bool sparse = false;
  for (int i = 0; i < count; ++i) {
    total_groups += (As[i].g.ntr + SH::NS - 1) / SH::NS;
    total_extra += long_row_workgroups(As[i]);
    sparse = sparse || As[i].nnz > 0;
  }
  size_t worst = 0;
  if (fused) {
    const int s = mfma_steps_per_split(total_groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, total_extra);
    const int nsplit = (nsteps + s - 1) / s;
    size_t total = (sparse ? up(((size_t)g0.n + 1) * 32) : 0) + (As[0].perm ? up((size_t)b * g0.n * 2) : 0);
    for (int i = 0; i < count; ++i)
      total += (As[i].nnz > 0 ? up(((size_t)(As[i].nnz / kSlotGrain) + 2) * 64) : 0) +
               up((size_t)nsplit * b * As[i].g.m * sizeof(float));
    worst = total;
  }
  for (int i = 0; i < count; ++i) {
    const DevMatrix& A = As[i];
    const int groups = (A.g.ntr + SH::NS - 1) / SH::NS;
    const int s = mfma_steps_per_split(groups, nsteps, wgs1 * kCUs, SH::WGS * kCUs, long_row_workgroups(A));
    const int nsplit = (nsteps + s - 1) / s;
    const size_t need = (A.nnz > 0 ? up(((size_t)A.g.n + 1) * 32) + up(((size_t)(A.nnz / kSlotGrain) + 2) * 64) : 0) +
                        (A.perm ? up((size_t)b * A.g.n * 2) : 0) + up((size_t)nsplit * b * A.g.m * sizeof(float));
    if (need > worst) worst = need;
  }
  return worst;
}

size_t mfma_workspace_bound(const DevMatrix* As, int count, int b, bool fused) {
  const Geometry& g = As[0].g;
#define SPQR_MFMA_CASE(W_, TR_, TC_, AX_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
    return mfma_scratch_bound<TR_, TC_>(As, count, b, fused);
  SPQR_MFMA_INSTANCES(SPQR_MFMA_CASE)
#undef SPQR_MFMA_CASE
  return 0;
}

hipError_t launch_prefill_scratch(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                                  const Workspace& ws) {
  const size_t need = prefill_workspace_bytes(A, b);
  if (ws.from_caller) {
    if (ws.p == nullptr || ws.bytes < need) return hipErrorNotSupported;
    return launch_prefill(A, X, b, Y, y_dtype, stream, ws.p);
  }
  // the dense copy is far too large for allocation nodes of a graph, and stream-ordered allocations wait on the host
  Scratch sc;
  if (scratch_get(&sc, need, current_device(), stream, false) != hipSuccess) return hipErrorNotSupported;
  const hipError_t e = launch_prefill(A, X, b, Y, y_dtype, stream, sc.p);
  const hipError_t ef = scratch_put(&sc, stream);
  return e == hipSuccess ? ef : e;
}

// ---- scratch for callers that cannot allocate ------------------------------------------------------------
// One array per device, resident from the moment the library's code is loaded on it until the process ends.
// In host code its name stands for the symbol, not for a device address: the address is asked per device
// (each GPU holds its own copy) and only that pointer is ever handed to kernels.  All calls on a device that
// use it share it: calls that overlap on one GPU (different streams) race.  Nothing in it has to start at
// zero: every word a batch call reads (the transposed batch with its zero line, the slots of the long rows,
// the partial results) is written earlier in the same call.
static __device__ __align__(256) uint8_t scratch[SPQR_STATIC_SCRATCH_BYTES];

hipError_t static_workspace(Workspace* ws) {
  static std::mutex lock;
  static uint8_t* ptr[kMaxDevices];          // the array's address on each device, nullptr = not asked yet
  const int dev = current_device();
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(lock);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    ptr[dev] = static_cast<uint8_t*>(p);
  }
  ws->from_caller = true;
  ws->p = ptr[dev];
  ws->bytes = SPQR_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}

// Tile shapes the matrix-core kernel is built for: the ones the vector kernel is tuned for.
bool mfma_has_instance(const Geometry& g) {
  const bool shape16 = g.tile_rows == 16 && g.tile_cols == 16;
  const bool shape8x32 = g.tile_rows == 8 && g.tile_cols == 32 && g.axis == 1;
  const bool shape32x8 = g.tile_rows == 32 && g.tile_cols == 8 && g.axis == 0;
  return g.layout == kBilevel && (g.w_bits == 3 || g.w_bits == 4) && (shape16 || shape8x32 || shape32x8);
}

hipError_t launch_mfma(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                       const Workspace& ws) {
  const Geometry& g = A.g;
#define SPQR_MFMA_CASE(W_, TR_, TC_, AX_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
    return launch_mfma_t<W_, TR_, TC_, AX_>(A, X, b, Y, y_dtype, stream, ws);
  SPQR_MFMA_INSTANCES(SPQR_MFMA_CASE)
#undef SPQR_MFMA_CASE
  return hipErrorNotSupported;
}

hipError_t launch_mfma_fused(const DevMatrix* As, int count, const uint16_t* X, int b, void* const* Ys, int y_dtype,
                             hipStream_t stream, const Workspace& ws) {
  const Geometry& g = As[0].g;
#define SPQR_MFMA_CASE(W_, TR_, TC_, AX_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
    return launch_mfma_fused_t<W_, TR_, TC_, AX_>(As, count, X, b, Ys, y_dtype, stream, ws);
  SPQR_MFMA_INSTANCES(SPQR_MFMA_CASE)
#undef SPQR_MFMA_CASE
  return hipErrorNotSupported;
}

}  // namespace spqr
