// Large batches (the prompt phase of Sec. 5, "Inference Time"): the weights are dequantised once per call into a
// dense binary16 copy in scratch, the outliers are added into it, and one tiled matrix-core kernel multiplies the
// whole batch with it (Sec. 4.2 describes the same order: 16-bit weights first, then the product).  The
// slices of 16 of the batch path read and dequantise the weights once per slice; here a weight is read once
// compressed, written once and read once per 128 vectors as binary16.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/spqr.h"
#include "spqr_kernels.h"
#include "spqr_tile.h"

namespace spqr {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Dense copy: Wd[m][ldw] binary16, ldw = n rounded up to 64, the columns behind n zero.
// One wavefront = one step of 64 tiles of a strip, one lane per tile (the loads of the GEMV); a lane turns
// its tile into binary16, w = s_hat * (q - z_hat) evaluated in binary32 and rounded once, and writes it row
// by row: consecutive lanes hold consecutive column blocks, so a row of the step is one contiguous run.
// ---------------------------------------------------------------------------
// LV: the statistic layout (1 bilevel, 2 integer zero-point, 3 binary16 statistics per group).
template <int W, int TR, int TC, int AXIS, int LV>
__global__ void __launch_bounds__(256)
dequant_tiles_f16_kernel(DevMatrix A, uint16_t* __restrict__ Wd, int ldw) {
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr int PPR = TC / 2, B2 = T::B2;
  constexpr float SCALE = (float)(1 << W);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int ntc = A.g.ntc, nsteps = (ntc + 63) >> 6;
  const int step = blockIdx.x * 4 + wave, strip = blockIdx.y;
  if (step >= nsteps) return;                // wave-uniform; the kernel has no barrier
  const int L = min(64, ntc - 64 * step);
  T t;
  load_tile<true>(t, A.packed + ((int64_t)strip * ntc + (int64_t)64 * step) * TILE_BYTES, L, min(lane, L - 1));
  const PairConsts kc = make_pair_consts<W>();
  const PairConsts k3 = make_pair_consts<3>();
  // w = fa * (1 + q/2^W) + fb with fa = 2^W * s_hat, fb = -s_hat * (2^W + z_hat), per group
  float fa[B2], fb[B2];
  if constexpr (LV == 3) {                   // dword g of the statistics: s_hat | z_hat << 16
#pragma unroll
    for (int g = 0; g < B2; ++g) {
      const float sh = h2f((uint16_t)(t.s[g] & 0xFFFF)), zh = h2f((uint16_t)(t.s[g] >> 16));
      fa[g] = SCALE * sh;
      fb[g] = -sh * (SCALE + zh);
    }
  } else {                                   // 3-bit codes, extracted as 1 + code/8; layout 2: z_hat = z_q (s_z = 1, z_z = 0)
    const uint32_t a2 = t.s[T::NC];
    const float s_s = h2f((uint16_t)(a2 & 0xFFFF)), z_s = h2f((uint16_t)(a2 >> 16));
    float s_z = 1.f, z_z = 0.f;
    if constexpr (LV == 1) {
      const uint32_t b2 = t.s[T::NC + 1];
      s_z = h2f((uint16_t)(b2 & 0xFFFF)); z_z = h2f((uint16_t)(b2 >> 16));
    }
    const float c1 = SCALE * 8.f * s_s, c2 = SCALE * (-s_s * z_s - 8.f * s_s);
    const float e1 = -8.f * s_z / SCALE, e2 = -(SCALE - s_z * z_z - 8.f * s_z) / SCALE;
#pragma unroll
    for (int p = 0; p < B2 / 2; ++p) {
      const half2_t sq = as_half2(pair_f16<3>(t.s, p, k3));
      const half2_t zq = as_half2(pair_f16<3>(t.s, B2 / 2 + p, k3));
      fa[2 * p] = fmaf((float)sq.x, c1, c2);
      fa[2 * p + 1] = fmaf((float)sq.y, c1, c2);
      fb[2 * p] = fa[2 * p] * fmaf((float)zq.x, e1, e2);
      fb[2 * p + 1] = fa[2 * p + 1] * fmaf((float)zq.y, e1, e2);
    }
  }
  if (lane >= L) return;                     // a lane behind the step's last tile held a copy of it
  uint16_t* out = Wd + ((int64_t)strip * TR) * ldw + ((int64_t)64 * step + lane) * TC;
#pragma unroll
  for (int r = 0; r < TR; ++r) {
    uint32_t o[PPR];
#pragma unroll
    for (int p = 0; p < PPR; ++p) {
      const half2_t q2 = as_half2(pair_f16<W>(t.c, r * PPR + p, kc));
      const int g0 = AXIS == 1 ? 2 * p : r, g1 = AXIS == 1 ? 2 * p + 1 : r;
      half2_t w;
      w.x = (_Float16)fmaf((float)q2.x, fa[g0], fb[g0]);
      w.y = (_Float16)fmaf((float)q2.y, fa[g1], fb[g1]);
      o[p] = __builtin_bit_cast(uint32_t, w);
    }
    u32x4* d = reinterpret_cast<u32x4*>(out + (int64_t)r * ldw);       // ldw and TC are multiples of 8: 16-byte aligned
#pragma unroll
    for (int k = 0; k < PPR / 4; ++k) {
      const u32x4 v = {o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]};
      d[k] = v;
    }
  }
}

// The zero columns [n, ldw) of every row (the matrix multiply reads whole blocks of 64 columns).
__global__ void __launch_bounds__(256) zero_pad_kernel(uint16_t* __restrict__ Wd, int m, int n, int ldw) {
  const int pad = ldw - n;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)m * pad) return;
  Wd[(i / pad) * ldw + n + (i % pad)] = 0;
}

// Wd[row][col] += val for every outlier (each position at most once: the sets the format allows have strictly
// increasing columns inside a row), one thread per entry; its row is found in the row pointers by bisection.
// A column index is clamped to n - 1, so that whatever an entry holds the write stays inside its row.
__global__ void __launch_bounds__(256) add_outliers_f16_kernel(DevMatrix A, uint16_t* __restrict__ Wd, int ldw) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= A.nnz) return;
  int lo = 0, hi = A.g.m;                    // row_ptr[lo] <= e < row_ptr[hi] for a valid prefix; lo stays below m anyway
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (A.row_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  const int col = min((int)A.col[e], A.g.n - 1);
  uint16_t* w = Wd + (int64_t)lo * ldw + col;
  *w = f2h_rne(h2f(*w) + h2f(A.val[e]));
}

// XP[v][j] = X[v][perm[j]]: the batch in the matrix's column order (act-order checkpoints).
__global__ void __launch_bounds__(256)
gather_x_kernel(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, uint16_t* __restrict__ XP, int n, int b) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  const int src = min(max(perm[j], 0), n - 1);
  for (int v = 0; v < b; ++v) XP[(int64_t)v * n + j] = X[(int64_t)v * n + src];
}

// ---------------------------------------------------------------------------
// Y[v][r] = sum_k X[v][k] * Wd[r][k] in binary32 on the matrix cores (v_mfma_f32_16x16x32_f16).
// A workgroup of 4 wavefronts owns 128 rows of Wd x BV vectors (BV = 128 or 64) and walks k in blocks of 64:
// both operands are K-contiguous, a block of each goes global -> registers -> LDS (row stride 144 bytes: the 16
// lanes of an operand read hit 16 different groups of 4 banks) one block ahead of the arithmetic, two LDS buffers, one
// barrier per block.  Wavefront (wr, wv) owns 64 rows x BV/2 vectors = 4 x BV/32 accumulator blocks: the MFMA's
// A operand is 16 rows of Wd (lane l: row l%16, k = 8(l/16).. +8), B 16 vectors of X, D[row 4(l/16)+i][vector l%16].
// Rows behind m and vectors behind b are clamped on load and dropped at the store; columns behind n are zero
// in Wd (ldw is a multiple of 64) and read as zero from X.
// ---------------------------------------------------------------------------
constexpr int kGemmBK = 64, kGemmLds = 72;     // k per block, LDS row stride in halves

// BR rows x BV vectors per workgroup (128 or 64 each); its four wavefronts are 2 x 2, each BR/2 rows x BV/2 vectors.
template <int BR, int BV>
__global__ void __launch_bounds__(256, 2)
gemm_f16_tn_kernel(const uint16_t* __restrict__ X, int b, int n, const uint16_t* __restrict__ Wd, int ldw, int m,
                   void* Y, int y_dtype, int blocks_per_split) {
  constexpr int BK = kGemmBK, LD = kGemmLds;
  constexpr int NRB = BR / 32;               // row blocks of 16 per wavefront
  constexpr int NVB = BV / 32;               // vector blocks of 16 per wavefront
  constexpr int WCH = BR * (BK / 8) / 256;   // 16-byte chunks per thread and block of k: Wd
  constexpr int XCH = BV * (BK / 8) / 256;   // ... X
  extern __shared__ __align__(16) uint8_t smem[];            // 2 buffers x (BR + BV) rows x LD halves
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);          // As[buf][BR * LD]
  uint16_t* Bs = As + 2 * BR * LD;                           // Bs[buf][BV * LD]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave & 1, wv = wave >> 1;
  const int i16 = lane & 15, g4 = lane >> 4;
  const int row0 = blockIdx.x * BR, vec0 = blockIdx.y * BV;
  // blocks of k of this workgroup: split blockIdx.z of gridDim.z (never empty: the host sizes the splits); with
  // several splits Y is the binary32 partial result [split][b][m]
  const int kt_lo = blockIdx.z * blocks_per_split, kt_hi = min(ldw / BK, kt_lo + blocks_per_split);
  if (gridDim.z > 1) Y = reinterpret_cast<float*>(Y) + (int64_t)blockIdx.z * b * m;

  // chunk c of a block: row c / 8 of the tile, k = 8 * (c % 8): 8 consecutive threads read 128 contiguous bytes
  const uint16_t* wsrc[WCH];
  const uint16_t* xsrc[XCH];
  int wdst[WCH], xdst[XCH], xk[XCH];
#pragma unroll
  for (int i = 0; i < WCH; ++i) {
    const int c = tid + 256 * i, r = c >> 3, kc = c & 7;
    wsrc[i] = Wd + (int64_t)min(row0 + r, m - 1) * ldw + 8 * kc;
    wdst[i] = r * LD + 8 * kc;
  }
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    const int c = tid + 256 * i, r = c >> 3, kc = c & 7;
    xsrc[i] = X + (int64_t)min(vec0 + r, b - 1) * n;
    xk[i] = 8 * kc;
    xdst[i] = r * LD + 8 * kc;
  }
  u32x4 wreg[WCH], xreg[XCH];
  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < WCH; ++i) wreg[i] = *reinterpret_cast<const u32x4*>(wsrc[i] + k0);
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int k = k0 + xk[i];              // n is a multiple of 8: a chunk is inside [0, n) or behind it
      const u32x4 v = *reinterpret_cast<const u32x4*>(xsrc[i] + min(k, n - 8));
      const u32x4 z = {0u, 0u, 0u, 0u};
      xreg[i] = k < n ? v : z;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < WCH; ++i) *reinterpret_cast<u32x4*>(As + buf * BR * LD + wdst[i]) = wreg[i];
#pragma unroll
    for (int i = 0; i < XCH; ++i) *reinterpret_cast<u32x4*>(Bs + buf * BV * LD + xdst[i]) = xreg[i];
  };

  float4_t D[NRB][NVB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) D[rb][vb] = float4_t{0.f, 0.f, 0.f, 0.f};

  fetch(kt_lo);
  stash(0);
  __syncthreads();
  for (int kt = kt_lo; kt < kt_hi; ++kt) {   // workgroup-uniform
    const int buf = (kt - kt_lo) & 1;
    if (kt + 1 < kt_hi) fetch(kt + 1);
    const uint16_t* a0 = As + buf * BR * LD + (wr * (BR / 2) + i16) * LD + 8 * g4;
    const uint16_t* b0 = Bs + buf * BV * LD + (wv * (BV / 2) + i16) * LD + 8 * g4;
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      half8_t af[NRB], bf[NVB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) af[rb] = *reinterpret_cast<const half8_t*>(a0 + rb * 16 * LD + 32 * ks);
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) bf[vb] = *reinterpret_cast<const half8_t*>(b0 + vb * 16 * LD + 32 * ks);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb)
          D[rb][vb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[rb], bf[vb], D[rb][vb], 0, 0, 0);
    }
    if (kt + 1 < kt_hi) stash(buf ^ 1);      // the other buffer: everyone left it at the previous barrier
    __syncthreads();
  }

  // D[rb][vb]: rows row0 + (BR/2) wr + 16 rb + 4 g4 .. +3, vector vec0 + (BV/2) wv + 16 vb + i16
#pragma unroll
  for (int vb = 0; vb < NVB; ++vb) {
    const int v = vec0 + wv * (BV / 2) + vb * 16 + i16;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const int r = row0 + wr * (BR / 2) + rb * 16 + 4 * g4;
      if (v < b && r < m) {                  // m is a multiple of 8: four rows are inside or outside together
        const int64_t at = (int64_t)v * m + r;
        if (y_dtype == SPQR_F32) {
          *reinterpret_cast<float4_t*>(reinterpret_cast<float*>(Y) + at) = D[rb][vb];
        } else {
          typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
          const u32x2 h = {(uint32_t)f2h_rne(D[rb][vb].x) | ((uint32_t)f2h_rne(D[rb][vb].y) << 16),
                           (uint32_t)f2h_rne(D[rb][vb].z) | ((uint32_t)f2h_rne(D[rb][vb].w) << 16)};
          *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(Y) + at) = h;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
static int padded_columns(int n) { return (n + kGemmBK - 1) / kGemmBK * kGemmBK; }

// Tiles of 256 codes in every statistic layout, and the 8 x 64 tiles of the bilevel layout (3-bit, group_axis 1).
bool prefill_has_instance(const Geometry& g) {
  if ((g.w_bits != 3 && g.w_bits != 4) || g.m % 8 != 0 || g.n % 8 != 0) return false;
  const bool shape16 = g.tile_rows == 16 && g.tile_cols == 16;
  const bool shape8x32 = g.tile_rows == 8 && g.tile_cols == 32 && g.axis == 1;
  const bool shape32x8 = g.tile_rows == 32 && g.tile_cols == 8 && g.axis == 0;
  const bool wide = g.tile_rows == 8 && g.tile_cols == 64 && g.axis == 1 && g.w_bits == 3 && g.layout == kBilevel;
  return shape16 || shape8x32 || shape32x8 || wide;
}

// Whether a batch of b vectors goes through the dense copy: the copy costs one pass over the compressed weights,
// one write of 2 bytes per weight and a scattered read-modify-write per outlier, whatever the batch; the slices of
// 16 cost a pass over the compressed weights each.  Measured on the 7B to 65B shapes (batches of 32 to 256, both
// paths forced): the copy wins from 48 vectors on layers of up to 120 M weights (4096^2 at 48: 34 against 56 us;
// 17920x6656: 144 against 156), from 64 on 8192^2 with 2 % outliers and from 96 on the layers of 180 M weights
// (22016x8192 at 64 / 96: 326 / 355 against 289 / 433); at 256 vectors it is 3.4 to 6.8 times faster.
bool prefill_wanted(const DevMatrix& A, int b) {
  const int forced = option(SPQR_OPT_BATCH_PATH);
  if (forced == SPQR_BATCH_PATH_DENSE) return true;
  if (forced != SPQR_BATCH_PATH_AUTO) return false;
  // formats without slices of 16 (the other statistic layouts, 8 x 64 tiles) pay a pass of the batch-1 kernel per
  // vector instead: the copy pays off from about a dozen vectors on
  if (!mfma_has_instance(A.g)) return b >= 12;
  const double from = (double)A.g.m * (double)A.g.n / 2.5e6 + (double)A.nnz / 1.5e5;
  return b >= 48 && (double)b >= from;
}

// Scratch of one call: the dense copy, the batch in column order if there is a permutation, the partial results if
// the multiply splits k (up to 8 splits: bounded without looking at the options).
size_t prefill_workspace_bytes(const DevMatrix& A, int b) {
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  return up((size_t)A.g.m * padded_columns(A.g.n) * 2) + (A.perm != nullptr ? up((size_t)b * A.g.n * 2) : 0) +
         up((size_t)8 * b * A.g.m * sizeof(float));
}

template <int W, int TR, int TC, int AXIS, int LV>
static hipError_t launch_dequant_tiles(const DevMatrix& A, uint16_t* Wd, int ldw, hipStream_t stream) {
  using T = TileRegs<W, TR, TC, AXIS, LV>;
  if (A.g.kw != T::KW || A.g.sd != T::SD || A.g.layout != LV) return hipErrorInvalidValue;   // the tile the kernel loads
  const int nsteps = (A.g.ntc + 63) / 64;
  hipLaunchKernelGGL((dequant_tiles_f16_kernel<W, TR, TC, AXIS, LV>), dim3((nsteps + 3) / 4, A.g.ntr), dim3(256), 0, stream,
                     A, Wd, ldw);
  return hipGetLastError();
}

// Y[i] = sum over the splits of P[split][i], in the order of the splits, rounded once to the output type.
__global__ void __launch_bounds__(256)
sum_splits_kernel(const float* __restrict__ P, int splits, int64_t count, void* __restrict__ Y, int y_dtype) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s = P[i];
  for (int k = 1; k < splits; ++k) s += P[(int64_t)k * count + i];
  if (y_dtype == SPQR_F32) reinterpret_cast<float*>(Y)[i] = s;
  else reinterpret_cast<uint16_t*>(Y)[i] = f2h_rne(s);
}

template <int BR, int BV>
static hipError_t launch_dense_gemm_t(const uint16_t* X, int b, int n, const uint16_t* Wd, int ldw, int m, void* Y,
                                      int y_dtype, int splits, int blocks_per_split, hipStream_t stream) {
  constexpr int lds = 2 * (BR + BV) * kGemmLds * 2;
  static PerDevice ready;                    // more than 64 KB of LDS per workgroup is an opt-in per kernel and device
  const int dev = current_device();
  if (!ready.get(dev)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_f16_tn_kernel<BR, BV>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    ready.set(dev, 1);
  }
  hipLaunchKernelGGL((gemm_f16_tn_kernel<BR, BV>), dim3((m + BR - 1) / BR, (b + BV - 1) / BV, splits), dim3(256), lds,
                     stream, X, b, n, Wd, ldw, m, Y, splits > 1 ? SPQR_F32 : y_dtype, blocks_per_split);
  return hipGetLastError();
}

// Tile and splits of the multiply.  128 rows x 128 vectors per workgroup (64 vectors for batches up to 64, 64 rows
// for matrices of up to 64 rows); where that leaves CUs without a workgroup (few rows, a small batch), the blocks of
// k are split over up to 8 workgroups of at least 8 blocks each, which write binary32 partial results that a second
// kernel adds in a fixed order.  Measured on the 7B to 65B shapes at 64 to 256 vectors: 128 rows with splits beat
// 64 rows without (8192x22016 at 128 vectors: 373 against 537 us for the whole call, 6656x17920 at 256: 265 against
// 327), 128 x 128 without splits beats 64 x 128 by 20 % where both fill the chip.  SPQR_OPT_DENSE_ROWS pins the
// rows for tuning runs.
struct DensePlan { int br, bv, splits, blocks_per_split; };
static DensePlan plan_dense_gemm(int b, int m, int ldw) {
  const int forced = option(SPQR_OPT_DENSE_ROWS);
  DensePlan p;
  p.br = (forced == 64 || forced == 128) ? forced : (m <= 64 ? 64 : 128);
  p.bv = b <= 64 ? 64 : 128;
  const int nk = ldw / kGemmBK;
  p.splits = 1; p.blocks_per_split = nk;
  const int64_t wgs = (int64_t)((m + p.br - 1) / p.br) * ((b + p.bv - 1) / p.bv);
  if (wgs < kCUs) {
    int s = (int)((2 * kCUs) / wgs);
    if (s > 8) s = 8;
    if (s > nk / 8) s = nk / 8;
    if (s > 1) {
      p.blocks_per_split = (nk + s - 1) / s;
      p.splits = (nk + p.blocks_per_split - 1) / p.blocks_per_split;   // no empty split
    }
  }
  return p;
}

// `partial`: plan.splits * b * m floats if the plan splits k, else unused.
static hipError_t launch_dense_gemm(const uint16_t* X, int b, int n, const uint16_t* Wd, int ldw, int m, void* Y,
                                    int y_dtype, float* partial, hipStream_t stream) {
  const DensePlan p = plan_dense_gemm(b, m, ldw);
  void* out = p.splits > 1 ? static_cast<void*>(partial) : Y;
  hipError_t e;
  if (p.bv == 128) e = p.br == 128 ? launch_dense_gemm_t<128, 128>(X, b, n, Wd, ldw, m, out, y_dtype, p.splits, p.blocks_per_split, stream)
                                   : launch_dense_gemm_t<64, 128>(X, b, n, Wd, ldw, m, out, y_dtype, p.splits, p.blocks_per_split, stream);
  else e = p.br == 128 ? launch_dense_gemm_t<128, 64>(X, b, n, Wd, ldw, m, out, y_dtype, p.splits, p.blocks_per_split, stream)
                       : launch_dense_gemm_t<64, 64>(X, b, n, Wd, ldw, m, out, y_dtype, p.splits, p.blocks_per_split, stream);
  if (e != hipSuccess || p.splits == 1) return e;
  const int64_t count = (int64_t)b * m;
  hipLaunchKernelGGL(sum_splits_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, partial, p.splits, count,
                     Y, y_dtype);
  return hipGetLastError();
}

// Y[b][m] = X[b][n] . W_hat^T for a large batch.  `scratch`: prefill_workspace_bytes(A, b) bytes, 256-byte aligned.
hipError_t launch_prefill(const DevMatrix& A, const uint16_t* X, int b, void* Y, int y_dtype, hipStream_t stream,
                          uint8_t* scratch) {
  const Geometry& g = A.g;
  if (!prefill_has_instance(g) || scratch == nullptr || b < 1) return hipErrorInvalidValue;
  // the output is written in groups of four rows: 16 bytes of binary32, 8 of binary16
  if (reinterpret_cast<uintptr_t>(Y) % (y_dtype == SPQR_F32 ? 16 : 8) != 0) return hipErrorInvalidValue;
  const int ldw = padded_columns(g.n);
  uint16_t* Wd = reinterpret_cast<uint16_t*>(scratch);
  const size_t wd_bytes = ((size_t)g.m * ldw * 2 + 255) & ~(size_t)255;
  const size_t xp_bytes = A.perm != nullptr ? ((size_t)b * g.n * 2 + 255) & ~(size_t)255 : 0;
  uint16_t* XP = A.perm != nullptr ? reinterpret_cast<uint16_t*>(scratch + wd_bytes) : nullptr;
  float* partial = reinterpret_cast<float*>(scratch + wd_bytes + xp_bytes);
  hipError_t e = hipErrorInvalidValue;
#define SPQR_CASE(W_, TR_, TC_, AX_, LV_) \
  if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_ && g.layout == LV_) \
    e = launch_dequant_tiles<W_, TR_, TC_, AX_, LV_>(A, Wd, ldw, stream);
#define SPQR_SHAPES(LV_) \
  SPQR_CASE(3, 16, 16, 1, LV_) SPQR_CASE(4, 16, 16, 1, LV_) SPQR_CASE(3, 8, 32, 1, LV_) SPQR_CASE(4, 8, 32, 1, LV_) \
  SPQR_CASE(3, 16, 16, 0, LV_) SPQR_CASE(4, 16, 16, 0, LV_) SPQR_CASE(3, 32, 8, 0, LV_) SPQR_CASE(4, 32, 8, 0, LV_)
  SPQR_SHAPES(1) SPQR_SHAPES(2) SPQR_SHAPES(3) SPQR_CASE(3, 8, 64, 1, 1)
#undef SPQR_SHAPES
#undef SPQR_CASE
  if (e != hipSuccess) return e;
  if (ldw > g.n) {
    const int64_t cells = (int64_t)g.m * (ldw - g.n);
    hipLaunchKernelGGL(zero_pad_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, stream, Wd, g.m, g.n, ldw);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (A.nnz > 0) {
    hipLaunchKernelGGL(add_outliers_f16_kernel, dim3((unsigned)((A.nnz + 255) / 256)), dim3(256), 0, stream, A, Wd, ldw);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const uint16_t* Xin = X;
  if (XP != nullptr) {
    hipLaunchKernelGGL(gather_x_kernel, dim3((g.n + 255) / 256), dim3(256), 0, stream, X, A.perm, XP, g.n, b);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    Xin = XP;
  }
  return launch_dense_gemm(Xin, b, g.n, Wd, ldw, g.m, Y, y_dtype, partial, stream);
}

}  // namespace spqr
