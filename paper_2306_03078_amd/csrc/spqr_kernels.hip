// HIP kernels for gfx950: fused SpQR decode + matvec, debug decode, validation.
//
// Hot path (Sec. 4.2 "Inference with SpQR", re-designed for CDNA4):
//   one workgroup owns one strip of tile_rows output rows; its wavefronts split
//   the input dimension in steps of 64 tiles; one lane owns one whole tile per
//   step, so every load instruction of a wavefront reads one contiguous run of
//   the packed buffer (16 bytes per lane) and a tile's statistics are decoded
//   once and reused by all of its rows.  x is staged once per workgroup in LDS
//   (it also serves the outlier gather).  Codes are turned into binary16 values
//   1 + q/2^b by one shift and one and-or per pair and multiplied with
//   v_dot2_f32_f16 (fp32 accumulation); the offset "1 +" is removed per tile.
//   The strip's outliers (a contiguous CSR range) are handled by the same
//   workgroup, so y is written once, without atomics, in a fixed order.
#include <hip/hip_runtime.h>

#include "../../include/spqr.h"
#include "spqr_device.h"
#include "spqr_kernels.h"

namespace spqr {

// ---------------------------------------------------------------------------
// Pair extraction for 256-code tiles held in registers.
// Returns the bit pattern of two binary16 numbers (1 + q_lo/2^W, 1 + q_hi/2^W).
// ---------------------------------------------------------------------------
template <int W>
__device__ __forceinline__ uint32_t pair_f16(const uint32_t* c, int q) {
  if constexpr (W == 4) {
    const uint32_t d = c[q >> 2];
    const int o = 4 * (q & 3);                       // code offset inside each half-word
    const uint32_t t = o < 6 ? (d << (6 - o)) : (d >> (o - 6));
    return (t & 0x03C003C0u) | 0x3C003C00u;          // mantissa bits 9..6
  } else {
    const int t3 = q >> 4, e = q & 15;
    if (e < 15) {
      const uint32_t d = c[3 * t3 + e / 5];
      const int o = 3 * (e % 5);
      const uint32_t t = o < 7 ? (d << (7 - o)) : (d >> (o - 7));
      return (t & 0x03800380u) | 0x3C003C00u;        // mantissa bits 9..7
    } else {
      const uint32_t d0 = c[3 * t3], d1 = c[3 * t3 + 1], d2 = c[3 * t3 + 2];
      uint32_t t = ((d0 >> 8) & 0x00800080u) | 0x3C003C00u;
      t |= (d1 >> 7) & 0x01000100u;
      t |= (d2 >> 6) & 0x02000200u;
      return t;
    }
  }
}

// 3-bit statistic code number idx from the statistic dwords of a tile.
__device__ __forceinline__ uint32_t stat3(const uint32_t* s, int idx) {
  const int q = idx >> 1, hi = (idx & 1) * 16;
  const int t3 = q >> 4, e = q & 15;
  if (e < 15) return (s[3 * t3 + e / 5] >> (3 * (e % 5) + hi)) & 7u;
  return ((s[3 * t3] >> (15 + hi)) & 1u) | (((s[3 * t3 + 1] >> (15 + hi)) & 1u) << 1)
       | (((s[3 * t3 + 2] >> (15 + hi)) & 1u) << 2);
}

// ---------------------------------------------------------------------------
// Fused GEMV for tiles of 256 codes.
//   W     code width (3, 4)
//   TR,TC tile rows / columns, TR*TC == 256
//   AXIS  0: groups are tile rows (beta2 = TR), 1: groups are tile columns (beta2 = TC)
// Grid: one workgroup per strip of TR rows; blockDim.x = 64 * (waves per workgroup).
// Dynamic LDS: n binary16 values of x (rounded up to 16 bytes).
// ---------------------------------------------------------------------------
template <int W, int TR, int TC, int AXIS>
struct TileRegs {
  static constexpr int KW = 256 * W / 128;
  static constexpr int B2 = AXIS == 0 ? TR : TC;
  static constexpr int SD = 3 * B2 / 16 + 2;
  static constexpr int SWF = SD / 4, SR = SD % 4;
  uint32_t c[4 * KW];
  uint32_t s[SD];
};

template <int W, int TR, int TC, int AXIS>
__device__ __forceinline__ void load_tile(TileRegs<W, TR, TC, AXIS>& t, const uint8_t* blk,
                                          int L, int lane) {
  using T = TileRegs<W, TR, TC, AXIS>;
#pragma unroll
  for (int k = 0; k < T::KW; ++k) {
    u32x4 v = *reinterpret_cast<const u32x4*>(blk + ((int64_t)k * L + lane) * 16);
    t.c[4 * k] = v.x; t.c[4 * k + 1] = v.y; t.c[4 * k + 2] = v.z; t.c[4 * k + 3] = v.w;
  }
  const uint8_t* sb = blk + (int64_t)16 * T::KW * L;
#pragma unroll
  for (int k = 0; k < T::SWF; ++k) {
    u32x4 v = *reinterpret_cast<const u32x4*>(sb + ((int64_t)k * L + lane) * 16);
    t.s[4 * k] = v.x; t.s[4 * k + 1] = v.y; t.s[4 * k + 2] = v.z; t.s[4 * k + 3] = v.w;
  }
  const uint8_t* rb = sb + (int64_t)16 * T::SWF * L;
#pragma unroll
  for (int k = 0; k < T::SR; ++k)
    t.s[4 * T::SWF + k] = *reinterpret_cast<const uint32_t*>(rb + ((int64_t)k * L + lane) * 4);
}

// One tile's contribution.  acc[r] accumulates, per output row r of the strip:
//   AXIS 1: sum_j (1 + q_rj/2^W) * u_j   with u_j = fp16(s_hat_j * x_j);  csum
//           accumulates sum_j (2^W + z_hat_j) * u_j, so y_r = 2^W*acc[r] - csum.
//   AXIS 0: s_hat_r * (2^W * sum_j (1 + q_rj/2^W) x_j - (2^W + z_hat_r) * sum_j x_j).
template <int W, int TR, int TC, int AXIS>
__device__ __forceinline__ void tile_fma(const TileRegs<W, TR, TC, AXIS>& t,
                                         const uint32_t* xpair /* TC/2 dwords in LDS */,
                                         float (&acc)[TR], float& csum) {
  using T = TileRegs<W, TR, TC, AXIS>;
  constexpr int PPR = TC / 2;
  constexpr float SCALE = (float)(1 << W);
  const uint32_t a = t.s[T::SD - 2], b = t.s[T::SD - 1];
  const float s_s = h2f((uint16_t)(a & 0xFFFF)), z_s = h2f((uint16_t)(a >> 16));
  const float s_z = h2f((uint16_t)(b & 0xFFFF)), z_z = h2f((uint16_t)(b >> 16));
  const float s_off = -s_s * z_s;             // s_hat = s_s*s_q + s_off
  const float z_off = -s_z * z_z + SCALE;     // 2^W + z_hat = s_z*z_q + z_off

  uint32_t xp[PPR];
#pragma unroll
  for (int p = 0; p < PPR; p += 4) {
    if constexpr (PPR % 4 == 0) {
      u32x4 v = *reinterpret_cast<const u32x4*>(xpair + p);
      xp[p] = v.x; xp[p + 1] = v.y; xp[p + 2] = v.z; xp[p + 3] = v.w;
    }
  }

  if constexpr (AXIS == 1) {
    uint32_t up[PPR];
#pragma unroll
    for (int p = 0; p < PPR; ++p) {
      const half2_t xv = as_half2(xp[p]);
      const float s0 = fmaf(s_s, (float)stat3(t.s, 2 * p), s_off);
      const float s1 = fmaf(s_s, (float)stat3(t.s, 2 * p + 1), s_off);
      const float z0 = fmaf(s_z, (float)stat3(t.s, T::B2 + 2 * p), z_off);
      const float z1 = fmaf(s_z, (float)stat3(t.s, T::B2 + 2 * p + 1), z_off);
      half2_t u;
      u.x = (_Float16)(s0 * (float)xv.x);
      u.y = (_Float16)(s1 * (float)xv.y);
      up[p] = __builtin_bit_cast(uint32_t, u);
      csum = fmaf(z0, (float)u.x, csum);
      csum = fmaf(z1, (float)u.y, csum);
    }
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      float d = acc[r];
#pragma unroll
      for (int p = 0; p < PPR; ++p)
        d = __builtin_amdgcn_fdot2(as_half2(pair_f16<W>(t.c, r * PPR + p)), as_half2(up[p]), d, false);
      acc[r] = d;
    }
  } else {
    float X = 0.f;
#pragma unroll
    for (int p = 0; p < PPR; ++p)
      X = __builtin_amdgcn_fdot2(as_half2(xp[p]), as_half2(0x3C003C00u), X, false);
#pragma unroll
    for (int r = 0; r < TR; ++r) {
      float d = 0.f;
#pragma unroll
      for (int p = 0; p < PPR; ++p)
        d = __builtin_amdgcn_fdot2(as_half2(pair_f16<W>(t.c, r * PPR + p)), as_half2(xp[p]), d, false);
      const float sh = fmaf(s_s, (float)stat3(t.s, r), s_off);
      const float zo = fmaf(s_z, (float)stat3(t.s, T::B2 + r), z_off);
      acc[r] = fmaf(sh, fmaf(SCALE, d, -zo * X), acc[r]);
    }
  }
}

// A 4-bit tile needs 32 code registers (twice, with the prefetch of the next
// step), which does not fit the 128 registers a 1024-thread workgroup allows.
template <int W> struct WavesPerGroup { static constexpr int MAX = W == 3 ? 16 : 8; };

template <int W, int TR, int TC, int AXIS>
__global__ void __launch_bounds__(64 * WavesPerGroup<W>::MAX)
gemv_tile256_kernel(DevMatrix A, const uint16_t* __restrict__ x, void* __restrict__ y, int y_dtype) {
  using T = TileRegs<W, TR, TC, AXIS>;
  static_assert(TR * TC == 256, "tile must hold 256 codes");
  static_assert((TC / 2) % 4 == 0, "x pairs are read as 16-byte LDS words");
  constexpr int TILE_BYTES = 16 * T::KW + 4 * T::SD;
  constexpr int MAX_WAVES = 16;
  constexpr int LIGHT_MAX = 512;             // rows with more outliers use the whole workgroup

  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);
  __shared__ float red[MAX_WAVES][TR];
  __shared__ float osum[TR];
  __shared__ float hred[MAX_WAVES];
  __shared__ int rp[TR + 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int strip = blockIdx.x;
  const int n = A.g.n, ntc = A.g.ntc;
  const int nsteps = (ntc + 63) >> 6;
  const uint8_t* strip_base = A.packed + (int64_t)strip * ntc * TILE_BYTES;

  // Issue the first tile load before anything else so it overlaps the staging.
  T cur;
  int step = wave;
  bool have = false;
  if (step < nsteps) {
    const int L = min(64, ntc - 64 * step);
    if (lane < L) { load_tile(cur, strip_base + (int64_t)64 * step * TILE_BYTES, L, lane); have = true; }
  }

  if (tid <= TR) rp[tid] = A.row_ptr[strip * TR + tid];

  // Stage x (binary16) in LDS, optionally through the input permutation.
  if (A.perm == nullptr) {
    const int nvec = n >> 3;                 // 16-byte chunks; n is a multiple of the tile width (even)
    const u32x4* src = reinterpret_cast<const u32x4*>(x);
    u32x4* dst = reinterpret_cast<u32x4*>(xs);
    for (int i = tid; i < nvec; i += nthreads) dst[i] = src[i];
    for (int j = (nvec << 3) + tid; j < n; j += nthreads) xs[j] = x[j];
  } else {
    for (int j = tid; j < n; j += nthreads) xs[j] = x[A.perm[j]];
  }
  __syncthreads();

  float acc[TR];
#pragma unroll
  for (int r = 0; r < TR; ++r) acc[r] = 0.f;
  float csum = 0.f;

  const uint32_t* xs32 = reinterpret_cast<const uint32_t*>(xs);
  while (step < nsteps) {                    // wave-uniform loop
    const int nstep = step + nwaves;
    T nxt;
    bool have_next = false;
    if (nstep < nsteps) {
      const int L = min(64, ntc - 64 * nstep);
      if (lane < L) { load_tile(nxt, strip_base + (int64_t)64 * nstep * TILE_BYTES, L, lane); have_next = true; }
    }
    if (have) tile_fma<W, TR, TC, AXIS>(cur, xs32 + (64 * step + lane) * (TC / 2), acc, csum);
    cur = nxt; have = have_next; step = nstep;
  }

  // ---- outliers of this strip: CSR entries [rp[0], rp[TR]) ------------------
  {
    const int l16 = tid & 15, g16 = tid >> 4, ngroups = nthreads >> 4;
    for (int r = g16; r < TR; r += ngroups) {
      const int a = rp[r], b = rp[r + 1];
      float p = 0.f;
      if (b - a <= LIGHT_MAX)
        for (int e = a + l16; e < b; e += 16) p = fmaf(h2f(A.val[e]), h2f(xs[A.col[e]]), p);
      p = row16_allreduce(p, lane);
      if (l16 == 0) osum[r] = p;
    }
    __syncthreads();
    for (int r = 0; r < TR; ++r) {           // workgroup-uniform
      const int a = rp[r], b = rp[r + 1];
      if (b - a > LIGHT_MAX) {
        float p = 0.f;
        for (int e = a + tid; e < b; e += nthreads) p = fmaf(h2f(A.val[e]), h2f(xs[A.col[e]]), p);
        p = wave_allreduce(p, lane);
        if (lane == 0) hred[wave] = p;
        __syncthreads();
        if (tid == 0) { float s = 0.f; for (int w = 0; w < nwaves; ++w) s += hred[w]; osum[r] = s; }
        __syncthreads();
      }
    }
  }

  // ---- dense partials: lanes -> rows, then waves -> workgroup ---------------
  if constexpr (AXIS == 1) {
#pragma unroll
    for (int r = 0; r < TR; ++r) acc[r] = fmaf((float)(1 << W), acc[r], -csum);
  }
  int row;
  const float rsum = wave_reduce_rows<TR>(acc, lane, &row);
  if ((lane & ((64 / TR) - 1)) == 0) red[wave][row] = rsum;
  __syncthreads();
  if (tid < TR) {
    float s = 0.f;
    for (int w = 0; w < nwaves; ++w) s += red[w][tid];
    s += osum[tid];
    const int64_t i = (int64_t)strip * TR + tid;
    if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
    else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
  }
}

// ---------------------------------------------------------------------------
// Generic fallback product: any supported geometry, one wavefront per output
// row, element-wise canonical decode.  Slow; used when no tuned kernel matches.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gemv_generic_kernel(DevMatrix A, const uint16_t* __restrict__ x, void* __restrict__ y, int y_dtype) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= A.g.m) return;                    // whole wavefront leaves together
  float s = 0.f;
  for (int j = lane; j < A.g.n; j += 64) {
    const float xv = h2f(x[A.perm ? A.perm[j] : j]);
    s = fmaf(dense_value(A.g, A.packed, i, j), xv, s);
  }
  for (int e = A.row_ptr[i] + lane; e < A.row_ptr[i + 1]; e += 64) {
    const int j = A.col[e];
    s = fmaf(h2f(A.val[e]), h2f(x[A.perm ? A.perm[j] : j]), s);
  }
  s = wave_allreduce(s, lane);
  if (lane == 0) {
    if (y_dtype == SPQR_F32) reinterpret_cast<float*>(y)[i] = s;
    else reinterpret_cast<uint16_t*>(y)[i] = f2h_rne(s);
  }
}

// ---------------------------------------------------------------------------
// Debug decode kernels.
// ---------------------------------------------------------------------------
__global__ void codes_u8_kernel(DevMatrix A, uint8_t* out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)A.g.m * A.g.n) return;
  const int i = (int)(idx / A.g.n), j = (int)(idx % A.g.n);
  out[idx] = (uint8_t)tile_code(A.g, A.packed, i / A.g.tile_rows, j / A.g.tile_cols,
                                i % A.g.tile_rows, j % A.g.tile_cols);
}

__global__ void stats_f32_kernel(DevMatrix A, float* out, int want_zero) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t grows = A.g.axis == 0 ? A.g.m : A.g.m / A.g.beta1;
  const int64_t gcols = A.g.axis == 0 ? A.g.n / A.g.beta1 : A.g.n;
  if (idx >= grows * gcols) return;
  const int gr = (int)(idx / gcols), gc = (int)(idx % gcols);
  int tr, tc, gi;
  if (A.g.axis == 0) { tr = gr / A.g.beta2; gi = gr % A.g.beta2; tc = gc; }
  else               { tr = gr; tc = gc / A.g.beta2; gi = gc % A.g.beta2; }
  float s_hat, z_hat;
  tile_group_stats(A.g, A.packed, tr, tc, gi, &s_hat, &z_hat);
  out[idx] = want_zero ? z_hat : s_hat;
}

template <typename OutT>
__device__ __forceinline__ void store_dense(OutT* out, int64_t idx, float v);
template <> __device__ __forceinline__ void store_dense<float>(float* out, int64_t idx, float v) { out[idx] = v; }
template <> __device__ __forceinline__ void store_dense<uint16_t>(uint16_t* out, int64_t idx, float v) { out[idx] = f2h_rne(v); }

template <typename OutT>
__global__ void dense_kernel(DevMatrix A, OutT* out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)A.g.m * A.g.n) return;
  store_dense<OutT>(out, idx, dense_value(A.g, A.packed, (int)(idx / A.g.n), (int)(idx % A.g.n)));
}

// Row of CSR entry e: largest i with row_ptr[i] <= e (row_ptr validated or trusted).
__device__ inline int csr_row_of(const int32_t* row_ptr, int m, int64_t e) {
  int lo = 0, hi = m;                        // invariant: row_ptr[lo] <= e < row_ptr[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (row_ptr[mid] <= e) lo = mid; else hi = mid;
  }
  return lo;
}

// Re-evaluates the positions that carry an outlier: dense value + outlier value,
// rounded once to the output type.
template <typename OutT>
__global__ void dense_outlier_kernel(DevMatrix A, OutT* out) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= A.nnz) return;
  const int i = csr_row_of(A.row_ptr, A.g.m, e);
  const int j = A.col[e];
  const float v = __fadd_rn(dense_value(A.g, A.packed, i, j), h2f(A.val[e]));
  store_dense<OutT>(out, (int64_t)i * A.g.n + j, v);
}

// ---------------------------------------------------------------------------
// Validation kernels.  *flag receives the first error class seen (any of them).
// ---------------------------------------------------------------------------
__global__ void fill_int_kernel(int* p, int v) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = v; }

__global__ void check_rowptr_kernel(DevMatrix A, int* flag) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i > A.g.m) return;
  const int64_t v = A.row_ptr[i];
  bool bad = v < 0 || v > A.nnz;
  if (i == 0 && v != 0) bad = true;
  if (i == A.g.m && v != A.nnz) bad = true;
  if (i < A.g.m && (int64_t)A.row_ptr[i + 1] < v) bad = true;
  if (i < A.g.m && (int64_t)A.row_ptr[i + 1] - v > A.g.n) bad = true;
  if (bad) atomicMin(flag, SPQR_ERR_CSR);
}

__global__ void check_entries_kernel(DevMatrix A, int check_csr, int check_finite, int* flag) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= A.nnz) return;
  if (check_csr) {
    const int i = csr_row_of(A.row_ptr, A.g.m, e);
    const int c = A.col[e];
    bool bad = c >= A.g.n;
    if (e > A.row_ptr[i] && A.col[e - 1] >= c) bad = true;
    if (bad) atomicMin(flag, SPQR_ERR_CSR);
  }
  if (check_finite && (A.val[e] & 0x7C00u) == 0x7C00u) atomicMax(flag + 1, 1);
}

__global__ void check_stats2_kernel(DevMatrix A, int* flag) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)A.g.ntr * A.g.ntc) return;
  const int tr = (int)(t / A.g.ntc), tc = (int)(t % A.g.ntc);
  const uint32_t a = ld32(A.packed, stat_dword_offset(A.g, tr, tc, A.g.sd - 2));
  const uint32_t b = ld32(A.packed, stat_dword_offset(A.g, tr, tc, A.g.sd - 1));
  const bool bad = (a & 0x7C00u) == 0x7C00u || (a & 0x7C000000u) == 0x7C000000u
                || (b & 0x7C00u) == 0x7C00u || (b & 0x7C000000u) == 0x7C000000u;
  if (bad) atomicMax(flag + 1, 1);
}

__global__ void check_perm_kernel(DevMatrix A, int* flag) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= A.g.n) return;
  const int p = A.perm[j];
  if (p < 0 || p >= A.g.n) atomicMax(flag + 2, 1);
}

// Device-side result words of spqr_pack_check: [0] CSR status, [1] non-finite, [2] perm.
__device__ int g_check_words[4];

// ---------------------------------------------------------------------------
// Launchers.
// ---------------------------------------------------------------------------
static inline int pick_waves(int nsteps, int max_waves) {
  if (nsteps <= max_waves) return nsteps < 1 ? 1 : nsteps;
  int best = max_waves; double best_eff = 0.0;
  for (int w = max_waves; w >= max_waves / 2; --w) {
    const int rounds = (nsteps + w - 1) / w;
    const double eff = (double)nsteps / ((double)rounds * w);
    if (eff > best_eff + 1e-9) { best_eff = eff; best = w; }
  }
  return best;
}

template <int W, int TR, int TC, int AXIS>
static hipError_t launch_tile256(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                                 hipStream_t stream) {
  const int nsteps = (A.g.ntc + 63) / 64;
  const int nw = pick_waves(nsteps, WavesPerGroup<W>::MAX);
  const size_t lds = ((size_t)A.g.n * 2 + 15) & ~(size_t)15;
  hipLaunchKernelGGL((gemv_tile256_kernel<W, TR, TC, AXIS>), dim3(A.g.ntr), dim3(64 * nw), lds,
                     stream, A, x, y, y_dtype);
  return hipGetLastError();
}

bool has_tuned_gemv(const Geometry& g) {
  if ((int64_t)g.n * 2 + 16 > 60 * 1024) return false;      // x must fit the LDS staging buffer
  if (g.tile_rows * g.tile_cols != 256) return false;
  if (g.axis == 1) return (g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 8 && g.tile_cols == 32);
  return (g.tile_rows == 16 && g.tile_cols == 16) || (g.tile_rows == 32 && g.tile_cols == 8);
}

hipError_t launch_gemv(const DevMatrix& A, const uint16_t* x, void* y, int y_dtype,
                       hipStream_t stream, bool force_generic) {
  const Geometry& g = A.g;
  if (!force_generic && has_tuned_gemv(g)) {
#define SPQR_CASE(W_, TR_, TC_, AX_) \
    if (g.w_bits == W_ && g.tile_rows == TR_ && g.tile_cols == TC_ && g.axis == AX_) \
      return launch_tile256<W_, TR_, TC_, AX_>(A, x, y, y_dtype, stream);
    SPQR_CASE(3, 16, 16, 1) SPQR_CASE(4, 16, 16, 1) SPQR_CASE(3, 8, 32, 1) SPQR_CASE(4, 8, 32, 1)
    SPQR_CASE(3, 16, 16, 0) SPQR_CASE(4, 16, 16, 0) SPQR_CASE(3, 32, 8, 0) SPQR_CASE(4, 32, 8, 0)
#undef SPQR_CASE
  }
  const int rows_per_block = 4;
  hipLaunchKernelGGL(gemv_generic_kernel, dim3((g.m + rows_per_block - 1) / rows_per_block),
                     dim3(64 * rows_per_block), 0, stream, A, x, y, y_dtype);
  return hipGetLastError();
}

hipError_t launch_dequant(const DevMatrix& A, int what, void* out, hipStream_t stream) {
  const int sel = what & 0xFF;
  const bool with_outliers = (what & SPQR_OUT_WITH_OUTLIERS) != 0;
  const int64_t total = (int64_t)A.g.m * A.g.n;
  const int bs = 256;
  const unsigned nb = (unsigned)((total + bs - 1) / bs);
  switch (sel) {
    case SPQR_OUT_CODES_U8:
      hipLaunchKernelGGL(codes_u8_kernel, dim3(nb), dim3(bs), 0, stream, A, (uint8_t*)out);
      break;
    case SPQR_OUT_SCALE_F32:
    case SPQR_OUT_ZERO_F32: {
      const int64_t groups = total / A.g.beta1;
      hipLaunchKernelGGL(stats_f32_kernel, dim3((unsigned)((groups + bs - 1) / bs)), dim3(bs), 0, stream,
                         A, (float*)out, sel == SPQR_OUT_ZERO_F32 ? 1 : 0);
      break;
    }
    case SPQR_OUT_DENSE_F32:
      hipLaunchKernelGGL(dense_kernel<float>, dim3(nb), dim3(bs), 0, stream, A, (float*)out);
      if (with_outliers && A.nnz > 0)
        hipLaunchKernelGGL(dense_outlier_kernel<float>, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs),
                           0, stream, A, (float*)out);
      break;
    case SPQR_OUT_DENSE_F16:
      hipLaunchKernelGGL(dense_kernel<uint16_t>, dim3(nb), dim3(bs), 0, stream, A, (uint16_t*)out);
      if (with_outliers && A.nnz > 0)
        hipLaunchKernelGGL(dense_outlier_kernel<uint16_t>, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs),
                           0, stream, A, (uint16_t*)out);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Runs the selected device checks and copies the three result words to the host.
hipError_t run_checks(const DevMatrix& A, bool csr, bool finite, bool perm, int host_words[3],
                      hipStream_t stream) {
  int* words = nullptr;
  hipError_t e = hipGetSymbolAddress((void**)&words, HIP_SYMBOL(g_check_words));
  if (e != hipSuccess) return e;
  for (int k = 0; k < 3; ++k)
    hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(64), 0, stream, words + k, 0);
  const int bs = 256;
  if (csr) {
    hipLaunchKernelGGL(check_rowptr_kernel, dim3((A.g.m + 1 + bs - 1) / bs), dim3(bs), 0, stream, A, words);
    // Entry checks index through row_ptr: only run them on a valid prefix array.
    e = hipMemcpyAsync(host_words, words, sizeof(int), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return e;
    if (host_words[0] != 0) { host_words[1] = host_words[2] = 0; return hipSuccess; }
  }
  if ((csr || finite) && A.nnz > 0)
    hipLaunchKernelGGL(check_entries_kernel, dim3((unsigned)((A.nnz + bs - 1) / bs)), dim3(bs), 0, stream,
                       A, csr ? 1 : 0, finite ? 1 : 0, words);
  if (finite) {
    const int64_t tiles = (int64_t)A.g.ntr * A.g.ntc;
    hipLaunchKernelGGL(check_stats2_kernel, dim3((unsigned)((tiles + bs - 1) / bs)), dim3(bs), 0, stream, A, words);
  }
  if (perm && A.perm)
    hipLaunchKernelGGL(check_perm_kernel, dim3((A.g.n + bs - 1) / bs), dim3(bs), 0, stream, A, words);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(host_words, words, 3 * sizeof(int), hipMemcpyDeviceToHost, stream);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(stream);
}

}  // namespace spqr
