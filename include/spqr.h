/*
 * spqr.h - C ABI of the SpQR inference library for AMD MI355X (gfx950).
 *
 * The library multiplies activations by a weight matrix W[m, n] (m = d_out,
 * n = d_in) that is stored in the Sparse-Quantized Representation of
 * "SpQR: A Sparse-Quantized Representation for Near-Lossless LLM Weight
 * Compression" (Sec. 4.2):
 *
 *   (1) a b_w-bit code Q_ij for EVERY weight (outlier positions included),
 *   (2) a 3-bit scale code and a 3-bit zero code per first-level group of
 *       beta1 weights, and four 16-bit scalars (s_s, z_s, s_z, z_z) per tile
 *       of beta2 first-level groups,
 *   (3) a CSR-style outlier set: per outlier a 16-bit value and a 16-bit
 *       column index, per row one 32-bit running count.
 *
 * Decode (Alg. 1, dequantize and fit_statistics):
 *       s_hat = s_s * (s_q - z_s)        z_hat = s_z * (z_q - z_z)
 *       W_hat_ij = s_hat_g * (Q_ij - z_hat_g)  (+ val_k where (i, j) is outlier k)
 *       y = W_hat . x      with fp32 accumulation.
 *
 * Group geometry (group_axis):
 *   0  a group is beta1 consecutive columns j of one row i (the paper's
 *      Alg. 1 sweeps column blocks of width beta1); a tile is beta2 rows x
 *      beta1 columns.
 *   1  a group is beta1 consecutive rows i of one column j; a tile is beta1
 *      rows x beta2 columns.
 *
 * Pointers are DEVICE pointers unless a parameter says "host".  The library
 * never frees or keeps caller memory.  The product and decode calls are
 * asynchronous on the given HIP stream (a hipStream_t passed as void*;
 * NULL = the default stream).  Who owns device scratch, and what that means:
 *   - spqr_gemv, spqr_gemv_fused, spqr_gemv_grouped, spqr_dequant_dense and
 *     batches of up to 3 vectors need no scratch: they allocate nothing and
 *     never synchronise;
 *   - spqr_gemm_smallbatch_ws / spqr_gemm_fused_ws take the scratch of the
 *     larger batches from the caller (spqr_workspace_bytes says how much):
 *     they allocate nothing, free nothing and never synchronise, on any stream,
 *     captured or not;
 *   - spqr_gemm_smallbatch / spqr_gemm_fused are conveniences over them with
 *     scratch the library owns: one buffer per stream, kept until the process
 *     ends and grown on demand, which does synchronise that stream and call
 *     hipFree / hipMalloc (see spqr_gemm_smallbatch);
 *   - spqr_gemm_smallbatch_noalloc keeps the scratch in a static device array
 *     (for callers that cannot allocate);
 *   - spqr_pack_check synchronises and allocates 16 bytes for the call.
 * Every entry point returns SPQR_OK (0) or a negative spqr_status; nothing
 * throws, aborts or prints.
 */
#ifndef SPQR_H_
#define SPQR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum spqr_status {
  SPQR_OK            =  0,
  SPQR_ERR_NULL      = -1,  /* a required pointer is NULL                          */
  SPQR_ERR_SHAPE     = -2,  /* m, n not positive multiples of the tile, n > 65536  */
  SPQR_ERR_PARAM     = -3,  /* bit widths / group sizes / axis / layout unsupported */
  SPQR_ERR_SIZE      = -4,  /* packed_bytes differs from spqr_packed_bytes(), nnz<0 */
  SPQR_ERR_ALIGN     = -5,  /* packed not 16-byte aligned, other arrays misaligned  */
  SPQR_ERR_CSR       = -6,  /* row_ptr not a valid prefix, column out of range or
                               not strictly increasing inside a row                */
  SPQR_ERR_NONFINITE = -7,  /* a 16-bit statistic or outlier value is inf / nan     */
  SPQR_ERR_BATCH     = -8,  /* batch outside [1, SPQR_MAX_BATCH]                    */
  SPQR_ERR_HIP       = -9,  /* a HIP runtime call or kernel launch failed           */
  SPQR_ERR_DTYPE     = -10, /* unknown output dtype / dequant selector              */
  SPQR_ERR_WORKSPACE = -11  /* the workspace is smaller than spqr_workspace_bytes() */
} spqr_status;

/* Values of spqr_matrix_t::layout_version: how a tile's statistics are stored.
 * 1 is the method's own bilevel format (Sec. 4.2); 2 and 3 are the two variants
 * the ablations of Sec. 5 evaluate. */
#define SPQR_LAYOUT_V1          1  /* 3-bit (s_q, z_q) per group, (s_s, z_s, s_z, z_z) per tile   */
#define SPQR_LAYOUT_ROUND_ZERO  2  /* "round zero": the 3-bit zero code IS the zero-point,
                                      z_hat = z_q; the tile keeps (s_s, z_s) only                */
#define SPQR_LAYOUT_STATS16     3  /* "16-bit statistics": binary16 (s_hat, z_hat) per group,
                                      nothing per tile; s_bits = z_bits = 16                     */
#define SPQR_MAX_BATCH  256

/* Output element types of y / Y. */
#define SPQR_F32 0   /* IEEE binary32 (used for parity)            */
#define SPQR_F16 1   /* IEEE binary16, round-to-nearest-even of the fp32 result */

/*
 * One matrix in SpQR form (Sec. 4.2; hyper-parameter names of App. B).
 *
 * Supported: w_bits in {3, 4}; s_bits = z_bits = 3 (16 for
 * SPQR_LAYOUT_STATS16); beta2 a multiple of 16; beta1 * beta2 * w_bits a
 * multiple of 128; tile width even; n <= 65536; m, n multiples of the tile.
 * Everything else returns SPQR_ERR_PARAM/SHAPE.
 *
 * `packed` holds parts (1) and (2), written by spqr_pack_host() /
 * spqr_pack_host_layout().  Layout SPQR_LAYOUT_V1:
 *   - the matrix is cut into tiles (tile_rows x tile_cols as above), ordered
 *     row-major over the tile grid; every run of up to 64 consecutive tiles of
 *     one tile-row forms a block of L <= 64 tiles starting at byte
 *     (first tile index) * tile_bytes;
 *   - a tile owns KW = tile_rows*tile_cols*w_bits/128 16-byte code words and
 *     SD = 3*beta2/16 + 2 statistic dwords; tile_bytes = 16*KW + 4*SD, which is
 *     exactly (b_w + 6/beta1 + 64/(beta1*beta2)) * beta1*beta2 / 8 (App. D Eq. 4);
 *   - inside a block, code word k of tile l sits at byte (k*L + l)*16; after
 *     all code words come the floor(SD/4) full statistic words, word k of tile
 *     l at (k*L + l)*16, then the SD%4 remaining dwords, dword k of tile l at
 *     (k*L + l)*4  (so each load instruction of a 64-lane wavefront reads one
 *     contiguous run);
 *   - codes are stored as pairs: pair q = r*(tile_cols/2) + p holds the codes
 *     of tile-local (row r, column 2p) in the low and (r, 2p+1) in the high
 *     16-bit half of a dword, at the same bit offset.  w_bits=4: dword q/4,
 *     offset 4*(q%4).  w_bits=3: triple t=q/16 of three dwords, e=q%16: for
 *     e<15 dword 3t+e/5 at offset 3*(e%5); for e=15 bit i of the low (high)
 *     code is bit 15 (31) of dword 3t+i;
 *   - the 2*beta2 statistic codes of a tile, in the order s_q[0..beta2),
 *     z_q[0..beta2) (group index along the tile), are stored as 3-bit pairs
 *     in the same way; the last two statistic dwords are s_s | z_s<<16 and
 *     s_z | z_z<<16 (binary16 bit patterns).
 * The other two layouts differ in the statistic dwords only:
 *   - SPQR_LAYOUT_ROUND_ZERO: SD = 3*beta2/16 + 1: the same code dwords, then
 *     s_s | z_s<<16; tile_bytes = (b_w + 6/beta1 + 32/(beta1*beta2)) * beta1*beta2/8;
 *   - SPQR_LAYOUT_STATS16: SD = beta2: dword g is s_hat_g | z_hat_g<<16 (binary16
 *     bit patterns) of group g of the tile; tile_bytes = (b_w + 32/beta1) * beta1*beta2/8
 *     (beta2 only shapes the tile).
 * Decode: SPQR_LAYOUT_ROUND_ZERO  s_hat = s_s * (s_q - z_s), z_hat = z_q;
 *         SPQR_LAYOUT_STATS16     s_hat, z_hat as stored.
 * Tiles of 256 codes have tuned batch-1 kernels in every layout; the slices of
 * 16 on the matrix cores exist for SPQR_LAYOUT_V1 only: the other layouts run a
 * few vectors as passes of the batch-1 kernel and a dozen and more through the
 * dense copy (see spqr_gemm_smallbatch).
 *
 * Outliers: row_ptr[m+1] is the exclusive prefix of per-row counts
 * (row_ptr[0] = 0, row_ptr[m] = nnz); col_idx / out_val are sorted by row then
 * strictly increasing column.  With nnz = 0, col_idx and out_val may be NULL;
 * row_ptr must still hold m+1 zeros.  col_idx and out_val must be 16-byte
 * aligned (SPQR_ERR_ALIGN otherwise): the product kernels read them in aligned
 * 16-byte granules of 8 entries.  The granule holding the last entry is read
 * whole; it shares its 16 aligned bytes, hence its page, with that entry, and
 * what lies behind entry nnz-1 is ignored.
 *
 * max_row_nnz is a hint for the launch plan only (never for correctness): an
 * upper estimate of the longest outlier row, 0 if unknown.  A matrix with rows
 * of thousands of outliers (Sec. 3.2 finds whole rows of sensitive weights)
 * gets wider workgroups for the strips that own them.
 *
 * perm (optional, NULL = identity) is an input permutation of length n: the
 * product is taken with x'[j] = x[perm[j]] (act-order checkpoints, Sec. 5).
 */
typedef struct spqr_matrix_t {
  int32_t m, n;
  int32_t w_bits, s_bits, z_bits;
  int32_t beta1, beta2;
  int32_t group_axis;
  int32_t layout_version;
  int32_t max_row_nnz;        /* optional hint, >= 0: the largest number of outliers in one row, 0 = unknown */
  const void*     packed;     /* device, 16-byte aligned */
  int64_t         packed_bytes;
  const int32_t*  row_ptr;    /* device, m+1 entries */
  const uint16_t* col_idx;    /* device, nnz entries, 16-byte aligned */
  const uint16_t* out_val;    /* device, nnz binary16 bit patterns, 16-byte aligned */
  int64_t         nnz;
  const int32_t*  perm;       /* device, n entries, or NULL */
} spqr_matrix_t;

/* ---- host-side helpers (no GPU needed) ---------------------------------- */

/* Bytes of the `packed` buffer for these parameters, or a negative
 * spqr_status.  Equals m*n*(b_w + (b_s+b_z)/beta1 + 64/(beta1*beta2))/8,
 * the outlier-free part of App. D Eq. 4, with no padding. */
int64_t spqr_packed_bytes(int32_t m, int32_t n, int32_t w_bits, int32_t s_bits,
                          int32_t z_bits, int32_t beta1, int32_t beta2,
                          int32_t group_axis);

/* The same for any layout_version (s_bits = z_bits = 16 for SPQR_LAYOUT_STATS16). */
int64_t spqr_packed_bytes_layout(int32_t layout_version, int32_t m, int32_t n, int32_t w_bits,
                                 int32_t s_bits, int32_t z_bits, int32_t beta1, int32_t beta2,
                                 int32_t group_axis);

/* Pack logical HOST arrays into layout V1 (HOST buffer `packed_out` of
 * spqr_packed_bytes() bytes, fully overwritten).
 *   Q      uint8 [m][n], codes < 2^w_bits
 *   s_q,z_q uint8, [m][n/beta1] for group_axis 0, [m/beta1][n] for axis 1, < 8
 *   s_s,z_s,s_z,z_z binary16 bit patterns, one per tile, [m/tile_rows][n/tile_cols]
 * Returns SPQR_ERR_PARAM if a code exceeds its bit width. */
int spqr_pack_host(int32_t m, int32_t n, int32_t w_bits, int32_t s_bits, int32_t z_bits,
                   int32_t beta1, int32_t beta2, int32_t group_axis,
                   const uint8_t* Q, const uint8_t* s_q, const uint8_t* z_q,
                   const uint16_t* s_s, const uint16_t* z_s,
                   const uint16_t* s_z, const uint16_t* z_z,
                   void* packed_out, int64_t packed_bytes);

/* The same for any layout_version (Sec. 5, ablations "round zero" and "16-bit
 * statistics"; SPQR_LAYOUT_V1 gives spqr_pack_host).  s_first / z_first, one
 * entry per first-level group in the shapes above: uint8 codes < 8 for layouts
 * 1 and 2, binary16 bit patterns (uint16) of s_hat / z_hat for layout 3.  The
 * per-tile arrays a layout does not store are ignored and may be NULL (s_z, z_z
 * for layout 2; all four for layout 3). */
int spqr_pack_host_layout(int32_t layout_version, int32_t m, int32_t n, int32_t w_bits,
                          int32_t s_bits, int32_t z_bits, int32_t beta1, int32_t beta2,
                          int32_t group_axis, const uint8_t* Q, const void* s_first,
                          const void* z_first, const uint16_t* s_s, const uint16_t* z_s,
                          const uint16_t* s_z, const uint16_t* z_z, void* packed_out,
                          int64_t packed_bytes);

const char* spqr_strerror(int status);

/* Library / layout version: (major<<16) | highest layout version understood. */
int32_t spqr_version(void);

/* ---- device entry points ------------------------------------------------- */

#define SPQR_CHECK_CSR        1u  /* O(nnz) validation of the outlier arrays (Sec. 4.2 ordering) */
#define SPQR_CHECK_NONFINITE  2u  /* reject inf/nan in 16-bit statistics and outlier values       */
#define SPQR_CHECK_PERM       4u  /* perm entries within [0, n)                                   */

/* Validate a descriptor: O(1) parameter / size / alignment checks always,
 * plus the device-side checks selected by `flags`.  Synchronises `stream`.
 * Writes nothing the caller owns. */
int spqr_pack_check(const spqr_matrix_t* A, uint32_t flags, void* stream);

/* y[m] = W_hat . x  (batch 1; the token-by-token decode of Sec. 4.2,
 * "Inference with SpQR", with the dense and the outlier part fused in one
 * kernel).  x: n binary16 values.  y: m elements of y_dtype, overwritten. */
int spqr_gemv(const spqr_matrix_t* A, const uint16_t* x_f16, void* y, int y_dtype,
              void* stream);

/* Y[b][m] = X[b][:] . W_hat^T for 1 <= b <= SPQR_MAX_BATCH (Sec. 4.2 dequantises
 * to 16 bit and multiplies; the sparse part is a product of its own).
 * Up to 3 vectors (4 on small layers): one launch of the batch-1 kernel's
 * NB-vector form.  More: either slices of up to 4 (weights read once per
 * slice), or, for tiles of 16x16, 8x32 (group_axis 1) and 32x8 (group_axis 0)
 * and a batch / layer large enough to pay for it, slices of up to 16: the
 * weights are read once per slice, dequantised to binary16 and multiplied on
 * the matrix cores, then a second kernel adds the outliers.  That path needs
 * device scratch, about (n+1)*32 + (nnz/256 + 2)*64 + splits*16*m*4 (+ 32*n
 * with a permutation) bytes per slice.
 * THIS entry point takes it from the library: one scratch buffer per stream
 * (up to 8 streams per device), kept until the process ends and grown on
 * demand -- growing synchronises the stream and calls hipFree and hipMalloc
 * inside the call -- and it holds the buffer's lock while the call is
 * enqueued: calls on different streams never share scratch, calls from several
 * host threads on one stream are enqueued one after the other.  On a stream
 * that is being captured the scratch is a stream-ordered allocation from the
 * device's default memory pool instead (allocation nodes of the graph, about
 * 10 us more per call), on further streams one from a pool of the library's
 * own.  If no scratch can be had, the slices of 4 run instead.  Callers that
 * must not allocate or synchronise use spqr_gemm_smallbatch_ws.
 * Large batches (48 vectors and more, 12 where no slices of 16 exist; the
 * prompt phase of Sec. 5 "Inference Time"; tiles of 256 codes in any layout
 * and 3-bit tiles of 8 x 64, Y 16-byte aligned): the matrix is
 * dequantised once into a dense binary16 copy in scratch (2 bytes per weight,
 * rows padded to a multiple of 64 columns; with a permutation b*n*2 bytes more),
 * the outliers are added into the copy, and one matrix-core kernel multiplies
 * the whole batch with it.  Where that much scratch cannot be had (a captured
 * call without a workspace, a workspace smaller than spqr_workspace_bytes says)
 * the slices of 16 run instead.
 * Results are deterministic (fixed summation order) on every path; the paths
 * differ by rounding only (all within the product tolerance).
 * X: [b][n] binary16 row-major.  Y: [b][m] of y_dtype, overwritten. */
int spqr_gemm_smallbatch(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y,
                         int y_dtype, void* stream);

/* Bytes of device scratch spqr_gemm_smallbatch_ws (count = 1) or
 * spqr_gemm_fused_ws need at most for these matrices and a batch of b; 0 if the
 * call takes kernels that need none.  A is a HOST array of `count` descriptor
 * pointers (1 <= count <= SPQR_MAX_FUSED; they must agree as for
 * spqr_gemm_fused).  Host arithmetic only; a negative return is an SPQR_ERR_*
 * code.  The value depends on the descriptors' shapes, nnz and perm, on b and
 * on the options of spqr_set_option, not on pointers or the stream. */
int64_t spqr_workspace_bytes(const spqr_matrix_t* const* A, int count, int b);

/* spqr_gemm_smallbatch with scratch the CALLER owns (Sec. 4.2's product, as
 * above): `workspace` is device memory, 256-byte aligned, of at least
 * spqr_workspace_bytes(&A, 1, b) bytes (SPQR_ERR_WORKSPACE if smaller; it may
 * be NULL when that is 0).  The call allocates nothing, frees nothing and
 * never synchronises; which kernels run does not depend on whether `stream`
 * is being captured, so a captured call records kernel nodes only.  The
 * workspace is written by the call's kernels and may be reused by the next
 * call on the same stream; calls that may overlap need workspaces of their
 * own.  Same results as spqr_gemm_smallbatch on the same path. */
int spqr_gemm_smallbatch_ws(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y,
                            int y_dtype, void* workspace, int64_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory at all (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc):
 * spqr_gemm_smallbatch with its scratch in a static device array of
 * SPQR_STATIC_SCRATCH_BYTES that the library's code object carries (every GPU
 * the library runs on holds it until the process ends).  A call whose
 * spqr_workspace_bytes(&A, 1, b) exceeds that size returns SPQR_ERR_WORKSPACE
 * and launches nothing.  No hipMalloc, hipFree or other allocating call is
 * made; the first call on a device asks the runtime for the array's address.
 * All calls on one GPU share the array: calls that may overlap on one GPU
 * (different streams) race on it -- give such callers spqr_gemm_smallbatch_ws.
 * Same results as spqr_gemm_smallbatch_ws. */
#define SPQR_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int spqr_gemm_smallbatch_noalloc(const spqr_matrix_t* A, const uint16_t* X_f16, int b, void* Y,
                                 int y_dtype, void* stream);

/* y[i][0..m_i) = W_hat_i . x for `count` (1..SPQR_MAX_FUSED) matrices that
 * share the input vector: the q/k/v or the gate/up projections of a decoder
 * block (Sec. 4.2 decodes token by token, layer by layer; matrices fed by the
 * same activations need not wait for one another).  A and y are HOST arrays of
 * `count` descriptor pointers / device output pointers.  The matrices must
 * agree in n, w_bits, s_bits, z_bits, beta1, beta2, group_axis, layout_version
 * and perm (SPQR_ERR_PARAM otherwise); m may differ.  When a tuned kernel
 * exists and perm is NULL all strips of all matrices run in ONE launch, each
 * workgroup doing exactly what it does in spqr_gemv; otherwise the call is
 * `count` launches of spqr_gemv.  Results equal spqr_gemv's. */
#define SPQR_MAX_FUSED 8
int spqr_gemv_fused(const spqr_matrix_t* const* A, int count, const uint16_t* x_f16,
                    void* const* y, int y_dtype, void* stream);

/* Y[i][b][m_i] = X[b][:] . W_hat_i^T for `count` matrices that share the batch X
 * (the q/k/v or gate/up projections of a decoder block at batch b): what
 * spqr_gemv_fused is for one vector.  Same agreement rules (SPQR_ERR_PARAM
 * otherwise), A and Y are HOST arrays.  Where the batch takes the matrix-core
 * path of spqr_gemm_smallbatch, all matrices share one transposition of the
 * batch, one dense launch and one finishing launch per slice of 16 vectors;
 * otherwise, and whenever `stream` is being captured into a graph, the call is
 * `count` calls of spqr_gemm_smallbatch (b == 1: one spqr_gemv_fused).  Scratch
 * as for spqr_gemm_smallbatch (library-owned; spqr_gemm_fused_ws takes the
 * caller's).  Same
 * arithmetic as spqr_gemm_smallbatch on the same path; only the order of the
 * partial sums over column ranges may differ. */
int spqr_gemm_fused(const spqr_matrix_t* const* A, int count, const uint16_t* X_f16, int b,
                    void* const* Y, int y_dtype, void* stream);

/* spqr_gemm_fused with scratch the caller owns: see spqr_gemm_smallbatch_ws;
 * the workspace holds at least spqr_workspace_bytes(A, count, b) bytes. */
int spqr_gemm_fused_ws(const spqr_matrix_t* const* A, int count, const uint16_t* X_f16, int b,
                       void* const* Y, int y_dtype, void* workspace, int64_t workspace_bytes,
                       void* stream);

/* y[i][0..m_i) = W_hat_i . x[i] for `count` (1..SPQR_MAX_GROUPED) matrices, each
 * with an input vector of its own: all projections of a decoder block whose
 * inputs are at hand (Sec. 5 times token-by-token generation: seven such
 * products per block), in as few launches as possible.  A, x_f16 and y are HOST
 * arrays.  Matrices that agree in w_bits, beta1, beta2, group_axis and layout,
 * have a tuned kernel and no permutation run in ONE launch (up to
 * SPQR_MAX_FUSED of them); the others take a launch each.  The input width n
 * with the most rows sizes that launch, and every workgroup of such a matrix
 * does what it does in spqr_gemv: those results equal spqr_gemv's bit for bit.
 * A matrix of another width joins the launch if the launch's LDS serves it: a
 * wider one needs max_row_nnz > 0 (the hint then tells that a workgroup's
 * outliers fit one round; an understated hint costs time, never correctness);
 * its partial sums over column ranges may meet in another order than in
 * spqr_gemv (same arithmetic otherwise).  A matrix that cannot join waits for
 * the next launch of the call.  No scratch, no allocation, no synchronisation. */
#define SPQR_MAX_GROUPED 16
int spqr_gemv_grouped(const spqr_matrix_t* const* A, int count, const uint16_t* const* x_f16,
                      void* const* y, int y_dtype, void* stream);

/* Process-wide switches for tuning runs and tests; production code never needs
 * them (all are 0 at start).  Returns SPQR_ERR_PARAM for an unknown option or
 * value.
 *   SPQR_OPT_BATCH_PATH    SPQR_BATCH_PATH_AUTO (0): the library's rule picks the
 *                          kernels of a batch; _VECTOR (1) / _MATRIX (2): slices
 *                          of 4 on the vector kernel / slices of 16 on the
 *                          matrix cores wherever both exist (and never the dense
 *                          copy); _DENSE (3): the dense-copy path of large
 *                          batches for any batch it exists for
 *   SPQR_OPT_FORCE_GENERIC 1: every product takes the element-wise fallback
 *                          kernel
 *   SPQR_OPT_BATCH_STEPS   k > 0: the matrix-core path's dense launch gives every
 *                          workgroup min(k, steps) steps of 64 tiles
 *   SPQR_OPT_DENSE_ROWS    64 or 128: rows per workgroup of the large-batch
 *                          multiply (0: the library's rule)
 *   SPQR_OPT_GEMV_PLAN     16 * P + R > 0: the batch-1 kernel runs with P
 *                          wavefronts per strip and R strips per workgroup
 *                          (clamped to what the matrix and the kernel allow) */
#define SPQR_OPT_BATCH_PATH     0
#define SPQR_OPT_FORCE_GENERIC  1
#define SPQR_OPT_BATCH_STEPS    2
#define SPQR_OPT_DENSE_ROWS     3
#define SPQR_OPT_GEMV_PLAN      4
#define SPQR_OPT_COUNT_         5
#define SPQR_BATCH_PATH_AUTO    0
#define SPQR_BATCH_PATH_VECTOR  1
#define SPQR_BATCH_PATH_MATRIX  2
#define SPQR_BATCH_PATH_DENSE   3
int spqr_set_option(int option, int value);

/* Debug decode (Alg. 1 `dequantize`, applied twice as in `fit_statistics`: first to
 * the statistic codes with the tile's second-level scalars, then to the weight
 * codes; Sec. 4.2's three parts of the representation).  `what` selects the output:
 *   SPQR_OUT_CODES_U8   uint8  [m][n]   the b_w-bit codes
 *   SPQR_OUT_SCALE_F32  float  group grid ([m][n/beta1] or [m/beta1][n]): s_hat
 *   SPQR_OUT_ZERO_F32   float  group grid: z_hat
 *   SPQR_OUT_DENSE_F32  float  [m][n]   s_hat*(Q - z_hat)
 *   SPQR_OUT_DENSE_F16  binary16 [m][n] the same, rounded to nearest even
 * OR-ing SPQR_OUT_WITH_OUTLIERS into a DENSE selector adds the outlier values
 * before the final rounding.  Decoded statistics are binary32: the code and the
 * second-level zero are widened, subtracted, then multiplied by the
 * second-level scale, each step rounded once (no fused multiply-add). */
#define SPQR_OUT_CODES_U8      0
#define SPQR_OUT_SCALE_F32     1
#define SPQR_OUT_ZERO_F32      2
#define SPQR_OUT_DENSE_F32     3
#define SPQR_OUT_DENSE_F16     4
#define SPQR_OUT_WITH_OUTLIERS 0x100
int spqr_dequant_dense(const spqr_matrix_t* A, int what, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif  /* SPQR_H_ */
