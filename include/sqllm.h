/*
 * sqllm.h — C ABI of the Dense-and-Sparse look-up-table matvec for AMD MI355X (gfx950).
 *
 * The library computes, for one linear layer and a small batch of activation vectors,
 *
 *        Y = D X + S X                                   (paper Sec. 4.2: W = D + S, W X = D X + S X)
 *
 *   D  (M x N)  dense part, stored as b-bit indices (b = 2, 3 or 4) into ONE look-up table of 2^b fp16
 *               values PER OUTPUT ROW:  D[i][j] = lut[i][ idx(i,j) ]
 *               (Sec. 4.3: what is stored are 3- or 4-bit indices, each naming an fp16 entry of a look-up table;
 *               Sec. 5, quantisation details: every output channel has a table of its own;
 *               App. F quantises to 2 bits with the same format).
 *   S  (M x N)  sparse part in compressed-sparse-row form with fp16 values (Sec. 4.2: outliers and
 *               sensitive values kept in FP16 and stored in CSR).
 *   X  (N x B)  fp16 activations, B = 1..16 vectors;  Y (M x B) fp16.
 *
 * STORAGE FORMAT (the paper does not fix one; this is the contract of this library)
 *   qidx   row i is a little-endian bit stream of N*b bits starting at byte i*N*b/8.  Element j owns stream
 *          bits [j*b, j*b+b), least-significant bit first; stream bit k is bit (k mod 8) of byte (k div 8).
 *          Rows follow each other without padding.  N must be a multiple of 128, so a row is a whole number
 *          of 32-byte (b=2), 48-byte (b=3) or 64-byte (b=4) groups of 128 elements.
 *   lut    fp16 [M][2^b], row-major.  No ordering of the entries is assumed.
 *   rowptr int32 [M+1], rowptr[0] = 0, non-decreasing, rowptr[M] = nnz.
 *   cols   int32 [nnz], 0 <= cols[p] < N.   vals  fp16 [nnz].  Duplicate (row, col) entries add up.
 *   x      fp16 [N][B] row-major (x[j*B + t]);   y  fp16 [M][B] row-major.
 *
 * ARITHMETIC  table look-ups are exact selections; products of fp16 values are accumulated in fp32; each
 *   y element is rounded to fp16 once.  The order of the fp32 additions is fixed for a given shape and
 *   launch configuration (no floating-point atomics are used), so results are reproducible run to run.
 *
 * OWNERSHIP / EXECUTION  every pointer is a caller-owned DEVICE pointer (unless stated otherwise) that must
 *   stay valid until the work enqueued on `stream` has finished.  The library never allocates, frees or
 *   synchronises: each call validates its arguments on the host, enqueues kernels on `stream`
 *   (a hipStream_t passed as void*, NULL = the default stream) and returns.  Device-side data (index
 *   ranges of cols, monotonicity of rowptr) is NOT validated; out-of-range columns are undefined behaviour.
 *   Finiteness is not validated either.  A non-finite activation x[j][t] reaches y[i][t] wherever the
 *   definition multiplies it by a weight (every row, through the dense term); in calls with B >= 3 the sparse
 *   term is formed by matrix instructions over groups of 16 rows, and a non-finite x[j][t] then also turns
 *   y[i][t] into NaN for the other rows of the group of a row holding a nonzero in column j (0 x Inf).
 *
 * ERRORS  every function returns an sqllm_status.  Arguments are validated on the host first and nothing is enqueued
 *   when validation fails.  An entry point that needs several kernel launches (batches of the one-thread-per-row
 *   kernel beyond 8 columns, more than 65535 rows in the parity exports, the offline pass) can fail in a later
 *   launch with SQLLM_ERR_HIP after earlier ones were enqueued; its outputs are then undefined.  A text for the last
 *   error of the calling thread is available from sqllm_last_error_string().
 *   M == 0 -> SQLLM_OK, nothing enqueued.  N must be positive: N == 0 (an empty sum) is SQLLM_ERR_SHAPE, the caller
 *   clears y itself.  The library holds gfx950 code only: on any other device the first call that would launch
 *   returns SQLLM_ERR_DEVICE (the architecture is looked up once per device and remembered).
 *
 * THREADS  the library keeps no mutable state other than the per-thread error text and a per-device "architecture
 *   checked" flag; calls from several threads and on several streams may overlap.
 *
 * ALIGNMENT  qidx and x must be 16-byte aligned; lut 16-byte; y, vals 2-byte; rowptr, cols 4-byte.
 */
#ifndef SQLLM_H
#define SQLLM_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SQLLM_OK = 0,
    SQLLM_ERR_NULL = 1,   /* a required pointer is NULL                                   */
    SQLLM_ERR_BITS = 2,   /* bits is not 2, 3 or 4                                        */
    SQLLM_ERR_SHAPE = 3,  /* M < 0, N <= 0, N % 128 != 0 (all widths), or N > SQLLM_MAX_N */
    SQLLM_ERR_ALIGN = 4,  /* a pointer violates the alignment rules above                 */
    SQLLM_ERR_NNZ = 5,    /* nnz < 0 or nnz >= 2^31                                       */
    SQLLM_ERR_BATCH = 6,  /* B outside 1..SQLLM_MAX_BATCH                                 */
    SQLLM_ERR_HIP = 7,    /* the HIP runtime reported an error (see the error string)     */
    SQLLM_ERR_DEVICE = 8  /* the current device is not a gfx950 GPU                       */
} sqllm_status;

#define SQLLM_MAX_BATCH 16
#define SQLLM_MAX_N 28672 /* widest row a workgroup covers with one 2048-column slice per wave (14 waves) */

/* Dense term only (Sec. 4.3, the LUT-based matrix-vector kernel):
 *   accumulate == 0:  y = D x          accumulate != 0:  y = fp16( fp32(y) + D x )                        */
int sqllm_lut_gemv(int M, int N, int bits, int B,
                   const void* qidx, const void* lut, const void* x, void* y,
                   int accumulate, void* stream);

/* Sparse term only (Sec. 4.3, the balanced CSR kernel: every thread of a workgroup takes the same number
 * of nonzeros regardless of which row they fall in, and rows shared by several threads are combined on
 * chip):   accumulate == 0:  y = S x        accumulate != 0:  y = fp16( fp32(y) + S x )
 * nnz == 0 is allowed (cols/vals may then be NULL; rowptr is not read).                                  */
int sqllm_csr_spmv(int M, int N, long long nnz, int B,
                   const int* rowptr, const int* cols, const void* vals,
                   const void* x, void* y, int accumulate, void* stream);

/* Both terms in ONE kernel launch (Sec. 4.3: dense and sparse kernels are launched in one call so that no
 * separate pass sums their outputs):  y = fp16( D x + S x ), summed in fp32.  nnz == 0 -> dense only.
 * B = 1 is the paper's matrix-vector case; B = 2..16 is still one launch (the products then run on the
 * matrix cores, every weight is decoded once for all columns), also for the dense-only and the sparse-only
 * entry points.                                                                                          */
int sqllm_dense_sparse_matvec(int M, int N, int bits, long long nnz, int B,
                              const void* qidx, const void* lut,
                              const int* rowptr, const int* cols, const void* vals, const void* plan,
                              const void* x, void* y, void* stream);

/* Plan of the sparse term: a one-time re-layout of the CSR arrays of a (static) weight matrix for the one-column kernel
 * (Sec. 4.3 / App. C balance the nonzeros over the threads at run time; weights do not change, so the balancing can be done
 * once).  The nonzeros of every block of four rows are stored as groups of 16 entries of one row -- column and fp16 value
 * packed into one 32-bit word -- at a position the kernel derives from its workgroup index, with an overflow list for heavy
 * rows.  With a plan the matvec requests its nonzeros at wave start (no row-pointer hop), reads 4 instead of 6 bytes per
 * nonzero (plus the padding of the groups) and sums a row's group with a fixed 16-lane reduction, cheap enough for the dense
 * waves to carry the sparse term.  It pays where the rows' nonzero counts are moderate (a workgroup whose rows hold far more
 * than the average goes through the overflow list, a second dependent fetch); a caller may build it per layer or not at all.
 *   sqllm_csr_plan_bytes   size of the plan buffer for (M, N, nnz), a multiple of 256; host pointer `bytes_out`.
 *   sqllm_csr_plan_build   fills `plan` (device, 256-byte aligned, at least that many bytes) from rowptr / cols / vals on
 *                          `stream`; N must not exceed 32768 columns (15-bit column field; SQLLM_MAX_N is below that).
 * `plan` arguments: NULL, or a plan built for exactly this (M, N, nnz) and these CSR arrays.  It is used by calls with B == 1
 * that have a dense term and nnz > 0 (sqllm_dense_sparse_matvec, sqllm_dense_sparse_matvec_multi); rowptr / cols / vals are
 * then not read and may be NULL.  Calls with B >= 2 ignore the plan and need the CSR arrays.  The result is within the same
 * tolerance of the definition with and without a plan; the order of the fp32 additions differs, so the last bit of y may. */
int sqllm_csr_plan_bytes(int M, int N, long long nnz, size_t* bytes_out);
int sqllm_csr_plan_build(int M, int N, long long nnz, const int* rowptr, const int* cols, const void* vals,
                         void* plan, size_t bytes, void* stream);

/* Several independent layers, one activation vector each (the per-token stack of matvecs of Sec. 4.3, last paragraph: q, k, v of
 * a decoder block share an input and do not depend on each other, gate and up likewise), in as few kernel launches as possible.
 *   layers   HOST pointer to `count` descriptors; every pointer inside a descriptor is a device pointer with the meaning,
 *            layout and alignment of the argument of the same name of sqllm_dense_sparse_matvec (B = 1).  All layers of one
 *            call have the same `bits`.  The descriptors are copied into the kernel arguments: the array may be reused or
 *            freed as soon as the call returns.
 * The layers of one call must not depend on each other and their y must not overlap; they may run in any order.  The call sorts
 * them into groups and gives each group launches of its own, of up to SQLLM_MAX_LAYERS_PER_LAUNCH layers with a plan, or half as
 * many without (their descriptors are larger, and a launch is fastest while its kernel arguments stay below 1 KiB).  A group is the
 * layers that agree in: plan or no plan; the waves per workgroup they need (one per 2048 columns: every workgroup of a launch has
 * the size of its widest layer, and starting surplus waves in the narrower ones costs more than a launch); without a plan, the
 * rows per workgroup of the layer's own launch, on which the summation order of its sparse term depends.  Layers with a plan
 * give the same bits whatever the rows per workgroup, so their launches choose it by size: eight rows when the launch is many
 * generations of workgroups, else what the layers' own launches would take.
 * Each y is bit for bit what a separate sqllm_dense_sparse_matvec call with the same arguments gives; what is saved is the launch
 * gap and the ramp-up and tail of every layer but the last of a launch, and in long launches part of the fixed work per row.
 * Errors as for sqllm_dense_sparse_matvec, reported for the first offending layer; nothing is enqueued if any layer fails
 * validation (more than 256 layers need a host allocation for the launch order: SQLLM_ERR_SHAPE if it fails).  count == 0 -> SQLLM_OK.                                                                                          */
typedef struct {
    int M, N, bits;
    long long nnz;
    const void* qidx;
    const void* lut;
    const int* rowptr;
    const int* cols;
    const void* vals;
    const void* plan; /* NULL or the layer's plan (see sqllm_csr_plan_build); a launch also ends where this changes */
    const void* x;
    void* y;
} sqllm_layer;
#define SQLLM_MAX_LAYERS_PER_LAUNCH 16
int sqllm_dense_sparse_matvec_multi(int count, const sqllm_layer* layers, void* stream);

/* The launches sqllm_dense_sparse_matvec_multi would make for these layers, for inspection and tests (host only: no GPU is
 * needed, nothing is enqueued, no pointer inside a descriptor is followed).
 *   launch_out    HOST int[count]: the number (0, 1, ...) of the launch layer l goes to, in the order the launches are enqueued;
 *                 -1 for a layer without rows
 *   rows_out      HOST int[count] or NULL: rows per workgroup of that launch (4 or 8; 0 for a layer without rows)
 *   launches_out  HOST int or NULL: number of launches
 * Validation and errors as for sqllm_dense_sparse_matvec_multi (SQLLM_ERR_NULL also for launch_out == NULL with count > 0).     */
int sqllm_multi_launch_order(int count, const sqllm_layer* layers, int* launch_out, int* rows_out, int* launches_out);

/* One thread per row over the CSR matrix — the "standard" kernel the paper's App. C compares the balanced
 * one against.  Same arguments and result as sqllm_csr_spmv; kept as the ablation baseline.              */
int sqllm_csr_spmv_rowwise(int M, int N, long long nnz, int B,
                           const int* rowptr, const int* cols, const void* vals,
                           const void* x, void* y, int accumulate, void* stream);

/* Parity exports: the same in-register decode as the matvec kernels, written out.
 *   idx_out  uint8 [M][N]  index of every element (Sec. 4.3, b-bit indices)
 *   w_out    fp16  [M][N]  lut[i][idx(i,j)]        (Sec. 4.3, dequantisation by table look-up)           */
int sqllm_unpack_indices(int M, int N, int bits, const void* qidx, void* idx_out, void* stream);
int sqllm_dequantize(int M, int N, int bits, const void* qidx, const void* lut, void* w_out, void* stream);

/* fp16 baseline the paper measures its speed-ups against (Tab. 3, FP16 row): y = W x with
 * W fp16 [M][N] row-major, fp32 accumulation, fp16 result.  N % 8 == 0, w and x 16-byte aligned.         */
int sqllm_fp16_gemv(int M, int N, int B, const void* w, const void* x, void* y, void* stream);

/* ---- Offline side: Dense-and-Sparse split and sensitivity-weighted k-means (Sec. 4.1, Eq. 4; Sec. 4.2) ----
 * One call turns an fp16 weight matrix into everything the matvec reads.  All pointers are device pointers.
 *   w      fp16   [M][N] row-major, finite values                      (in)
 *   sens   uint16 [M][N] per-weight sensitivity: the diagonal Fisher information of Eq. 4 scaled to 16 bits by the
 *                        caller; only ratios inside a row matter for the tables, the order across the matrix for
 *                        the extraction                                  (in)
 *   n_lo, n_hi, n_sens   Sec. 4.2 thresholds as counts: T_min is the n_lo-th smallest weight of the matrix, T_max the
 *                        n_hi-th largest, and the sensitivity threshold the n_sens-th largest sensitivity (0-based).
 *                        A weight is extracted iff w < T_min or w > T_max or its sensitivity is above the threshold
 *                        (strict comparisons: ties stay dense, so at most n_lo + n_hi + n_sens entries are extracted;
 *                        -0 counts as smaller than +0).  All three 0 -> nothing is extracted.
 *   max_iter             upper bound on the centroid updates per row; iteration stops earlier when no weight changes
 *                        its cluster.
 *   workspace            sqllm_quantize_workspace_bytes(M, N) bytes of scratch, 4-byte aligned; contents are
 *                        overwritten; calls sharing a workspace must not overlap.
 *   qidx, lut            out: packed indices and fp16 tables (ascending per row) in the layout described above.
 *                        Per row the tables minimise sum_j sens_j (w_j - lut[idx_j])^2 over the dense weights by
 *                        Lloyd iterations from an equal-count start; idx_j is the nearest table entry (ties to the
 *                        lower index).  An extracted position gets the index of the entry nearest to zero.
 *   rowptr, cols, vals   out: CSR of the extracted weights (their full fp16 values, columns ascending);
 *                        rowptr int32 [M + 1]; cols / vals need room for n_lo + n_hi + n_sens entries;
 *                        the number written is rowptr[M].
 *   iters                out, may be NULL: int32 [M], centroid updates performed per row.
 * The results are a pure function of the inputs (integer accumulation, fixed-precision decisions): run-to-run
 * identical.  Errors as for the other entry points; M * N must be below 2^32.                                   */
long long sqllm_quantize_workspace_bytes(int M, int N);
int sqllm_quantize_layer(int M, int N, int bits, int max_iter, const void* w, const void* sens,
                         long long n_lo, long long n_hi, long long n_sens, void* workspace, long long workspace_bytes,
                         void* qidx, void* lut, int* rowptr, int* cols, void* vals, int* iters, void* stream);

/* The same offline pass for callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: no workspace argument, the 5.2 KB of scratch live in a device array the library
 * itself holds (one copy on every GPU the library is loaded on, until the process ends).  Arguments, results and errors
 * as for sqllm_quantize_layer; additionally M * N must not exceed SQLLM_NOALLOC_MAX_WEIGHTS (SQLLM_ERR_SHAPE otherwise).
 * The call allocates and frees nothing.  All calls on one GPU share that GPU's scratch array (it is cleared by the
 * call's first kernel): calls that overlap on one GPU -- different streams, different threads -- race and give
 * undefined results; calls on one stream, or ordered by events, are fine.                                        */
#define SQLLM_NOALLOC_MAX_WEIGHTS (1ll << 31)
int sqllm_quantize_layer_noalloc(int M, int N, int bits, int max_iter, const void* w, const void* sens,
                                 long long n_lo, long long n_hi, long long n_sens,
                                 void* qidx, void* lut, int* rowptr, int* cols, void* vals, int* iters, void* stream);

/* Bytes the method moves for one matvec (indices + tables + CSR arrays + x + y); used for GB/s figures.  */
long long sqllm_algorithmic_bytes(int M, int N, int bits, long long nnz, int B);

/* Sec. 4.2 gives the extraction as percentages (outliers by value, plus a share picked by sensitivity); the offline entry
 * point takes counts.  This host-only helper turns the shares into those counts: half of the outlier share on each tail,
 * n_lo = n_hi = floor(outlier_frac * M * N / 2), and n_sens = floor(sens_frac * M * N).  Shares must be >= 0 and sum to
 * less than 1.  The three results are host pointers.                                                                   */
int sqllm_extraction_counts(int M, int N, double outlier_frac, double sens_frac,
                            long long* n_lo, long long* n_hi, long long* n_sens);

const char* sqllm_last_error_string(void); /* host pointer, valid until the thread's next failing call */
const char* sqllm_status_string(int status);
int sqllm_version(void);                   /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* SQLLM_H */
