/*
 * CPU ORACLE for the Dense-and-Sparse look-up-table matvec — TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this file; the GPU
 * library shares no code with it.  It is the plain definition of what the inference path computes,
 * written out step by step in fp64:
 *
 *   W X = D X + S X                                        (Sec. 4.2, Dense-and-Sparse decomposition)
 *   D[i][j] = lut[i][ idx(i,j) ]                           (Sec. 4.3: b-bit indices into a table of
 *                                                           fp16 values; Sec. 5 "Quantization Details":
 *                                                           one table per output channel i)
 *   S in compressed-sparse-row form, fp16 values           (Sec. 4.2)
 *
 *   y[i][t]      = sum_j D[i][j] x[j][t] + sum_{p in row i} vals[p] x[cols[p]][t]
 *   absdot[i][t] = sum_j |D[i][j] + S[i][j]| |x[j][t]|     (scale of the accepted error)
 *
 * Storage format assumed (the paper leaves it open): row i of the index matrix is a little-endian
 * bit stream of N*b bits at byte offset i*N*b/8; element j owns stream bits [j*b, j*b+b), least
 * significant first; stream bit k is bit (k mod 8) of byte (k div 8).
 *
 * Deliberately naive: indices are read ONE BIT AT A TIME, nothing is blocked, fused or reordered.
 * Pinned by tests/test_oracle_*.py: hand-computed byte patterns, exact rational brute force,
 * numpy / scipy special cases, closed forms, the generator's reconstruction invariant.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* fp16 bit pattern -> the real number it denotes (subnormals, infinities and NaN included) */
double orc_half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0)        v = (double)frac * 0x1p-24;                 /* subnormal: frac * 2^-24 */
    else if (expo == 31)  v = frac ? NAN : INFINITY;
    else                  v = (1.0 + (double)frac * 0x1p-10) * ldexp(1.0, expo - 15);
    return sign ? -v : v;
}

static inline int stream_bit(const uint8_t *row, int64_t k) { return (row[k >> 3] >> (k & 7)) & 1; }

/* index of element j of a row: bits [j*b, j*b+b) of the row's stream, LSB first */
static inline int row_index(const uint8_t *row, int bits, int64_t j) {
    int v = 0;
    for (int t = 0; t < bits; ++t) v |= stream_bit(row, j * bits + t) << t;
    return v;
}

/* idx_out[i][j] = unpacked index */
void orc_unpack(int M, int N, int bits, const uint8_t *qidx, uint8_t *idx_out) {
    const int64_t row_bytes = (int64_t)N * bits / 8;
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j)
            idx_out[(int64_t)i * N + j] = (uint8_t)row_index(qidx + i * row_bytes, bits, j);
}

/* w_out[i][j] = lut[i][idx(i,j)] as an fp16 bit pattern (dequantisation is a pure selection) */
void orc_dequant(int M, int N, int bits, const uint8_t *qidx, const uint16_t *lut, uint16_t *w_out) {
    const int64_t row_bytes = (int64_t)N * bits / 8;
    const int K = 1 << bits;
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j)
            w_out[(int64_t)i * N + j] = lut[(int64_t)i * K + row_index(qidx + i * row_bytes, bits, j)];
}

/*
 * y[i][t] and absdot[i][t] for rows i in [row_begin, row_end).  Outputs are M x B row-major; rows outside
 * the range are left untouched.  qidx == NULL skips the dense term, nnz == 0 / rowptr == NULL the sparse one.
 * absdot may be NULL.  Duplicate (row, col) entries of the CSR matrix add up.
 */
void orc_matvec_rows(int M, int N, int bits, int B, int row_begin, int row_end,
                     const uint8_t *qidx, const uint16_t *lut,
                     int64_t nnz, const int32_t *rowptr, const int32_t *cols, const uint16_t *vals,
                     const uint16_t *x, double *y, double *absdot) {
    const int64_t row_bytes = (int64_t)N * bits / 8;
    const int K = 1 << bits;
    const int have_sparse = (nnz > 0 && rowptr && cols && vals);
    (void)M;
    #pragma omp parallel
    {
        double *weff = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        #pragma omp for schedule(static)
        for (int i = row_begin; i < row_end; ++i) {
            /* effective row of W in fp64: dense part ... */
            for (int j = 0; j < N; ++j)
                weff[j] = qidx ? orc_half_to_double(lut[(int64_t)i * K + row_index(qidx + i * row_bytes, bits, j)]) : 0.0;
            for (int t = 0; t < B; ++t) {
                double acc = 0.0;
                for (int j = 0; j < N; ++j) acc += weff[j] * orc_half_to_double(x[(int64_t)j * B + t]);
                /* ... plus the sparse term, entry by entry */
                if (have_sparse)
                    for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
                        acc += orc_half_to_double(vals[p]) * orc_half_to_double(x[(int64_t)cols[p] * B + t]);
                y[(int64_t)i * B + t] = acc;
            }
            if (absdot) {
                if (have_sparse)
                    for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) weff[cols[p]] += orc_half_to_double(vals[p]);
                for (int t = 0; t < B; ++t) {
                    double a = 0.0;
                    for (int j = 0; j < N; ++j) a += fabs(weff[j]) * fabs(orc_half_to_double(x[(int64_t)j * B + t]));
                    absdot[(int64_t)i * B + t] = a;
                }
            }
        }
        free(weff);
    }
}

void orc_matvec(int M, int N, int bits, int B, const uint8_t *qidx, const uint16_t *lut,
                int64_t nnz, const int32_t *rowptr, const int32_t *cols, const uint16_t *vals,
                const uint16_t *x, double *y, double *absdot) {
    orc_matvec_rows(M, N, bits, B, 0, M, qidx, lut, nnz, rowptr, cols, vals, x, y, absdot);
}

/* plain fp16 matrix times vector, fp64 (oracle for the fp16 comparison baseline) */
void orc_fp16_matvec(int M, int N, int B, const uint16_t *w, const uint16_t *x, double *y, double *absdot) {
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i)
        for (int t = 0; t < B; ++t) {
            double acc = 0.0, a = 0.0;
            for (int j = 0; j < N; ++j) {
                double wv = orc_half_to_double(w[(int64_t)i * N + j]), xv = orc_half_to_double(x[(int64_t)j * B + t]);
                acc += wv * xv; a += fabs(wv) * fabs(xv);
            }
            y[(int64_t)i * B + t] = acc;
            if (absdot) absdot[(int64_t)i * B + t] = a;
        }
}

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
