/*
 * sqgen — seeded synthetic generator of Dense-and-Sparse quantised layers.
 *
 * Stand-in for the paper's offline quantiser (Sec. 4.1-4.2): it produces, for an
 * M x N layer, the triple the inference kernels read (Sec. 4.3): a packed b-bit
 * index matrix, one look-up table of 2^b fp16 centroids per output row, and a
 * CSR matrix of fp16 outliers.  It is input plumbing for BOTH the CPU oracle and
 * the GPU library and contains none of the inference arithmetic (no unpacking,
 * no look-up, no dot products).
 *
 * Recipe (all choices are this build's, the paper fixes none of them):
 *   W0[i][j]  = fp16( 0.02 * T4 ),  T4 = Z / sqrt(V/4), Z ~ N(0,1) (Box-Muller),
 *               V ~ chi^2_4 = -2 ln(U1 U2); four counter-based uniforms per element.
 *   sparse set: either the global top-nnz |w| of the matrix (ties: row-major order)
 *               or per-row top-c_i |w| with prescribed skewed counts c_i
 *               (a seeded subset of ceil(h*M) "heavy" rows shares round(s*nnz)).
 *   centroids:  k-th of 2^b = order statistic at rank floor((k+0.5)/2^b * n_i) of the
 *               row's remaining values; made strictly ascending by one-ulp bumps.
 *   indices:    nearest centroid (ties -> lower index); at an extracted position the
 *               index of the centroid nearest to zero (the sparse entry then carries
 *               the full original value, so W_eff = lut[idx] + s there).
 *   packing:    row i is a little-endian bit stream; element j owns stream bits
 *               [j*b, j*b+b), least significant bit first; stream bit k is bit k%8
 *               of byte k/8.  Rows are laid end to end, no padding.
 *
 * Every output is a deterministic function of (shape, bits, frac, skew, seed): the
 * random stream is addressed by element index, so the thread count does not matter.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------- counter-based uniforms ---------------- */
static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31; return z;
}
static inline uint64_t rng_u64(uint64_t seed, uint64_t stream, uint64_t ctr) {
    uint64_t k = mix64(seed + 0x9E3779B97F4A7C15ull * (stream + 1));
    return mix64(k ^ mix64(ctr + 0xD1B54A32D192ED03ull));
}
static inline double rng_u01(uint64_t seed, uint64_t stream, uint64_t ctr) {
    /* strictly inside (0,1) */
    return ((double)(rng_u64(seed, stream, ctr) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

/* ---------------- fp16 helpers (bit patterns) ---------------- */
static uint16_t float_to_half_rne(float f) {
    uint32_t x; memcpy(&x, &f, 4);
    uint32_t sign = (x >> 16) & 0x8000u;
    uint32_t ax = x & 0x7FFFFFFFu;
    if (ax >= 0x7F800000u) return (uint16_t)(sign | (ax > 0x7F800000u ? 0x7E00u : 0x7C00u));
    if (ax >= 0x477FF000u) return (uint16_t)(sign | 0x7BFFu);   /* clamp to max finite */
    if (ax < 0x33000001u) return (uint16_t)sign;               /* rounds to zero */
    int e = (int)(ax >> 23) - 127;
    uint32_t man = (ax & 0x7FFFFFu) | 0x800000u;
    int shift; uint32_t base;
    if (e < -14) { shift = 13 + (-14 - e); base = 0; }          /* subnormal half */
    else         { shift = 13; base = (uint32_t)(e + 15) << 10; man &= 0x7FFFFFu; }
    uint32_t q = man >> shift;
    uint32_t rem = man & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    uint32_t h = base + q;
    if (rem > half || (rem == half && (q & 1u))) h += 1;        /* carries propagate correctly */
    if (h > 0x7BFFu) h = 0x7BFFu;
    return (uint16_t)(sign | h);
}
static double half_to_double(uint16_t h) {
    int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m + 1024), e - 25);
    return s ? -v : v;
}
/* monotone key: a < b as reals  <=>  key(a) < key(b)  (with -0 < +0) */
static inline uint16_t half_key(uint16_t h) { return (h & 0x8000u) ? (uint16_t)~h : (uint16_t)(h | 0x8000u); }
static inline uint16_t key_half(uint16_t k) { return (k & 0x8000u) ? (uint16_t)(k & 0x7FFFu) : (uint16_t)~k; }

/* LSD radix sort of 16-bit keys, ascending */
static void sort_u16(uint16_t *a, uint16_t *tmp, int n) {
    int cnt[256];
    for (int pass = 0; pass < 2; ++pass) {
        int sh = pass * 8;
        memset(cnt, 0, sizeof cnt);
        for (int i = 0; i < n; ++i) cnt[(a[i] >> sh) & 255]++;
        int s = 0;
        for (int k = 0; k < 256; ++k) { int c = cnt[k]; cnt[k] = s; s += c; }
        for (int i = 0; i < n; ++i) tmp[cnt[(a[i] >> sh) & 255]++] = a[i];
        memcpy(a, tmp, (size_t)n * 2);
    }
}

/* ---------------- public: raw weights and activations ---------------- */
void sqgen_weights(int M, int N, uint64_t seed, uint16_t *w16) {
    const int64_t total = (int64_t)M * N;
    #pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        double u1 = rng_u01(seed, 0, 4 * (uint64_t)e + 0);
        double u2 = rng_u01(seed, 0, 4 * (uint64_t)e + 1);
        double u3 = rng_u01(seed, 0, 4 * (uint64_t)e + 2);
        double u4 = rng_u01(seed, 0, 4 * (uint64_t)e + 3);
        double z = sqrt(-2.0 * log(u3)) * cos(6.283185307179586476925 * u4);
        double v = -2.0 * log(u1 * u2);
        double t = z / sqrt(v / 4.0);
        w16[e] = float_to_half_rne((float)(0.02 * t));
    }
}

/* x[j][t], N x B row-major, N(0,1) rounded to fp16 */
void sqgen_x(int N, int B, uint64_t seed, uint16_t *x16) {
    const int64_t total = (int64_t)N * B;
    for (int64_t e = 0; e < total; ++e) {
        double u1 = rng_u01(seed, 1, 2 * (uint64_t)e + 0);
        double u2 = rng_u01(seed, 1, 2 * (uint64_t)e + 1);
        double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
        x16[e] = float_to_half_rne((float)z);
    }
}

/* Synthetic per-weight sensitivities (stand-in for the diagonal Fisher information of Sec. 4.1, which needs a
 * model and calibration data): squared-gradient-like values g^2 with g = z1 * exp(0.75 z2), heavy-tailed so that
 * a few weights of every row dominate, scaled by 64 and stored as 16-bit unsigned integers (saturating). */
void sqgen_sens(int M, int N, uint64_t seed, uint16_t *s16) {
    const int64_t total = (int64_t)M * N;
    #pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        double u1 = rng_u01(seed, 7, 4 * (uint64_t)e + 0);
        double u2 = rng_u01(seed, 7, 4 * (uint64_t)e + 1);
        double u3 = rng_u01(seed, 7, 4 * (uint64_t)e + 2);
        double u4 = rng_u01(seed, 7, 4 * (uint64_t)e + 3);
        double z1 = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
        double z2 = sqrt(-2.0 * log(u3)) * cos(6.283185307179586476925 * u4);
        double v = floor(64.0 * z1 * z1 * exp(1.5 * z2));
        s16[e] = (uint16_t)(v > 65535.0 ? 65535.0 : v);
    }
}

/* number of sparse entries for a sparsity level */
int64_t sqgen_nnz(int M, int N, double frac) { return llround(frac * (double)M * (double)N); }

/* ---------------- per-row extraction counts ---------------- */
typedef struct { uint64_t key; int row; } keyrow;
static int cmp_keyrow(const void *a, const void *b) {
    const keyrow *x = a, *y = b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return (x->row > y->row) - (x->row < y->row);
}

/* skewed counts: ceil(h*M) seeded "heavy" rows share round(s*nnz) evenly (remainder to the
 * lowest row ids of the group), the other rows share the rest the same way. */
int sqgen_counts_skewed(int M, int N, int64_t nnz, double h, double s, uint64_t seed, int32_t *counts) {
    int nh = (int)ceil(h * (double)M - 1e-9);
    if (nh < 0) nh = 0; if (nh > M) nh = M;
    int64_t heavy_total = (nh > 0) ? llround(s * (double)nnz) : 0;
    if (nh == M) heavy_total = nnz;
    int64_t light_total = nnz - heavy_total;
    keyrow *kr = malloc(sizeof(keyrow) * (size_t)M);
    uint8_t *is_heavy = calloc((size_t)M, 1);
    if (!kr || !is_heavy) { free(kr); free(is_heavy); return -1; }
    for (int i = 0; i < M; ++i) { kr[i].key = rng_u64(seed, 2, (uint64_t)i); kr[i].row = i; }
    qsort(kr, (size_t)M, sizeof(keyrow), cmp_keyrow);
    for (int r = 0; r < nh; ++r) is_heavy[kr[r].row] = 1;
    int nl = M - nh;
    int64_t hb = nh ? heavy_total / nh : 0, hr = nh ? heavy_total % nh : 0;
    int64_t lb = nl ? light_total / nl : 0, lr = nl ? light_total % nl : 0;
    int64_t seen_h = 0, seen_l = 0; int ok = 0;
    for (int i = 0; i < M; ++i) {
        int64_t c;
        if (is_heavy[i]) { c = hb + (seen_h < hr); ++seen_h; }
        else             { c = lb + (seen_l < lr); ++seen_l; }
        if (c > N) ok = -2;
        counts[i] = (int32_t)c;
    }
    free(kr); free(is_heavy);
    return ok;
}

/* global rule: the nnz largest |w| of the whole matrix; ties at the threshold are taken in
 * row-major order.  Writes per-row counts and a per-element flag (1 = extracted). */
int sqgen_select_global(int M, int N, int64_t nnz, const uint16_t *w16, int32_t *counts, uint8_t *flag) {
    const int64_t total = (int64_t)M * N;
    int64_t *hist = calloc(32768, sizeof(int64_t));
    if (!hist) return -1;
    for (int64_t e = 0; e < total; ++e) hist[w16[e] & 0x7FFFu]++;
    int64_t above = 0; int T = 32768;             /* T = threshold abs pattern */
    while (T > 0 && above + hist[T - 1] <= nnz) { --T; above += hist[T]; }
    /* now: count(abs >= T) = above <= nnz, and adding pattern T-1 would exceed nnz */
    int64_t ties_needed = nnz - above; int tie_pat = T - 1;
    free(hist);
    memset(flag, 0, (size_t)total);
    for (int i = 0; i < M; ++i) {
        int c = 0;
        for (int j = 0; j < N; ++j) {
            int a = w16[(int64_t)i * N + j] & 0x7FFF;
            int take = 0;
            if (a >= T) take = 1;
            else if (a == tie_pat && ties_needed > 0) { take = 1; --ties_needed; }
            if (take) { flag[(int64_t)i * N + j] = 1; ++c; }
        }
        counts[i] = c;
    }
    return 0;
}

/* per-row rule: the counts[i] largest |w| of row i; ties at the threshold -> lower column first */
void sqgen_select_rows(int M, int N, const uint16_t *w16, const int32_t *counts, uint8_t *flag) {
    #pragma omp parallel
    {
        uint16_t *k = malloc((size_t)N * 2), *tmp = malloc((size_t)N * 2);
        #pragma omp for schedule(dynamic, 16)
        for (int i = 0; i < M; ++i) {
            const uint16_t *w = w16 + (int64_t)i * N; uint8_t *f = flag + (int64_t)i * N;
            int c = counts[i];
            memset(f, 0, (size_t)N);
            if (c <= 0) continue;
            for (int j = 0; j < N; ++j) k[j] = w[j] & 0x7FFFu;
            sort_u16(k, tmp, N);
            int T = k[N - c];                         /* c-th largest abs pattern */
            int gt = 0; for (int j = 0; j < N; ++j) gt += ((w[j] & 0x7FFF) > T);
            int ties = c - gt;
            for (int j = 0; j < N; ++j) {
                int a = w[j] & 0x7FFF;
                if (a > T) f[j] = 1;
                else if (a == T && ties > 0) { f[j] = 1; --ties; }
            }
        }
        free(k); free(tmp);
    }
}

/* ---------------- quantise + pack ---------------- */
/* Inputs: w16, flag (1 = goes to the sparse matrix), counts (per-row sum of flag).
 * Outputs: qidx (M*N*bits/8 bytes), lut (M * 2^bits fp16), rowptr (M+1), cols/vals (nnz),
 * optional idx_out (M*N bytes) and wgen_out (M*N doubles = lut[idx] + extracted value). */
int sqgen_quantize(int M, int N, int bits, const uint16_t *w16, const uint8_t *flag, const int32_t *counts,
                   uint8_t *qidx, uint16_t *lut, int32_t *rowptr, int32_t *cols, uint16_t *vals,
                   uint8_t *idx_out, double *wgen_out) {
    if (bits < 1 || bits > 8) return -1;
    const int K = 1 << bits;
    if (((int64_t)N * bits) % 8 != 0) return -2;
    const int64_t row_bytes = (int64_t)N * bits / 8;
    rowptr[0] = 0;
    for (int i = 0; i < M; ++i) rowptr[i + 1] = rowptr[i] + counts[i];
    int err = 0;
    #pragma omp parallel
    {
        uint16_t *k = malloc((size_t)N * 2), *tmp = malloc((size_t)N * 2);
        uint8_t *idx = malloc((size_t)N);
        #pragma omp for schedule(dynamic, 16)
        for (int i = 0; i < M; ++i) {
            const uint16_t *w = w16 + (int64_t)i * N; const uint8_t *f = flag + (int64_t)i * N;
            /* remaining values, sorted ascending as reals */
            int n = 0;
            for (int j = 0; j < N; ++j) if (!f[j]) k[n++] = half_key(w[j]);
            if (n < 1) { err = 1; continue; }
            sort_u16(k, tmp, n);
            uint16_t cen[256]; double cend[256];
            for (int c = 0; c < K; ++c) {
                int64_t r = (int64_t)floor(((double)c + 0.5) / (double)K * (double)n);
                if (r >= n) r = n - 1;
                uint16_t key = k[r];
                if (c > 0) {                          /* keep strictly ascending as reals */
                    uint16_t prev = half_key(cen[c - 1]);
                    while (key <= prev || half_to_double(key_half(key)) <= cend[c - 1]) ++key;
                }
                cen[c] = key_half(key); cend[c] = half_to_double(cen[c]);
                lut[(int64_t)i * K + c] = cen[c];
            }
            int zero_idx = 0;                         /* centroid nearest to zero, ties -> lower */
            for (int c = 1; c < K; ++c) if (fabs(cend[c]) < fabs(cend[zero_idx])) zero_idx = c;
            int p = rowptr[i];
            for (int j = 0; j < N; ++j) {
                if (f[j]) { idx[j] = (uint8_t)zero_idx; cols[p] = j; vals[p] = w[j]; ++p; continue; }
                double v = half_to_double(w[j]);
                int best = 0; double bd = fabs(v - cend[0]);
                for (int c = 1; c < K; ++c) { double d = fabs(v - cend[c]); if (d < bd) { bd = d; best = c; } }
                idx[j] = (uint8_t)best;
            }
            if (wgen_out) {
                double *wg = wgen_out + (int64_t)i * N;
                for (int j = 0; j < N; ++j) wg[j] = cend[idx[j]] + (f[j] ? half_to_double(w[j]) : 0.0);
            }
            if (idx_out) memcpy(idx_out + (int64_t)i * N, idx, (size_t)N);
            /* pack, one bit at a time */
            uint8_t *q = qidx + (int64_t)i * row_bytes;
            memset(q, 0, (size_t)row_bytes);
            for (int j = 0; j < N; ++j)
                for (int t = 0; t < bits; ++t)
                    if ((idx[j] >> t) & 1) { int64_t sb = (int64_t)j * bits + t; q[sb >> 3] |= (uint8_t)(1u << (sb & 7)); }
        }
        free(k); free(tmp); free(idx);
    }
    return err;
}

/* pack an arbitrary index matrix (tests build hand-made layers with it) */
int sqgen_pack(int M, int N, int bits, const uint8_t *idx, uint8_t *qidx) {
    if (((int64_t)N * bits) % 8 != 0) return -2;
    const int64_t row_bytes = (int64_t)N * bits / 8;
    memset(qidx, 0, (size_t)(row_bytes * M));
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j)
            for (int t = 0; t < bits; ++t)
                if ((idx[(int64_t)i * N + j] >> t) & 1) {
                    int64_t sb = (int64_t)j * bits + t;
                    qidx[i * row_bytes + (sb >> 3)] |= (uint8_t)(1u << (sb & 7));
                }
    return 0;
}

int sqgen_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
