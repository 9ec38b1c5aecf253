// Offline side for gfx950: Dense-and-Sparse split and sensitivity-weighted k-means (paper Sec. 4.1-4.2) -- device code.
//
// What is computed, per weight matrix W (fp16, M x N) with per-weight sensitivities s (16-bit unsigned, the
// stand-in for the diagonal Fisher information of Eq. 4):
//   1. Thresholds (Sec. 4.2, "T_min / T_max from the percentile of the distribution"): the n_lo-th smallest and
//      the n_hi-th largest weight and the n_sens-th largest sensitivity of the whole matrix, found exactly with two
//      passes of 256-bin histograms over monotone 16-bit keys (high byte, then low byte inside the selected bin).
//   2. The split: a weight goes to the sparse matrix S iff it lies strictly outside [T_min, T_max] or its
//      sensitivity is strictly above the sensitivity threshold; S is written in CSR (count per row, scan, ordered fill).
//   3. Per output row, weighted 1-D k-means over the remaining weights (Eq. 4: minimise sum_j s_j (w_j - Q(w_j))^2
//      over 2^b values) by Lloyd iterations: equal-count start, nearest-centroid assignment, sensitivity-weighted
//      means.  Every integer decision is taken in fp32 exactly as written below and the weighted sums are exact
//      64-bit integers, so the result does not depend on the order of the additions.  The row is sorted once and
//      the iterations move the K - 1 cluster boundaries (see quant_kmeans_kernel).
//   4. fp16 tables, final indices (nearest table entry in exact arithmetic, ties to the lower index; an extracted
//      position gets the entry nearest to zero) and the packed index stream in the layout the matvec reads.
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>

#include "sqllm_kernels.h"

namespace sqllm {

typedef uint32_t u32;
typedef unsigned long long u64;
typedef long long i64;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

// monotone key: a < b as reals  =>  key(a) < key(b)  (-0 sorts below +0)
__device__ __forceinline__ u32 half_key(u32 h) { return (h & 0x8000u) ? (~h & 0xFFFFu) : (h | 0x8000u); }
__device__ __forceinline__ u32 key_half(u32 k) { return (k & 0x8000u) ? (k & 0x7FFFu) : (~k & 0xFFFFu); }
__device__ __forceinline__ float half_bits_to_f32(u32 h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }
// exact value of a finite fp16 bit pattern times 2^24
__device__ __forceinline__ i64 half_to_fixed(u32 h) {
    const u32 e = (h >> 10) & 31u, m = h & 1023u;
    const i64 mag = e == 0 ? (i64)m : ((i64)(m + 1024u) << (e - 1u));
    return (h & 0x8000u) ? -mag : mag;
}

// Workspace layout (32-bit words)
constexpr int kWsHist1W = 0, kWsHist1S = 256, kWsHist2 = 512 /* 3 x 256 */, kWsSel = 1280 /* 3 x (bin, residual lo, residual hi) + pad */,
              kWsThr = 1296 /* key_min, key_max, s_thr */, kWsWords = 1312;

__global__ void __launch_bounds__(256) quant_clear_kernel(u32* ws) {
    for (int i = threadIdx.x + blockIdx.x * blockDim.x; i < kWsWords; i += blockDim.x * gridDim.x) ws[i] = 0;
}

// pass 1: histograms of the high bytes of all weight keys and of all sensitivities
__global__ void __launch_bounds__(256) quant_hist1_kernel(long long units, const u32x4* __restrict__ w, const u32x4* __restrict__ s, u32* __restrict__ ws) {
    // eight copies of each histogram, picked by the lane, so that the lanes of a wave seldom add to one address
    __shared__ u32 hw8[8][256], hs8[8][256];
#pragma unroll
    for (int c = 0; c < 8; ++c) { hw8[c][threadIdx.x] = 0; hs8[c][threadIdx.x] = 0; }
    u32* hw = hw8[threadIdx.x & 7];
    u32* hs = hs8[threadIdx.x & 7];
    __syncthreads();
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < units; i += (long long)gridDim.x * blockDim.x) {
        const u32x4 wv = w[i], sv = s[i];
        const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            atomicAdd(&hw[half_key(wd[k] & 0xFFFFu) >> 8], 1u); atomicAdd(&hw[half_key(wd[k] >> 16) >> 8], 1u);
            atomicAdd(&hs[(sd[k] & 0xFFFFu) >> 8], 1u); atomicAdd(&hs[sd[k] >> 24], 1u);
        }
    }
    __syncthreads();
    u32 tw = 0, ts = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) { tw += hw8[c][threadIdx.x]; ts += hs8[c][threadIdx.x]; }
    if (tw) atomicAdd(&ws[kWsHist1W + threadIdx.x], tw);
    if (ts) atomicAdd(&ws[kWsHist1S + threadIdx.x], ts);
}

// Bin holding the element of rank r (0-based) in a 256-bin histogram, and the rank inside that bin; called by all 256
// threads of the block, thread t owning bin t.  The bin is the one whose running count first exceeds r.
__device__ __forceinline__ void select_bin(u32 mine, u64 r, u64* scan /* [256] in LDS */, u32& bin, u64& residual) {
    const int t = threadIdx.x;
    scan[t] = mine;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const u64 v = t >= off ? scan[t - off] : 0;
        __syncthreads();
        scan[t] += v;
        __syncthreads();
    }
    const u64 incl = scan[t], excl = incl - mine;
    __shared__ u32 sel_bin;
    __shared__ u64 sel_res;
    if (t == 0) { sel_bin = 255; sel_res = 0; }                      // rank past the end (cannot happen for valid counts)
    __syncthreads();
    if (r >= excl && r < incl) { sel_bin = (u32)t; sel_res = r - excl; }
    __syncthreads();
    bin = sel_bin; residual = sel_res;
    __syncthreads();
}

__global__ void __launch_bounds__(256) quant_select1_kernel(u64 total, u64 n_lo, u64 n_hi, u64 n_sens, u32* ws) {
    __shared__ u64 scan[256];
    const u32 hw = ws[kWsHist1W + threadIdx.x], hs = ws[kWsHist1S + threadIdx.x];
    for (int t = 0; t < 3; ++t) {
        const u64 rank = t == 0 ? n_lo : (t == 1 ? total - 1 - n_hi : total - 1 - n_sens);
        u32 bin; u64 res;
        select_bin(t < 2 ? hw : hs, rank, scan, bin, res);
        if (threadIdx.x == 0) { ws[kWsSel + 4 * t] = bin; ws[kWsSel + 4 * t + 1] = (u32)res; ws[kWsSel + 4 * t + 2] = (u32)(res >> 32); }
    }
}

// pass 2: histograms of the low bytes inside the three selected bins
__global__ void __launch_bounds__(256) quant_hist2_kernel(long long units, const u32x4* __restrict__ w, const u32x4* __restrict__ s, u32* __restrict__ ws) {
    __shared__ u32 h[3][256];
    h[0][threadIdx.x] = 0; h[1][threadIdx.x] = 0; h[2][threadIdx.x] = 0;
    const u32 bin_min = ws[kWsSel], bin_max = ws[kWsSel + 4], bin_s = ws[kWsSel + 8];
    __syncthreads();
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < units; i += (long long)gridDim.x * blockDim.x) {
        const u32x4 wv = w[i], sv = s[i];
        const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const u32 key = half_key(hh ? wd[k] >> 16 : wd[k] & 0xFFFFu), sv16 = hh ? sd[k] >> 16 : sd[k] & 0xFFFFu;
                if ((key >> 8) == bin_min) atomicAdd(&h[0][key & 255u], 1u);
                if ((key >> 8) == bin_max) atomicAdd(&h[1][key & 255u], 1u);
                if ((sv16 >> 8) == bin_s) atomicAdd(&h[2][sv16 & 255u], 1u);
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 3; ++t)
        if (h[t][threadIdx.x]) atomicAdd(&ws[kWsHist2 + 256 * t + threadIdx.x], h[t][threadIdx.x]);
}

__global__ void __launch_bounds__(256) quant_select2_kernel(u32* ws) {
    __shared__ u64 scan[256];
    for (int t = 0; t < 3; ++t) {
        const u64 r = (u64)ws[kWsSel + 4 * t + 1] | ((u64)ws[kWsSel + 4 * t + 2] << 32);
        u32 lo; u64 res;
        select_bin(ws[kWsHist2 + 256 * t + threadIdx.x], r, scan, lo, res);
        if (threadIdx.x == 0) ws[kWsThr + t] = (ws[kWsSel + 4 * t] << 8) | lo;
    }
}

__device__ __forceinline__ bool is_extracted(u32 wbits, u32 sv, u32 key_min, u32 key_max, u32 s_thr) {
    const u32 key = half_key(wbits);
    return key < key_min || key > key_max || sv > s_thr;
}

// extracted entries per row -> rowptr[row + 1]; one wave per row
__global__ void __launch_bounds__(256) quant_count_kernel(int M, int N, const uint16_t* __restrict__ w, const uint16_t* __restrict__ s, const u32* __restrict__ ws, int* __restrict__ rowptr) {
    const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const u32 key_min = ws[kWsThr], key_max = ws[kWsThr + 1], s_thr = ws[kWsThr + 2];
    const u32x4* wr = reinterpret_cast<const u32x4*>(w + (size_t)row * N);
    const u32x4* sr = reinterpret_cast<const u32x4*>(s + (size_t)row * N);
    int cnt = 0;
    for (int i = lane; i < N / 8; i += 64) {
        const u32x4 wv = wr[i], sv = sr[i];
        const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
            cnt += (int)is_extracted(wd[k] & 0xFFFFu, sd[k] & 0xFFFFu, key_min, key_max, s_thr) + (int)is_extracted(wd[k] >> 16, sd[k] >> 16, key_min, key_max, s_thr);
    }
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off, 64);
    if (lane == 0) rowptr[row + 1] = cnt;
    if (row == 0 && lane == 0) rowptr[0] = 0;
}

// in-place inclusive scan of rowptr[1 .. M]; one block of 1024 threads
__global__ void __launch_bounds__(1024) quant_scan_kernel(int M, int* __restrict__ rowptr) {
    __shared__ int sums[1024];
    const int per = (M + 1023) / 1024;
    const int b = threadIdx.x * per, e = min(b + per, M);
    int local = 0;
    for (int i = b; i < e; ++i) local += rowptr[i + 1];
    sums[threadIdx.x] = local;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {                       // Hillis-Steele inclusive scan
        const int v = threadIdx.x >= off ? sums[threadIdx.x - off] : 0;
        __syncthreads();
        sums[threadIdx.x] += v;
        __syncthreads();
    }
    int run = sums[threadIdx.x] - local;
    for (int i = b; i < e; ++i) { run += rowptr[i + 1]; rowptr[i + 1] = run; }
}

// Sum of a 32-bit integer over the 64 lanes with DPP moves (no LDS traffic), returned as a uniform value.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_add(int v) { return v + __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false); }
__device__ __forceinline__ int wave_sum_i32(int v) {
    v = dpp_add<0xB1>(v);            // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);            // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);           // row_half_mirror
    v = dpp_add<0x140>(v);           // row_mirror: every lane holds the sum of its row of 16
    v = dpp_add<0x142, 0xA>(v);      // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);      // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    return __builtin_amdgcn_readlane(v, 63);
}
// The three sums a boundary needs over the lanes' (sensitivity, product) pairs -- sum s, sum of the low words and sum of
// the high words of the products p = s * w * 2^24 -- from four 32-bit reductions: s < 2^16 and |p| < 2^57, so the 16-bit
// halves of the low word and the (signed) high word all add up over 64 lanes without overflow.
__device__ __forceinline__ void wave_sums(u32 sv, i64 p, u64& s0, u64& lo, u64& hi) {
    const u32 plo = (u32)((u64)p & 0xFFFFFFFFull);
    const int phi = (int)(p >> 32);
    const u32 a = (u32)wave_sum_i32((int)(plo & 0xFFFFu)), b = (u32)wave_sum_i32((int)(plo >> 16));
    s0 = (u64)(u32)wave_sum_i32((int)sv);
    lo = (u64)a + ((u64)b << 16);
    hi = (u64)(i64)wave_sum_i32(phi);
}

__device__ __forceinline__ u32 umin(u32 a, u32 b) { return a < b ? a : b; }
__device__ __forceinline__ u32 umax(u32 a, u32 b) { return a < b ? b : a; }

// The sort is a bitonic network in its all-ascending form: the merge of size k first compares word i of the lower half
// with its MIRROR image k - 1 - i in the upper half, then runs the usual half-cleaners of distance k/4, k/8, ... 1.  Every
// comparator puts the smaller word at the lower index, so words past the end of the row, thought of as +infinity, never
// move and comparators reaching past the end are simply skipped: the cost follows N, not the next power of two.
// Steps with distances below 16 stay inside aligned blocks of 16 words; a thread runs them in registers:
// FULL: the whole merges k = 2, 4, 8, 16 (start of the sort);  otherwise the half-cleaners 8, 4, 2, 1 of a later merge.
template <bool FULL>
__device__ __forceinline__ void sort_block_steps(u32* __restrict__ A, int blk) {
    u32 v[16];
    u32x4* src = reinterpret_cast<u32x4*>(A + 16 * blk);
#pragma unroll
    for (int i = 0; i < 4; ++i) { const u32x4 t4 = src[i]; v[4 * i] = t4.x; v[4 * i + 1] = t4.y; v[4 * i + 2] = t4.z; v[4 * i + 3] = t4.w; }
    auto cx = [&](int a, int b) { const u32 lo = umin(v[a], v[b]), hi = umax(v[a], v[b]); v[a] = lo; v[b] = hi; };
    if constexpr (FULL) {
#pragma unroll
        for (int k = 2; k <= 16; k <<= 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {                                // mirror step of merge k
                const int base = (i / (k / 2)) * k, off = i % (k / 2);
                cx(base + off, base + k - 1 - off);
            }
#pragma unroll
            for (int j = k >> 2; j > 0; j >>= 1) {
#pragma unroll
                for (int i = 0; i < 8; ++i) cx(2 * i - (i & (j - 1)), 2 * i - (i & (j - 1)) + j);
            }
        }
    } else {
#pragma unroll
        for (int j = 8; j > 0; j >>= 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) cx(2 * i - (i & (j - 1)), 2 * i - (i & (j - 1)) + j);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) src[i] = u32x4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
}

// One block of 256 threads per row.  In one dimension the clusters of Lloyd's method are intervals of the sorted
// weights, so the row is sorted once and every iteration only moves K - 1 boundaries:
//   * LDS holds the row's dense weights as (key << 16 | sensitivity), sorted ascending by a bitonic network
//     (extracted positions are 0xFFFFFFFF and end up behind the dense ones; the network skips what lies past the row),
//     and the running sums (sum s, low and high words of sum s w 2^24) in front of every chunk of 64 sorted weights.
//   * A boundary position p_k = #{ j : fp32(2 w_j) <= fp32(c_k + c_{k+1}) } is found by a 64-way search (every lane
//     probes one position per round, three rounds cover 2^18 weights); the sums in front of p_k are the chunk's running
//     sums plus a wave reduction over the part of the chunk before p_k; cluster sums are differences of neighbours.
//     These are the same decisions and the same exact integer sums as a pass over all weights, hence the same result.
//   * "No weight changed its cluster" is "no boundary position moved".
// The final indices and the packed stream are produced from the row as it lies in memory.
template <int BITS, int T>
__global__ void __launch_bounds__(T) quant_kmeans_kernel(int M, int N, int NP, int max_iter, const uint16_t* __restrict__ w, const uint16_t* __restrict__ sens,
                                                         const u32* __restrict__ ws, const int* __restrict__ rowptr, void* __restrict__ qidx,
                                                         uint16_t* __restrict__ lut, int* __restrict__ cols, uint16_t* __restrict__ vals, int* __restrict__ iters) {
    constexpr int K = 1 << BITS;
    extern __shared__ __align__(16) char smem[];
    u32* A = reinterpret_cast<u32*>(smem);                           // [N]; NP (the next power of two) only bounds the sort's merges
    const int NC = N / 64;
    u64* c0 = reinterpret_cast<u64*>(A + N);                        // [NC + 1] running sum of s in front of chunk c
    u64* clo = c0 + (NC + 1);                                        // low words of s * w * 2^24
    u64* chi = clo + (NC + 1);                                       // high words (two's complement)
    __shared__ u64 F0[K + 1], Flo[K + 1], Fhi[K + 1];
    __shared__ float cen[K], thr2[K];
    __shared__ i64 cfix[K];
    __shared__ int scan[T], pos[K + 1], prevpos[K + 1], flag;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, row = blockIdx.x;
    const u32 key_min = ws[kWsThr], key_max = ws[kWsThr + 1], s_thr = ws[kWsThr + 2];
    const uint16_t* __restrict__ wrow = w + (size_t)row * N;
    const uint16_t* __restrict__ srow = sens + (size_t)row * N;

    // ---- 1. the row into LDS as sortable words; extracted positions become 0xFFFFFFFF
    {
        const u32x4* wr = reinterpret_cast<const u32x4*>(wrow);
        const u32x4* sr = reinterpret_cast<const u32x4*>(srow);
        for (int i = tid; i < N / 8; i += T) {
            u32 out[8];
            {
                const u32x4 wv = wr[i], sv = sr[i];
                const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32 w0 = wd[k] & 0xFFFFu, w1 = wd[k] >> 16, s0 = sd[k] & 0xFFFFu, s1 = sd[k] >> 16;
                    out[2 * k] = is_extracted(w0, s0, key_min, key_max, s_thr) ? 0xFFFFFFFFu : (half_key(w0) << 16) | s0;
                    out[2 * k + 1] = is_extracted(w1, s1, key_min, key_max, s_thr) ? 0xFFFFFFFFu : (half_key(w1) << 16) | s1;
                }
            }
            reinterpret_cast<u32x4*>(A)[2 * i] = u32x4{out[0], out[1], out[2], out[3]};
            reinterpret_cast<u32x4*>(A)[2 * i + 1] = u32x4{out[4], out[5], out[6], out[7]};
        }
    }
    __syncthreads();

    // ---- 2. CSR entries of the row, columns ascending: thread t owns the columns [t C, (t + 1) C)
    const int C = (N + T - 1) / T;
    const int jb = min(tid * C, N), je = min(jb + C, N);
    int mine = 0;
    for (int j = jb; j < je; ++j) mine += A[j] == 0xFFFFFFFFu;
    scan[tid] = mine;
    __syncthreads();
    for (int off = 1; off < T; off <<= 1) {
        const int v = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    const int n_dense = N - scan[T - 1];
    {
        int o = rowptr[row] + scan[tid] - mine;
        for (int j = jb; j < je; ++j)
            if (A[j] == 0xFFFFFFFFu) { cols[o] = j; vals[o] = wrow[j]; ++o; }
    }
    __syncthreads();

    // ---- 3. sort, ascending (see sort_block_steps): only the first N words take part; distances >= 16 go through LDS,
    //         one step per barrier
    for (int blk = tid; blk < N / 16; blk += T) sort_block_steps<true>(A, blk);       // merges k = 2 .. 16
    __syncthreads();
    // Steps with distances >= 16 through LDS.  A thread takes four NEIGHBOURING comparators at a time -- their lower words
    // are one 16-byte chunk and so are their upper words (in reverse order for the mirror step) -- and kSortBatch such
    // quads per round: all loads, then all stores.  Index arithmetic, LDS instructions and round trips are shared by four
    // comparators, and the 16-byte accesses of neighbouring lanes are conflict-free.
    constexpr int kSortBatch = 2;
    auto lds_step = [&](auto quad_of, bool mirror) {
        for (int g0 = tid; g0 < NP / 8; g0 += kSortBatch * T) {
            int a[kSortBatch], b[kSortBatch];
            u32x4 va[kSortBatch], vb[kSortBatch];
            bool live[kSortBatch];
#pragma unroll
            for (int u = 0; u < kSortBatch; ++u) {
                quad_of(4 * (g0 + u * T), a[u], b[u]);                   // first words of the two chunks (multiples of 4)
                live[u] = g0 + u * T < NP / 8 && b[u] < N;               // a < b always; N is a multiple of 4
                if (live[u]) { va[u] = *reinterpret_cast<const u32x4*>(A + a[u]); vb[u] = *reinterpret_cast<const u32x4*>(A + b[u]); }
            }
#pragma unroll
            for (int u = 0; u < kSortBatch; ++u) {
                if (live[u]) {
                    const u32x4 x = va[u];
                    const u32x4 y = mirror ? u32x4{vb[u].w, vb[u].z, vb[u].y, vb[u].x} : vb[u];
                    const u32x4 lo = {umin(x.x, y.x), umin(x.y, y.y), umin(x.z, y.z), umin(x.w, y.w)};
                    const u32x4 hi = {umax(x.x, y.x), umax(x.y, y.y), umax(x.z, y.z), umax(x.w, y.w)};
                    *reinterpret_cast<u32x4*>(A + a[u]) = lo;
                    *reinterpret_cast<u32x4*>(A + b[u]) = mirror ? u32x4{hi.w, hi.z, hi.y, hi.x} : hi;
                }
            }
            if (a[0] >= N) break;                                        // a grows with the quad index
        }
        __syncthreads();
    };
    for (int k = 32; k <= NP; k <<= 1) {
        const int hk = k >> 1;
        // mirror step: word off of the lower half against word k - 1 - off of the upper half of every group of k; the four
        // partners of the words off .. off + 3 are the chunk that starts at k - 4 - off, read backwards
        lds_step([&](int i, int& a, int& b) { const int base = (i / hk) * k, off = i & (hk - 1); a = base + off; b = base + k - 4 - off; }, true);
        for (int j = k >> 2; j >= 16; j >>= 1)
            lds_step([&](int i, int& a, int& b) { a = 2 * i - (i & (j - 1)); b = a + j; }, false);
        for (int blk = tid; blk < N / 16; blk += T) sort_block_steps<false>(A, blk);  // half-cleaners 8, 4, 2, 1
        __syncthreads();
    }

    // ---- 4. running sums in front of every chunk of 64 sorted weights
    const int nchunks = (n_dense + 63) / 64;
    for (int c = wave; c < nchunks; c += T / 64) {
        const int j = c * 64 + lane;
        u32 sv = 0;
        i64 p = 0;
        if (j < n_dense) {
            const u32 v = A[j];
            sv = v & 0xFFFFu;
            p = (i64)sv * half_to_fixed(key_half(v >> 16));
        }
        u64 s0, lo, hi;
        wave_sums(sv, p, s0, lo, hi);
        if (lane == 0) { c0[c + 1] = s0; clo[c + 1] = lo; chi[c + 1] = hi; }
    }
    __syncthreads();
    if (wave == 0) {
        // running sums over the chunks: every lane of wave 0 takes a run of consecutive chunks, the runs are chained with
        // a prefix sum across the lanes
        const int per = (nchunks + 63) / 64;
        const int cb = min(1 + lane * per, nchunks + 1), ce = min(cb + per, nchunks + 1);
        u64 t0 = 0, tl = 0, th = 0;
        for (int c = cb; c < ce; ++c) { t0 += c0[c]; tl += clo[c]; th += chi[c]; }
        u64 p0 = t0, pl = tl, ph = th;
        for (int off = 1; off < 64; off <<= 1) {
            const u64 u0 = (u64)__shfl_up((long long)p0, off, 64), ul = (u64)__shfl_up((long long)pl, off, 64), uh = (u64)__shfl_up((long long)ph, off, 64);
            if (lane >= off) { p0 += u0; pl += ul; ph += uh; }
        }
        u64 r0 = p0 - t0, rl = pl - tl, rh = ph - th;                    // sums in front of the lane's run
        for (int c = cb; c < ce; ++c) { r0 += c0[c]; rl += clo[c]; rh += chi[c]; c0[c] = r0; clo[c] = rl; chi[c] = rh; }
        if (lane == 0) { c0[0] = 0; clo[0] = 0; chi[0] = 0; }
    }
    // ---- 5. equal-count start
    if (tid < K) {
        const u64 rank = ((u64)(2 * tid + 1) * (u64)n_dense) / (u64)(2 * K);
        cen[tid] = n_dense > 0 ? half_bits_to_f32(key_half(A[rank] >> 16)) : 0.f;
    }
    if (tid <= K) prevpos[tid] = -1;
    __syncthreads();

    // ---- 6. Lloyd iterations on the boundaries
    int it = 0;
    if (n_dense > 0) {
        for (;;) {
            if (tid < K - 1) thr2[tid] = __fadd_rn(cen[tid], cen[tid + 1]);
            if (tid == 0) flag = 0;
            __syncthreads();
            for (int k = wave; k < K - 1; k += T / 64) {                 // uniform per wave
                const float t = thr2[k];
                // p = #{ j < n_dense : 2 w_j <= t }: rounds of 64 probes; invariant: the answer lies in [lo, lo + len]
                int lo = 0, len = n_dense;
                while (len > 0) {
                    const int step = (len + 63) / 64;                    // probe positions lo + step (l + 1) - 1
                    const int j = lo + step * (lane + 1) - 1;
                    bool le = false;
                    if (j < lo + len) le = !(t < 2.0f * half_bits_to_f32(key_half(A[j] >> 16)));
                    const int cnt = __builtin_popcountll(__ballot(le));  // probes with 2 w <= t form a prefix
                    lo += cnt * step;
                    len = min(step - 1, n_dense - lo);                   // the next probe after the prefix is > t (or past the end)
                    if (len < 0) len = 0;
                }
                const int p = lo;
                const int c = p >> 6, inside = p & 63;
                u32 sv = 0;
                i64 pr = 0;
                if (lane < inside) {
                    const u32 v = A[c * 64 + lane];
                    sv = v & 0xFFFFu;
                    pr = (i64)sv * half_to_fixed(key_half(v >> 16));
                }
                u64 s0, l, h;
                wave_sums(sv, pr, s0, l, h);
                if (lane == 0) {
                    pos[k + 1] = p; F0[k + 1] = c0[c] + s0; Flo[k + 1] = clo[c] + l; Fhi[k + 1] = chi[c] + h;
                    if (p != prevpos[k + 1]) flag = 1;
                }
            }
            if (tid == 0) {
                pos[0] = 0; F0[0] = 0; Flo[0] = 0; Fhi[0] = 0;
                pos[K] = n_dense; F0[K] = c0[nchunks]; Flo[K] = clo[nchunks]; Fhi[K] = chi[nchunks];
            }
            __syncthreads();
            const bool stop = flag == 0 || it == max_iter;
            if (!stop && tid < K) {
                const u64 s0 = F0[tid + 1] - F0[tid];
                if (s0 > 0) {
                    const double s1 = (double)(i64)(Fhi[tid + 1] - Fhi[tid]) * 4294967296.0 + (double)(Flo[tid + 1] - Flo[tid]);
                    cen[tid] = (float)(s1 * 5.9604644775390625e-08 / (double)s0);
                }
            }
            if (tid <= K) prevpos[tid] = pos[tid];
            __syncthreads();
            if (stop) break;
            ++it;
        }
    }

    // ---- 7. fp16 tables; final indices from the row as it lies in memory, packed 32 per thread
    if (tid < K) {
        const uint16_t hb = __builtin_bit_cast(uint16_t, (_Float16)cen[tid]);
        lut[(size_t)row * K + tid] = hb;
        cfix[tid] = half_to_fixed(hb);
    }
    if (tid == 0 && iters) iters[row] = it;
    __syncthreads();
    {
        i64 tf[K - 1];
#pragma unroll
        for (int k = 0; k < K - 1; ++k) tf[k] = cfix[k] + cfix[k + 1];
        u32 zero = 0;
        i64 best = cfix[0] < 0 ? -cfix[0] : cfix[0];
#pragma unroll
        for (int k = 1; k < K; ++k) {
            const i64 a = cfix[k] < 0 ? -cfix[k] : cfix[k];
            if (a < best) { best = a; zero = k; }
        }
        u32* out = static_cast<u32*>(qidx) + (size_t)row * ((size_t)N * BITS / 32);
        for (int ch = tid; ch < N / 32; ch += T) {
            u32 q[BITS];
#pragma unroll
            for (int k = 0; k < BITS; ++k) q[k] = 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const u32x4 wv = reinterpret_cast<const u32x4*>(wrow + ch * 32)[g], sv = reinterpret_cast<const u32x4*>(srow + ch * 32)[g];
                const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                for (int e8 = 0; e8 < 8; ++e8) {
                    const u32 wb = (e8 & 1) ? wd[e8 >> 1] >> 16 : wd[e8 >> 1] & 0xFFFFu;
                    const u32 sb = (e8 & 1) ? sd[e8 >> 1] >> 16 : sd[e8 >> 1] & 0xFFFFu;
                    u32 a = zero;
                    if (!is_extracted(wb, sb, key_min, key_max, s_thr)) {
                        const i64 w2 = 2 * half_to_fixed(wb);
                        a = 0;
#pragma unroll
                        for (int k = 0; k < K - 1; ++k) a += tf[k] < w2;
                    }
                    const int e = g * 8 + e8, bitpos = e * BITS;
                    q[bitpos >> 5] |= a << (bitpos & 31);
                    if ((bitpos & 31) + BITS > 32) q[(bitpos >> 5) + 1] |= a >> (32 - (bitpos & 31));
                }
            }
#pragma unroll
            for (int k = 0; k < BITS; ++k) out[(size_t)ch * BITS + k] = q[k];
        }
    }
}

// ---------------------------------------------------------------------------------------------- launcher
size_t quantize_workspace_bytes() { return (size_t)kWsWords * 4; }

// Scratch of the entry point that allocates nothing: the same 5.2 KB workspace, held by the library itself in device memory
// of every GPU the code object is loaded on.  In host code the array's name only stands for the symbol; its device address
// is asked for once per device (with that device current) and remembered.
static __device__ __align__(256) u32 scratch[kWsWords];

hipError_t quantize_static_scratch(void** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> ptrs[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    void* p = dev >= 0 && dev < kMaxDevices ? ptrs[dev].load(std::memory_order_acquire) : nullptr;
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        if (dev >= 0 && dev < kMaxDevices) ptrs[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

hipError_t launch_quantize(const QuantArgs& a, hipStream_t s) {
    u32* ws = static_cast<u32*>(a.workspace);
    const long long units = (long long)a.M * a.N / 8;
    const u64 total = (u64)a.M * (u64)a.N;
    // every block ends with up to 512 global atomic adds to the same 512 counters: 1024 blocks rather than 2048
    // (4096x4096: the two histogram kernels 47 + 27 -> 36 + 23 us)
    const int hist_blocks = (int)min((long long)1024, (units + 255) / 256);
    hipLaunchKernelGGL(quant_clear_kernel, dim3(4), dim3(256), 0, s, ws);
    hipLaunchKernelGGL(quant_hist1_kernel, dim3(hist_blocks), dim3(256), 0, s, units, static_cast<const u32x4*>(a.w), static_cast<const u32x4*>(a.sens), ws);
    hipLaunchKernelGGL(quant_select1_kernel, dim3(1), dim3(256), 0, s, total, (u64)a.n_lo, (u64)a.n_hi, (u64)a.n_sens, ws);
    hipLaunchKernelGGL(quant_hist2_kernel, dim3(hist_blocks), dim3(256), 0, s, units, static_cast<const u32x4*>(a.w), static_cast<const u32x4*>(a.sens), ws);
    hipLaunchKernelGGL(quant_select2_kernel, dim3(1), dim3(256), 0, s, ws);
    hipLaunchKernelGGL(quant_count_kernel, dim3((a.M + 3) / 4), dim3(256), 0, s, a.M, a.N, static_cast<const uint16_t*>(a.w), static_cast<const uint16_t*>(a.sens), ws, a.rowptr);
    hipLaunchKernelGGL(quant_scan_kernel, dim3(1), dim3(1024), 0, s, a.M, a.rowptr);
    int NP = 128;
    while (NP < a.N) NP <<= 1;
    const size_t lds = (size_t)a.N * 4 + (size_t)(a.N / 64 + 1) * 24;
    // Threads per row by the row's LDS footprint (the kernel is bound by LDS and barrier latency, so it wants 16 or more
    // waves per compute unit): 256 up to 4096 weights (eight workgroups per unit), 512 up to 16384 (2-4 workgroups), 1024
    // beyond (one).  Measured: 4096x11008 2.24 -> 1.79 ms and 8192x8192 2.30 -> 2.08 ms with 512 instead of 256 threads,
    // 8192x22016 9.95 -> 8.39 ms with 1024 instead of 512; 4096x4096 0.61 -> 0.67 ms with 512 (so 256 there).
    auto go = [](auto kernel) { return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024); };
    const int threads = a.N > 16384 ? 1024 : (a.N > 4096 ? 512 : 256);
#define SQ_LAUNCH_KMEANS(B_, T_)                                                                                                     \
    {                                                                                                                                \
        static bool enabled = false;                                                                                                 \
        if (!enabled) { const hipError_t e = go(&quant_kmeans_kernel<B_, T_>); if (e != hipSuccess) return e; enabled = true; }      \
        hipLaunchKernelGGL((quant_kmeans_kernel<B_, T_>), dim3(a.M), dim3(T_), lds, s, a.M, a.N, NP, a.max_iter,                       \
                           static_cast<const uint16_t*>(a.w), static_cast<const uint16_t*>(a.sens), ws, a.rowptr, a.qidx,           \
                           static_cast<uint16_t*>(a.lut), a.cols, static_cast<uint16_t*>(a.vals), a.iters);                         \
    }
#define SQ_LAUNCH_KMEANS_T(B_)                                                                                                      \
    { if (threads == 1024) SQ_LAUNCH_KMEANS(B_, 1024) else if (threads == 512) SQ_LAUNCH_KMEANS(B_, 512) else SQ_LAUNCH_KMEANS(B_, 256) }
    if (a.bits == 2) SQ_LAUNCH_KMEANS_T(2) else if (a.bits == 3) SQ_LAUNCH_KMEANS_T(3) else SQ_LAUNCH_KMEANS_T(4)
#undef SQ_LAUNCH_KMEANS_T
#undef SQ_LAUNCH_KMEANS
    return hipGetLastError();
}

}  // namespace sqllm
