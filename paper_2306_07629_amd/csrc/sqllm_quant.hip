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
//      64-bit integers (LDS integer atomics), so the result does not depend on the order of the additions.
//   4. fp16 tables, final indices (nearest table entry in exact arithmetic, ties to the lower index; an extracted
//      position gets the entry nearest to zero) and the packed index stream in the layout the matvec reads.
#include <hip/hip_runtime.h>
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
    __shared__ u32 hw[256], hs[256];
    hw[threadIdx.x] = 0; hs[threadIdx.x] = 0;
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
    if (hw[threadIdx.x]) atomicAdd(&ws[kWsHist1W + threadIdx.x], hw[threadIdx.x]);
    if (hs[threadIdx.x]) atomicAdd(&ws[kWsHist1S + threadIdx.x], hs[threadIdx.x]);
}

// bin holding the element of rank r (0-based) in a 256-bin histogram, and the rank inside that bin
__device__ inline void select_bin(const u32* hist, u64 r, u32& bin, u64& residual) {
    u64 cum = 0;
    bin = 255; residual = 0;
    for (u32 b = 0; b < 256; ++b) {
        const u64 h = hist[b];
        if (r < cum + h) { bin = b; residual = r - cum; return; }
        cum += h;
    }
}

__global__ void quant_select1_kernel(u64 total, u64 n_lo, u64 n_hi, u64 n_sens, u32* ws) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const u64 ranks[3] = {n_lo, total - 1 - n_hi, total - 1 - n_sens};
    for (int t = 0; t < 3; ++t) {
        u32 bin; u64 res;
        select_bin(ws + (t < 2 ? kWsHist1W : kWsHist1S), ranks[t], bin, res);
        ws[kWsSel + 4 * t] = bin; ws[kWsSel + 4 * t + 1] = (u32)res; ws[kWsSel + 4 * t + 2] = (u32)(res >> 32);
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

__global__ void quant_select2_kernel(u32* ws) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    for (int t = 0; t < 3; ++t) {
        const u64 r = (u64)ws[kWsSel + 4 * t + 1] | ((u64)ws[kWsSel + 4 * t + 2] << 32);
        u32 lo; u64 res;
        select_bin(ws + kWsHist2 + 256 * t, r, lo, res);
        ws[kWsThr + t] = (ws[kWsSel + 4 * t] << 8) | lo;
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

// sum over the 64 lanes, valid in every lane
__device__ __forceinline__ int wave_sum_all(int v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One block of 256 threads per row.  LDS: the row's weights and sensitivities (bit patterns), one byte of index per
// weight (0xFF marks an extracted position while the iterations run), and the per-cluster sums.
template <int BITS>
__global__ void __launch_bounds__(256) quant_kmeans_kernel(int M, int N, int max_iter, const uint16_t* __restrict__ w, const uint16_t* __restrict__ sens,
                                                         const u32* __restrict__ ws, const int* __restrict__ rowptr, void* __restrict__ qidx,
                                                         uint16_t* __restrict__ lut, int* __restrict__ cols, uint16_t* __restrict__ vals, int* __restrict__ iters) {
    constexpr int K = 1 << BITS, T = 256;
    extern __shared__ __align__(16) char smem[];
    uint16_t* wl = reinterpret_cast<uint16_t*>(smem);                // [N]
    uint16_t* sl = wl + N;                                          // [N]
    uint8_t* il = reinterpret_cast<uint8_t*>(sl + N);               // [N]
    __shared__ u64 S0[K], S1lo[K], S1hi[K];
    __shared__ float cen[K], thr2[K];
    __shared__ i64 cfix[K];
    __shared__ int counts[K], scan[T], flags[2];
    __shared__ u32 prefix[K];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, row = blockIdx.x;
    const u32 key_min = ws[kWsThr], key_max = ws[kWsThr + 1], s_thr = ws[kWsThr + 2];

    // ---- 1. the row into LDS; mark extracted positions
    {
        const u32x4* wr = reinterpret_cast<const u32x4*>(w + (size_t)row * N);
        const u32x4* sr = reinterpret_cast<const u32x4*>(sens + (size_t)row * N);
        for (int i = tid; i < N / 8; i += T) {
            const u32x4 wv = wr[i], sv = sr[i];
            reinterpret_cast<u32x4*>(wl)[i] = wv; reinterpret_cast<u32x4*>(sl)[i] = sv;
            const u32 wd[4] = {wv.x, wv.y, wv.z, wv.w}, sd[4] = {sv.x, sv.y, sv.z, sv.w};
            u32 m[2] = {0, 0};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 a = is_extracted(wd[k] & 0xFFFFu, sd[k] & 0xFFFFu, key_min, key_max, s_thr) ? 0xFFu : 0xFEu;
                const u32 b = is_extracted(wd[k] >> 16, sd[k] >> 16, key_min, key_max, s_thr) ? 0xFFu : 0xFEu;
                m[k >> 1] |= (a | (b << 8)) << (16 * (k & 1));
            }
            reinterpret_cast<u32*>(il)[2 * i] = m[0]; reinterpret_cast<u32*>(il)[2 * i + 1] = m[1];
        }
        if (tid < K) { S0[tid] = 0; S1lo[tid] = 0; S1hi[tid] = 0; counts[tid] = 0; }
    }
    __syncthreads();

    // ---- 2. CSR entries of the row, columns ascending: thread t owns the columns [t C, (t + 1) C)
    const int C = (N + T - 1) / T;
    const int jb = min(tid * C, N), je = min(jb + C, N);
    int mine = 0;
    for (int j = jb; j < je; ++j) mine += il[j] == 0xFF;
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
            if (il[j] == 0xFF) { cols[o] = j; vals[o] = wl[j]; ++o; }
    }

    // ---- 3. equal-count start: centroid k = the dense weight of rank floor((2k + 1) n / (2K)); K bitwise searches over
    //         the 16-bit keys run together (largest v with #{keys < v} <= rank)
    if (tid < K) prefix[tid] = 0;
    __syncthreads();
    if (n_dense > 0) {
        for (int bit = 15; bit >= 0; --bit) {
            u32 cand[K];
            int cnt[K];
#pragma unroll
            for (int k = 0; k < K; ++k) { cand[k] = prefix[k] | (1u << bit); cnt[k] = 0; }
            for (int j = tid; j < N; j += T) {
                if (il[j] != 0xFF) {
                    const u32 key = half_key(wl[j]);
#pragma unroll
                    for (int k = 0; k < K; ++k) cnt[k] += key < cand[k];
                }
            }
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int tot = wave_sum_all(cnt[k]);
                if (lane == 0) atomicAdd(&counts[k], tot);
            }
            __syncthreads();
            if (tid < K) {
                const u64 rank = ((u64)(2 * tid + 1) * (u64)n_dense) / (u64)(2 * K);
                if ((u64)counts[tid] <= rank) prefix[tid] |= 1u << bit;
                counts[tid] = 0;
            }
            __syncthreads();
        }
    }
    if (tid < K) cen[tid] = n_dense > 0 ? half_bits_to_f32(key_half(prefix[tid])) : 0.f;
    if (tid == 0) { flags[0] = 0; flags[1] = 0; }
    __syncthreads();

    // ---- 4. Lloyd iterations
    int it = 0;
    for (;;) {
        if (tid < K - 1) thr2[tid] = __fadd_rn(cen[tid], cen[tid + 1]);
        __syncthreads();
        float t[K - 1];
#pragma unroll
        for (int k = 0; k < K - 1; ++k) t[k] = thr2[k];
        int changed = 0;
        for (int j = tid; j < N; j += T) {
            const u32 old = il[j];
            if (old != 0xFF) {
                const u32 wb = wl[j];
                const float two_w = 2.0f * half_bits_to_f32(wb);
                u32 a = 0;
#pragma unroll
                for (int k = 0; k < K - 1; ++k) a += t[k] < two_w;
                changed |= a != old;
                il[j] = (uint8_t)a;
                const u64 sv = sl[j];
                const i64 p = (i64)sv * half_to_fixed(wb);
                atomicAdd(&S0[a], sv);
                atomicAdd(&S1lo[a], (u64)p & 0xFFFFFFFFull);
                atomicAdd(&S1hi[a], (u64)(p >> 32));
            }
        }
        if (changed) flags[it & 1] = 1;                              // benign race: every writer stores 1
        __syncthreads();
        const bool any_changed = flags[it & 1] != 0;
        const bool stop = !any_changed || it == max_iter;
        if (!stop && tid < K) {
            if (S0[tid] > 0) {
                const double s1 = (double)(i64)S1hi[tid] * 4294967296.0 + (double)S1lo[tid];
                cen[tid] = (float)(s1 * 5.9604644775390625e-08 / (double)S0[tid]);
            }
        }
        if (tid < K) { S0[tid] = 0; S1lo[tid] = 0; S1hi[tid] = 0; }
        if (tid == 0) flags[(it + 1) & 1] = 0;
        __syncthreads();
        if (stop) break;
        ++it;
    }

    // ---- 5. fp16 tables and final indices
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
        for (int j = tid; j < N; j += T) {
            u32 a = zero;
            if (il[j] != 0xFF) {
                const i64 w2 = 2 * half_to_fixed(wl[j]);
                a = 0;
#pragma unroll
                for (int k = 0; k < K - 1; ++k) a += tf[k] < w2;
            }
            il[j] = (uint8_t)a;
        }
    }
    __syncthreads();

    // ---- 6. packed index stream: element j owns bits [j b, j b + b) of the row, least significant bit first
    {
        u32* out = static_cast<u32*>(qidx) + (size_t)row * ((size_t)N * BITS / 32);
        for (int ch = tid; ch < N / 32; ch += T) {
            u32 q[BITS];
#pragma unroll
            for (int k = 0; k < BITS; ++k) q[k] = 0;
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const u32 v = il[ch * 32 + e];
                const int bitpos = e * BITS;
                q[bitpos >> 5] |= v << (bitpos & 31);
                if ((bitpos & 31) + BITS > 32) q[(bitpos >> 5) + 1] |= v >> (32 - (bitpos & 31));
            }
#pragma unroll
            for (int k = 0; k < BITS; ++k) out[(size_t)ch * BITS + k] = q[k];
        }
    }
}

// ---------------------------------------------------------------------------------------------- launcher
size_t quantize_workspace_bytes() { return (size_t)kWsWords * 4; }

hipError_t launch_quantize(const QuantArgs& a, hipStream_t s) {
    u32* ws = static_cast<u32*>(a.workspace);
    const long long units = (long long)a.M * a.N / 8;
    const u64 total = (u64)a.M * (u64)a.N;
    const int hist_blocks = (int)min((long long)2048, (units + 255) / 256);
    hipLaunchKernelGGL(quant_clear_kernel, dim3(4), dim3(256), 0, s, ws);
    hipLaunchKernelGGL(quant_hist1_kernel, dim3(hist_blocks), dim3(256), 0, s, units, static_cast<const u32x4*>(a.w), static_cast<const u32x4*>(a.sens), ws);
    hipLaunchKernelGGL(quant_select1_kernel, dim3(1), dim3(64), 0, s, total, (u64)a.n_lo, (u64)a.n_hi, (u64)a.n_sens, ws);
    hipLaunchKernelGGL(quant_hist2_kernel, dim3(hist_blocks), dim3(256), 0, s, units, static_cast<const u32x4*>(a.w), static_cast<const u32x4*>(a.sens), ws);
    hipLaunchKernelGGL(quant_select2_kernel, dim3(1), dim3(64), 0, s, ws);
    hipLaunchKernelGGL(quant_count_kernel, dim3((a.M + 3) / 4), dim3(256), 0, s, a.M, a.N, static_cast<const uint16_t*>(a.w), static_cast<const uint16_t*>(a.sens), ws, a.rowptr);
    hipLaunchKernelGGL(quant_scan_kernel, dim3(1), dim3(1024), 0, s, a.M, a.rowptr);
    const size_t lds = (size_t)a.N * 5;
    hipError_t e = hipSuccess;
    if (a.bits == 3) {
        static bool enabled = false;
        if (!enabled) { e = hipFuncSetAttribute(reinterpret_cast<const void*>(&quant_kmeans_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024); enabled = true; }
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((quant_kmeans_kernel<3>), dim3(a.M), dim3(256), lds, s, a.M, a.N, a.max_iter, static_cast<const uint16_t*>(a.w), static_cast<const uint16_t*>(a.sens),
                           ws, a.rowptr, a.qidx, static_cast<uint16_t*>(a.lut), a.cols, static_cast<uint16_t*>(a.vals), a.iters);
    } else {
        static bool enabled = false;
        if (!enabled) { e = hipFuncSetAttribute(reinterpret_cast<const void*>(&quant_kmeans_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024); enabled = true; }
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((quant_kmeans_kernel<4>), dim3(a.M), dim3(256), lds, s, a.M, a.N, a.max_iter, static_cast<const uint16_t*>(a.w), static_cast<const uint16_t*>(a.sens),
                           ws, a.rowptr, a.qidx, static_cast<uint16_t*>(a.lut), a.cols, static_cast<uint16_t*>(a.vals), a.iters);
    }
    return hipGetLastError();
}

}  // namespace sqllm
