// Dense-and-Sparse look-up-table matvec for gfx950 (CDNA4, wave64) — device code.
//
// What is computed (paper Sec. 4.2-4.3):  y = D x + S x,  D[i][j] = lut[i][idx(i,j)] with b-bit indices and
// one fp16 table per output row, S in CSR with fp16 values.  The storage format is described in sqllm.h.
//
// Work decomposition
//   * A wave owns a slice of 2048 consecutive columns: lane l holds the 32 activations
//     x[2048 w + 32 l .. +32) in registers for the whole kernel, so x is read once per workgroup.
//   * A workgroup has W = ceil(N / 2048) waves (one per slice) and walks over `rows_per_wg` consecutive
//     rows.  For every row each lane loads its 32 indices (12 bytes for b = 3, 16 bytes for b = 4: the
//     wave reads 768 / 1024 contiguous bytes per row), decodes them in registers and accumulates in fp32.
//   * Table look-ups never touch LDS memory: the row's table lives in ONE register spread over the 64
//     lanes and is read with ds_bpermute_b32 (a cross-lane gather that has no bank conflicts).
//       b = 3: lane e holds the pair (lut[e & 7], lut[e >> 3]); a 6-bit field of the stream (two
//              neighbouring indices) selects a ready-made fp16 pair that feeds v_dot2_f32_f16.
//       b = 4: lane e holds lut[e & 15]; one look-up per index, fp16 x fp16 -> fp32 fused multiply-add.
//     The gather address is (field << 2); the hardware uses address bits [7:2] only, so a single shift (or a
//     funnel shift where a field straddles two dwords) per look-up is all the integer work there is.
//   * Per row the 64 lane sums are reduced with DPP adds, the W slice sums are combined through LDS in a
//     fixed order, the CSR term is added, and y is rounded to fp16 once.
//   * CSR term (balanced): the nonzeros of the workgroup's rows form one contiguous range of the CSR
//     arrays; thread t takes nonzeros t, t + T, t + 2T, ... of that range whatever rows they fall in
//     (equal work per thread), products are combined per row with a segmented scan inside the wave and
//     accumulated into wave-private LDS slots, so no floating-point atomics are needed and the result does
//     not depend on timing.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sqllm_kernels.h"

namespace sqllm {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kLaneElems = 32;                      // indices per lane per row
constexpr int kSliceCols = kWave * kLaneElems;      // 2048 columns per wave

// ---------------------------------------------------------------------------------------------- helpers
__device__ __forceinline__ u32 funnel_shr(u32 hi, u32 lo, u32 sh) { return __builtin_amdgcn_alignbit(hi, lo, sh); }

__device__ __forceinline__ u32 lane_gather(u32 byte_addr, u32 table) {
    return (u32)__builtin_amdgcn_ds_bpermute((int)byte_addr, (int)table);
}

__device__ __forceinline__ half2_t as_half2(u32 v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ u32 as_u32(half2_t v) { return __builtin_bit_cast(u32, v); }

// sum over the 64 lanes; the total ends up in every lane
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// ---------------------------------------------------------------------------------------------- decode
// A lane's share of one row: BITS dwords = 32 indices.
template <int BITS>
struct LaneChunk {
    u32 q[BITS];
};

template <int BITS>
__device__ __forceinline__ LaneChunk<BITS> load_chunk(const u32* __restrict__ p, bool live) {
    LaneChunk<BITS> c;
#pragma unroll
    for (int k = 0; k < BITS; ++k) c.q[k] = 0;
    if (live) {
#pragma unroll
        for (int k = 0; k < BITS; ++k) c.q[k] = __builtin_nontemporal_load(p + k);
    }
    return c;
}

// b = 3.  Gather addresses of the 16 index PAIRS of a lane: pair p owns bits [6p, 6p+6) of the 96-bit
// chunk; the address must carry that field in bits [7:2].
__device__ __forceinline__ void pair_addresses(const LaneChunk<3>& c, u32 (&a)[16]) {
    const u32 q0 = c.q[0], q1 = c.q[1], q2 = c.q[2];
    a[0] = q0 << 2;   a[1] = q0 >> 4;   a[2] = q0 >> 10;  a[3] = q0 >> 16;  a[4] = q0 >> 22;
    a[5] = funnel_shr(q1, q0, 28);                      // bits 30..35 straddle dwords 0 and 1
    a[6] = q1 >> 2;   a[7] = q1 >> 8;   a[8] = q1 >> 14;  a[9] = q1 >> 20;
    a[10] = funnel_shr(q2, q1, 26);                     // bits 60..65 straddle dwords 1 and 2
    a[11] = q2;       a[12] = q2 >> 6;  a[13] = q2 >> 12; a[14] = q2 >> 18; a[15] = q2 >> 24;
}

// b = 4.  Gather address of index k (0..31) of a lane: field bits [4k, 4k+4) -> address bits [5:2]
// (bits [7:6] then carry part of the next index; the table is replicated four times so they do not matter).
__device__ __forceinline__ u32 elem_address(const LaneChunk<4>& c, int k) {
    const u32 q = c.q[k >> 3];
    const int pos = k & 7;
    return pos == 0 ? (q << 2) : (q >> (4 * pos - 2));
}

// The row's table, one register across the wave.
template <int BITS>
__device__ __forceinline__ u32 load_table(const uint16_t* __restrict__ lut_row, int lane);

template <>
__device__ __forceinline__ u32 load_table<3>(const uint16_t* __restrict__ lut_row, int lane) {
    const u32 lo = lut_row[lane & 7], hi = lut_row[lane >> 3];
    return lo | (hi << 16);
}
template <>
__device__ __forceinline__ u32 load_table<4>(const uint16_t* __restrict__ lut_row, int lane) {
    const u32 v = lut_row[lane & 15];
    return v | (v << 16);
}

// ---------------------------------------------------------------------------------------------- x in registers
// xr[t][p] = (x[j0 + 2p][t], x[j0 + 2p + 1][t]) for the lane's 32 columns j0 .. j0 + 31.
template <int NB>
__device__ __forceinline__ void load_x(const uint16_t* __restrict__ x, int B, int bn, int j0, bool live, u32 (&xr)[NB][16]) {
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int p = 0; p < 16; ++p) xr[t][p] = 0;
    if (!live) return;
    if (NB == 1 && B == 1) {
        const uint4* src = reinterpret_cast<const uint4*>(x + j0);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint4 v = src[k];
            xr[0][4 * k + 0] = v.x; xr[0][4 * k + 1] = v.y; xr[0][4 * k + 2] = v.z; xr[0][4 * k + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            if (t < bn) {
#pragma unroll
                for (int p = 0; p < 16; ++p) {
                    const u32 lo = x[(size_t)(j0 + 2 * p) * B + t], hi = x[(size_t)(j0 + 2 * p + 1) * B + t];
                    xr[t][p] = lo | (hi << 16);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- dense row slice
template <int BITS, int NB>
__device__ __forceinline__ void accumulate_chunk(const LaneChunk<BITS>& c, u32 table, const u32 (&xr)[NB][16], float (&acc)[NB]);

template <int NB>
__device__ __forceinline__ void accumulate_chunk3(const LaneChunk<3>& c, u32 table, const u32 (&xr)[NB][16], float (&acc)[NB]) {
    u32 a[16];
    pair_addresses(c, a);
    u32 w[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) w[p] = lane_gather(a[p], table);
#pragma unroll
    for (int p = 0; p < 16; ++p)
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[t] = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[t][p]), acc[t], false);
}

template <int NB>
__device__ __forceinline__ void accumulate_chunk4(const LaneChunk<4>& c, u32 table, const u32 (&xr)[NB][16], float (&acc)[NB]) {
#pragma unroll
    for (int k = 0; k < 32; k += 2) {
        const u32 w0 = lane_gather(elem_address(c, k), table);
        const u32 w1 = lane_gather(elem_address(c, k + 1), table);
        const float f0 = (float)as_half2(w0).x, f1 = (float)as_half2(w1).x;
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            const half2_t xv = as_half2(xr[t][k >> 1]);
            acc[t] = __builtin_fmaf(f0, (float)xv.x, acc[t]);
            acc[t] = __builtin_fmaf(f1, (float)xv.y, acc[t]);
        }
    }
}

template <int BITS, int NB>
__device__ __forceinline__ void accumulate_any(const LaneChunk<BITS>& c, u32 table, const u32 (&xr)[NB][16], float (&acc)[NB]) {
    if constexpr (BITS == 3) accumulate_chunk3<NB>(c, table, xr, acc);
    else accumulate_chunk4<NB>(c, table, xr, acc);
}

// ---------------------------------------------------------------------------------------------- the matvec kernel
// grid.x = ceil(M / rows_per_wg); block = W * 64 threads, W = ceil(N / 2048) when dense, any W when sparse only.
// dynamic LDS: float part[W][rows_per_wg][NB]  +  int srp[rows_per_wg + 1]
template <int BITS, int NB, int RB>
__global__ void __launch_bounds__(1024) matvec_kernel(MatvecArgs g) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int W = blockDim.x >> 6, T = blockDim.x;
    const int rows = g.rows_per_wg;
    const int r0 = blockIdx.x * rows;
    const int nrows = min(rows, g.M - r0);
    float* part = reinterpret_cast<float*>(lds_raw);                       // [W][rows][NB]
    int* srp = reinterpret_cast<int*>(part + (size_t)W * rows * NB);       // [rows + 1]
    const int B = g.B, bn = g.bn;                                         // x, y row stride; live batch columns
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(g.x) + g.bt0;

    const bool sparse = g.nnz > 0;
    if (sparse)
        for (int k = tid; k <= nrows; k += T) srp[k] = g.rowptr[r0 + k];

    // ---- dense term: this wave's 2048-column slice of every row of the block
    if (g.qidx != nullptr) {
        const int j0 = wave * kSliceCols + lane * kLaneElems;
        const bool live = j0 < g.N;
        u32 xr[NB][16];
        load_x<NB>(x, B, bn, j0, live, xr);
        const size_t row_dwords = (size_t)g.N * BITS / 32;
        const u32* __restrict__ qbase = static_cast<const u32*>(g.qidx) + (size_t)r0 * row_dwords + (size_t)(j0 / 32) * BITS;
        const uint16_t* __restrict__ lbase = static_cast<const uint16_t*>(g.lut) + (size_t)r0 * (1 << BITS);
        for (int rb = 0; rb < nrows; rb += RB) {
            LaneChunk<BITS> c[RB];
            u32 table[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                const bool ok = rb + u < nrows;                              // uniform
                c[u] = load_chunk<BITS>(qbase + (size_t)(rb + u) * row_dwords, live && ok);
                table[u] = ok ? load_table<BITS>(lbase + (size_t)(rb + u) * (1 << BITS), lane) : 0u;
            }
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                float acc[NB];
#pragma unroll
                for (int t = 0; t < NB; ++t) acc[t] = 0.f;
                accumulate_any<BITS, NB>(c[u], table[u], xr, acc);
#pragma unroll
                for (int t = 0; t < NB; ++t) {
                    const float s = wave_sum(acc[t]);
                    if (lane == 0 && rb + u < nrows) part[((size_t)wave * rows + rb + u) * NB + t] = s;
                }
            }
        }
    } else {
        for (int k = lane; k < nrows * NB; k += kWave) part[(size_t)wave * rows * NB + k] = 0.f;
    }
    __syncthreads();

    // ---- sparse term: nonzeros [P0, P1) of the block's rows, dealt out evenly to the T threads
    if (sparse) {
        const int P0 = srp[0], P1 = srp[nrows];
        const int* __restrict__ cols = g.cols;
        const uint16_t* __restrict__ vals = static_cast<const uint16_t*>(g.vals);
        float* mine = part + (size_t)wave * rows * NB;
        for (int pbase = P0 + wave * kWave; pbase < P1; pbase += T) {       // uniform per wave
            const int p = pbase + lane;
            const bool ok = p < P1;
            int r = nrows;                                                   // sentinel row for idle lanes
            float prod[NB];
#pragma unroll
            for (int t = 0; t < NB; ++t) prod[t] = 0.f;
            if (ok) {
                const int c = cols[p];
                const float v = (float)__builtin_bit_cast(half_t, vals[p]);
                int lo = 0, hi = nrows;                                      // largest r with srp[r] <= p
                while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (srp[mid] <= p) lo = mid; else hi = mid; }
                r = lo;
#pragma unroll
                for (int t = 0; t < NB; ++t)
                    if (t < bn) prod[t] = v * (float)__builtin_bit_cast(half_t, x[(size_t)c * B + t]);
            }
            // segmented inclusive scan over lanes (rows are non-decreasing with the lane index)
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int r_up = __shfl_up(r, d, kWave);
#pragma unroll
                for (int t = 0; t < NB; ++t) {
                    const float v_up = __shfl_up(prod[t], d, kWave);
                    if (lane >= d && r_up == r) prod[t] += v_up;
                }
            }
            const int r_next = __shfl_down(r, 1, kWave);
            const bool tail = ok && (lane == kWave - 1 || r_next != r);
            if (tail) {
#pragma unroll
                for (int t = 0; t < NB; ++t) mine[(size_t)r * NB + t] += prod[t];
            }
        }
        __syncthreads();
    }

    // ---- combine the W partial sums in a fixed order, round once
    uint16_t* __restrict__ y = static_cast<uint16_t*>(g.y) + g.bt0;
    for (int k = tid; k < nrows * NB; k += T) {
        const int r = k / NB, t = k - r * NB;
        if (t >= bn) continue;
        float s = 0.f;
        for (int w = 0; w < W; ++w) s += part[((size_t)w * rows + r) * NB + t];
        const size_t o = (size_t)(r0 + r) * B + t;
        if (g.accumulate) s += (float)__builtin_bit_cast(half_t, y[o]);
        y[o] = __builtin_bit_cast(uint16_t, (half_t)s);
    }
}

// ---------------------------------------------------------------------------------------------- standard CSR kernel
// one thread per row (the kernel the paper's App. C calls "standard")
template <int NB>
__global__ void __launch_bounds__(256) csr_rowwise_kernel(MatvecArgs g) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= g.M) return;
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(g.x) + g.bt0;
    const uint16_t* __restrict__ vals = static_cast<const uint16_t*>(g.vals);
    uint16_t* __restrict__ y = static_cast<uint16_t*>(g.y) + g.bt0;
    float acc[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) acc[t] = 0.f;
    if (g.nnz > 0) {
        for (int p = g.rowptr[i]; p < g.rowptr[i + 1]; ++p) {
            const int c = g.cols[p];
            const float v = (float)__builtin_bit_cast(half_t, vals[p]);
#pragma unroll
            for (int t = 0; t < NB; ++t)
                if (t < g.bn) acc[t] += v * (float)__builtin_bit_cast(half_t, x[(size_t)c * g.B + t]);
        }
    }
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        if (t >= g.bn) continue;
        const size_t o = (size_t)i * g.B + t;
        float s = acc[t];
        if (g.accumulate) s += (float)__builtin_bit_cast(half_t, y[o]);
        y[o] = __builtin_bit_cast(uint16_t, (half_t)s);
    }
}

// ---------------------------------------------------------------------------------------------- parity exports
// Same load + address arithmetic + gather as the matvec; one wave per (row, slice).
template <int BITS>
__global__ void __launch_bounds__(64) decode_kernel(int M, int N, const void* qidx, const void* lut, void* idx_out, void* w_out) {
    const int lane = threadIdx.x;
    const int row = blockIdx.y, slice = blockIdx.x;
    const int j0 = slice * kSliceCols + lane * kLaneElems;
    const bool live = j0 < N;
    const size_t row_dwords = (size_t)N * BITS / 32;
    const u32* p = static_cast<const u32*>(qidx) + (size_t)row * row_dwords + (size_t)(j0 / 32) * BITS;
    const LaneChunk<BITS> c = load_chunk<BITS>(p, live);
    u32 idx[32], wbits[32];
    if constexpr (BITS == 3) {
        u32 a[16];
        pair_addresses(c, a);
        // identity tables: gathering them returns the lane number the address selects = the 6-bit field
        const u32 table = lut ? load_table<3>(static_cast<const uint16_t*>(lut) + (size_t)row * 8, lane) : 0u;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const u32 field = lane_gather(a[k], (u32)lane);
            idx[2 * k] = field & 7; idx[2 * k + 1] = field >> 3;
            const u32 w = lane_gather(a[k], table);
            wbits[2 * k] = w & 0xFFFF; wbits[2 * k + 1] = w >> 16;
        }
    } else {
        const u32 table = lut ? load_table<4>(static_cast<const uint16_t*>(lut) + (size_t)row * 16, lane) : 0u;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const u32 a = elem_address(c, k);
            idx[k] = lane_gather(a, (u32)lane) & 15;
            wbits[k] = lane_gather(a, table) & 0xFFFF;
        }
    }
    if (!live) return;
    if (idx_out) {
        uint8_t* o = static_cast<uint8_t*>(idx_out) + (size_t)row * N + j0;
#pragma unroll
        for (int k = 0; k < 32; ++k) o[k] = (uint8_t)idx[k];
    }
    if (w_out) {
        uint16_t* o = static_cast<uint16_t*>(w_out) + (size_t)row * N + j0;
#pragma unroll
        for (int k = 0; k < 32; ++k) o[k] = (uint16_t)wbits[k];
    }
}

// ---------------------------------------------------------------------------------------------- fp16 baseline
// y = W x, W fp16 row-major.  One wave per row group; lane reads 16 bytes (8 weights) per step.
template <int NB, int RB>
__global__ void __launch_bounds__(256) fp16_gemv_kernel(int M, int N, int B, const void* wv, const void* xv, void* yv) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * (blockDim.x >> 6) + wave) * RB;
    if (row0 >= M) return;
    const uint16_t* __restrict__ w = static_cast<const uint16_t*>(wv);
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(xv);
    float acc[RB][NB];
#pragma unroll
    for (int u = 0; u < RB; ++u)
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[u][t] = 0.f;
    for (int j = lane * 8; j < N; j += kWave * 8) {
        u32 xr[NB][4];
        if (NB == 1) {
            const uint4 v = *reinterpret_cast<const uint4*>(x + j);
            xr[0][0] = v.x; xr[0][1] = v.y; xr[0][2] = v.z; xr[0][3] = v.w;
        } else {
#pragma unroll
            for (int t = 0; t < NB; ++t)
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    xr[t][p] = t < B ? ((u32)x[(size_t)(j + 2 * p) * B + t] | ((u32)x[(size_t)(j + 2 * p + 1) * B + t] << 16)) : 0u;
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            if (row0 + u >= M) continue;
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(w + (size_t)(row0 + u) * N + j));
            const u32 wr[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int t = 0; t < NB; ++t) acc[u][t] = __builtin_amdgcn_fdot2(as_half2(wr[p]), as_half2(xr[t][p]), acc[u][t], false);
        }
    }
    uint16_t* __restrict__ y = static_cast<uint16_t*>(yv);
#pragma unroll
    for (int u = 0; u < RB; ++u)
#pragma unroll
        for (int t = 0; t < NB; ++t) {
            const float s = wave_sum(acc[u][t]);
            if (lane == 0 && row0 + u < M && t < B) y[(size_t)(row0 + u) * B + t] = __builtin_bit_cast(uint16_t, (half_t)s);
        }
}

// ---------------------------------------------------------------------------------------------- launchers
template <int BITS, int NB>
static hipError_t launch_matvec_t(const MatvecArgs& g, int waves, hipStream_t s) {
    constexpr int RB = (NB == 1) ? 4 : (NB == 2 ? 2 : 1);
    const int grid = (g.M + g.rows_per_wg - 1) / g.rows_per_wg;
    const size_t lds = (size_t)waves * g.rows_per_wg * NB * sizeof(float) + (size_t)(g.rows_per_wg + 1) * sizeof(int);
    hipLaunchKernelGGL((matvec_kernel<BITS, NB, RB>), dim3(grid), dim3(waves * kWave), lds, s, g);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_matvec_b(const MatvecArgs& g0, int waves, hipStream_t s) {
    // at most four batch columns per launch (their activations must fit in registers)
    for (int t0 = 0; t0 < g0.B; t0 += 4) {
        MatvecArgs g = g0;
        g.bt0 = t0; g.bn = min(4, g0.B - t0);
        hipError_t e;
        if (g.bn == 1) e = launch_matvec_t<BITS, 1>(g, waves, s);
        else if (g.bn == 2) e = launch_matvec_t<BITS, 2>(g, waves, s);
        else e = launch_matvec_t<BITS, 4>(g, waves, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_matvec(const MatvecArgs& g, int waves, hipStream_t s) {
    return g.bits == 3 ? launch_matvec_b<3>(g, waves, s) : launch_matvec_b<4>(g, waves, s);
}

hipError_t launch_csr_rowwise(const MatvecArgs& g0, hipStream_t s) {
    MatvecArgs g = g0;
    g.bt0 = 0; g.bn = g.B;
    const int grid = (g.M + 255) / 256;
    if (g.B == 1) hipLaunchKernelGGL((csr_rowwise_kernel<1>), dim3(grid), dim3(256), 0, s, g);
    else if (g.B == 2) hipLaunchKernelGGL((csr_rowwise_kernel<2>), dim3(grid), dim3(256), 0, s, g);
    else if (g.B <= 4) hipLaunchKernelGGL((csr_rowwise_kernel<4>), dim3(grid), dim3(256), 0, s, g);
    else hipLaunchKernelGGL((csr_rowwise_kernel<8>), dim3(grid), dim3(256), 0, s, g);
    return hipGetLastError();
}

hipError_t launch_decode(int M, int N, int bits, const void* qidx, const void* lut, void* idx_out, void* w_out, hipStream_t s) {
    const int slices = (N + kSliceCols - 1) / kSliceCols;
    // grid.y is limited to 65535 rows per launch
    for (int m0 = 0; m0 < M; m0 += 65535) {
        const int m = min(65535, M - m0);
        const size_t qoff = (size_t)m0 * N * bits / 8;
        const void* q = static_cast<const char*>(qidx) + qoff;
        const void* l = lut ? static_cast<const char*>(lut) + (size_t)m0 * (1 << bits) * 2 : nullptr;
        void* io = idx_out ? static_cast<char*>(idx_out) + (size_t)m0 * N : nullptr;
        void* wo = w_out ? static_cast<char*>(w_out) + (size_t)m0 * N * 2 : nullptr;
        if (bits == 3) hipLaunchKernelGGL((decode_kernel<3>), dim3(slices, m), dim3(kWave), 0, s, m, N, q, l, io, wo);
        else hipLaunchKernelGGL((decode_kernel<4>), dim3(slices, m), dim3(kWave), 0, s, m, N, q, l, io, wo);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_fp16_gemv(int M, int N, int B, const void* w, const void* x, void* y, hipStream_t s) {
    constexpr int RB = 2, WAVES = 4;
    const int grid = (M + WAVES * RB - 1) / (WAVES * RB);
    if (B == 1) hipLaunchKernelGGL((fp16_gemv_kernel<1, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    else if (B == 2) hipLaunchKernelGGL((fp16_gemv_kernel<2, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    else if (B <= 4) hipLaunchKernelGGL((fp16_gemv_kernel<4, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    else hipLaunchKernelGGL((fp16_gemv_kernel<8, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    return hipGetLastError();
}

}  // namespace sqllm
