// Dense-and-Sparse look-up-table matvec for gfx950 (CDNA4, wave64) — device code.
//
// What is computed (paper Sec. 4.2-4.3):  y = D x + S x,  D[i][j] = lut[i][idx(i,j)] with b-bit indices and
// one fp16 table per output row, S in CSR with fp16 values.  The storage format is described in sqllm.h.
//
// Work decomposition of the matvec kernel
//   * A workgroup owns R consecutive rows (R = 4 or 8, compile time) and all N columns.
//   * Dense waves: wave w owns the 2048-column slice [2048 w, 2048 w + 2048): lane l keeps the 32 activations
//     x[2048 w + 32 l .. +32) in registers for the whole kernel (x is read once per workgroup) and, per row,
//     loads its 32 indices (12 bytes for b = 3, 16 bytes for b = 4; the wave reads 768 / 1024 contiguous
//     bytes of the row).  D rows are requested up front, row u + D when row u has been handed to the look-ups.
//   * Dequantisation goes through PAIR TABLES in LDS: for every row of the block the workgroup first builds
//       b = 3:  64 entries,  entry (a | c << 3) = (lut[a], lut[c]) as two fp16 in one dword   (256 B / row)
//       b = 4: 256 entries,  entry (a | c << 4) = (lut[a], lut[c])                            (1 KB / row)
//       b = 2:  16 entries,  entry (a | c << 2) = (lut[a], lut[c])                            (64 B / row)
//     so ONE ds_read_b32, addressed by a 6- or 8-bit field of the index stream (two neighbouring indices),
//     returns a ready-made fp16 pair for v_dot2_f32_f16 (two products, fp32 accumulate).  Measured on MI355X
//     a wave-wide look-up occupies the LDS for ~4 cycles (64 entries) / ~7 cycles (256 entries, bank
//     conflicts), against ~7.3 for a ds_bpermute-based register table.  The field extraction is a shift + mask
//     (a funnel shift where a 3-bit pair straddles two dwords; a byte select for b = 4).
//   * Per row the 64 lane sums are reduced with DPP adds (no LDS traffic), the slice sums of the W waves
//     are combined through LDS in a fixed order, the CSR term is added, and y is rounded to fp16 once.
//   * Sparse wave (balanced CSR, cf. Sec. 4.3): one extra wave per workgroup handles the nonzeros of the
//     block's rows while the dense waves stream.  The nonzeros of R consecutive rows are one contiguous
//     range of the CSR arrays; lane l takes nonzeros l, l + 64, ... of that range whatever rows they fall in
//     (equal work per lane), finds each one's row by comparing against the R + 1 row pointers held in
//     scalar registers, and the products are combined per row with a segmented scan built from DPP moves.
//     Only the last lane of each row segment touches the row's LDS accumulator, so no floating-point
//     atomics are needed and the result does not depend on timing.
//   * With a plan of the sparse term (a one-time re-layout of the CSR arrays, see PlanView) there is no sparse wave: every
//     dense wave fetches one 64-entry batch of the workgroup's slot at wave start, gathers its activations once its last
//     index row has been requested, and sums the four 16-entry row groups of the batch with fixed 16-lane reductions.
//   * matvec_multi_kernel / matvec_planned_multi_kernel run the workgroups of up to 16 layers in one grid: a workgroup
//     finds its layer from the first-block table in the kernel arguments and then runs the same per-block code, so every y
//     is bit for bit that of a launch of its own.
// Batches: two to sixteen activation columns go to matvec_b16_kernel, which runs the dense and the sparse term on the
// matrix cores (every lane decodes its own row, MFMAs replace the packed dot products); its header describes the
// lane mapping.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <type_traits>

#include "sqllm_kernels.h"

namespace sqllm {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32;
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
typedef u32 u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kLaneElems = 32;                      // indices per lane per row
constexpr int kSliceCols = kWave * kLaneElems;      // 2048 columns per wave
constexpr int kMaxDenseWaves = 14;                  // N <= 28672 (two more waves of the block take the sparse term)

// ---------------------------------------------------------------------------------------------- helpers
__device__ __forceinline__ u32 funnel_shr(u32 hi, u32 lo, u32 sh) { return __builtin_amdgcn_alignbit(hi, lo, sh); }
__device__ __forceinline__ half2_t as_half2(u32 v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ float half_bits_to_float(uint16_t h) { return (float)__builtin_bit_cast(half_t, h); }
__device__ __forceinline__ uint16_t float_to_half_bits(float f) { return __builtin_bit_cast(uint16_t, (half_t)f); }

// DPP controls (gfx9 encoding)
constexpr int kQuadXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kQuadXor2 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kWaveShl1 = 0x130;       // lane i reads lane i + 1
constexpr int kRowRor4 = 0x124, kRowRor8 = 0x128;
constexpr int kRowMirror = 0x140, kRowHalfMirror = 0x141;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f(float old, float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_i(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xF, false);
}

// Sum over the 64 lanes without LDS traffic; the total is valid in lane 63.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
    v += dpp_f<kQuadXor1>(0.f, v);
    v += dpp_f<kQuadXor2>(0.f, v);
    v += dpp_f<kRowHalfMirror>(0.f, v);
    v += dpp_f<kRowMirror>(0.f, v);                 // every lane: sum of its row of 16
    v += dpp_f<kRowBcast15, 0xA>(0.f, v);           // rows 1 and 3 add the row before them
    v += dpp_f<kRowBcast31, 0xC>(0.f, v);           // rows 2 and 3 add lane 31 (= rows 0 + 1)
    return v;
}

// ---------------------------------------------------------------------------------------------- index stream
// A lane's share of one row: BITS dwords = 32 indices.
template <int BITS>
struct LaneChunk {
    u32 q[BITS];
};

template <int BITS>
__device__ __forceinline__ LaneChunk<BITS> load_chunk(const u32* __restrict__ p) {
    LaneChunk<BITS> c;
#pragma unroll
    for (int k = 0; k < BITS; ++k) c.q[k] = __builtin_nontemporal_load(p + k);
    return c;
}

// the same from a uniform row pointer and the lane's dword offset inside the row: the address is formed by the load instruction
// (scalar base + 32-bit vector offset) instead of 64-bit vector arithmetic
template <int BITS>
__device__ __forceinline__ LaneChunk<BITS> load_chunk_at(const u32* __restrict__ row, u32 lane_dword) {
    LaneChunk<BITS> c;
    const u32* p = reinterpret_cast<const u32*>(reinterpret_cast<const char*>(row) + (size_t)(lane_dword * 4u));
#pragma unroll
    for (int k = 0; k < BITS; ++k) c.q[k] = __builtin_nontemporal_load(p + k);
    return c;
}

// Byte offsets (entry * 4) into the row's pair table of the 16 index pairs of a lane.
//   b = 3: pair p owns bits [6p, 6p + 6) of the 96-bit chunk; two of them straddle a dword boundary.
//   b = 4: pair p is byte p of the 128-bit chunk.
__device__ __forceinline__ void pair_offsets(const LaneChunk<3>& c, u32 (&a)[16]) {
    const u32 q0 = c.q[0], q1 = c.q[1], q2 = c.q[2];
    a[0] = (q0 << 2) & 0xFC;   a[1] = (q0 >> 4) & 0xFC;   a[2] = (q0 >> 10) & 0xFC;  a[3] = (q0 >> 16) & 0xFC;
    a[4] = (q0 >> 22) & 0xFC;
    a[5] = funnel_shr(q1, q0, 28) & 0xFC;               // bits 30..35 straddle dwords 0 and 1
    a[6] = (q1 >> 2) & 0xFC;   a[7] = (q1 >> 8) & 0xFC;   a[8] = (q1 >> 14) & 0xFC;  a[9] = (q1 >> 20) & 0xFC;
    a[10] = funnel_shr(q2, q1, 26) & 0xFC;              // bits 60..65 straddle dwords 1 and 2
    a[11] = q2 & 0xFC;         a[12] = (q2 >> 6) & 0xFC;  a[13] = (q2 >> 12) & 0xFC; a[14] = (q2 >> 18) & 0xFC;
    a[15] = (q2 >> 24) & 0xFC;
}
__device__ __forceinline__ void pair_offsets(const LaneChunk<4>& c, u32 (&a)[16]) {
#pragma unroll
    for (int p = 0; p < 16; ++p) a[p] = ((c.q[p >> 2] >> (8 * (p & 3))) & 0xFF) << 2;
}
//   b = 2: pair p is nibble p of the 64-bit chunk.
__device__ __forceinline__ void pair_offsets(const LaneChunk<2>& c, u32 (&a)[16]) {
#pragma unroll
    for (int p = 0; p < 16; ++p) a[p] = ((c.q[p >> 3] >> (4 * (p & 7))) & 0xF) << 2;
}

// the offset of pair p alone (p a compile-time constant after unrolling): the same values as pair_offsets
__device__ __forceinline__ u32 pair_offset_of(const LaneChunk<3>& c, int p) {
    const u32 q0 = c.q[0], q1 = c.q[1], q2 = c.q[2];
    switch (p) {
        case 0: return (q0 << 2) & 0xFC;
        case 1: return (q0 >> 4) & 0xFC;
        case 2: return (q0 >> 10) & 0xFC;
        case 3: return (q0 >> 16) & 0xFC;
        case 4: return (q0 >> 22) & 0xFC;
        case 5: return funnel_shr(q1, q0, 28) & 0xFC;
        case 6: return (q1 >> 2) & 0xFC;
        case 7: return (q1 >> 8) & 0xFC;
        case 8: return (q1 >> 14) & 0xFC;
        case 9: return (q1 >> 20) & 0xFC;
        case 10: return funnel_shr(q2, q1, 26) & 0xFC;
        case 11: return q2 & 0xFC;
        case 12: return (q2 >> 6) & 0xFC;
        case 13: return (q2 >> 12) & 0xFC;
        case 14: return (q2 >> 18) & 0xFC;
        default: return (q2 >> 24) & 0xFC;
    }
}
__device__ __forceinline__ u32 pair_offset_of(const LaneChunk<4>& c, int p) { return ((c.q[p >> 2] >> (8 * (p & 3))) & 0xFF) << 2; }
__device__ __forceinline__ u32 pair_offset_of(const LaneChunk<2>& c, int p) { return ((c.q[p >> 3] >> (4 * (p & 7))) & 0xF) << 2; }

template <int BITS>
struct TableShape {
    static constexpr int kEntryBits = 2 * BITS;               // a table entry holds the pair of two neighbouring indices: 4, 6 or 8 bits
    static constexpr int kEntries = 1 << kEntryBits;          // 16, 64 or 256
    static constexpr int kTableDwords = kEntries;             // LDS dwords of one row's table (one dword = two fp16 per entry)
    static constexpr int kRowBytes = 2 << BITS;               // bytes of one row's fp16 table: 8, 16 or 32
    static constexpr int kRawUnit = kRowBytes < 16 ? kRowBytes : 16;   // bytes of fp16 table one lane fetches
};

// Pair tables of R rows from their fp16 tables staged in LDS (raw[u << BITS | k]); executed by ONE wave.
template <int BITS, int R>
__device__ __forceinline__ void build_tables(u32* __restrict__ tables, const uint16_t* __restrict__ raw, int lane) {
    constexpr int E = TableShape<BITS>::kEntries, K = 1 << BITS;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        const u32 lo = raw[u * K + (lane & (K - 1))];           // the same for all entries of this lane
#pragma unroll
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            if (E >= kWave || e < E) {
                const u32 hi = raw[u * K + (e >> BITS)];
                tables[u * E + e] = lo | (hi << 16);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------- x in registers
// xr[p] = (x[j0 + 2p], x[j0 + 2p + 1]) for the lane's 32 columns j0 .. j0 + 31 (j0 is in range, x is one column).
__device__ __forceinline__ void load_x(const uint16_t* __restrict__ x, u32 j0, u32 (&xr)[16]) {
    const u32x4* src = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(x) + (size_t)(j0 * 2u));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const u32x4 v = src[k];
        xr[4 * k + 0] = v.x; xr[4 * k + 1] = v.y; xr[4 * k + 2] = v.z; xr[4 * k + 3] = v.w;
    }
}

// table look-ups of one row slice: 16 dwords, each an fp16 pair
template <int BITS>
__device__ __forceinline__ void lookup_chunk(const LaneChunk<BITS>& c, const u32* __restrict__ table, u32 (&w)[16]) {
    u32 a[16];
    pair_offsets(c, a);
    const char* tb = reinterpret_cast<const char*>(table);
#pragma unroll
    for (int p = 0; p < 16; ++p) w[p] = *reinterpret_cast<const u32*>(tb + a[p]);
}

// 16 packed dot products (two fp16 products each, fp32 accumulate) in two accumulator chains
__device__ __forceinline__ float dot_chunk(const u32 (&w)[16], const u32 (&xr)[16]) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int p = 0; p < 16; p += 2) {
        a0 = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[p]), a0, false);
        a1 = __builtin_amdgcn_fdot2(as_half2(w[p + 1]), as_half2(xr[p + 1]), a1, false);
    }
    return a0 + a1;
}

// Joint reduction of C per-lane values over the lanes of each 16-lane row (C = 4 or 8).  On return v[0] holds, in the lanes
// named by row_block_slot(), the sum of one input v[c] over the 16 lanes of the lane's row.  Butterfly steps halve the number of
// live values (3 VALU per produced value instead of a full 4-step reduction per input).  The association of the additions is
// the same for every c and both C -- quads first (lane ^ 1, lane ^ 2), then quad k with quad k ^ 2, then the two pair sums:
// ((q0 + q2) + (q1 + q3)) up to commutativity -- so a row's sum does not depend on how many rows its workgroup owns, and
// projections stacked into one call give bit for bit the dense term of separate calls.
template <int C>
__device__ __forceinline__ void row_block_reduce(float (&v)[C], int lane) {
    static_assert(C == 4 || C == 8, "block size");
    {   // lane bit 0, partner lane ^ 1: v[k] <- class 2 k + (lane & 1)
        const bool hi = lane & 1;
#pragma unroll
        for (int k = 0; k < C / 2; ++k) {
            const float keep = hi ? v[2 * k + 1] : v[2 * k], send = hi ? v[2 * k] : v[2 * k + 1];
            v[k] = keep + dpp_f<kQuadXor1>(0.f, send);
        }
    }
    {   // lane bit 1, partner lane ^ 2: v[k] <- class 4 k + (lane & 3)
        const bool hi = lane & 2;
#pragma unroll
        for (int k = 0; k < C / 4; ++k) {
            const float keep = hi ? v[2 * k + 1] : v[2 * k], send = hi ? v[2 * k] : v[2 * k + 1];
            v[k] = keep + dpp_f<kQuadXor2>(0.f, send);
        }
    }
    // lane bit 3 (a rotation by 8 lanes pairs lane l with lane l ^ 8): quads k and k ^ 2
    if constexpr (C == 8) {
        const bool hi = lane & 8;
        const float keep = hi ? v[1] : v[0], send = hi ? v[0] : v[1];
        v[0] = keep + dpp_f<kRowRor8>(0.f, send);            // lanes 0..7: class lane & 3; lanes 8..15: class 4 + (lane & 3)
    } else {
        v[0] += dpp_f<kRowRor8>(0.f, v[0]);
    }
    // lane bit 2: a rotation by 4 lanes hands quad k the pair sum of quad k - 1, which holds the same class for odd k
    v[0] += dpp_f<kRowRor4>(0.f, v[0]);
}
// lane of a 16-lane row that holds class c after row_block_reduce<C>: a lane of quad 1 (c < 4) or quad 3 (c >= 4)
__device__ __forceinline__ bool row_block_valid(int lane) { return (lane & 4) != 0; }
template <int C>
__device__ __forceinline__ int row_block_class(int lane) { return (C == 8 && (lane & 8)) ? 4 + (lane & 3) : (lane & 3); }

// ---------------------------------------------------------------------------------------------- sparse term
// Balanced CSR (cf. Sec. 4.3).  The nonzeros of the block's R rows are ONE contiguous range [P0, P1) of the
// CSR arrays.  It is cut into batches of 64; batch b goes to wave (b mod NW) and lane l of that wave takes
// nonzero P0 + 64 b + l, whatever row it falls in -- every lane of the block gets the same amount of work
// and a heavy row is spread over all waves.  A wave handles up to UB batches per round: first all column /
// value loads, then all activation gathers, then the reduction, so a round costs two memory round trips
// (which the dense decode of the same wave overlaps).  Products are combined per row inside the wave (plain
// DPP reduction when a batch lies in one row, segmented DPP scan otherwise) and only the last lane of a row
// segment adds to the wave's private LDS slot of that row: no floating-point atomics, fixed summation order.
// (One LDS float add per nonzero instead of the scan was measured: lanes meeting in a slot are served one after the other,
// 22016x8192 fused 19.4 -> 24.9 us.)
template <int UB>
struct SparseRegs {
    int c[UB];
    uint16_t vb[UB];
    uint16_t xv[UB];
};

struct SparseRange {
    int P0, P1, nbatch;
};

// Loads of one round are unconditional (indices clamped into [P0, P1), surplus lanes and batches are masked
// in the reduction), so that all of them are in flight at once.
template <int UB>
__device__ __forceinline__ void sparse_issue_cols_vals(const MatvecArgs& g, const SparseRange& sr, int b0, int NW, int lane, SparseRegs<UB>& q) {
    const int* __restrict__ cols = g.cols;
    const uint16_t* __restrict__ vals = static_cast<const uint16_t*>(g.vals);
#pragma unroll
    for (int k = 0; k < UB; ++k) {
        const int p = min(sr.P0 + (b0 + k * NW) * kWave + lane, sr.P1 - 1);
        q.c[k] = cols[p];
        q.vb[k] = vals[p];
    }
}

template <int UB>
__device__ __forceinline__ void sparse_issue_gathers(const uint16_t* __restrict__ x, SparseRegs<UB>& q) {
#pragma unroll
    for (int k = 0; k < UB; ++k) q.xv[k] = x[q.c[k]];
}

// LDS float add without a returned value: queued in order behind the wave's earlier LDS operations.  Only one
// wave ever touches a given slot and its lanes address distinct slots, so the summation order is fixed.
__device__ __forceinline__ void lds_add(float* slot, float v) { (void)__hip_atomic_fetch_add(slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

template <int R, int UB>
__device__ __forceinline__ void sparse_reduce(const SparseRange& sr, const int (&rp)[R + 1], int b0, int NW, int lane, const SparseRegs<UB>& q, float* __restrict__ slots) {
    int carry_row = -1;                                              // uniform: row whose sum is still in registers
    float carry = 0.f;
#pragma unroll
    for (int k = 0; k < UB; ++k) {
        const int b = b0 + k * NW;
        if (b < sr.nbatch) {                                         // uniform
            const int p_first = sr.P0 + b * kWave, p_last = min(p_first + kWave, sr.P1) - 1;
            const int p = p_first + lane;
            const bool ok = p <= p_last;
            float v = ok ? half_bits_to_float(q.vb[k]) * half_bits_to_float(q.xv[k]) : 0.f;
            int row_first = 0, row_last = 0;                         // rows of the batch's first / last nonzero
#pragma unroll
            for (int i = 1; i < R; ++i) { row_first += (p_first >= rp[i]) ? 1 : 0; row_last += (p_last >= rp[i]) ? 1 : 0; }
            if (row_first == row_last) {
                // the whole batch lies in one row: plain wave reduction, summed in registers across batches
                if (carry_row != row_first) {
                    if (carry_row >= 0 && lane == kWave - 1) lds_add(slots + carry_row, carry);
                    carry_row = row_first;
                    carry = 0.f;
                }
                carry += wave_sum_to_lane63(v);
            } else {
                int row = 0;                                         // number of i in 1..R-1 with rp[i] <= p
#pragma unroll
                for (int i = 1; i < R; ++i) row += (p >= rp[i]) ? 1 : 0;
                if (!ok) row = R;                                    // idle lanes form their own segment
                // segmented inclusive scan (rows are non-decreasing with the lane index)
#define SQ_SEG_STEP(CTRL, MASK)                                                        \
                {                                                                      \
                    const int r_up = dpp_i<CTRL, MASK>(-1, row);                       \
                    const float v_up = dpp_f<CTRL, MASK>(0.f, v);                      \
                    v += (r_up == row) ? v_up : 0.f;                                   \
                }
                SQ_SEG_STEP(kRowShr1, 0xF)
                SQ_SEG_STEP(kRowShr2, 0xF)
                SQ_SEG_STEP(kRowShr4, 0xF)
                SQ_SEG_STEP(kRowShr8, 0xF)
                SQ_SEG_STEP(kRowBcast15, 0xA)
                SQ_SEG_STEP(kRowBcast31, 0xC)
#undef SQ_SEG_STEP
                const int row_next = dpp_i<kWaveShl1>(-2, row);
                if (ok && row_next != row) lds_add(slots + row, v);  // last lane of its row segment
            }
        }
    }
    if (carry_row >= 0 && lane == kWave - 1) lds_add(slots + carry_row, carry);
}

template <int R, int U>
__device__ __forceinline__ void sparse_round(const MatvecArgs& g, const uint16_t* __restrict__ x, const SparseRange& sr, const int (&rp)[R + 1],
                                             int b0, int NW, int lane, float* __restrict__ slots) {
    SparseRegs<U> q;
    sparse_issue_cols_vals<U>(g, sr, b0, NW, lane, q);
    sparse_issue_gathers<U>(x, q);
    sparse_reduce<R, U>(sr, rp, b0, NW, lane, q, slots);
}

// ---------------------------------------------------------------------------------------------- the matvec kernel (one activation column)
// grid.x = ceil(M / R); block = (W + S) waves.  W = ceil(N / 2048) dense waves (0 without a dense term), wave w
// owning column slice w; S sparse waves (1 next to a dense term, kSparseOnlyWaves alone, 0 when nnz == 0).
// The sparse wave works through the first UB batches of the block's nonzeros while the dense waves stream
// (that is all of them except in blocks holding a very heavy row); whatever is left is dealt out to ALL
// waves once the dense waves have finished their rows, so a heavy row never serialises on one wave.
// The dense path is straight-line code: out-of-range lanes and rows load clamped (valid) addresses and are
// neutralised by zero activations / by not being stored.
constexpr int kSparseOnlyWaves = 4;

template <int R>
__device__ __forceinline__ void load_row_pointers(const MatvecArgs& g, int r0, int nrows, bool sparse, int (&rp)[R + 1], SparseRange& sr) {
#pragma unroll
    for (int k = 0; k <= R; ++k) rp[k] = sparse ? g.rowptr[r0 + min(k, nrows)] : 0;   // uniform -> scalar loads
    sr.P0 = rp[0]; sr.P1 = rp[R]; sr.nbatch = (sr.P1 - sr.P0 + kWave - 1) / kWave;
}

// The work of one workgroup: rows [R block, R block + R) of layer g, carried by the workgroup's first NW waves
// (W dense waves, then the sparse wave).
// Total of one output row over the workgroup's partial sums: `na` values a[i * R + row] followed by `nb` values b[i * R + row].
// Eight lanes per row (lane = 8 row + p) each add every eighth value in order, then the eight are combined by a butterfly whose
// every lane forms the same sums; the order depends on the counts only, not on R.  Valid in all eight lanes of a row < R.
template <int R>
__device__ __forceinline__ float block_row_total(const float* __restrict__ a, int na, const float* __restrict__ b, int nb, int lane) {
    const int row = lane >> 3, p = lane & 7;
    float s = 0.f;
    if (row < R) {
        for (int i = p; i < na + nb; i += 8) s += i < na ? a[i * R + row] : b[(i - na) * R + row];
    }
    s += dpp_f<kQuadXor1>(0.f, s);
    s += dpp_f<kQuadXor2>(0.f, s);
    s += dpp_f<kRowHalfMirror>(0.f, s);
    return s;
}

template <int BITS, int R, int D>
__device__ __forceinline__ void matvec_block(const MatvecArgs& g, int block, int NW) {
    static_assert(D >= 2 && D <= R && (R == 4 || R == 8), "prefetch depth, rows per workgroup");
    constexpr int E = TableShape<BITS>::kEntries, K = 1 << BITS;
    constexpr int kRawUnit = TableShape<BITS>::kRawUnit;             // bytes of fp16 tables one lane fetches (16, or 8 for b = 2)
    constexpr int UB = 8;                                            // sparse batches per wave and round
    constexpr int TD = TableShape<BITS>::kTableDwords;
    __shared__ __align__(8) u32 tables[R * TD];
    __shared__ __align__(16) uint16_t raw[R * K];
    __shared__ float part[kMaxDenseWaves * 4 * R];                   // dense:  [wave][16-lane row][r]
    __shared__ float spart[(kMaxDenseWaves + 1) * R];                // sparse: [wave][r]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
    const bool dense = g.qidx != nullptr, sparse = g.nnz > 0;
    const int W = dense ? (g.N + kSliceCols - 1) / kSliceCols : 0;
    const int r0 = block * R;
    const int nrows = min(R, g.M - r0);
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(g.x);

    int rp[R + 1];
    SparseRange sr;
    load_row_pointers<R>(g, r0, nrows, sparse, rp, sr);              // consumed late by the dense waves
    float* myslots = spart + wave * R;
    if (lane < R) myslots[lane] = 0.f;
    int next_batch = 0;                                              // first batch not yet handled (uniform)

    if (wave < W) {
        // ---- dense wave.  Issue order: (wave 0: fp16 tables), activations, first D rows of the index stream.
        // wave 0 fetches the fp16 tables of the block's rows (LPR lanes per row) and builds their pair tables
        constexpr int LPR = TableShape<BITS>::kRowBytes / kRawUnit;
        const int my_rows = wave == 0 ? R : 0;
        const int bu = lane / LPR;                                    // row of the block this lane fetches a piece of
        u32x4 rawv = {0, 0, 0, 0};
        if (lane < my_rows * LPR) {
            const int row = min(r0 + bu, g.M - 1);
            const char* src = static_cast<const char*>(g.lut) + (size_t)row * TableShape<BITS>::kRowBytes + (lane % LPR) * kRawUnit;
            if constexpr (kRawUnit == 16) {
                rawv = *reinterpret_cast<const u32x4*>(src);
            } else {
                const u32x2 v = *reinterpret_cast<const u32x2*>(src);
                rawv.x = v.x; rawv.y = v.y;
            }
        }
        const u32 j0 = (u32)wave * kSliceCols + (u32)lane * kLaneElems;
        const bool live = j0 < (u32)g.N;
        const u32 j0c = live ? j0 : (u32)g.N - kLaneElems;
        u32 xr[16];
        load_x(x, j0c, xr);
        const size_t row_dwords = (size_t)g.N * BITS / 32;
        const u32 lane_dword = (j0c >> 5) * BITS;                    // the lane's 32 indices inside a row of the index stream
        const u32* __restrict__ qrow0 = static_cast<const u32*>(g.qidx);
        auto row_ptr = [&](int u) {
            const u32 row = (u32)__builtin_amdgcn_readfirstlane(min(r0 + u, g.M - 1));   // uniform: the 64-bit product stays on the scalar unit
            return qrow0 + (size_t)row * row_dwords;
        };
        LaneChunk<BITS> c[R];
#pragma unroll
        for (int u = 0; u < D; ++u) c[u] = load_chunk_at<BITS>(row_ptr(u), lane_dword);
        if (!live) {
#pragma unroll
            for (int p = 0; p < 16; ++p) xr[p] = 0;
        }
        if (my_rows > 0) {                                            // uniform
            if (lane < my_rows * LPR) {
                if constexpr (kRawUnit == 16) *reinterpret_cast<u32x4*>(raw + bu * K + (lane % LPR) * 8) = rawv;
                else *reinterpret_cast<u32x2*>(raw + bu * K) = u32x2{rawv.x, rawv.y};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            build_tables<BITS, R>(tables, raw, lane);
        }
        __syncthreads();
        // software pipeline: the look-ups of row u + 1 are in flight while the products of row u are formed;
        // row u + D of the index stream is requested when row u has been handed to the look-ups
        float acc[R];
        u32 w[16];
        lookup_chunk<BITS>(c[0], tables, w);
        if constexpr (D < R) c[D] = load_chunk_at<BITS>(row_ptr(D), lane_dword);
#pragma unroll
        for (int u = 0; u < R; ++u) {
            if (u + 1 + D < R) c[(u + 1 + D) % R] = load_chunk_at<BITS>(row_ptr(u + 1 + D), lane_dword);
            // The look-ups of row u + 1 are issued one at a time between the products of row u (the product of a pair, two field
            // extractions, one look-up) instead of as a block of 16 -- the workgroups of a launch run in step, and blocks of
            // look-ups from all of them fill the LDS queue while the vector ALUs idle.
            // One set of 16 registers holds the pairs of both rows: the look-up of pair p of row u + 1 goes into the register the
            // product of pair p of row u has just read (two sets cost 8 to 16 registers per lane, i.e. a wave per SIMD).  The products
            // run in the two accumulator chains of dot_chunk; the scheduling barrier after every step keeps the order.
            {
                float a0 = 0.f, a1 = 0.f;
                const char* tb = reinterpret_cast<const char*>(tables + (u + 1 < R ? u + 1 : 0) * TD);
#pragma unroll
                for (int p = 0; p < 16; ++p) {
                    if (p & 1) a1 = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[p]), a1, false);
                    else a0 = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[p]), a0, false);
                    if (u + 1 < R) {
                        w[p] = *reinterpret_cast<const u32*>(tb + pair_offset_of(c[u + 1], p));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                acc[u] = a0 + a1;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // reduce the R row sums jointly over each 16-lane row of the wave
        row_block_reduce<R>(acc, lane);
        if (row_block_valid(lane) && (R == 8 || !(lane & 8))) part[(wave * 4 + (lane >> 4)) * R + row_block_class<R>(lane)] = acc[0];
        next_batch = UB;                                             // the sparse wave takes batches 0 .. UB-1
    } else {
        // ---- sparse wave(s)
        if (dense) {
            // columns and values of the first batches are requested BEFORE the dense waves' table barrier: the row pointers arrive
            // together with the fp16 tables, so the second hop of the chain (row pointers -> columns / values -> gathers -> scan)
            // runs while the tables are built instead of after (22016x8192 fused 21.3 -> 20.5 us)
            if (sr.nbatch > 2) {
                SparseRegs<UB> q;
                sparse_issue_cols_vals<UB>(g, sr, 0, 1, lane, q);
                __syncthreads();
                sparse_issue_gathers<UB>(x, q);
                sparse_reduce<R, UB>(sr, rp, 0, 1, lane, q, myslots);
            } else if (sr.nbatch > 0) {
                SparseRegs<2> q;
                sparse_issue_cols_vals<2>(g, sr, 0, 1, lane, q);
                __syncthreads();
                sparse_issue_gathers<2>(x, q);
                sparse_reduce<R, 2>(sr, rp, 0, 1, lane, q, myslots);
            } else {
                __syncthreads();
            }
            next_batch = UB;
        }
    }
    // ---- what is left of the sparse term (everything in a sparse-only launch): batch b goes to wave
    //      (b - next_batch) mod NW, UB batches per wave and round
    for (int b0 = next_batch + wave; b0 < sr.nbatch; b0 += NW * UB)   // uniform
        sparse_round<R, UB>(g, x, sr, rp, b0, NW, lane, myslots);
    __syncthreads();

    // combine the slice sums and the sparse partial sums in a fixed order, round once
    uint16_t* __restrict__ y = static_cast<uint16_t*>(g.y);
    if (wave == 0) {
        float s = block_row_total<R>(part, 4 * W, spart, sparse ? NW : 0, lane);
        const int row = lane >> 3;
        if ((lane & 7) == 0 && row < nrows) {
            if (g.accumulate) s += half_bits_to_float(y[r0 + row]);
            y[r0 + row] = float_to_half_bits(s);
        }
    }
}

// ---------------------------------------------------------------------------------------------- sparse term from a plan
// A plan (sqllm_kernels.h: PlanLayout) holds the nonzeros of every block of four rows (a "quad") as groups of 16 entries of one
// row, four groups to a batch of 64 lanes, the first C batches of a quad in a slot found from the quad index alone.  A workgroup
// of R rows serves R / 4 quads, each exactly as a four-row workgroup would (same batches on the same waves in the same order),
// so the sparse sums -- like the dense ones -- do not depend on R.  Against the
// CSR arrays this removes the first hop of the dependent chain (row pointers -> columns / values -> gathers), halves the loads
// per nonzero (column and value share a dword) and replaces the segmented scan by a fixed 16-lane reduction -- cheap enough for
// the dense waves to carry the sparse term themselves, so a workgroup needs no extra wave.
struct PlanView {
    const u32* slot_entries;    // [quads][C][64]
    const uint8_t* slot_tags;   // [quads][C][4]  one tag byte per group
    const int* ov_desc;         // [quads][2]     first overflow batch, overflow batches
    const u32* ov_entries;      // [ov batches][64]
    const uint8_t* ov_tags;     // [ov batches][4]
    int C;
    int ov_cap;                 // batches the overflow sections hold
};

constexpr int kPlanRows = 4;   // rows of a plan block ("quad"), whatever the rows per workgroup of the kernel that reads it

__device__ __forceinline__ PlanView plan_view(const void* plan, int M, long long nnz, int C) {
    // the offsets of plan_layout() on the host; C comes with the kernel arguments (its formula needs a 64-bit division)
    const size_t n_q = (size_t)((M + kPlanRows - 1) / kPlanRows);
    const size_t ov_cap = (size_t)((nnz / 16 + M) / 4) + n_q + 1;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    const char* b = static_cast<const char*>(plan);
    PlanView v;
    size_t o = 0;
    v.slot_entries = reinterpret_cast<const u32*>(b + o); o += up(n_q * C * 256);
    v.slot_tags = reinterpret_cast<const uint8_t*>(b + o); o += up(n_q * C * 4);
    v.ov_desc = reinterpret_cast<const int*>(b + o);      o += up(n_q * 8);
    v.ov_entries = reinterpret_cast<const u32*>(b + o);   o += up(ov_cap * 256);
    v.ov_tags = reinterpret_cast<const uint8_t*>(b + o);
    v.C = C;
    v.ov_cap = (int)ov_cap;
    return v;
}

// sum over each 16-lane row, valid in its lane 15
__device__ __forceinline__ float row16_sum_to_lane15(float v) {
    v += dpp_f<kRowShr1>(0.f, v);
    v += dpp_f<kRowShr2>(0.f, v);
    v += dpp_f<kRowShr4>(0.f, v);
    v += dpp_f<kRowShr8>(0.f, v);
    return v;
}

// one batch: entry, gathered activation and the tag byte of the lane's group (valid << 7 | (count - 1) << 3 | row) per lane ->
// the row sums go to the wave's slots
__device__ __forceinline__ void plan_batch_reduce(u32 entry, u32 xv, u32 tb, int lane, float* __restrict__ slots) {
    const bool ok = (tb & 0x80u) && (u32)(lane & 15) <= ((tb >> 3) & 15u);
    float v = ok ? half_bits_to_float((uint16_t)(entry >> 16)) * half_bits_to_float((uint16_t)xv) : 0.f;
    v = row16_sum_to_lane15(v);
    // one add per group, in group order (instructions of a wave reach the LDS in order): a fixed order of additions per slot
#pragma unroll
    for (int gi = 0; gi < 4; ++gi)
        if (lane == 16 * gi + 15 && (tb & 0x80u)) lds_add(slots + (tb & 7u), v);
}

template <int BITS, int R, int D>
__device__ __forceinline__ void matvec_planned_block(const MatvecArgs& g, int block, int W) {
    static_assert(D >= 2 && D <= R && (R == 4 || R == 8), "prefetch depth, rows per workgroup");
    constexpr int K = 1 << BITS;
    constexpr int kRawUnit = TableShape<BITS>::kRawUnit;
    constexpr int Q = R / kPlanRows;                                 // quads of the plan per workgroup; C <= W: one slot batch per wave and quad
    constexpr int UP = Q == 1 ? 2 : 1;                               // overflow batches per wave and quad requested ahead
    constexpr int TD = TableShape<BITS>::kTableDwords;
    __shared__ __align__(8) u32 tables[R * TD];
    __shared__ __align__(16) uint16_t raw[R * K];
    __shared__ float part[kMaxDenseWaves * 4 * R];                   // dense:  [wave][16-lane row][r]
    __shared__ float spart[kMaxDenseWaves * R];                      // sparse: [wave][r]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r0 = block * R;
    const int nrows = min(R, g.M - r0);
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(g.x);
    const PlanView pv = plan_view(g.plan, g.M, g.nnz, g.plan_c);
    const int n_quads = (g.M + kPlanRows - 1) / kPlanRows;
    float* myslots = spart + wave * R;
    if (lane < R) myslots[lane] = 0.f;

    // ---- Issue order: (wave 0: fp16 tables), activations, first D rows of the index stream, this wave's slot batches
    constexpr int LPR = TableShape<BITS>::kRowBytes / kRawUnit;
    const int my_rows = wave == 0 ? R : 0;
    const int bu = lane / LPR;
    u32x4 rawv = {0, 0, 0, 0};
    if (lane < my_rows * LPR) {
        const int row = min(r0 + bu, g.M - 1);
        const char* src = static_cast<const char*>(g.lut) + (size_t)row * TableShape<BITS>::kRowBytes + (lane % LPR) * kRawUnit;
        if constexpr (kRawUnit == 16) {
            rawv = *reinterpret_cast<const u32x4*>(src);
        } else {
            const u32x2 v = *reinterpret_cast<const u32x2*>(src);
            rawv.x = v.x; rawv.y = v.y;
        }
    }
    const u32 j0 = (u32)wave * kSliceCols + (u32)lane * kLaneElems;
    const bool live = j0 < (u32)g.N;
    const u32 j0c = live ? j0 : (u32)g.N - kLaneElems;
    u32 xr[16];
    load_x(x, j0c, xr);
    const size_t row_dwords = (size_t)g.N * BITS / 32;
    const u32 lane_dword = (j0c >> 5) * BITS;                        // the lane's 32 indices inside a row of the index stream
    const u32* __restrict__ qrow0 = static_cast<const u32*>(g.qidx); // row pointers below are uniform: r0 and M are
    auto row_ptr = [&](int u) {
        const u32 row = (u32)__builtin_amdgcn_readfirstlane(min(r0 + u, g.M - 1));   // keeps the 64-bit product on the scalar unit
        return qrow0 + (size_t)row * row_dwords;
    };
    LaneChunk<BITS> c[R];
#pragma unroll
    for (int u = 0; u < D; ++u) c[u] = load_chunk_at<BITS>(row_ptr(u), lane_dword);
    // The slot batch of this wave in quad q is batch `wave` of that quad's slot; past the slot (wave >= C) the last batch is
    // re-read and ignored.  Entries, tag bytes (one per group, fetched by the group's own lanes) and the overflow descriptors all
    // come through vector loads: a scalar load would have to be waited for together with every LDS operation of the wave.
    u32 ent[Q], tags[Q], sx[Q], oe[Q][UP], ot[Q][UP];
    int ovd[Q], ov_first[Q], ov_nb[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int quad = min(block * Q + q, n_quads - 1);            // a workgroup at the end of M may have no second quad
        const size_t sb = (size_t)quad * pv.C + min(wave, pv.C - 1);
        ent[q] = pv.slot_entries[sb * 64 + lane];
        tags[q] = pv.slot_tags[sb * 4 + (lane >> 4)];
        ovd[q] = pv.ov_desc[2 * quad + (lane & 1)];                  // lane 0: first overflow batch, lane 1: their number
        ov_first[q] = 0; ov_nb[q] = 0;
    }
    if (!live) {
#pragma unroll
        for (int p = 0; p < 16; ++p) xr[p] = 0;
    }
    if (my_rows > 0) {                                                // uniform
        if (lane < my_rows * LPR) {
            if constexpr (kRawUnit == 16) *reinterpret_cast<u32x4*>(raw + bu * K + (lane % LPR) * 8) = rawv;
            else *reinterpret_cast<u32x2*>(raw + bu * K) = u32x2{rawv.x, rawv.y};
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        build_tables<BITS, R>(tables, raw, lane);
    }
    __syncthreads();
    float acc[R];
    u32 w[16];                                                       // the pairs of the current row; each is replaced by the next row's once its product is formed
    lookup_chunk<BITS>(c[0], tables, w);
    if constexpr (D < R) c[D] = load_chunk_at<BITS>(row_ptr(D), lane_dword);
#pragma unroll
    for (int u = 0; u < R; ++u) {
        if (u + 1 < R) {
            if (u + 1 + D < R) c[(u + 1 + D) % R] = load_chunk_at<BITS>(row_ptr(u + 1 + D), lane_dword);
        }
        // The activations of the slot batches are gathered once the last row of the index stream has been requested: memory
        // results return in request order, so gathers issued earlier would stand between the wave and its next rows, and a
        // gather has to wait for its entry first (the scheduling barrier keeps the compiler from moving that wait, and with it
        // the request for the last row, the other way round).
        // With them go the requests for this wave's first overflow batches (a workgroup with a heavy row has some): their
        // place is known once the descriptor has arrived, which it has when the entries have.
        if (u + 1 + D == R - 1 || (D == R - 1 && u == 0)) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < Q; ++q) sx[q] = x[ent[q] & 0x7FFFu];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                ov_first[q] = __builtin_amdgcn_readlane(ovd[q], 0);
                ov_nb[q] = __builtin_amdgcn_readlane(ovd[q], 1);
#pragma unroll
                for (int k = 0; k < UP; ++k) {
                    const int b = min(ov_first[q] + min(wave + k * W, max(ov_nb[q] - 1, 0)), pv.ov_cap - 1);
                    oe[q][k] = pv.ov_entries[(size_t)b * 64 + lane];
                    ot[q][k] = pv.ov_tags[(size_t)b * 4 + (lane >> 4)];
                }
            }
        }
        // products of row u in the two accumulator chains of dot_chunk; the look-ups of row u + 1 take over its registers one by one
        // (as in matvec_block)
        {
            float a0 = 0.f, a1 = 0.f;
            const char* tb = reinterpret_cast<const char*>(tables + (u + 1 < R ? u + 1 : 0) * TD);
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                if (p & 1) a1 = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[p]), a1, false);
                else a0 = __builtin_amdgcn_fdot2(as_half2(w[p]), as_half2(xr[p]), a0, false);
                if (u + 1 < R) {
                    w[p] = *reinterpret_cast<const u32*>(tb + pair_offset_of(c[u + 1], p));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            acc[u] = a0 + a1;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    row_block_reduce<R>(acc, lane);
    if (row_block_valid(lane) && (R == 8 || !(lane & 8))) part[(wave * 4 + (lane >> 4)) * R + row_block_class<R>(lane)] = acc[0];
    // ---- sparse term, quad by quad: this wave's slot batch, then its share of the quad's overflow batches (batches wave, wave + W,
    // wave + 2 W, ... in this order whatever UP and R are)
    constexpr int UO = 8;                                            // batches per wave and round in the loop for very heavy rows
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        float* qslots = myslots + q * kPlanRows;
        const bool have = block * Q + q < n_quads;                   // uniform; the last workgroup of an odd number of quads has one
        const int nb = have ? ov_nb[q] : 0, first = ov_first[q];
        if (wave < pv.C && have) plan_batch_reduce(ent[q], sx[q], tags[q], lane, qslots);     // uniform
        if (wave < nb) {                                                                      // uniform
            u32 ox[UP];
#pragma unroll
            for (int k = 0; k < UP; ++k) ox[k] = x[oe[q][k] & 0x7FFFu];
#pragma unroll
            for (int k = 0; k < UP; ++k)
                if (wave + k * W < nb) plan_batch_reduce(oe[q][k], ox[k], ot[q][k], lane, qslots);
        }
        // what a very heavy row leaves after that: UO batches per wave and round, all requested before the first is used (the
        // workgroup that owns such a row ends last, and every round costs it two memory latencies)
        for (int ob = wave + UP * W; ob < nb; ob += UO * W) {                                 // uniform
            u32 e2[UO], t2[UO], x2[UO];
#pragma unroll
            for (int k = 0; k < UO; ++k) {
                const int b = min(ob + k * W, nb - 1);
                e2[k] = pv.ov_entries[(size_t)(first + b) * 64 + lane];
                t2[k] = pv.ov_tags[(size_t)(first + b) * 4 + (lane >> 4)];
            }
#pragma unroll
            for (int k = 0; k < UO; ++k) x2[k] = x[e2[k] & 0x7FFFu];
#pragma unroll
            for (int k = 0; k < UO; ++k)
                if (ob + k * W < nb) plan_batch_reduce(e2[k], x2[k], t2[k], lane, qslots);
        }
    }
    __syncthreads();
    uint16_t* __restrict__ y = static_cast<uint16_t*>(g.y);
    if (wave == 0) {
        const float s = block_row_total<R>(part, 4 * W, spart, W, lane);
        const int row = lane >> 3;
        if ((lane & 7) == 0 && row < nrows) y[r0 + row] = float_to_half_bits(s);
    }
}

template <int BITS, int R, int D>
__global__ void __launch_bounds__(1024) matvec_planned_kernel(MatvecArgs g) {
    matvec_planned_block<BITS, R, D>(g, blockIdx.x, blockDim.x >> 6);
}

// The arguments of a multi-layer launch as the kernel takes them (by value): only the fields its class reads, and room for 8 or
// 16 layers, whichever the launch needs.  The block stays under 1 KiB (16 planned layers: 968 bytes, 8 CSR layers: 616): launches
// with a larger one were measured 7 to 17 % slower over a whole decode step, whatever the layout of the fields, and a small block
// is a little faster than a large one below that size too.
struct PlannedLayer { int M, N, nnz, plan_c; const void *qidx, *lut, *x; void* y; const void* plan; };                            // 56 bytes
struct CsrLayer { int M, N, nnz, pad; const void *qidx, *lut, *x; void* y; const int* rowptr; const int* cols; const void* vals; };   // 72 bytes
template <class L, int K>
struct MultiKernArgs {
    int count;
    int first_block[K + 1];
    L layer[K];
};
template <class L, int K>
__device__ __forceinline__ int layer_of_block(const MultiKernArgs<L, K>& m) {
    int l = 0;
#pragma unroll
    for (int k = 1; k < K; ++k) l += (k < m.count && (int)blockIdx.x >= m.first_block[k]) ? 1 : 0;   // uniform
    return l;
}

template <int BITS, int R, int D, int K>
__global__ void __launch_bounds__(1024) matvec_planned_multi_kernel(MultiKernArgs<PlannedLayer, K> m) {
    const int l = layer_of_block(m);
    MatvecArgs g;
    const PlannedLayer& a = m.layer[l];
    g.M = a.M; g.N = a.N; g.bits = BITS; g.B = 1; g.bt0 = 0; g.bn = 1; g.accumulate = 0; g.nnz = a.nnz;
    g.qidx = a.qidx; g.lut = a.lut; g.rowptr = nullptr; g.cols = nullptr; g.vals = nullptr; g.x = a.x; g.y = a.y; g.plan = a.plan; g.plan_c = a.plan_c;
    const int W = (g.N + kSliceCols - 1) / kSliceCols;
    if ((int)(threadIdx.x >> 6) >= W) return;
    matvec_planned_block<BITS, R, D>(g, (int)blockIdx.x - m.first_block[l], W);
}

// ---- building a plan from the CSR arrays: count the batches of every workgroup, scan the overflow, fill
__device__ __forceinline__ int plan_groups_of(int cnt) { return (cnt + 15) >> 4; }

template <int R>
__global__ void __launch_bounds__(256) plan_count_kernel(int M, int n_wg, int C, const int* __restrict__ rowptr, int* __restrict__ ov_desc) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= n_wg) return;
    int groups = 0;
    for (int i = 0; i < R; ++i) {
        const int r = b * R + i;
        if (r < M) groups += plan_groups_of(rowptr[r + 1] - rowptr[r]);
    }
    const int nb = (groups + 3) >> 2;
    ov_desc[2 * b + 1] = nb > C ? nb - C : 0;
}

// exclusive scan of the overflow counts over the workgroups (one block; n_wg is a few thousand)
__global__ void __launch_bounds__(1024) plan_scan_kernel(int n_wg, int* __restrict__ ov_desc) {
    __shared__ int sums[1024];
    const int t = threadIdx.x;
    const int per = (n_wg + 1023) / 1024;
    const int lo = min(t * per, n_wg), hi = min(lo + per, n_wg);
    int s = 0;
    for (int b = lo; b < hi; ++b) s += ov_desc[2 * b + 1];
    sums[t] = s;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        const int v = t >= d ? sums[t - d] : 0;
        __syncthreads();
        sums[t] += v;
        __syncthreads();
    }
    int run = sums[t] - s;
    for (int b = lo; b < hi; ++b) { ov_desc[2 * b] = run; run += ov_desc[2 * b + 1]; }
}

// one wave per workgroup of the matvec: lane l fills entry l of every batch
template <int R>
__global__ void __launch_bounds__(64) plan_fill_kernel(int M, int C, const int* __restrict__ rowptr, const int* __restrict__ cols, const uint16_t* __restrict__ vals,
                                                       u32* __restrict__ slot_entries, uint8_t* __restrict__ slot_tags, const int* __restrict__ ov_desc,
                                                       u32* __restrict__ ov_entries, uint8_t* __restrict__ ov_tags) {
    const int b = blockIdx.x, lane = threadIdx.x;
    int gp[R + 1], rs[R + 1];                                        // first group / first nonzero of every row of the workgroup (uniform)
    gp[0] = 0;
#pragma unroll
    for (int i = 0; i <= R; ++i) rs[i] = rowptr[min(b * R + i, M)];
#pragma unroll
    for (int i = 0; i < R; ++i) gp[i + 1] = gp[i] + plan_groups_of(rs[i + 1] - rs[i]);
    const int groups = gp[R], nb = (groups + 3) >> 2;
    const int ov_first = ov_desc[2 * b];
    const int total = max(nb, C);                                    // unused slot batches are cleared
    for (int k = 0; k < total; ++k) {
        const int gidx = 4 * k + (lane >> 4);
        u32 entry = 0, tag = 0;
        if (gidx < groups) {
            int i = 0;
#pragma unroll
            for (int t = 1; t < R; ++t) i += gidx >= gp[t] ? 1 : 0;
            const int j = gidx - gp[i];
            const int left = rs[i + 1] - rs[i] - 16 * j;              // >= 1
            const int cnt = left < 16 ? left : 16;
            const int p = rs[i] + 16 * j + (lane & 15);
            if ((lane & 15) < cnt) entry = ((u32)cols[p] & 0x7FFFu) | ((u32)vals[p] << 16);
            tag = 0x80u | ((u32)(cnt - 1) << 3) | (u32)i;
        }
        if (k < C) {
            slot_entries[((size_t)b * C + k) * 64 + lane] = entry;
            if ((lane & 15) == 0) slot_tags[((size_t)b * C + k) * 4 + (lane >> 4)] = (uint8_t)tag;
        } else {
            ov_entries[((size_t)ov_first + k - C) * 64 + lane] = entry;
            if ((lane & 15) == 0) ov_tags[((size_t)ov_first + k - C) * 4 + (lane >> 4)] = (uint8_t)tag;
        }
    }
}

template <int BITS, int R, int D>
__global__ void __launch_bounds__(1024) matvec_kernel(MatvecArgs g) {
    matvec_block<BITS, R, D>(g, blockIdx.x, blockDim.x >> 6);
}

// Several independent layers in ONE launch (one activation column each): the grid is the concatenation of the layers' grids,
// workgroup b belongs to the layer l with first_block[l] <= b < first_block[l + 1].  The launch has as many waves per workgroup
// as its widest layer needs; in a narrower layer the surplus waves leave at once (a finished wave no longer takes part in the
// workgroup's barriers).  That is correct but slow -- two-wave layers in six-wave workgroups took 30 % longer than in a launch of
// their own -- so the host gives every wave count launches of its own and the early exit is only a guard.  Every layer is computed by the same code, in the same order of operations, as in a launch of its own,
// so the results are bit for bit those of separate calls -- what is saved is the launch and the ramp between them: the last
// workgroups of a layer run beside the first of the next.
template <int BITS, int R, int D, int K>
__global__ void __launch_bounds__(1024) matvec_multi_kernel(MultiKernArgs<CsrLayer, K> m) {
    const int l = layer_of_block(m);
    MatvecArgs g;
    const CsrLayer& a = m.layer[l];
    g.M = a.M; g.N = a.N; g.bits = BITS; g.B = 1; g.bt0 = 0; g.bn = 1; g.accumulate = 0; g.nnz = a.nnz;
    g.qidx = a.qidx; g.lut = a.lut; g.rowptr = a.rowptr; g.cols = a.cols; g.vals = a.vals; g.x = a.x; g.y = a.y; g.plan = nullptr;
    const int NW = (g.N + kSliceCols - 1) / kSliceCols + (g.nnz > 0 ? 1 : 0);
    if ((int)(threadIdx.x >> 6) >= NW) return;
    matvec_block<BITS, R, D>(g, (int)blockIdx.x - m.first_block[l], NW);
}

// ---------------------------------------------------------------------------------------------- up to sixteen activation columns on the matrix cores
// y[M][B] = (D + S) x[N][B] for 1 <= B <= 16 as a product of 16 x 16 tiles (v_mfma_f32_16x16x16_f16).  The
// instruction multiplies A (16 rows x 16 k) by B (16 k x 16 columns): lane l supplies A[l % 16][4 (l / 16) + e]
// and B[4 (l / 16) + e][l % 16], e = 0..3, and keeps D[4 (l / 16) + e][l % 16].
//   * A workgroup owns R = 16 RG rows and all N columns; its NW waves deal the 128-column windows of the row out
//     among themselves (wave w takes windows w, w + NW, ...).  In a window, lane (r, q) = (l % 16, l / 16) loads
//     the 32 indices of row r of each row group at columns 128 t + 32 q + [0, 32), looks them up in that row's
//     pair table -- the same decode as with one column -- and feeds weights 4 m .. 4 m + 3 to MFMA m (m = 0..7);
//     as B operand the same lane holds the activations of batch column r at the same 32 columns, gathered from x
//     with 16-bit loads (any row stride B <= 16, any parity) once per window and used for all RG row groups.
//   * The sparse term runs on the matrix cores as well: 16 consecutive nonzeros are one MFMA whose A operand
//     holds value p in the row of nonzero p (a lane compares p against the two row pointers of ITS row) and
//     whose B operand holds the activations of column cols[p].  The steps of a row group -- aligned groups of 16
//     nonzeros overlapping its CSR range -- are dealt out to the waves like the windows, so a heavy row is
//     spread over all waves and no reduction other than the accumulators is needed.
//   * Accumulators of the waves are combined through LDS in a fixed order; y is rounded to fp16 once.
typedef _Float16 half4v_t __attribute__((ext_vector_type(4)));
typedef float float4v_t __attribute__((ext_vector_type(4)));

template <int E>
__device__ __forceinline__ u32 quad_bcast(u32 v) {
    return (u32)__builtin_amdgcn_mov_dpp((int)v, E * 0x55, 0xF, 0xF, true);   // quad_perm: every lane reads lane E of its quad
}

constexpr int kB16StageBytes = 16 * 400;                  // one window of x for 16 columns: 16 planes of 64 row pairs (fast path), or the window as it lies in memory plus the shifts of its quarters (4224 bytes)

// Entry-major tables.  Lane l of a 16-lane group decodes its OWN matrix row, so the 32 lanes the LDS serves together
// read 32 different (row, entry) addresses; with one table after the other every row's entries overlay the same
// banks and the look-up takes ~7.5 cycles (hardware counters: 58 % of the LDS cycles were bank conflicts).  Here entry
// e of the block's row rho lives at byte (e R + rho) * kEntryBytes: a row owns one bank, rows never
// collide with each other and only the two lanes of one row can (2 passes per 32 lanes, as with one shared table).
// LDS addresses of the 16 entries of a lane's chunk: entry index times the entry stride 1 << S, OR the
// row's offset `base` < 1 << S (the tables start at LDS address 0: the kernel has no other static or dynamic LDS before them):
template <int S>
__device__ __forceinline__ void entry_offsets(const LaneChunk<3>& c, u32 base, u32 (&a)[16]) {
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int bit = 6 * p, d = bit >> 5, pos = bit & 31;
        const u32 f = pos + 6 <= 32 ? (c.q[d] >> pos) & 63u : funnel_shr(c.q[(d + 1) % 3], c.q[d], pos) & 63u;   // a pair never starts in the last 6 bits of dword 2
        a[p] = (f << S) | base;
    }
}
template <int S>
__device__ __forceinline__ void entry_offsets(const LaneChunk<4>& c, u32 base, u32 (&a)[16]) {
#pragma unroll
    for (int p = 0; p < 16; ++p) a[p] = (((c.q[p >> 2] >> (8 * (p & 3))) & 0xFFu) << S) | base;
}
template <int S>
__device__ __forceinline__ void entry_offsets(const LaneChunk<2>& c, u32 base, u32 (&a)[16]) {
#pragma unroll
    for (int p = 0; p < 16; ++p) a[p] = (((c.q[p >> 3] >> (4 * (p & 7))) & 0xFu) << S) | base;
}
template <int BITS, int S>
__device__ __forceinline__ void lookup_chunk_at(const LaneChunk<BITS>& c, u32 base, u32 (&w)[16]) {
    u32 a[16];
    entry_offsets<S>(c, base, a);
#pragma unroll
    for (int p = 0; p < 16; ++p) w[p] = *reinterpret_cast<const __attribute__((address_space(3))) u32*>(a[p]);
}

// Sparse term of the 16-column kernel.  Step j covers the nonzeros [16 j, 16 j + 16); the steps overlapping the CSR
// range of row group rg are first[rg] .. first[rg] + count[rg] - 1, and flat step f of the block runs through the
// row groups in order.  A wave handles NS flat steps f0, f0 + NW, ... per round: all column / value loads, then all
// activation gathers, then the products.  Slots past the block's last step re-read step 0 and contribute nothing.
template <int RG, int NS>
struct B16SparseSlots {
    int srg[NS], sj[NS];      // uniform: row group (-1: none) and step of each slot
    u32 col[NS], val[NS];     // lane e of a quad holds nonzero 16 j + 4 q + e
};

template <int RG, int NS>
__device__ __forceinline__ void b16_sparse_issue(const MatvecArgs& g, const int (&first)[RG], const int (&count)[RG], int total, int f0, int NW,
                                                 int lane, B16SparseSlots<RG, NS>& S) {
    const int last_nz = (int)g.nnz - 1;
    const uint16_t* __restrict__ vals = static_cast<const uint16_t*>(g.vals);
    const int e4 = 4 * (lane >> 4) + (lane & 3);
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        int f = f0 + k * NW;
        S.srg[k] = -1; S.sj[k] = 0;
        if (f < total) {
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                if (S.srg[k] < 0) {
                    if (f < count[rg]) { S.srg[k] = rg; S.sj[k] = first[rg] + f; }
                    else f -= count[rg];
                }
            }
        }
        const int pl = min(16 * S.sj[k] + e4, last_nz);
        S.col[k] = (u32)g.cols[pl];
        S.val[k] = vals[pl];
    }
}

// QT (B a multiple of 4): the activations of a step are gathered with ONE 8-byte load per lane -- lane e of a quad reads
// the four columns 4 (n / 4) .. + 3 of the x row of ITS nonzero -- and a 4 x 4 transposition inside the quad (three quad
// permutes) hands every lane its own column of all four nonzeros; otherwise four 16-bit loads per lane.
template <int RG, int NS, bool QT>
__device__ __forceinline__ void b16_sparse_finish(const uint16_t* __restrict__ x, int B, int nb, u32 xmask, int lane, const int (&lo)[RG], const int (&hi)[RG],
                                                  const B16SparseSlots<RG, NS>& S, float4v_t (&acc)[RG]) {
    const int q = lane >> 4;
    const char* xb = reinterpret_cast<const char*>(x);
    u32 xa[NS][2], aa[NS][2];
    if constexpr (QT) {
        const u32 cg = 4u * ((u32)nb >> 2);                          // first column of the lane's group of four (0 for absent columns)
        const bool odd = (lane & 1) != 0, upper = (lane & 2) != 0;
        const u32 sel = odd ? 0x03020706u : 0x05040100u;
        u32x2 d[NS];
#pragma unroll
        for (int k = 0; k < NS; ++k) d[k] = *reinterpret_cast<const u32x2*>(xb + 2u * (S.col[k] * (u32)B + cg));   // byte offsets fit 32 bits
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            // rows = the quad's four nonzeros, columns = the group's four batch columns; first the 2 x 2 blocks of halves ...
            const u32 p0 = (u32)__builtin_amdgcn_mov_dpp((int)d[k].x, 0xB1, 0xF, 0xF, true), p1 = (u32)__builtin_amdgcn_mov_dpp((int)d[k].y, 0xB1, 0xF, 0xF, true);
            const u32 e0 = __builtin_amdgcn_perm(p0, d[k].x, sel), e1 = __builtin_amdgcn_perm(p1, d[k].y, sel);
            // ... then the dwords between lanes 2 apart
            const u32 send = upper ? e0 : e1;
            const u32 recv = (u32)__builtin_amdgcn_mov_dpp((int)send, 0x4E, 0xF, 0xF, true);
            xa[k][0] = (upper ? recv : e0) & xmask;
            xa[k][1] = (upper ? e1 : recv) & xmask;
        }
    } else {
#pragma unroll
        for (int k = 0; k < NS; ++k) {
            // byte offsets fit 32 bits: N * B * 2 < 2^20
            const u32 c0 = quad_bcast<0>(S.col[k]), c1 = quad_bcast<1>(S.col[k]), c2 = quad_bcast<2>(S.col[k]), c3 = quad_bcast<3>(S.col[k]);
            const u32 x0 = *reinterpret_cast<const uint16_t*>(xb + 2u * (c0 * (u32)B + (u32)nb)), x1 = *reinterpret_cast<const uint16_t*>(xb + 2u * (c1 * (u32)B + (u32)nb));
            const u32 x2 = *reinterpret_cast<const uint16_t*>(xb + 2u * (c2 * (u32)B + (u32)nb)), x3 = *reinterpret_cast<const uint16_t*>(xb + 2u * (c3 * (u32)B + (u32)nb));
            xa[k][0] = (x0 | (x1 << 16)) & xmask;
            xa[k][1] = (x2 | (x3 << 16)) & xmask;
        }
    }
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        const int p0 = 16 * S.sj[k] + 4 * q;
        int l = 0, h = 0;
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) { if (S.srg[k] == rg) { l = lo[rg]; h = hi[rg]; } }
        const u32 v0 = quad_bcast<0>(S.val[k]), v1 = quad_bcast<1>(S.val[k]), v2 = quad_bcast<2>(S.val[k]), v3 = quad_bcast<3>(S.val[k]);
        // value p goes to the row whose CSR range holds p: 0 <= p - l < h - l as one unsigned comparison
        const u32 span = (u32)(h - l), d0 = (u32)(p0 - l);
        const u32 a0 = d0 < span ? v0 : 0u, a1 = d0 + 1u < span ? v1 : 0u, a2 = d0 + 2u < span ? v2 : 0u, a3 = d0 + 3u < span ? v3 : 0u;
        aa[k][0] = a0 | (a1 << 16);
        aa[k][1] = a2 | (a3 << 16);
    }
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        const half4v_t a = __builtin_bit_cast(half4v_t, u32x2{aa[k][0], aa[k][1]});
        const half4v_t b = __builtin_bit_cast(half4v_t, u32x2{xa[k][0], xa[k][1]});
#pragma unroll
        for (int rg = 0; rg < RG; ++rg)
            if (S.srg[k] == rg) acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, acc[rg], 0, 0, 0);   // uniform branch
    }
}

// B4 = 1..4: the batch is exactly 4 B4 columns (4, 8, 12 or 16); B4 = 5: exactly 2 columns -- the activations take the
// fast paths below;  B4 == 0: any batch up to 16, activations staged as they lie in memory.
template <int BITS, int RG, int B4>
__global__ void __launch_bounds__(1024) matvec_b16_kernel(MatvecArgs g) {
    constexpr int R = 16 * RG, K = 1 << BITS;
    constexpr int TD = TableShape<BITS>::kTableDwords;
    constexpr int kRawUnit = TableShape<BITS>::kRawUnit;
    constexpr int kRawLanes = R * TableShape<BITS>::kRowBytes / kRawUnit;
    constexpr int kWinCols = 128;
    extern __shared__ __align__(2048) char smem16[];
    u32* tables = reinterpret_cast<u32*>(smem16);                                   // R tables, each 4 TD bytes (a power of two)
    uint16_t* raw = reinterpret_cast<uint16_t*>(smem16 + R * TD * 4);               // fp16 tables as loaded
    char* stage0 = smem16 + R * TD * 4 + R * K * 2;                                 // per wave: staging of one x window, later its partial sums

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform, and known to be: addresses derived from it stay in scalar registers
    const int NW = blockDim.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int r0 = blockIdx.x * R;
    const int nrows = min(R, g.M - r0);
    const int B = g.B;
    const bool dense = g.qidx != nullptr, sparse = g.nnz > 0;
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(g.x);
    const int nwin = dense ? g.N / kWinCols : 0;
    char* stage = stage0 + wave * kB16StageBytes;
    const int NWD = dense ? NW : 0;                                  // every wave takes windows of the dense term (if there is one) ...
    const bool sparse_wave = sparse;                                 // ... and afterwards a share of the sparse term

    // ---- fp16 tables of the block's rows -> LDS
    if (dense && tid < kRawLanes) {
        const int u = tid * kRawUnit / TableShape<BITS>::kRowBytes;
        const int row = min(r0 + u, g.M - 1);
        const char* src = static_cast<const char*>(g.lut) + (size_t)row * TableShape<BITS>::kRowBytes + (tid * kRawUnit) % TableShape<BITS>::kRowBytes;
        if constexpr (kRawUnit == 16) *reinterpret_cast<u32x4*>(raw + tid * 8) = *reinterpret_cast<const u32x4*>(src);
        else *reinterpret_cast<u32x2*>(raw + tid * 4) = *reinterpret_cast<const u32x2*>(src);
    }
    // row pointers of the lane's own row in every row group (rows past M are empty)
    int lo[RG], hi[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        lo[rg] = sparse_wave ? g.rowptr[min(r0 + 16 * rg + r, g.M)] : 0;
        hi[rg] = sparse_wave ? g.rowptr[min(r0 + 16 * rg + r + 1, g.M)] : 0;
    }
    const size_t row_dwords = (size_t)g.N * BITS / 32;
    const int nb = r < B ? r : 0;                                    // lanes of absent columns read column 0 and are zeroed
    const u32 xmask = r < B ? 0xFFFFFFFFu : 0u;
    auto load_idx = [&](int t, LaneChunk<BITS> (&c)[RG]) {
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            const int row = min(r0 + 16 * rg + r, g.M - 1);
            c[rg] = load_chunk<BITS>(static_cast<const u32*>(g.qidx) + (size_t)row * row_dwords + (size_t)(4 * t + q) * BITS);
        }
    };
    // Activations of a window: the 128 rows of x are 64 B contiguous dwords.  They are copied to LDS as they lie in
    // memory (coalesced loads, 16 B dwords per quarter of the window, every quarter shifted by 32 bytes so that the four
    // lane groups read different banks), and each lane then picks the 32 halves of ITS column with 16-bit reads.
    // Load slot (qq, ii) covers dwords 64 ii + lane of quarter qq; slots past the quarter re-read its last dword.
    const int qd = 16 * B;                                           // dwords of one quarter (32 rows of x)
    u32 eoff[4];                                                     // byte offset of the lane's dword in load slot ii of a quarter
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) eoff[ii] = 4u * (u32)min(64 * ii + lane, qd - 1);
    const u32 stage_lds = (u32)(size_t)stage;                        // LDS byte address of the wave's staging area (uniform)
    constexpr int kEntryBytes = 4;                                    // one pair of fp16 per entry
    constexpr int kStrideLog2 = (RG == 2 ? 5 : 4) + 2;               // log2(R * kEntryBytes): bytes from one entry to the next
    const u32 tab0 = (u32)r * kEntryBytes;                           // the lane's row of row group 0; the tables start at LDS address 0
    constexpr int BT = B4 == 5 ? 2 : 4 * B4, kPitch = 256 + 16;      // fast path: columns, bytes of one column's 64 row pairs (+ bank shift)
    constexpr u32 kPitchQ = 400;                                     // plane pitch of the 8- and 16-column paths: 64 row pairs + up to 24 dwords of rotation
    auto load_xblock = [&](int t, u32 (&v)[16]) {
        if constexpr (B4 == 4 || B4 == 2) {
            // fully coalesced: load i of lane l is the 16-byte unit 64 i + l of the window (half a row of 16 columns, or
            // a whole row of 8); the neighbouring row sits two lanes (one lane) further and is fetched with a quad permute
            const u32x4* src = reinterpret_cast<const u32x4*>(x + (size_t)t * kWinCols * BT) + lane;
#pragma unroll
            for (int i = 0; i < B4; ++i) {
                const u32x4 v4 = src[64 * i];
                v[4 * i] = v4.x; v[4 * i + 1] = v4.y; v[4 * i + 2] = v4.z; v[4 * i + 3] = v4.w;
            }
        } else if constexpr (B4 > 0) {
            // lane l fetches rows 2 l and 2 l + 1 of the window: 4 BT contiguous bytes
            const char* src = reinterpret_cast<const char*>(x + (size_t)t * kWinCols * BT) + (u32)lane * 4u * BT;
            if constexpr (BT == 2) {
                const u32x2 v2 = *reinterpret_cast<const u32x2*>(src);
                v[0] = v2.x; v[1] = v2.y;
            } else {
#pragma unroll
                for (int i = 0; i < BT / 4; ++i) {
                    const u32x4 v4 = reinterpret_cast<const u32x4*>(src)[i];
                    v[4 * i] = v4.x; v[4 * i + 1] = v4.y; v[4 * i + 2] = v4.z; v[4 * i + 3] = v4.w;
                }
            }
        } else {
            const char* src = reinterpret_cast<const char*>(x + (size_t)t * kWinCols * B);   // uniform
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const char* sq = src + (size_t)(4 * qq * qd);        // uniform
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) v[4 * qq + ii] = *reinterpret_cast<const u32*>(sq + eoff[ii]);
            }
        }
    };
    const u32 rd0 = stage_lds + 4u * q * qd + 32u * q + 2u * nb;     // slow path: row 32 q of the window, column nb
    auto stage_x = [&](const u32 (&v)[16], u32 (&xb)[16]) {
        if constexpr (B4 == 4 || B4 == 2) {
            // own row k and its neighbour k ^ 1 (lane ^ 2 for 16 columns, lane ^ 1 for 8): the lane of the even row forms
            // the pair (x[k][n], x[k + 1][n]) of the even column n of each dword, the lane of the odd row that of the odd column
            const bool keven = B4 == 4 ? (lane & 2) == 0 : (lane & 1) == 0;
            const u32 sel = keven ? 0x05040100u : 0x03020706u;
            // Plane n holds the 64 row pairs of column n, rotated by rot(n) dwords (planes of kPitchQ = 100 dwords, so a
            // rotated plane needs no wrap-around).  The rotation makes BOTH sides conflict-free: the 32 lanes the LDS
            // serves together write 8 (16) consecutive row pairs of 4 (2) planes whose bank offsets 4 n + rot(n) are 0, 8,
            // 16, 24 (0, 16) apart, and 8 neighbouring lanes read 16 bytes of 8 planes whose offsets are the 8 multiples
            // of 4.  Without it every write was a 4-way conflict (counters: 61 % of the LDS cycles).
            //   16 columns: rot(n) = 4 + 4 [n%4 == 1] - 4 [n%4 == 2] + 16 [n >= 8];   8 columns: rot(n) = 12 - 4 (n / 2) + 12 (n % 2)
            const u32 odd = keven ? 0u : 1u, h = (u32)lane & 1u;
            const u32 wr = B4 == 4 ? stage_lds + (8u * h + odd) * kPitchQ + ((u32)(lane >> 2) + 4u * odd + 16u * h) * 4u
                                   : stage_lds + odd * kPitchQ + ((u32)(lane >> 1) + 12u * odd) * 4u;
#pragma unroll
            for (int i = 0; i < B4; ++i)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const u32 own = v[4 * i + d];
                    const u32 other = (u32)__builtin_amdgcn_mov_dpp((int)own, B4 == 4 ? 0x4E : 0xB1, 0xF, 0xF, true);   // quad_perm [2,3,0,1] / [1,0,3,2]
                    const u32 pair = __builtin_amdgcn_perm(other, own, sel);
                    const u32 off = B4 == 4 ? (u32)(2 * d) * kPitchQ + 64u * i + 16u * (1 - (d & 1))
                                            : (u32)(2 * d) * kPitchQ + 128u * i + 4u * (12 - 4 * d);
                    *reinterpret_cast<__attribute__((address_space(3))) u32*>(wr + off) = pair;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const u32 n3 = (u32)nb & 3u;
            const u32 rot = B4 == 4 ? 4u + (n3 == 1u ? 4u : 0u) - (n3 == 2u ? 4u : 0u) + 16u * ((u32)nb >> 3)
                                    : 12u - 4u * (((u32)nb & 7u) >> 1) + 12u * ((u32)nb & 1u);
            const u32 rd = stage_lds + (u32)nb * kPitchQ + ((u32)q * 16u + rot) * 4u;
            const u32 xm = B4 == 4 ? 0xFFFFFFFFu : xmask;            // with 16 columns every lane's column exists
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 v4 = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(rd + 16u * i);
                xb[4 * i] = v4.x & xm; xb[4 * i + 1] = v4.y & xm; xb[4 * i + 2] = v4.z & xm; xb[4 * i + 3] = v4.w & xm;
            }
        } else if constexpr (B4 > 0) {
            // v[d], d < BT / 2: columns 2 d, 2 d + 1 of row 2 l; v[BT / 2 + d]: the same of row 2 l + 1.  The pair
            // (x[2 l][n], x[2 l + 1][n]) goes to dword l of column n's plane; lane (n, q) then reads 64 bytes of plane n.
#pragma unroll
            for (int n = 0; n < BT; ++n) {
                const u32 pair = __builtin_amdgcn_perm(v[BT / 2 + n / 2], v[n / 2], (n & 1) ? 0x07060302u : 0x05040100u);
                *reinterpret_cast<__attribute__((address_space(3))) u32*>(stage_lds + (u32)n * kPitch + (u32)lane * 4u) = pair;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const u32 rd = stage_lds + (u32)nb * kPitch + (u32)q * 64u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 v4 = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(rd + 16u * i);
                xb[4 * i] = v4.x & xmask; xb[4 * i + 1] = v4.y & xmask; xb[4 * i + 2] = v4.z & xmask; xb[4 * i + 3] = v4.w & xmask;
            }
        } else {
            // the strides are recomputed from a copy of B the compiler cannot see through: hoisted out of the window
            // loop the 48 addresses would occupy 48 registers for the whole kernel
            u32 Bl = (u32)B;
            asm volatile("" : "+s"(Bl));
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const u32 base = stage_lds + 64u * qq * Bl + 32u * qq;   // uniform
#pragma unroll
                for (int ii = 0; ii < 4; ++ii)
                    *reinterpret_cast<__attribute__((address_space(3))) u32*>(base + eoff[ii]) = v[4 * qq + ii];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const u32 a = *reinterpret_cast<const __attribute__((address_space(3))) uint16_t*>(rd0 + (u32)(2 * p) * 2u * Bl);
                const u32 b = *reinterpret_cast<const __attribute__((address_space(3))) uint16_t*>(rd0 + (u32)(2 * p + 1) * 2u * Bl);
                xb[p] = (a | (b << 16)) & xmask;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // ---- the first two windows of this wave are requested before the tables are built
    LaneChunk<BITS> c0[RG], c1[RG], c2[RG];
    u32 xb[16], xv[16];
    int t = dense ? wave : 0;                                        // wave w takes windows w, w + NWD, ... (NWD <= nwin)
    const int last_t = t < nwin ? wave + ((nwin - 1 - wave) / NWD) * NWD : 0;   // this wave's last window
    if (t < nwin) {
        load_xblock(t, xv);
        load_idx(t, c0);
        load_idx(min(t + NWD, last_t), c1);
    }
    __syncthreads();
    if (dense)
        for (int o = tid; o < R * TableShape<BITS>::kEntries; o += blockDim.x) {
            // consecutive threads write consecutive rows of one entry (conflict-free); see entry_offsets for the layout
            const int rho = o % R, e = o / R;
            const uint16_t* rr = raw + rho * K;
            const u32 lo16 = rr[e & (K - 1)], hi16 = rr[e >> BITS];
            tables[o] = lo16 | (hi16 << 16);
        }
    __syncthreads();

    float4v_t acc[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) acc[rg] = float4v_t{0.f, 0.f, 0.f, 0.f};

    // ---- dense term: windows t, t + NW, ...  Indices are requested two windows ahead, activations one window ahead
    //      (from L2) and staged while the matrix cores work on the current window.  Past the wave's last window the
    //      requests repeat that window (valid addresses, results unused) instead of branching around loads.
    if (t < nwin) {
        stage_x(xv, xb);
        load_xblock(min(t + NWD, last_t), xv);
    }
    for (; t < nwin; t += NWD) {
        load_idx(min(t + 2 * NWD, last_t), c2);
        u32 w[2][16];
        lookup_chunk_at<BITS, kStrideLog2>(c0[0], tab0, w[0]);
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            if (rg + 1 < RG) lookup_chunk_at<BITS, kStrideLog2>(c0[rg + 1], tab0 + 16u * (rg + 1) * kEntryBytes, w[(rg + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const half4v_t a = __builtin_bit_cast(half4v_t, u32x2{w[rg & 1][2 * m], w[rg & 1][2 * m + 1]});
                const half4v_t b = __builtin_bit_cast(half4v_t, u32x2{xb[2 * m], xb[2 * m + 1]});
                acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, acc[rg], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        stage_x(xv, xb);                                             // window t + NWD
        load_xblock(min(t + 2 * NWD, last_t), xv);
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) { c0[rg] = c1[rg]; c1[rg] = c2[rg]; }
    }

    // ---- sparse term, after the dense windows: every wave takes steps wave, wave + NW, ... of the block (a heavy row
    //      is spread over all waves); rounds of 4 steps per wave, of 8 while more than 4 NW steps are left, of 12 beyond
    //      8 NW (16 would spill; 8192x8192 at 16 columns: 23.1 -> 22.2 us with the rounds of 12)
    if (sparse_wave) {
        int first[RG], count[RG], total = 0;                         // uniform
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            const int P0 = __builtin_amdgcn_readlane(lo[rg], 0), P1 = __builtin_amdgcn_readlane(hi[rg], 15);
            first[rg] = P0 >> 4;
            count[rg] = P1 > P0 ? ((P1 - 1) >> 4) - (P0 >> 4) + 1 : 0;
            total += count[rg];
        }
        int f0 = wave;
        while (f0 < total) {
            if (total - f0 > 8 * NW) {
                B16SparseSlots<RG, 12> S;
                b16_sparse_issue<RG, 12>(g, first, count, total, f0, NW, lane, S);
                b16_sparse_finish<RG, 12, (B4 >= 1 && B4 <= 4)>(x, B, nb, xmask, lane, lo, hi, S, acc);
                f0 += 12 * NW;
            } else if (total - f0 > 4 * NW) {
                B16SparseSlots<RG, 8> S;
                b16_sparse_issue<RG, 8>(g, first, count, total, f0, NW, lane, S);
                b16_sparse_finish<RG, 8, (B4 >= 1 && B4 <= 4)>(x, B, nb, xmask, lane, lo, hi, S, acc);
                f0 += 8 * NW;
            } else {
                B16SparseSlots<RG, 4> S;
                b16_sparse_issue<RG, 4>(g, first, count, total, f0, NW, lane, S);
                b16_sparse_finish<RG, 4, (B4 >= 1 && B4 <= 4)>(x, B, nb, xmask, lane, lo, hi, S, acc);
                f0 += 4 * NW;
            }
        }
    }

    // ---- combine the waves' accumulators in a fixed order: lane (r, q) holds rows 4 q + e of column r
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        const float v[4] = {acc[rg].x, acc[rg].y, acc[rg].z, acc[rg].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) reinterpret_cast<float*>(stage)[(16 * rg + 4 * q + e) * 16 + r] = v[e];
    }
    __syncthreads();
    uint16_t* __restrict__ y = static_cast<uint16_t*>(g.y);
    for (int o = tid; o < R * 16; o += blockDim.x) {
        const int row = o >> 4, n = o & 15;
        if (row < nrows && n < B) {
            float sum = 0.f;
            for (int wv = 0; wv < NW; ++wv) sum += reinterpret_cast<const float*>(stage0 + wv * kB16StageBytes)[row * 16 + n];
            const size_t yo = (size_t)(r0 + row) * B + n;
            if (g.accumulate) sum += half_bits_to_float(y[yo]);
            y[yo] = float_to_half_bits(sum);
        }
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
            const float v = half_bits_to_float(vals[p]);
#pragma unroll
            for (int t = 0; t < NB; ++t)
                if (t < g.bn) acc[t] += v * half_bits_to_float(x[(size_t)c * g.B + t]);
        }
    }
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        if (t >= g.bn) continue;
        const size_t o = (size_t)i * g.B + t;
        float s = acc[t];
        if (g.accumulate) s += half_bits_to_float(y[o]);
        y[o] = float_to_half_bits(s);
    }
}

// ---------------------------------------------------------------------------------------------- parity exports
// Same load, field extraction, table build and look-up as the matvec; one wave per (row, slice).
// Without a table (lut == nullptr) the fp16 table is replaced by the bit patterns 0, 1, 2, ... so that the
// look-up returns the indices themselves.
template <int BITS>
__global__ void __launch_bounds__(64) decode_kernel(int M, int N, const void* qidx, const void* lut, void* idx_out, void* w_out) {
    constexpr int K = 1 << BITS;
    __shared__ __align__(8) u32 table[TableShape<BITS>::kTableDwords];
    __shared__ __align__(16) uint16_t raw[K < 8 ? 8 : K];
    const int lane = threadIdx.x;
    const int row = blockIdx.y, slice = blockIdx.x;
    const int j0 = slice * kSliceCols + lane * kLaneElems;
    const bool live = j0 < N;
    const int j0c = live ? j0 : N - kLaneElems;
    const size_t row_dwords = (size_t)N * BITS / 32;
    const u32* p = static_cast<const u32*>(qidx) + (size_t)row * row_dwords + (size_t)(j0c / 32) * BITS;
    const LaneChunk<BITS> c = load_chunk<BITS>(p);
    if (lane < K) raw[lane] = lut ? static_cast<const uint16_t*>(lut)[(size_t)row * K + lane] : (uint16_t)lane;
    __syncthreads();
    build_tables<BITS, 1>(table, raw, lane);
    __syncthreads();
    u32 w[16];
    lookup_chunk<BITS>(c, table, w);
    if (!live) return;
    if (idx_out) {
        uint8_t* o = static_cast<uint8_t*>(idx_out) + (size_t)row * N + j0;
#pragma unroll
        for (int k = 0; k < 16; ++k) { o[2 * k] = (uint8_t)(w[k] & 0xFF); o[2 * k + 1] = (uint8_t)(w[k] >> 16); }
    }
    if (w_out) {
        u32* o = reinterpret_cast<u32*>(static_cast<uint16_t*>(w_out) + (size_t)row * N + j0);
#pragma unroll
        for (int k = 0; k < 16; ++k) o[k] = w[k];
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
            const u32x4 v = *reinterpret_cast<const u32x4*>(x + j);
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
            const float s = wave_sum_to_lane63(acc[u][t]);
            if (lane == 63 && row0 + u < M && t < B) y[(size_t)(row0 + u) * B + t] = float_to_half_bits(s);
        }
}

// ---------------------------------------------------------------------------------------------- launchers
template <int BITS, int R, int D>
static hipError_t launch_matvec_r(const MatvecArgs& g, hipStream_t s) {
    const int W = g.qidx ? (g.N + kSliceCols - 1) / kSliceCols : 0;
    const int S = g.nnz > 0 ? (W ? 1 : kSparseOnlyWaves) : (W ? 0 : 1);
    hipLaunchKernelGGL((matvec_kernel<BITS, R, D>), dim3((g.M + R - 1) / R), dim3((W + S) * kWave), 0, s, g);
    return hipGetLastError();
}

// One activation column.  Rows per workgroup, measured (fused, 0.45 % sparse): 4 rows win on 22016x8192 (19.3 against 19.4 us),
// 8192x8192 (11.0 against 13.4) and 11008x4096 (8.8 against 9.8); rows of eight or more slices -- 8192x22016 with its 11 waves per
// workgroup, of which a compute unit holds only two -- want 8 rows (25.1 against 27.3 us): the fixed cost of a workgroup (tables,
// barriers, the final combination) is then spread over twice the stream.
template <int BITS>
static hipError_t launch_matvec_one(const MatvecArgs& g, hipStream_t s) {
    return g.qidx && multi_rows_per_workgroup(g.N) == 8 ? launch_matvec_r<BITS, 8, 2>(g, s) : launch_matvec_r<BITS, 4, 2>(g, s);
}

PlanLayout plan_layout(int M, int N, long long nnz) {
    PlanLayout L;
    L.R = kPlanRows;                                                // blocks of four rows, whatever the kernel's rows per workgroup
    L.n_wg = (M + L.R - 1) / L.R;
    const long long n_wg = L.n_wg;
    const long long groups = nnz / 16 + M / 2 + 1;                  // a row of c nonzeros has ceil(c / 16) groups
    const int W = (N + kSliceCols - 1) / kSliceCols;
    long long C = n_wg > 0 ? (groups * 115 / 100 + 4 * n_wg - 1) / (4 * n_wg) : 1;   // 15 % above the mean; a wave carries at most one slot batch per block
    L.C = (int)(C < 1 ? 1 : (C > W ? W : C));
    L.ov_cap = (nnz / 16 + M) / 4 + n_wg + 1;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    size_t o = 0;
    L.off_slot_entries = o; o += up((size_t)n_wg * L.C * 256);
    L.off_slot_tags = o;    o += up((size_t)n_wg * L.C * 4);
    L.off_ov_desc = o;      o += up((size_t)n_wg * 8);
    L.off_ov_entries = o;   o += up((size_t)L.ov_cap * 256);
    L.off_ov_tags = o;      o += up((size_t)L.ov_cap * 4);
    L.bytes = o;
    return L;
}

hipError_t launch_plan_build(int M, int N, long long nnz, const int* rowptr, const int* cols, const void* vals, void* plan, hipStream_t s) {
    const PlanLayout L = plan_layout(M, N, nnz);
    if (L.n_wg == 0) return hipSuccess;
    char* b = static_cast<char*>(plan);
    u32* slot_entries = reinterpret_cast<u32*>(b + L.off_slot_entries);
    uint8_t* slot_tags = reinterpret_cast<uint8_t*>(b + L.off_slot_tags);
    int* ov_desc = reinterpret_cast<int*>(b + L.off_ov_desc);
    u32* ov_entries = reinterpret_cast<u32*>(b + L.off_ov_entries);
    uint8_t* ov_tags = reinterpret_cast<uint8_t*>(b + L.off_ov_tags);
    const uint16_t* v16 = static_cast<const uint16_t*>(vals);
    hipLaunchKernelGGL((plan_count_kernel<kPlanRows>), dim3((L.n_wg + 255) / 256), dim3(256), 0, s, M, L.n_wg, L.C, rowptr, ov_desc);
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, s, L.n_wg, ov_desc);
    hipLaunchKernelGGL((plan_fill_kernel<kPlanRows>), dim3(L.n_wg), dim3(64), 0, s, M, L.C, rowptr, cols, v16, slot_entries, slot_tags, ov_desc, ov_entries, ov_tags);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_matvec_planned(const MatvecArgs& g0, hipStream_t s) {
    MatvecArgs g = g0;
    g.plan_c = plan_layout(g.M, g.N, g.nnz).C;
    const int W = (g.N + kSliceCols - 1) / kSliceCols;
    if (multi_rows_per_workgroup(g.N) == 8) hipLaunchKernelGGL((matvec_planned_kernel<BITS, 8, 2>), dim3((g.M + 7) / 8), dim3(W * kWave), 0, s, g);
    else hipLaunchKernelGGL((matvec_planned_kernel<BITS, 4, 2>), dim3((g.M + 3) / 4), dim3(W * kWave), 0, s, g);
    return hipGetLastError();
}

template <int BITS, int R, int K, bool PLANNED>
static hipError_t launch_multi_k(const MultiArgs& m, hipStream_t s) {
    int total = 0, waves = 1, w2 = 1;
    typedef typename std::conditional<PLANNED, PlannedLayer, CsrLayer>::type L;
    MultiKernArgs<L, K> k;
    memset(&k, 0, sizeof k);
    k.count = m.count;
    for (int l = 0; l < m.count; ++l) {
        const LayerArgs& a = m.layer[l];
        k.first_block[l] = total;
        total += (a.M + R - 1) / R;
        w2 = max(w2, (a.N + kSliceCols - 1) / kSliceCols);
        waves = max(waves, (a.N + kSliceCols - 1) / kSliceCols + (a.nnz > 0 ? 1 : 0));
        L& d = k.layer[l];
        d.M = a.M; d.N = a.N; d.nnz = (int)a.nnz; d.qidx = a.qidx; d.lut = a.lut; d.x = a.x; d.y = a.y;
        if constexpr (PLANNED) {
            d.plan = a.plan;
            d.plan_c = plan_layout(a.M, a.N, a.nnz).C;
        } else {
            d.rowptr = a.rowptr; d.cols = a.cols; d.vals = a.vals;
        }
    }
    for (int l = m.count; l <= K; ++l) k.first_block[l] = total;
    if (total == 0) return hipSuccess;
    if constexpr (PLANNED) hipLaunchKernelGGL((matvec_planned_multi_kernel<BITS, R, 2, K>), dim3(total), dim3(w2 * kWave), 0, s, k);
    else hipLaunchKernelGGL((matvec_multi_kernel<BITS, R, 2, K>), dim3(total), dim3(waves * kWave), 0, s, k);
    return hipGetLastError();
}
template <int BITS, int R>
static hipError_t launch_multi_r(const MultiArgs& m, hipStream_t s) {
    if (m.count < 1 || m.count > kMaxLayersPerLaunch) return hipErrorInvalidValue;
    const bool planned = m.layer[0].plan != nullptr;
    for (int l = 0; l < m.count; ++l)
        if ((m.layer[l].plan != nullptr) != planned) return hipErrorInvalidValue;   // one class per launch
    if (!planned && m.count > kMaxCsrLayersPerLaunch) return hipErrorInvalidValue;
    if (m.count <= 8) return planned ? launch_multi_k<BITS, R, 8, true>(m, s) : launch_multi_k<BITS, R, 8, false>(m, s);
    return launch_multi_k<BITS, R, 16, true>(m, s);
}

int multi_rows_per_workgroup(int N) { return (N + kSliceCols - 1) / kSliceCols >= 8 ? 8 : 4; }

hipError_t launch_matvec_multi(const MultiArgs& m, int bits, int R, hipStream_t s) {
    if (R == 8) return bits == 2 ? launch_multi_r<2, 8>(m, s) : (bits == 3 ? launch_multi_r<3, 8>(m, s) : launch_multi_r<4, 8>(m, s));
    return bits == 2 ? launch_multi_r<2, 4>(m, s) : (bits == 3 ? launch_multi_r<3, 4>(m, s) : launch_multi_r<4, 4>(m, s));
}

// up to 16 columns in one launch: 32 rows per workgroup when that still gives every compute unit a workgroup
// Measured (8192x8192, 11008x4096, 4096x4096, 22016x8192 at 16 columns): 8 waves per workgroup beat 16 (fused 23.4 / 22.2 /
// 9.8 us against 24.3 / 27.6 / 11.0) and 4 (the sparse term then has too few waves); 32 rows per workgroup beat 16 from
// M = 8192 on (dense 15.1 against 19.6 us: the activations a workgroup stages serve twice the rows).
constexpr int kB16Waves = 8;
constexpr int kB16TwoGroupsMinM = 8192;
template <int BITS, int RG, int B4>
static hipError_t launch_matvec_b16_r(const MatvecArgs& g, hipStream_t s) {
    constexpr int R = 16 * RG;
    const int nwin = g.qidx ? g.N / 128 : 0;
    const int NW = nwin ? (nwin < kB16Waves ? nwin : kB16Waves) : kB16Waves;   // without a dense term all waves share the sparse steps
    const size_t lds = (size_t)R * TableShape<BITS>::kTableDwords * 4 + (size_t)R * (2 << BITS) + (size_t)NW * kB16StageBytes;
    // raised on every launch: the attribute belongs to the current device's copy of the kernel, and the call is a host-side table update
    const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(&matvec_b16_kernel<BITS, RG, B4>), hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL((matvec_b16_kernel<BITS, RG, B4>), dim3((g.M + R - 1) / R), dim3(NW * kWave), lds, s, g);
    return hipGetLastError();
}
template <int BITS, int RG>
static hipError_t launch_matvec_b16_b(const MatvecArgs& g, hipStream_t s) {
    // batches of exactly 2, 4, 8, 12 or 16 columns: pairs of rows of x are whole 8- or 16-byte units and take the fast
    // activation paths
    switch (g.B) {
        case 2: return launch_matvec_b16_r<BITS, RG, 5>(g, s);
        case 4: return launch_matvec_b16_r<BITS, RG, 1>(g, s);
        case 8: return launch_matvec_b16_r<BITS, RG, 2>(g, s);
        case 12: return launch_matvec_b16_r<BITS, RG, 3>(g, s);
        case 16: return launch_matvec_b16_r<BITS, RG, 4>(g, s);
        default: return launch_matvec_b16_r<BITS, RG, 0>(g, s);
    }
}
template <int BITS>
static hipError_t launch_matvec_b16(const MatvecArgs& g, hipStream_t s) {
    return g.M >= kB16TwoGroupsMinM ? launch_matvec_b16_b<BITS, 2>(g, s) : launch_matvec_b16_b<BITS, 1>(g, s);
}

hipError_t launch_matvec(const MatvecArgs& g, hipStream_t s) {
    // one column: the vector-ALU kernel; two or more: one launch of the 16-column kernel (every weight is decoded once for all
    // columns), also without a dense term
    if (g.B == 1 && g.plan && g.qidx && g.nnz > 0 && !g.accumulate)
        return g.bits == 2 ? launch_matvec_planned<2>(g, s) : (g.bits == 3 ? launch_matvec_planned<3>(g, s) : launch_matvec_planned<4>(g, s));
    if (g.B == 1) return g.bits == 2 ? launch_matvec_one<2>(g, s) : (g.bits == 3 ? launch_matvec_one<3>(g, s) : launch_matvec_one<4>(g, s));
    return g.bits == 2 ? launch_matvec_b16<2>(g, s) : (g.bits == 3 ? launch_matvec_b16<3>(g, s) : launch_matvec_b16<4>(g, s));
}

hipError_t launch_csr_rowwise(const MatvecArgs& g0, hipStream_t s) {
    const int grid = (g0.M + 255) / 256;
    for (int t0 = 0; t0 < g0.B; t0 += 8) {                           // windows of at most eight columns
        MatvecArgs g = g0;
        g.bt0 = t0; g.bn = min(8, g0.B - t0);
        if (g.bn == 1) hipLaunchKernelGGL((csr_rowwise_kernel<1>), dim3(grid), dim3(256), 0, s, g);
        else if (g.bn == 2) hipLaunchKernelGGL((csr_rowwise_kernel<2>), dim3(grid), dim3(256), 0, s, g);
        else if (g.bn <= 4) hipLaunchKernelGGL((csr_rowwise_kernel<4>), dim3(grid), dim3(256), 0, s, g);
        else hipLaunchKernelGGL((csr_rowwise_kernel<8>), dim3(grid), dim3(256), 0, s, g);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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
        if (bits == 2) hipLaunchKernelGGL((decode_kernel<2>), dim3(slices, m), dim3(kWave), 0, s, m, N, q, l, io, wo);
        else if (bits == 3) hipLaunchKernelGGL((decode_kernel<3>), dim3(slices, m), dim3(kWave), 0, s, m, N, q, l, io, wo);
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
    else if (B <= 8) hipLaunchKernelGGL((fp16_gemv_kernel<8, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    else hipLaunchKernelGGL((fp16_gemv_kernel<16, RB>), dim3(grid), dim3(WAVES * kWave), 0, s, M, N, B, w, x, y);
    return hipGetLastError();
}

}  // namespace sqllm
