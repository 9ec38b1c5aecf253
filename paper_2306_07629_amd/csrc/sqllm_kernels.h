// Internal interface between the host-side C ABI (sqllm_api.cpp) and the device code (sqllm_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

namespace sqllm {

struct MatvecArgs {
    int M, N, bits, B;
    int bt0, bn;            // one-thread-per-row CSR kernel only: batch columns [bt0, bt0 + bn) are computed by this launch (bn <= 8)
    int accumulate;
    long long nnz;
    const void* qidx;       // nullptr -> no dense term
    const void* lut;
    const int* rowptr;      // only read when nnz > 0
    const int* cols;
    const void* vals;
    const void* x;
    void* y;
    const void* plan;       // nullptr, or the plan of the sparse term (one-column kernel only): rowptr / cols / vals are then not read
    int plan_c;             // slot batches per workgroup of that plan (set by the launcher)
};

// ---- Plan of the sparse term (built once per matrix, caller-owned device buffer).  The nonzeros of every block of four
// consecutive rows are re-laid-out as GROUPS of 16 entries of one row (zero-padded), four groups to a BATCH of 64 lanes:
//   entry  u32 = column (15 bits) | fp16 value << 16          tag byte of a group = valid << 7 | (count - 1) << 3 | row within the block
// The first `C` batches of block b sit in a fixed slot (batch b C + k), so the kernel can request them at wave start from its
// workgroup index alone; what does not fit (a heavy row) goes to an overflow region described by one (first batch, batches) pair
// per block.  Every offset below follows from (M, N, nnz) alone, so the host never has to read the plan.  The block size does
// not depend on the rows per workgroup of the kernel: a workgroup of eight rows serves two blocks, each in the order a workgroup
// of four would, so y does not depend on that choice.
struct PlanLayout {
    int R;                      // rows per block (4)
    int n_wg;                   // blocks = ceil(M / R)
    int C;                      // slot batches per block
    long long ov_cap;           // capacity of the overflow region in batches
    size_t off_slot_entries, off_slot_tags, off_ov_desc, off_ov_entries, off_ov_tags, bytes;
};
PlanLayout plan_layout(int M, int N, long long nnz);
hipError_t launch_plan_build(int M, int N, long long nnz, const int* rowptr, const int* cols, const void* vals, void* plan, hipStream_t s);

// Several independent one-column layers in one launch.  The host-side description below is turned by the launcher into the
// compact argument block the kernel takes by value (only the fields of its class, room for 8 or 16 layers as needed).
constexpr int kMaxLayersPerLaunch = 16;      // layers with a plan
constexpr int kMaxCsrLayersPerLaunch = 8;    // layers whose sparse term is read from the CSR arrays (more fields per layer)
struct LayerArgs {
    int M, N;
    long long nnz;
    const void* qidx;
    const void* lut;
    const int* rowptr;
    const int* cols;
    const void* vals;
    const void* x;
    void* y;
    const void* plan;       // all layers of a launch have a plan, or none has
};
struct MultiArgs {
    int count;
    LayerArgs layer[kMaxLayersPerLaunch];
};
int multi_rows_per_workgroup(int N);             // rows per workgroup of the one-column kernel for rows of N columns (4 or 8)
hipError_t launch_matvec_multi(const MultiArgs& m, int bits, int rows_per_workgroup, hipStream_t s);

// Offline side (sqllm_quant.hip): everything is a caller-owned device pointer.
struct QuantArgs {
    int M, N, bits, max_iter;
    long long n_lo, n_hi, n_sens;
    const void* w;          // fp16 [M][N]
    const void* sens;       // uint16 [M][N]
    void* workspace;        // quantize_workspace_bytes() bytes
    void* qidx;             // out: packed indices
    void* lut;              // out: fp16 [M][2^bits]
    int* rowptr;            // out: [M + 1]
    int* cols;              // out: capacity n_lo + n_hi + n_sens
    void* vals;             // out: fp16, same capacity
    int* iters;             // out, optional: [M]
};
size_t quantize_workspace_bytes();
hipError_t quantize_static_scratch(void** device_ptr);   // the library's own workspace on the current device (no allocation)
hipError_t launch_quantize(const QuantArgs& a, hipStream_t s);

hipError_t launch_matvec(const MatvecArgs& g, hipStream_t s);
hipError_t launch_csr_rowwise(const MatvecArgs& g, hipStream_t s);
hipError_t launch_decode(int M, int N, int bits, const void* qidx, const void* lut, void* idx_out, void* w_out, hipStream_t s);
hipError_t launch_fp16_gemv(int M, int N, int B, const void* w, const void* x, void* y, hipStream_t s);

}  // namespace sqllm
