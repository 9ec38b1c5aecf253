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
};

// Several independent one-column layers in one launch (passed by value as kernel arguments)
constexpr int kMaxLayersPerLaunch = 8;
struct MultiArgs {
    int count;
    int first_block[kMaxLayersPerLaunch + 1];   // filled by the launcher: workgroups of layer l are first_block[l] .. first_block[l + 1] - 1
    int M[kMaxLayersPerLaunch], N[kMaxLayersPerLaunch];
    long long nnz[kMaxLayersPerLaunch];
    const void* qidx[kMaxLayersPerLaunch];
    const void* lut[kMaxLayersPerLaunch];
    const int* rowptr[kMaxLayersPerLaunch];
    const int* cols[kMaxLayersPerLaunch];
    const void* vals[kMaxLayersPerLaunch];
    const void* x[kMaxLayersPerLaunch];
    void* y[kMaxLayersPerLaunch];
};
int multi_rows_per_workgroup(int N);             // rows per workgroup of the one-column kernel for rows of N columns (4 or 8)
hipError_t launch_matvec_multi(MultiArgs& m, int bits, hipStream_t s);

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
