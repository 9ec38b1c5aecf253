// Internal interface between the host-side C ABI (sqllm_api.cpp) and the device code (sqllm_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

namespace sqllm {

struct MatvecArgs {
    int M, N, bits, B;
    int bt0, bn;            // batch columns [bt0, bt0 + bn) are computed by this launch (bn <= 4)
    int rows_per_wg;        // requested rows per workgroup; the launcher rounds it to 2, 4, 8 or 16
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

hipError_t launch_matvec(const MatvecArgs& g, hipStream_t s);
hipError_t launch_csr_rowwise(const MatvecArgs& g, hipStream_t s);
hipError_t launch_decode(int M, int N, int bits, const void* qidx, const void* lut, void* idx_out, void* w_out, hipStream_t s);
hipError_t launch_fp16_gemv(int M, int N, int B, const void* w, const void* x, void* y, hipStream_t s);

}  // namespace sqllm
