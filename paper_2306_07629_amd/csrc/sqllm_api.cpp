// Host side of the C ABI declared in sqllm.h: argument validation (everything that can be decided without
// touching the device is decided here, before any HIP call), choice of launch shape, error reporting.
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <vector>

#include "sqllm.h"
#include "sqllm_kernels.h"

namespace {

thread_local char g_err[256] = "no error";

int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return status;
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_shape(int M, int N, int B) {
    if (M < 0) return fail(SQLLM_ERR_SHAPE, "M = %d is negative", M);
    // One rule for every width: a lane of the kernels decodes 32 indices and a wave 2048, and the 16-column kernel walks a row in
    // windows of 128 columns; 4-bit rows that are whole 16-byte words but not whole 128-column windows (N % 32 == 0 only) are
    // therefore not accepted.  N == 0 is rejected as well: there is no row to read, the caller can clear y itself.
    if (N <= 0 || N % 128 != 0) return fail(SQLLM_ERR_SHAPE, "N = %d must be a positive multiple of 128", N);
    if (N > SQLLM_MAX_N) return fail(SQLLM_ERR_SHAPE, "N = %d exceeds SQLLM_MAX_N = %d", N, SQLLM_MAX_N);
    if (B < 1 || B > SQLLM_MAX_BATCH) return fail(SQLLM_ERR_BATCH, "B = %d outside 1..%d", B, SQLLM_MAX_BATCH);
    return SQLLM_OK;
}

int check_bits(int bits) {
    if (bits < 2 || bits > 4) return fail(SQLLM_ERR_BITS, "bits = %d, only 2, 3 and 4 are supported", bits);
    return SQLLM_OK;
}

int check_dense_ptrs(const void* qidx, const void* lut) {
    if (!qidx || !lut) return fail(SQLLM_ERR_NULL, "qidx / lut must not be NULL");
    if (misaligned(qidx, 16) || misaligned(lut, 16)) return fail(SQLLM_ERR_ALIGN, "qidx and lut must be 16-byte aligned");
    return SQLLM_OK;
}

int check_xy(const void* x, const void* y) {
    if (!x || !y) return fail(SQLLM_ERR_NULL, "x / y must not be NULL");
    if (misaligned(x, 16)) return fail(SQLLM_ERR_ALIGN, "x must be 16-byte aligned");
    if (misaligned(y, 2)) return fail(SQLLM_ERR_ALIGN, "y must be 2-byte aligned");
    return SQLLM_OK;
}

int check_sparse(long long nnz, const int* rowptr, const int* cols, const void* vals) {
    if (nnz < 0 || nnz > 0x7FFFFFFFll) return fail(SQLLM_ERR_NNZ, "nnz = %lld outside 0..2^31-1", nnz);
    if (nnz == 0) return SQLLM_OK;
    if (!rowptr || !cols || !vals) return fail(SQLLM_ERR_NULL, "rowptr / cols / vals must not be NULL when nnz > 0");
    if (misaligned(rowptr, 4) || misaligned(cols, 4) || misaligned(vals, 2))
        return fail(SQLLM_ERR_ALIGN, "rowptr and cols must be 4-byte aligned, vals 2-byte aligned");
    return SQLLM_OK;
}

int check_plan(long long nnz, const void* plan) {
    if (nnz < 0 || nnz > 0x7FFFFFFFll) return fail(SQLLM_ERR_NNZ, "nnz = %lld outside 0..2^31-1", nnz);
    if (misaligned(plan, 256)) return fail(SQLLM_ERR_ALIGN, "plan must be 256-byte aligned");
    return SQLLM_OK;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(SQLLM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// The kernels are built for gfx950 only.  The architecture of the current device is looked up once per device (a host-side
// query, no kernel) and remembered; any other architecture is refused before a launch could fail with a generic HIP error.
constexpr int kMaxDevices = 64;
std::atomic<int> g_arch_ok[kMaxDevices];      // 0 unknown, 1 gfx950, -1 something else

int check_device() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    int state = dev >= 0 && dev < kMaxDevices ? g_arch_ok[dev].load(std::memory_order_relaxed) : 0;
    if (state == 0) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess) return hip_fail(e, "hipGetDeviceProperties");
        state = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
        if (dev >= 0 && dev < kMaxDevices) g_arch_ok[dev].store(state, std::memory_order_relaxed);
        if (state < 0) return fail(SQLLM_ERR_DEVICE, "device %d is %s, this library holds gfx950 code only", dev, prop.gcnArchName);
    }
    if (state < 0) return fail(SQLLM_ERR_DEVICE, "device %d is not a gfx950 GPU", dev);
    return SQLLM_OK;
}

int run_matvec(int M, int N, int bits, long long nnz, int B, const void* qidx, const void* lut, const int* rowptr,
               const int* cols, const void* vals, const void* plan, const void* x, void* y, int accumulate, void* stream) {
    if (M == 0) return SQLLM_OK;
    int st;
    if ((st = check_device())) return st;
    sqllm::MatvecArgs g;
    memset(&g, 0, sizeof g);
    g.M = M; g.N = N; g.bits = bits; g.B = B; g.bt0 = 0; g.bn = B;
    g.accumulate = accumulate; g.nnz = nnz;
    g.qidx = qidx; g.lut = lut; g.rowptr = rowptr; g.cols = cols; g.vals = vals; g.x = x; g.y = y; g.plan = plan;
    const hipError_t e = sqllm::launch_matvec(g, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "matvec launch");
    return SQLLM_OK;
}

}  // namespace

extern "C" {

int sqllm_lut_gemv(int M, int N, int bits, int B, const void* qidx, const void* lut, const void* x, void* y,
                   int accumulate, void* stream) {
    int st;
    if ((st = check_bits(bits)) || (st = check_shape(M, N, B)) || (st = check_dense_ptrs(qidx, lut)) || (st = check_xy(x, y))) return st;
    return run_matvec(M, N, bits, 0, B, qidx, lut, nullptr, nullptr, nullptr, nullptr, x, y, accumulate, stream);
}

int sqllm_csr_spmv(int M, int N, long long nnz, int B, const int* rowptr, const int* cols, const void* vals,
                   const void* x, void* y, int accumulate, void* stream) {
    int st;
    if ((st = check_shape(M, N, B)) || (st = check_sparse(nnz, rowptr, cols, vals)) || (st = check_xy(x, y))) return st;
    return run_matvec(M, N, 3, nnz, B, nullptr, nullptr, rowptr, cols, vals, nullptr, x, y, accumulate, stream);
}

int sqllm_dense_sparse_matvec(int M, int N, int bits, long long nnz, int B, const void* qidx, const void* lut,
                              const int* rowptr, const int* cols, const void* vals, const void* plan, const void* x, void* y, void* stream) {
    int st;
    const bool planned = plan != nullptr && B == 1 && nnz > 0;       // the CSR arrays are then not read
    if ((st = check_bits(bits)) || (st = check_shape(M, N, B)) || (st = check_dense_ptrs(qidx, lut)) ||
        (st = planned ? check_plan(nnz, plan) : check_sparse(nnz, rowptr, cols, vals)) || (st = check_xy(x, y))) return st;
    return run_matvec(M, N, bits, nnz, B, qidx, lut, rowptr, cols, vals, planned ? plan : nullptr, x, y, 0, stream);
}

int sqllm_csr_plan_bytes(int M, int N, long long nnz, size_t* bytes_out) {
    int st;
    if ((st = check_shape(M, N, 1))) return st;
    if (nnz < 0 || nnz > 0x7FFFFFFFll) return fail(SQLLM_ERR_NNZ, "nnz = %lld outside 0..2^31-1", nnz);
    if (!bytes_out) return fail(SQLLM_ERR_NULL, "bytes_out must not be NULL");
    *bytes_out = sqllm::plan_layout(M, N, nnz).bytes;
    return SQLLM_OK;
}

int sqllm_csr_plan_build(int M, int N, long long nnz, const int* rowptr, const int* cols, const void* vals,
                         void* plan, size_t bytes, void* stream) {
    int st;
    if ((st = check_shape(M, N, 1)) || (st = check_sparse(nnz, rowptr, cols, vals))) return st;
    if (!plan) return fail(SQLLM_ERR_NULL, "plan must not be NULL");
    if (!rowptr) return fail(SQLLM_ERR_NULL, "rowptr must not be NULL");
    if (misaligned(plan, 256)) return fail(SQLLM_ERR_ALIGN, "plan must be 256-byte aligned");
    const size_t need = sqllm::plan_layout(M, N, nnz).bytes;
    if (bytes < need) return fail(SQLLM_ERR_SHAPE, "plan buffer of %zu bytes, %zu needed", bytes, need);
    if (M == 0) return SQLLM_OK;
    if ((st = check_device())) return st;
    const hipError_t e = sqllm::launch_plan_build(M, N, nnz, rowptr, cols, vals, plan, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "plan build launch");
    return SQLLM_OK;
}

// workgroups of eight rows from which a planned multi-layer launch counts as many generations (256 compute units hold about 1800)
static const long long kManyGenerationsBlocks = 4096;

}  // extern "C"

namespace {

int validate_layers(int count, const sqllm_layer* layers) {
    if (count < 0) return fail(SQLLM_ERR_SHAPE, "count = %d is negative", count);
    if (count == 0) return SQLLM_OK;
    if (!layers) return fail(SQLLM_ERR_NULL, "layers must not be NULL");
    int st;
    for (int l = 0; l < count; ++l) {
        const sqllm_layer& L = layers[l];
        const bool planned = L.plan != nullptr && L.nnz > 0;
        if ((st = check_bits(L.bits)) || (st = check_shape(L.M, L.N, 1)) || (st = check_dense_ptrs(L.qidx, L.lut)) ||
            (st = planned ? check_plan(L.nnz, L.plan) : check_sparse(L.nnz, L.rowptr, L.cols, L.vals)) || (st = check_xy(L.x, L.y))) {
            char msg[200];
            snprintf(msg, sizeof msg, "%s", g_err);
            return fail(st, "layer %d: %s", l, msg);
        }
        if (L.bits != layers[0].bits) return fail(SQLLM_ERR_BITS, "layer %d: bits = %d, layer 0 has %d (one width per call)", l, L.bits, layers[0].bits);
    }
    return SQLLM_OK;
}

// Sorts the layers of a call into launches and hands each to fn(indices of its layers, their number, planned, rows per workgroup).
// A launch holds layers of one group.  Groups differ in
//   * plan or no plan (different kernels);
//   * without a plan, the rows per workgroup of the layer's own launch: with the sparse term read from the CSR arrays the
//     batches of a workgroup depend on its rows, so such a layer keeps that number and every y stays bit for bit that of a
//     call of its own.  With a plan y does not depend on the rows per workgroup, and the launch takes eight rows when it is
//     many generations of workgroups (fewer, longer workgroups amortise their fixed work; the other layers' workgroups
//     hide their start-up), else what the layers' own launches would take;
//   * the waves per workgroup the layer needs (one per 2048 columns): all workgroups of a launch have the size of its widest
//     layer and the surplus waves of a narrower layer leave at once, but starting them is not free -- a 7B-shaped step with the
//     two-wave and six-wave layers in common launches took 820 us, in launches of their own 630 us.
// The layers of a call are independent, so they may run in any order: groups are taken in the order of their first layer.
// Layers without rows belong to no launch.
template <class Fn>
int for_each_launch(int count, const sqllm_layer* layers, Fn&& fn) {
    auto planned_of = [](const sqllm_layer& L) { return L.plan != nullptr && L.nnz > 0; };
    auto key_of = [&](const sqllm_layer& L) {
        if (L.M <= 0) return -1;
        const int waves = (L.N + 2047) / 2048 + (L.nnz > 0 && !planned_of(L) ? 1 : 0);   // without a plan one more wave walks the CSR arrays
        return ((planned_of(L) ? 1 : 2 * sqllm::multi_rows_per_workgroup(L.N)) << 16) | waves;
    };
    int key_few[256];                                               // a decode step of a 7B-shaped model is 224 layers: no allocation for it
    std::vector<int> key_many;
    int* key = key_few;
    if (count > 256) {
        try {
            key_many.resize(count);
        } catch (...) {
            return fail(SQLLM_ERR_SHAPE, "count = %d: out of host memory for the launch order", count);
        }
        key = key_many.data();
    }
    for (int l = 0; l < count; ++l) key[l] = key_of(layers[l]);
    for (int first = 0; first < count; ++first) {
        const int kk = key[first];
        if (kk < 0) continue;
        const int cls = kk >> 16;
        const bool planned = cls == 1;
        const int cap = planned ? sqllm::kMaxLayersPerLaunch : sqllm::kMaxCsrLayersPerLaunch;
        const int rule = sqllm::multi_rows_per_workgroup(layers[first].N);   // the same for every layer of the group
        int l = first;
        while (l < count) {
            int idx[sqllm::kMaxLayersPerLaunch], n = 0;
            long long blocks8 = 0;
            for (; l < count && n < cap; ++l) {
                if (key[l] != kk) continue;
                key[l] = -1;                                        // taken
                idx[n++] = l;
                blocks8 += (layers[l].M + 7) / 8;
            }
            if (n == 0) break;
            // a launch of one layer is that layer's own launch, with its own rule
            const int rows = planned ? ((rule == 8 || (n > 1 && blocks8 >= kManyGenerationsBlocks)) ? 8 : 4) : cls / 2;
            const int st = fn(idx, n, planned, rows);
            if (st) return st;
        }
    }
    return SQLLM_OK;
}

}  // namespace

extern "C" {

int sqllm_dense_sparse_matvec_multi(int count, const sqllm_layer* layers, void* stream) {
    static_assert(SQLLM_MAX_LAYERS_PER_LAUNCH == sqllm::kMaxLayersPerLaunch, "header and kernels disagree");
    int st;
    if ((st = validate_layers(count, layers))) return st;
    bool any = false;
    for (int l = 0; l < count; ++l) any = any || layers[l].M > 0;
    if (!any) return SQLLM_OK;
    if ((st = check_device())) return st;
    return for_each_launch(count, layers, [&](const int* idx, int n, bool planned, int rows) -> int {
        if (n == 1) {
            // the single-layer kernel starts a little earlier: it does not have to find its layer in the kernel arguments first
            const sqllm_layer& L = layers[idx[0]];
            return run_matvec(L.M, L.N, L.bits, L.nnz, 1, L.qidx, L.lut, L.rowptr, L.cols, L.vals, planned ? L.plan : nullptr, L.x, L.y, 0, stream);
        }
        sqllm::MultiArgs m;
        memset(&m, 0, sizeof m);
        m.count = n;
        for (int k = 0; k < n; ++k) {
            const sqllm_layer& L = layers[idx[k]];
            sqllm::LayerArgs& a = m.layer[k];
            a.M = L.M; a.N = L.N; a.nnz = L.nnz; a.qidx = L.qidx; a.lut = L.lut; a.rowptr = L.rowptr; a.cols = L.cols;
            a.vals = L.vals; a.x = L.x; a.y = L.y; a.plan = planned ? L.plan : nullptr;
        }
        const hipError_t e = sqllm::launch_matvec_multi(m, layers[0].bits, rows, static_cast<hipStream_t>(stream));
        return e != hipSuccess ? hip_fail(e, "multi-layer matvec launch") : SQLLM_OK;
    });
}

int sqllm_multi_launch_order(int count, const sqllm_layer* layers, int* launch_out, int* rows_out, int* launches_out) {
    int st;
    if ((st = validate_layers(count, layers))) return st;
    if (count > 0 && !launch_out) return fail(SQLLM_ERR_NULL, "launch_out must not be NULL");
    for (int l = 0; l < count; ++l) {
        launch_out[l] = -1;
        if (rows_out) rows_out[l] = 0;
    }
    int launches = 0;
    if (count > 0) {
        st = for_each_launch(count, layers, [&](const int* idx, int n, bool, int rows) -> int {
            for (int k = 0; k < n; ++k) {
                launch_out[idx[k]] = launches;
                if (rows_out) rows_out[idx[k]] = rows;
            }
            ++launches;
            return SQLLM_OK;
        });
        if (st) return st;
    }
    if (launches_out) *launches_out = launches;
    return SQLLM_OK;
}

int sqllm_csr_spmv_rowwise(int M, int N, long long nnz, int B, const int* rowptr, const int* cols, const void* vals,
                           const void* x, void* y, int accumulate, void* stream) {
    int st;
    if ((st = check_shape(M, N, B)) || (st = check_sparse(nnz, rowptr, cols, vals)) || (st = check_xy(x, y))) return st;
    if (M == 0) return SQLLM_OK;
    if ((st = check_device())) return st;
    sqllm::MatvecArgs g;
    memset(&g, 0, sizeof g);
    g.M = M; g.N = N; g.bits = 3; g.B = B; g.bn = B; g.accumulate = accumulate; g.nnz = nnz;
    g.rowptr = rowptr; g.cols = cols; g.vals = vals; g.x = x; g.y = y;
    const hipError_t e = sqllm::launch_csr_rowwise(g, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "csr_rowwise launch");
    return SQLLM_OK;
}

int sqllm_unpack_indices(int M, int N, int bits, const void* qidx, void* idx_out, void* stream) {
    int st;
    if ((st = check_bits(bits)) || (st = check_shape(M, N, 1))) return st;
    if (!qidx || !idx_out) return fail(SQLLM_ERR_NULL, "qidx / idx_out must not be NULL");
    if (misaligned(qidx, 16)) return fail(SQLLM_ERR_ALIGN, "qidx must be 16-byte aligned");
    if (M == 0) return SQLLM_OK;
    if ((st = check_device())) return st;
    const hipError_t e = sqllm::launch_decode(M, N, bits, qidx, nullptr, idx_out, nullptr, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "unpack launch");
    return SQLLM_OK;
}

int sqllm_dequantize(int M, int N, int bits, const void* qidx, const void* lut, void* w_out, void* stream) {
    int st;
    if ((st = check_bits(bits)) || (st = check_shape(M, N, 1)) || (st = check_dense_ptrs(qidx, lut))) return st;
    if (!w_out) return fail(SQLLM_ERR_NULL, "w_out must not be NULL");
    if (misaligned(w_out, 2)) return fail(SQLLM_ERR_ALIGN, "w_out must be 2-byte aligned");
    if (M == 0) return SQLLM_OK;
    if ((st = check_device())) return st;
    const hipError_t e = sqllm::launch_decode(M, N, bits, qidx, lut, nullptr, w_out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "dequantize launch");
    return SQLLM_OK;
}

int sqllm_fp16_gemv(int M, int N, int B, const void* w, const void* x, void* y, void* stream) {
    if (M < 0) return fail(SQLLM_ERR_SHAPE, "M = %d is negative", M);
    if (N <= 0 || N % 8 != 0) return fail(SQLLM_ERR_SHAPE, "N = %d must be a positive multiple of 8", N);
    if (B < 1 || B > SQLLM_MAX_BATCH) return fail(SQLLM_ERR_BATCH, "B = %d outside 1..%d", B, SQLLM_MAX_BATCH);
    if (!w) return fail(SQLLM_ERR_NULL, "w must not be NULL");
    if (misaligned(w, 16)) return fail(SQLLM_ERR_ALIGN, "w must be 16-byte aligned");
    int st;
    if ((st = check_xy(x, y))) return st;
    if (M == 0) return SQLLM_OK;
    if ((st = check_device())) return st;
    const hipError_t e = sqllm::launch_fp16_gemv(M, N, B, w, x, y, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "fp16_gemv launch");
    return SQLLM_OK;
}

long long sqllm_algorithmic_bytes(int M, int N, int bits, long long nnz, int B) {
    long long b = (long long)M * N * bits / 8 + (long long)M * (1ll << bits) * 2 + (long long)B * ((long long)N + M) * 2;
    if (nnz > 0) b += nnz * 6 + ((long long)M + 1) * 4;
    return b;
}

long long sqllm_quantize_workspace_bytes(int M, int N) {
    (void)M; (void)N;
    return (long long)sqllm::quantize_workspace_bytes();
}

namespace {
int run_quantize(int M, int N, int bits, int max_iter, const void* w, const void* sens, long long n_lo, long long n_hi, long long n_sens,
                 void* workspace, bool own_scratch, void* qidx, void* lut, int* rowptr, int* cols, void* vals, int* iters, void* stream) {
    int st;
    if ((st = check_bits(bits)) || (st = check_shape(M, N, 1))) return st;
    if (M == 0) return SQLLM_OK;
    const long long total = (long long)M * N;
    if (total >= (1ll << 32)) return fail(SQLLM_ERR_SHAPE, "M * N = %lld does not fit the 32-bit histogram counters", total);
    if (max_iter < 0) return fail(SQLLM_ERR_SHAPE, "max_iter = %d is negative", max_iter);
    if (n_lo < 0 || n_hi < 0 || n_sens < 0 || n_lo >= total || n_hi >= total || n_sens >= total || n_lo + n_hi + n_sens >= (1ll << 31))
        return fail(SQLLM_ERR_NNZ, "extraction counts (%lld, %lld, %lld) out of range for %lld weights", n_lo, n_hi, n_sens, total);
    if (!w || !sens || (!own_scratch && !workspace) || !qidx || !lut || !rowptr) return fail(SQLLM_ERR_NULL, "a required pointer is NULL");
    if (n_lo + n_hi + n_sens > 0 && (!cols || !vals)) return fail(SQLLM_ERR_NULL, "cols / vals are NULL although entries may be extracted");
    if (((uintptr_t)w | (uintptr_t)sens | (uintptr_t)qidx | (uintptr_t)lut) & 15) return fail(SQLLM_ERR_ALIGN, "w, sens, qidx and lut must be 16-byte aligned");
    if (((uintptr_t)workspace | (uintptr_t)rowptr | (uintptr_t)cols | (uintptr_t)iters) & 3) return fail(SQLLM_ERR_ALIGN, "workspace, rowptr, cols and iters must be 4-byte aligned");
    if ((uintptr_t)vals & 1) return fail(SQLLM_ERR_ALIGN, "vals must be 2-byte aligned");
    if ((st = check_device())) return st;
    if (own_scratch) {
        const hipError_t e = sqllm::quantize_static_scratch(&workspace);
        if (e != hipSuccess) return hip_fail(e, "address of the library's scratch array");
    }
    sqllm::QuantArgs a;
    memset(&a, 0, sizeof a);
    a.M = M; a.N = N; a.bits = bits; a.max_iter = max_iter; a.n_lo = n_lo; a.n_hi = n_hi; a.n_sens = n_sens;
    a.w = w; a.sens = sens; a.workspace = workspace; a.qidx = qidx; a.lut = lut; a.rowptr = rowptr; a.cols = cols; a.vals = vals; a.iters = iters;
    const hipError_t e = sqllm::launch_quantize(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "quantize launch");
    return SQLLM_OK;
}
}  // namespace

int sqllm_quantize_layer(int M, int N, int bits, int max_iter, const void* w, const void* sens,
                         long long n_lo, long long n_hi, long long n_sens, void* workspace, long long workspace_bytes,
                         void* qidx, void* lut, int* rowptr, int* cols, void* vals, int* iters, void* stream) {
    if (M != 0 && workspace && workspace_bytes < (long long)sqllm::quantize_workspace_bytes())
        return fail(SQLLM_ERR_SHAPE, "workspace of %lld bytes, %lld needed", workspace_bytes, (long long)sqllm::quantize_workspace_bytes());
    return run_quantize(M, N, bits, max_iter, w, sens, n_lo, n_hi, n_sens, workspace, false, qidx, lut, rowptr, cols, vals, iters, stream);
}

int sqllm_quantize_layer_noalloc(int M, int N, int bits, int max_iter, const void* w, const void* sens,
                                 long long n_lo, long long n_hi, long long n_sens,
                                 void* qidx, void* lut, int* rowptr, int* cols, void* vals, int* iters, void* stream) {
    if ((long long)M * N > SQLLM_NOALLOC_MAX_WEIGHTS)
        return fail(SQLLM_ERR_SHAPE, "M * N = %lld exceeds SQLLM_NOALLOC_MAX_WEIGHTS = %lld", (long long)M * N, (long long)SQLLM_NOALLOC_MAX_WEIGHTS);
    return run_quantize(M, N, bits, max_iter, w, sens, n_lo, n_hi, n_sens, nullptr, true, qidx, lut, rowptr, cols, vals, iters, stream);
}

int sqllm_extraction_counts(int M, int N, double outlier_frac, double sens_frac, long long* n_lo, long long* n_hi, long long* n_sens) {
    if (!n_lo || !n_hi || !n_sens) return fail(SQLLM_ERR_NULL, "n_lo / n_hi / n_sens must not be NULL");
    if (M < 0 || N < 0) return fail(SQLLM_ERR_SHAPE, "M = %d, N = %d: negative", M, N);
    if (!(outlier_frac >= 0.0 && sens_frac >= 0.0 && outlier_frac + sens_frac < 1.0))
        return fail(SQLLM_ERR_NNZ, "shares %g + %g outside [0, 1)", outlier_frac, sens_frac);
    const double total = (double)M * (double)N;
    *n_lo = *n_hi = (long long)(outlier_frac * total / 2.0);      // half of the outlier share on each tail
    *n_sens = (long long)(sens_frac * total);
    return SQLLM_OK;
}

const char* sqllm_last_error_string(void) { return g_err; }

const char* sqllm_status_string(int status) {
    switch (status) {
        case SQLLM_OK: return "SQLLM_OK";
        case SQLLM_ERR_NULL: return "SQLLM_ERR_NULL";
        case SQLLM_ERR_BITS: return "SQLLM_ERR_BITS";
        case SQLLM_ERR_SHAPE: return "SQLLM_ERR_SHAPE";
        case SQLLM_ERR_ALIGN: return "SQLLM_ERR_ALIGN";
        case SQLLM_ERR_NNZ: return "SQLLM_ERR_NNZ";
        case SQLLM_ERR_BATCH: return "SQLLM_ERR_BATCH";
        case SQLLM_ERR_HIP: return "SQLLM_ERR_HIP";
        case SQLLM_ERR_DEVICE: return "SQLLM_ERR_DEVICE";
        default: return "SQLLM_ERR_UNKNOWN";
    }
}

int sqllm_version(void) { return 100; }

}  // extern "C"
