// Measured ceilings of the GPU the library runs on, for pricing the query kernels against what the
// machine actually delivers besides its published peaks: a streaming read of a buffer far larger
// than every cache (HBM read bandwidth) and a loop of independent fp32 matrix-core instructions
// (v_mfma_f32_16x16x4_f32 rate).  Measurement infrastructure only; not on the query path.
#include <hip/hip_runtime.h>

#include "pqt_index.hpp"

using pqt_host::DeviceGuard;
using pqt_host::fail;

namespace pqt {

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* src, size_t n16, uint32_t* sink) {
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;           // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* sink) {
    v4f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    const float a = (float)(threadIdx.x & 3), b = (float)(threadIdx.x & 7);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == -1.0f) sink[0] = s;
}

}  // namespace pqt

extern "C" int pqt_measure_peaks(int device, double* hbm_read_gb_per_s, double* mfma_f32_tflop_per_s) {
    if (!hbm_read_gb_per_s || !mfma_f32_tflop_per_s) return fail(PQT_EINVAL, "pqt_measure_peaks: null argument");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev)
        return fail(PQT_EHIP, "GPU %d is not available (%d visible)", device, ndev);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", device);
    const size_t bytes = (size_t)4 << 30;            // 4 GiB: sixteen times the last-level cache
    void* buf = nullptr;
    uint32_t* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    auto done = [&]() {
        (void)hipFree(buf); (void)hipFree(sink);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    };
#define PEAK_TRY(expr)                                                                                        \
    do {                                                                                                      \
        hipError_t e_ = (expr);                                                                               \
        if (e_ != hipSuccess) {                                                                               \
            done();                                                                                           \
            return fail(e_ == hipErrorOutOfMemory ? PQT_ENOMEM : PQT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
        }                                                                                                     \
    } while (0)
    PEAK_TRY(hipMalloc(&buf, bytes));
    PEAK_TRY(hipMalloc(reinterpret_cast<void**>(&sink), 16));
    PEAK_TRY(hipMemset(buf, 1, bytes));
    PEAK_TRY(hipEventCreate(&e0));
    PEAK_TRY(hipEventCreate(&e1));
    float ms = 0.0f;
    double best_bw = 0.0, best_fl = 0.0;
    for (int rep = 0; rep < 4; ++rep) {              // first repetition warms up
        PEAK_TRY(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(pqt::stream_read_kernel, dim3(256 * 16), dim3(256), 0, 0, static_cast<const uint4*>(buf), bytes / 16, sink);
        PEAK_TRY(hipEventRecord(e1, 0));
        PEAK_TRY(hipEventSynchronize(e1));
        PEAK_TRY(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0 && ms > 0.0f) best_bw = best_bw > bytes / (ms * 1e-3) / 1e9 ? best_bw : bytes / (ms * 1e-3) / 1e9;
    }
    const int iters = 20000, blocks = 256 * 8;       // 8 workgroups of 4 wavefronts per CU
    for (int rep = 0; rep < 4; ++rep) {
        PEAK_TRY(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(pqt::mfma_loop_kernel, dim3(blocks), dim3(256), 0, 0, iters, reinterpret_cast<float*>(sink));
        PEAK_TRY(hipEventRecord(e1, 0));
        PEAK_TRY(hipEventSynchronize(e1));
        PEAK_TRY(hipEventElapsedTime(&ms, e0, e1));
        const double flop = (double)blocks * 4 * iters * 8 * (2.0 * 16 * 16 * 4);
        if (rep > 0 && ms > 0.0f) best_fl = best_fl > flop / (ms * 1e-3) / 1e12 ? best_fl : flop / (ms * 1e-3) / 1e12;
    }
#undef PEAK_TRY
    done();
    *hbm_read_gb_per_s = best_bw;
    *mfma_f32_tflop_per_s = best_fl;
    return PQT_OK;
}
