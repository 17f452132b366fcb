// Achievable peaks of the device the library runs on, measured with plain kernels: a streaming copy (HBM) and
// register-resident loops of the two fp32 MFMA shapes the einsum kernels use.  Measurement aid for benchmarks: the
// roofline fractions are quoted against the datasheet figures and against these.
#include "device_common.hpp"

namespace einet_impl {

namespace {

__global__ void k_peak_copy(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

typedef float floatx16p __attribute__((ext_vector_type(16)));

// NACC independent accumulator chains per wave, operands in registers, nothing else in the loop
template <int NACC>
__global__ __launch_bounds__(256) void k_peak_mfma32(float* out, int iters, float a, float b) {
    floatx16p acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void k_peak_mfma16(float* out, int iters, float a, float b) {
    floatx4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// best of `reps` timed launches, in seconds; negative on a HIP error
template <class F>
double best_time(F&& launch, int reps, hipStream_t s) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return -1.0;
    }
    double best = -1.0;
    launch();                                           // warm-up
    for (int r = 0; r < reps; ++r) {
        (void)hipEventRecord(e0, s);
        launch();
        (void)hipEventRecord(e1, s);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            best = -1.0;
            break;
        }
        if (best < 0.0 || ms * 1e-3 < best) best = ms * 1e-3;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return best;
}

}  // namespace

// out[0]: copy rate, GB/s read + written; out[1]: 32x32x2 fp32 MFMA, TFLOP/s; out[2]: 16x16x4 fp32 MFMA, TFLOP/s
// (one wave per SIMD, four chains); out[3]: 16x16x4 with four waves per SIMD.
hipError_t measure_peaks(const void* src, void* dst, size_t bytes, int reps, double* out, hipStream_t s) {
    const size_t n = bytes / 16;
    const int cus = EINET_NUM_CUS;
    double t = best_time([&] {
        hipLaunchKernelGGL(k_peak_copy, dim3(cus * 16), dim3(256), 0, s, static_cast<const float4*>(src),
                           static_cast<float4*>(dst), n);
    }, reps, s);
    if (t <= 0.0) return hipErrorUnknown;
    out[0] = 2.0 * (double)n * 16.0 / t / 1e9;
    float* o = static_cast<float*>(dst);                // (needs room for 4 * cus * 256 floats: checked by the caller)
    const int iters = 4000;
    t = best_time([&] { hipLaunchKernelGGL(k_peak_mfma32<2>, dim3(cus), dim3(256), 0, s, o, iters, 1.0f, 0.5f); }, reps, s);
    if (t <= 0.0) return hipErrorUnknown;
    out[1] = (double)cus * 4 * iters * 8 * 2 * 4096.0 / t / 1e12;
    t = best_time([&] { hipLaunchKernelGGL(k_peak_mfma16<4>, dim3(cus), dim3(256), 0, s, o, iters, 1.0f, 0.5f); }, reps, s);
    if (t <= 0.0) return hipErrorUnknown;
    out[2] = (double)cus * 4 * iters * 8 * 4 * 2048.0 / t / 1e12;
    t = best_time([&] { hipLaunchKernelGGL(k_peak_mfma16<4>, dim3(cus * 4), dim3(256), 0, s, o, iters, 1.0f, 0.5f); }, reps, s);
    if (t <= 0.0) return hipErrorUnknown;
    out[3] = (double)cus * 16 * iters * 8 * 4 * 2048.0 / t / 1e12;
    return hipGetLastError();
}

}  // namespace einet_impl
