// Stand-ins for the device side, so that the host code of the library (structure compiler, argument checks, table
// upload, layer loops) runs in a CPU process under AddressSanitizer and UBSan: the kernel launchers do nothing, the
// few HIP runtime calls of api.cpp act on host memory.  Test infrastructure only; nothing here is part of the
// library.
#include <cstring>

#include "../../paper_2004_06231_amd/csrc/kernels.hpp"

extern "C" {
hipError_t hipGetLastError() { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) {
    std::memcpy(dst, src, n);
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = reinterpret_cast<hipEvent_t>(new int(0)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<int*>(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
}

namespace einet_impl {
void launch_leaf_derive(const float*, float*, const Dims&, hipStream_t) {}
void launch_leaf_forward(const DevTables&, int, int, const float*, const uint8_t*, int, const float*, float*, double*,
                         const Dims&, hipStream_t) {}
void launch_einsum_forward(const DevTables&, int, int, bool, const float*, float*, double*, float*, float*, const Dims&,
                           hipStream_t) {}
void launch_mixing_forward(const DevTables&, int, int, int, const float*, float*, double*, float*, const Dims&,
                           hipStream_t) {}
void launch_root_forward(const DevTables&, int, const float*, float*, double*, float*, float*, const Dims&, hipStream_t) {}
void launch_root_backward(const DevTables&, int, const int32_t*, float*, PartialSumList*, bool, const float*, float*,
                          const float*, const double*, const float*, float*, const Dims&, hipStream_t) {}
void launch_sum_partial_stats(const PartialSumList&, float*, bool, hipStream_t) {}
void launch_region_assemble(const DevTables&, int, int, bool, float*, const float*, const Dims&, hipStream_t) {}
void launch_einsum_backward(const DevTables&, int, int, bool, bool, const float*, float*, const float*, const double*,
                            const float*, const float*, float*, float*, PartialSumList*, bool, const Dims&, hipStream_t) {}
void launch_tail_backward(const DevTables&, int, int, int, int, int, const float*, const uint8_t*, int, const float*,
                          const float*, const double*, const float*, const float*, bool, float*, int64_t, int64_t, int64_t,
                          int64_t, float*, size_t, const Dims&, hipStream_t) {}
void launch_em_update(const DevTables&, int, int, bool, float*, float*, float*, int64_t, int64_t, int64_t, float, float,
                      float, float, const Dims&, hipStream_t) {}
void launch_fill(float*, float, int64_t, hipStream_t) {}
void launch_init_params(const DevTables&, int, float*, int64_t, uint64_t, float, float, const Dims&, hipStream_t) {}
void launch_sample_init(int32_t*, int, int, hipStream_t) {}
void launch_sample_regions(const DevTables&, int, int, bool, const float*, const float*, const double*, const float*,
                           const float*, int, int32_t*, const Dims&, hipStream_t) {}
void launch_sample_leaves(const DevTables&, int, const float*, const uint8_t*, int, const float*, const float*,
                          const int32_t*, float*, const Dims&, hipStream_t) {}
hipError_t static_scratch_address(void** ptr) {
    static double arena[1 << 21];
    *ptr = arena;
    return hipSuccess;
}
hipError_t measure_peaks(const void*, void*, size_t, int, double* out, hipStream_t) {
    out[0] = out[1] = out[2] = out[3] = 1.0;
    return hipSuccess;
}
void launch_mixture_logp(const float*, const float*, int, int, float*, hipStream_t) {}
}  // namespace einet_impl
