// Shared by the HIP translation units: the data layout of the arenas and small device helpers.
//
// Activations live in a node-major arena A[node][b][k] (float32, log domain):
// every region and every simple sum owns one dense [B][K] block, so a layer's
// "gather" of left and right inputs (Sec. 3.3) is an index lookup.  A block does
// not hold the log-densities themselves but their residuals against one offset
// per (node, sample), Off[node][b] (float64):
//     log-density[node][b][k] = Off[node][b] + A[node][b][k].
// Leaves take their largest entry as offset; an einsum output takes the offsets of
// its children plus the two shifts of Eq. 4, so that its residual is log S~ in
// [log of the smallest weight, 0]; a mixing output takes the largest offset of its
// children.  Log-densities of large scopes have magnitudes of 1e3..1e5, where a
// float32 resolves 1e-4..1e-2; the residuals stay small, and the posteriors of the
// top-down pass (exponentials of differences) keep full float32 precision.  The
// posterior arena G has the same shape; Gp holds what einsum item e sends down:
// blocks e*nb .. e*nb+nb-1 ([b][k] each, nb = 1 + ceil(K/4)), the first for its
// left child, the others, one per workgroup of the item's top-down launch, shares
// for its right child.  A child sums the blocks of its parents when it is
// processed: no atomics anywhere.
#ifndef EINET_DEVICE_COMMON_HPP
#define EINET_DEVICE_COMMON_HPP

#include "kernels.hpp"

#include <cmath>

namespace einet_impl {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int EINET_NUM_CUS = 256;        // compute units of an MI355X: workgroups of a one-per-unit launch
constexpr int EINET_MAX_DEVICES = 16;     // per-device once-flags of the launchers

// Raises the dynamic-LDS limit of a kernel.  A refusal is not kept as the thread's last error: the launch
// that needs the memory then fails and reports it, instead of a later, unrelated call.
template <class Kernel>
inline void allow_dynamic_lds(Kernel kernel, size_t bytes) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)bytes) != hipSuccess)
        (void)hipGetLastError();
}

// Workgroups of a launch are handed to the 8 XCDs round-robin by blockIdx.x, and every XCD has an L2 of its own.
// This renumbering gives each XCD a contiguous range of work items, so that neighbouring items (the workgroups
// of one partition, which read the same child rows) meet in one L2.  It is a bijection on [0, gridDim.x).
__device__ __forceinline__ int xcd_contiguous_block() {
    const int n = gridDim.x, x = blockIdx.x & 7, q = n >> 3, r = n & 7;
    return x * q + min(x, r) + (blockIdx.x >> 3);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace einet_impl

#endif
