// Launchers of the HIP kernels (device code lives in kernels.hip).  All pointers
// are device pointers; every launcher only enqueues work on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/einet.h"

namespace einet_impl {

// Device copies of the plan tables (pointers into the bound workspace).
struct DevTables {
    const int32_t *ein_left, *ein_right, *ein_out, *ein_kout, *ein_woff;
    const int32_t *mix_node, *mix_kout, *mix_cptr, *mix_child, *mix_voff;
    const int32_t *leaf_node, *leaf_replica, *leaf_sptr, *leaf_var, *lv_leaf, *lv_var;
    const int32_t *rb_node, *rb_kout, *rb_mix, *rb_pptr, *rb_pslot;
    const int32_t *row_off, *row_len;
};

struct Dims {
    int B, D, C, R, K, T, TD, family;
};

void launch_leaf_derive(const float* phi, float* theta, const Dims& d, hipStream_t s);
void launch_leaf_forward(const DevTables& t, int n_leaves, const float* x, const uint8_t* mask, int mask_mode,
                         const float* theta, float* A, const Dims& d, hipStream_t s);
void launch_einsum_forward(const DevTables& t, int first, int count, const float* params, float* A, const Dims& d,
                           hipStream_t s);
void launch_mixing_forward(const DevTables& t, int first, int count, const float* params, float* A, const Dims& d,
                           hipStream_t s);
void launch_copy_root(const float* A, float* logp, const Dims& d, hipStream_t s);

void launch_region_backward(const DevTables& t, int first, int count, bool is_root_layer, const float* params,
                            float* stats, const float* A, float* G, const float* Gp, const Dims& d, hipStream_t s);
void launch_einsum_backward(const DevTables& t, int first, int count, const float* params, float* stats,
                            const float* A, const float* G, float* Gp, const Dims& d, hipStream_t s);
void launch_leaf_backward(const DevTables& t, int n_lv, const float* x, const uint8_t* mask, int mask_mode,
                          const float* G, float* stats, int64_t phi_off, int64_t den_off, int64_t tot_off,
                          const Dims& d, hipStream_t s);

void launch_update_rows(const DevTables& t, int n_rows, float* params, float* stats, float step, float w_floor,
                        hipStream_t s);
void launch_update_leaves(float* params, float* stats, int64_t phi_off, int64_t den_off, int64_t tot_off, float step,
                          float min_var, float max_var, const Dims& d, hipStream_t s);
void launch_fill(float* p, float value, int64_t n, hipStream_t s);

}  // namespace einet_impl
