// C ABI of libeinet (see include/einet.h): argument checks, workspace layout,
// and the per-layer launch sequence.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <cstring>
#include <algorithm>
#include <string>
#include <vector>

#include "../../include/einet.h"
#include "kernels.hpp"
#include "structure.hpp"

using namespace einet_impl;

struct einet {
    einet_spec spec{};
    RegionGraph graph;
    Plan plan;
    mutable std::string err;

    // workspace layout (bytes from the start of the workspace)
    std::vector<int32_t> blob;      // all index tables, concatenated
    size_t off_theta = 0, off_A = 0, off_Off = 0, off_amax = 0, off_G = 0, off_Gp = 0, off_part = 0, ws_bytes = 0;
    // Scratch for the statistics blocks of virtual items (bwd_virtual_items: a region per layer, since the blocks
    // of a top-down pass are summed at its end) and, after that sum, of the leaf statistics' batch groups
    // (leaf_stats_groups), which share the memory.
    bool has_part = false;
    size_t part_floats = 0;
    static constexpr size_t NO_PART = ~size_t(0);
    std::vector<size_t> part_off;   // per einsum layer: floats from off_part to its region, or NO_PART
    struct TableOffsets {
#define X(name) size_t name;
        EINET_TABLES(X)
#undef X
    } to{};

    // optional per-launch timing (einet_profile_*)
    bool profiling = false;
    struct Timed { int cls; hipEvent_t start, stop; int64_t work; };
    std::vector<Timed> timed;
    struct Launch { int cls; float ms; int64_t work; };
    std::vector<Launch> last_launches;   // the launches of the last einet_profile_read, in order
    int profile_dropped = 0;        // launches that could not be bracketed (event creation failed)

    // true while the einsum-weight statistics are logically zero: einet_em_update does not clear them,
    // the next einet_em_accumulate overwrites them instead of adding
    bool weight_stats_zero = false;

    // The posterior of the root is 1 for every sample.  Its entries (b, 0), b < root_ones_batch, of the posterior
    // arena hold that value from an earlier E-step (the arena is laid out for the batch size of the call, the
    // root first, so a call with B samples leaves exactly the first B of them alone); 0 after einet_bind and
    // after einet_sample, which uses the arena for the choices.
    int root_ones_batch = 0;

    bool bound = false;
    float* params = nullptr;
    float* stats = nullptr;
    char* ws = nullptr;
    DevTables dt{};
};

namespace {

std::string g_create_error;

size_t append(std::vector<int32_t>& blob, const std::vector<int32_t>& v) {
    while (blob.size() % 64) blob.push_back(0);   // 256-byte alignment of every table
    size_t off = blob.size();
    blob.insert(blob.end(), v.begin(), v.end());
    if (v.empty()) blob.push_back(0);
    return off;
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

int fail(const einet_t* h, int code, const std::string& msg) {
    if (h) h->err = msg;
    else g_create_error = msg;
    return code;
}

int check_hip(const einet_t* h, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(h, EINET_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
    return EINET_OK;
}

Dims dims_of(const einet_t* h, int B) {
    Dims d;
    d.B = B;
    d.D = h->graph.num_vars;
    d.C = h->plan.C;
    d.R = h->graph.num_replica;
    d.K = h->plan.K;
    d.T = h->plan.T;
    d.TD = h->plan.TD;
    d.family = h->plan.family;
    d.P = h->plan.leaf_param;
    return d;
}

int check_batch_args(einet_t* h, const float* x, const uint8_t* mask, int mask_mode, int B) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    if (B < 1) return fail(h, EINET_ERR_INVALID_ARG, "B must be at least 1");
    if (B > h->spec.max_batch) return fail(h, EINET_ERR_BATCH_TOO_LARGE, "B exceeds max_batch given to einet_create");
    if (!x) return fail(h, EINET_ERR_INVALID_ARG, "x_dev is NULL");
    if (mask_mode != EINET_MASK_NONE && mask_mode != EINET_MASK_SHARED && mask_mode != EINET_MASK_PER_SAMPLE)
        return fail(h, EINET_ERR_INVALID_ARG, "unknown mask_mode");
    if ((mask_mode != EINET_MASK_NONE) != (mask != nullptr))
        return fail(h, EINET_ERR_INVALID_ARG, "mask_dev must be NULL exactly when mask_mode is EINET_MASK_NONE");
    return EINET_OK;
}

enum KernelClass {
    KC_LEAF_FWD, KC_EINSUM_FWD, KC_MIXING_FWD, KC_REGION_BWD, KC_EINSUM_BWD, KC_LEAF_BWD, KC_UPDATE, KC_SAMPLE, KC_ROOT_FWD,
    KC_ROOT_BWD, KC_COUNT
};
int check_update_args(einet_t* h, float step, float min_var, float max_var, float w_floor) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    if (!(step > 0.f && step <= 1.f)) return fail(h, EINET_ERR_INVALID_ARG, "step must be in (0, 1]");
    if (!(min_var >= 0.f) || !(max_var >= min_var) || !(w_floor >= 0.f))
        return fail(h, EINET_ERR_INVALID_ARG, "need 0 <= min_var <= max_var and w_floor >= 0");
    return EINET_OK;
}

const char* const kKernelClassNames[KC_COUNT] = {"leaf_forward", "einsum_forward", "mixing_forward", "region_backward",
                                                 "einsum_backward", "leaf_mixing_backward", "em_update",
                                                 "sampling", "root_forward", "root_backward"};

// Runs `launch` (which enqueues kernels on s); when profiling, brackets it with two events.
template <class F>
void run(einet_t* h, int cls, hipStream_t s, F&& launch, int64_t work = 0) {
    if (!h->profiling) {
        launch();
        return;
    }
    einet::Timed t{cls, nullptr, nullptr, work};
    if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) {
        (void)hipGetLastError();
        if (t.start) (void)hipEventDestroy(t.start);
        h->profile_dropped += 1;          // einet_profile_read reports it: the totals would be short
        launch();
        return;
    }
    (void)hipEventRecord(t.start, s);
    launch();
    (void)hipEventRecord(t.stop, s);
    h->timed.push_back(t);
}

// Where the activations of a forward pass live: residuals A [node][B][K], offsets Off [node][B], shifts
// amax [item][2][B].
struct Arena {
    float* A;
    double* Off;
    float* amax;
};

Arena workspace_arena(const einet_t* h) {
    return Arena{reinterpret_cast<float*>(h->ws + h->off_A), reinterpret_cast<double*>(h->ws + h->off_Off),
                 reinterpret_cast<float*>(h->ws + h->off_amax)};
}

// Work tag of the launches of einsum layer l in the profile: output entries summed over its items (the algorithmic
// flop of a launch are 2 B K^2 times this bottom-up and 4 B K^2 times this top-down) times 2^24, plus the items.
int64_t layer_outputs(const Plan& p, int l) {
    int64_t n = 0;
    for (int e = p.ein_layer_ptr[l]; e < p.ein_layer_ptr[l + 1]; ++e) n += p.ein_kout[e];
    return (n << 24) | (int64_t)(p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l]);
}

// Leaf layer, then einsum (+ mixing) layers bottom-up; fills the arena.
void forward(einet_t* h, const Arena& ar, const float* x, const uint8_t* mask, int mask_mode, float* logp,
             const Dims& d, hipStream_t s) {
    const Plan& p = h->plan;
    float* A = ar.A;
    double* Off = ar.Off;
    const float* theta = reinterpret_cast<const float*>(h->ws + h->off_theta);
    run(h, KC_LEAF_FWD, s, [&] {
        launch_leaf_forward(h->dt, (int)p.leaf_node.size(), p.max_leaf_scope, x, mask, mask_mode, theta, A, Off, d, s);
    });
    for (int l = 0; l < p.num_layers; ++l) {
        const int count = p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l];
        if (l == p.num_layers - 1 && root_kernels_apply(count, p.K)) {
            // the root's partitions and the root's mixture in one launch
            run(h, KC_ROOT_FWD, s, [&] { launch_root_forward(h->dt, count, h->params, A, Off, ar.amax, logp, d, s); },
                layer_outputs(p, l));
            break;
        }
        run(h, KC_EINSUM_FWD, s, [&] {
            launch_einsum_forward(h->dt, p.ein_layer_ptr[l], p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l],
                                  p.ein_layer_full[l] != 0, h->params, A, Off, ar.amax, logp, d, s);
        }, layer_outputs(p, l));
        if (p.mix_layer_ptr[l + 1] > p.mix_layer_ptr[l])
            run(h, KC_MIXING_FWD, s, [&] {
                int most = 0;                         // partitions of the widest region of this layer
                for (int i = p.mix_layer_ptr[l]; i < p.mix_layer_ptr[l + 1]; ++i)
                    most = std::max(most, p.mix_cptr[i + 1] - p.mix_cptr[i]);
                launch_mixing_forward(h->dt, p.mix_layer_ptr[l], p.mix_layer_ptr[l + 1] - p.mix_layer_ptr[l], most,
                                      h->params, A, Off, logp, d, s);
            });
    }
}

}  // namespace

extern "C" {

int einet_create(const einet_spec* spec, einet_t** out) {
    if (!spec || !out) return fail(nullptr, EINET_ERR_INVALID_ARG, "spec or out is NULL");
    *out = nullptr;
    if (spec->K < 1 || spec->K > 64) return fail(nullptr, EINET_ERR_INVALID_ARG, "K must be in 1..64");
    if (spec->channels < 1) return fail(nullptr, EINET_ERR_INVALID_ARG, "channels must be at least 1");
    if (spec->max_batch < 1) return fail(nullptr, EINET_ERR_INVALID_ARG, "max_batch must be at least 1");
    if (spec->leaf_family < EINET_LEAF_BERNOULLI || spec->leaf_family > EINET_LEAF_CATEGORICAL)
        return fail(nullptr, EINET_ERR_INVALID_ARG, "unknown leaf_family");
    if (spec->leaf_family == EINET_LEAF_BINOMIAL && (spec->leaf_param < 1 || spec->leaf_param > 4095))
        return fail(nullptr, EINET_ERR_INVALID_ARG, "binomial leaves need leaf_param (trials) in 1..4095");
    if (spec->leaf_family == EINET_LEAF_CATEGORICAL && (spec->leaf_param < 2 || spec->leaf_param > 256))
        return fail(nullptr, EINET_ERR_INVALID_ARG, "categorical leaves need leaf_param (values) in 2..256");
    einet_t* h = new einet();
    h->spec = *spec;
    std::string err;
    bool ok = false;
    if (spec->structure == EINET_STRUCTURE_RAT) {
        if (spec->num_vars < 2 || spec->depth < 1 || spec->depth > 24 || spec->num_replica < 1) {
            delete h;
            return fail(nullptr, EINET_ERR_INVALID_ARG, "random binary trees need num_vars >= 2, depth in 1..24, num_replica >= 1");
        }
        ok = build_rat(spec->num_vars, spec->depth, spec->num_replica, spec->seed, h->graph, err);
    } else if (spec->structure == EINET_STRUCTURE_PD) {
        bool good = spec->height >= 1 && spec->width >= 1 && spec->num_deltas >= 1 &&
                    spec->num_deltas <= EINET_MAX_DELTAS && (spec->axes & 3) && !(spec->axes & ~3);
        for (int i = 0; good && i < spec->num_deltas; ++i) good = spec->deltas[i] >= 1;
        if (!good) {
            delete h;
            return fail(nullptr, EINET_ERR_INVALID_ARG, "Poon-Domingos needs height, width >= 1, 1..8 positive deltas, axes in 1..3");
        }
        ok = build_pd(spec->height, spec->width, spec->deltas, spec->num_deltas, spec->axes, h->graph, err);
    } else {
        delete h;
        return fail(nullptr, EINET_ERR_INVALID_ARG, "unknown structure kind");
    }
    if (ok) ok = compile_plan(h->graph, spec->K, spec->channels, spec->leaf_family, spec->leaf_param, h->plan, err);
    if (!ok) {
        delete h;
        return fail(nullptr, EINET_ERR_BAD_STRUCTURE, err);
    }
    // workspace layout
    const Plan& p = h->plan;
    auto& b = h->blob;
    auto& t = h->to;
#define X(name) t.name = append(b, p.name);
    EINET_TABLES(X)
#undef X
    const size_t K = p.K, mb = spec->max_batch;
    size_t off = align256(b.size() * sizeof(int32_t));
    h->off_theta = off;
    off = align256(off + sizeof(float) * size_t(h->graph.num_vars) * p.C * h->graph.num_replica * p.TD * K);
    h->off_A = off;
    off = align256(off + sizeof(float) * size_t(p.num_nodes) * mb * K);
    h->off_Off = off;
    off = align256(off + sizeof(double) * size_t(p.num_nodes) * mb);
    h->off_amax = off;
    off = align256(off + sizeof(float) * 2 * p.ein_left.size() * mb);
    h->off_G = off;
    off = align256(off + sizeof(float) * size_t(p.num_nodes) * mb * K);
    h->off_Gp = off;
    off = align256(off + sizeof(float) * gp_blocks_per_item(p.K) * p.ein_left.size() * mb * K);
    h->part_off.assign(p.num_layers, einet::NO_PART);
    for (int l = 0; l < p.num_layers; ++l) {         // (the root's layer, the last, has a kernel of its own)
        const int count = p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l];
        const size_t need = l + 1 < p.num_layers ? bwd_partial_bound(count, (int)p.K, (int)mb, p.ein_layer_full[l] != 0)
                                                 : root_bwd_partial_bound(count, (int)p.K, (int)mb);
        if (need == 0) continue;
        h->has_part = true;
        h->part_off[l] = h->part_floats;
        h->part_floats += (need + 63) & ~size_t(63);
    }
    {
        const int lg = leaf_stats_groups_max((int)p.leaf_node.size(), p.max_leaf_scope, p.C, (int)p.K, (int)mb);
        if (lg > 1 && p.family != EINET_LEAF_CATEGORICAL) {
            h->has_part = true;
            const size_t need = (size_t)lg * (size_t)(p.n_stats - p.phi_offset);
            if (need > h->part_floats) h->part_floats = need;
        }
    }
    if (h->has_part) {
        h->off_part = off;
        off = align256(off + sizeof(float) * h->part_floats);
    }
    h->ws_bytes = off;
    *out = h;
    return EINET_OK;
}

void einet_destroy(einet_t* h) {
    if (!h) return;
    for (auto& t : h->timed) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    delete h;
}

const char* einet_last_error(const einet_t* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int einet_sizes(const einet_t* h, size_t* n_params, size_t* n_stats, size_t* workspace_bytes) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (n_params) *n_params = (size_t)h->plan.n_params;
    if (n_stats) *n_stats = (size_t)h->plan.n_stats;
    if (workspace_bytes) *workspace_bytes = h->ws_bytes;
    return EINET_OK;
}

int einet_structure(const einet_t* h, einet_structure_view* v) {
    if (!h || !v) return EINET_ERR_INVALID_ARG;
    const Plan& p = h->plan;
    v->num_vars = h->graph.num_vars;
    v->num_regions = (int32_t)h->graph.scope.size();
    v->num_partitions = (int32_t)h->graph.partition.size();
    v->num_replica = h->graph.num_replica;
    v->num_layers = p.num_layers;
    v->K = p.K;
    v->channels = p.C;
    v->num_suff_stats = p.T;
    v->scope_ptr = p.scope_ptr.data();
    v->scope_var = p.scope_var.data();
    v->region_replica = h->graph.replica.data();
    v->partition = p.partition_flat.data();
    v->layer_ptr = p.layer_ptr.data();
    v->layer_partition = p.layer_partition.data();
    v->w_offset = p.w_offset.data();
    v->v_offset = p.v_offset.data();
    v->phi_offset = p.phi_offset;
    v->den_offset = p.den_offset;
    v->tot_offset = p.tot_offset;
    return EINET_OK;
}

int einet_bind(einet_t* h, float* params_dev, float* stats_dev, void* workspace_dev, void* stream) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!params_dev || !stats_dev || !workspace_dev) return fail(h, EINET_ERR_INVALID_ARG, "NULL device buffer");
    if (reinterpret_cast<uintptr_t>(workspace_dev) % 256) return fail(h, EINET_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (reinterpret_cast<uintptr_t>(params_dev) % 16 || reinterpret_cast<uintptr_t>(stats_dev) % 16)
        return fail(h, EINET_ERR_INVALID_ARG, "params and stats must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(workspace_dev, h->blob.data(), h->blob.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(h, EINET_ERR_HIP, std::string("uploading index tables: ") + hipGetErrorString(e));
    // Statistics that an M-step has consumed but not cleared in memory stay logically zero when the very same
    // buffer is bound again; any other buffer is taken to hold statistics to be continued.
    const bool same_stats = h->bound && h->stats == stats_dev;
    h->params = params_dev;
    h->stats = stats_dev;
    h->ws = static_cast<char*>(workspace_dev);
    const int32_t* base = reinterpret_cast<const int32_t*>(h->ws);
    const auto& t = h->to;
#define X(name) h->dt.name = base + t.name;
    EINET_TABLES(X)
#undef X
    h->bound = true;
    h->root_ones_batch = 0;
    h->weight_stats_zero = same_stats && h->weight_stats_zero;
    return EINET_OK;
}

int einet_refresh(einet_t* h, void* stream) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    launch_leaf_derive(h->params + h->plan.phi_offset, reinterpret_cast<float*>(h->ws + h->off_theta), dims_of(h, 0),
                       static_cast<hipStream_t>(stream));
    return check_hip(h, "einet_refresh");
}

int einet_init_params(einet_t* h, uint64_t seed, float leaf_lo, float leaf_hi, void* stream) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    if (!(leaf_lo <= leaf_hi)) return fail(h, EINET_ERR_INVALID_ARG, "need leaf_lo <= leaf_hi");
    const bool prob = h->plan.family == EINET_LEAF_BERNOULLI || h->plan.family == EINET_LEAF_BINOMIAL;
    if (prob && !(leaf_lo > 0.f && leaf_hi < 1.f))
        return fail(h, EINET_ERR_INVALID_ARG, "Bernoulli and binomial leaves need 0 < leaf_lo <= leaf_hi < 1");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims d = dims_of(h, 0);
    launch_init_params(h->dt, (int)h->plan.row_off.size(), h->params, h->plan.phi_offset, seed, leaf_lo, leaf_hi, d, s);
    launch_leaf_derive(h->params + h->plan.phi_offset, reinterpret_cast<float*>(h->ws + h->off_theta), d, s);
    return check_hip(h, "einet_init_params");
}

int einet_logp(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B, float* logp_dev,
               void* stream) {
    int rc = check_batch_args(h, x_dev, mask_dev, mask_mode, B);
    if (rc != EINET_OK) return rc;
    if (!logp_dev) return fail(h, EINET_ERR_INVALID_ARG, "logp_dev is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims d = dims_of(h, B);
    forward(h, workspace_arena(h), x_dev, mask_dev, mask_mode, logp_dev, d, s);
    return check_hip(h, "einet_logp");
}

int einet_logp_static(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B, float* logp_dev,
                      void* stream) {
    int rc = check_batch_args(h, x_dev, mask_dev, mask_mode, B);
    if (rc != EINET_OK) return rc;
    if (!logp_dev) return fail(h, EINET_ERR_INVALID_ARG, "logp_dev is NULL");
    const Plan& p = h->plan;
    const size_t K = p.K, nb = (size_t)B;
    const size_t bytes_A = align256(sizeof(float) * size_t(p.num_nodes) * nb * K);
    const size_t bytes_Off = align256(sizeof(double) * size_t(p.num_nodes) * nb);
    const size_t bytes_amax = align256(sizeof(float) * 2 * p.ein_left.size() * nb);
    const size_t need = bytes_A + bytes_Off + bytes_amax;
    if (need > EINET_STATIC_SCRATCH_BYTES)
        return fail(h, EINET_ERR_BATCH_TOO_LARGE,
                    "einet_logp_static: this model needs " + std::to_string(need) + " bytes of activations for B = " +
                        std::to_string(B) + ", the fixed arena holds " + std::to_string(EINET_STATIC_SCRATCH_BYTES));
    void* base = nullptr;
    const hipError_t e = static_scratch_address(&base);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(h, EINET_ERR_HIP, std::string("einet_logp_static: address of the fixed arena: ") + hipGetErrorString(e));
    }
    char* c = static_cast<char*>(base);
    const Arena ar{reinterpret_cast<float*>(c), reinterpret_cast<double*>(c + bytes_A),
                   reinterpret_cast<float*>(c + bytes_A + bytes_Off)};
    forward(h, ar, x_dev, mask_dev, mask_mode, logp_dev, dims_of(h, B), static_cast<hipStream_t>(stream));
    return check_hip(h, "einet_logp_static");
}

int einet_em_accumulate(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B,
                        float* logp_dev, void* stream) {
    int rc = check_batch_args(h, x_dev, mask_dev, mask_mode, B);
    if (rc != EINET_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims d = dims_of(h, B);
    const Plan& p = h->plan;
    forward(h, workspace_arena(h), x_dev, mask_dev, mask_mode, logp_dev, d, s);
    const float* A = reinterpret_cast<const float*>(h->ws + h->off_A);
    const double* Off = reinterpret_cast<const double*>(h->ws + h->off_Off);
    float* G = reinterpret_cast<float*>(h->ws + h->off_G);
    float* Gp = reinterpret_cast<float*>(h->ws + h->off_Gp);
    // top-down: posteriors of the regions of sum layer l (root first), then the einsum items below them
    const float* amax = reinterpret_cast<const float*>(h->ws + h->off_amax);
    PartialSumList sums;
    auto layer_part = [&](int l) -> float* {
        return h->part_off[l] == einet::NO_PART ? nullptr
                                                : reinterpret_cast<float*>(h->ws + h->off_part) + h->part_off[l];
    };
    for (int l = p.num_layers - 1, step = 0; l >= 0; --l, ++step) {
        // (the top sum layer is the root alone: nothing to launch when its ones are still in place; nor for a layer
        // whose einsum kernel adds up the parents' blocks itself)
        const bool direct = p.ein_layer_direct[l] != 0;
        if (!direct && (step > 0 || B > h->root_ones_batch))
            run(h, KC_REGION_BWD, s, [&] {
                launch_region_assemble(h->dt, p.rb_layer_ptr[step], p.rb_layer_ptr[step + 1] - p.rb_layer_ptr[step],
                                       step == 0, G, Gp, d, s);
            });
        if (step == 0) {
            // the root's partitions (one output entry each; the root's posterior is 1, its block in G is read by the
            // mixing statistics only): a launch of their own kind, timed as a class of its own
            run(h, KC_ROOT_BWD, s, [&] {
                launch_root_backward(h->dt, p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l], h->dt.ein_woff + p.ein_layer_ptr[l],
                                     layer_part(l), &sums,
                                     !h->weight_stats_zero, h->params, h->stats, A, Off, amax, Gp, d, s);
                if (l == 0) launch_sum_partial_stats(sums, h->stats, !h->weight_stats_zero, s);
            }, layer_outputs(p, l));
            continue;
        }
        run(h, KC_EINSUM_BWD, s, [&] {
            launch_einsum_backward(h->dt, p.ein_layer_ptr[l], p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l],
                                   p.ein_layer_full[l] != 0, !h->weight_stats_zero, h->params, h->stats, A, Off, amax, G, Gp,
                                   layer_part(l), &sums, direct, d, s);
            // after the last layer: the statistics blocks of the launches that ran virtual items, all layers in one
            // launch (before the leaf statistics, whose batch groups use the same scratch)
            if (l == 0) launch_sum_partial_stats(sums, h->stats, !h->weight_stats_zero, s);
        }, layer_outputs(p, l));
    }
    const int leaf_step = p.num_layers;
    if (!p.leaves_direct)
        run(h, KC_REGION_BWD, s, [&] {
            launch_region_assemble(h->dt, p.rb_layer_ptr[leaf_step],
                                   p.rb_layer_ptr[leaf_step + 1] - p.rb_layer_ptr[leaf_step], false, G, Gp, d, s);
        });
    run(h, KC_LEAF_BWD, s, [&] {
        launch_tail_backward(h->dt, (int)p.lv_leaf.size(), (int)p.leaf_node.size(), p.max_leaf_scope,
                             (int)p.mix_node.size(), p.max_mix_children, x_dev, mask_dev,
                             mask_mode, h->params, A, Off, G, Gp, p.leaves_direct, h->stats, p.phi_offset, p.den_offset,
                             p.tot_offset, p.n_stats,
                             h->has_part ? reinterpret_cast<float*>(h->ws + h->off_part) : nullptr, h->part_floats, d, s);
    });
    rc = check_hip(h, "einet_em_accumulate");
    // (after a failed launch nothing is known about the arena or the statistics: the root's ones are written
    // again next time, and the statistics are added to, never overwritten)
    h->weight_stats_zero = false;
    h->root_ones_batch = rc == EINET_OK ? B : 0;
    return rc;
}

int einet_em_update(einet_t* h, float step, float min_var, float max_var, float w_floor, void* stream) {
    int rc = check_update_args(h, step, min_var, max_var, w_floor);
    if (rc != EINET_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims d = dims_of(h, 0);
    const Plan& p = h->plan;
    run(h, KC_UPDATE, s, [&] {
        launch_em_update(h->dt, (int)p.row_off.size(), p.n_weight_rows, h->weight_stats_zero, h->params, h->stats,
                         reinterpret_cast<float*>(h->ws + h->off_theta), p.phi_offset, p.den_offset, p.tot_offset,
                         step, min_var, max_var, w_floor, d, s);
    });
    rc = check_hip(h, "einet_em_update");
    if (rc == EINET_OK) h->weight_stats_zero = true;
    return rc;
}

int einet_em_reset(einet_t* h, void* stream) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    launch_fill(h->stats, 0.f, h->plan.n_stats, static_cast<hipStream_t>(stream));
    const int rc = check_hip(h, "einet_em_reset");
    h->weight_stats_zero = rc == EINET_OK;
    return rc;
}

int einet_em_epoch(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int64_t N, int batch,
                   float step, float min_var, float max_var, float w_floor, float* logp_dev, void* stream) {
    int rc = check_batch_args(h, x_dev, mask_dev, mask_mode, batch);
    if (rc != EINET_OK) return rc;
    if (N < 1) return fail(h, EINET_ERR_INVALID_ARG, "N must be at least 1");
    rc = check_update_args(h, step, min_var, max_var, w_floor);
    if (rc != EINET_OK) return rc;
    const size_t sample = (size_t)h->graph.num_vars * h->plan.C;
    for (int64_t b0 = 0; b0 < N; b0 += batch) {
        const int nb = (int)(N - b0 < batch ? N - b0 : batch);
        const uint8_t* m = mask_mode == EINET_MASK_PER_SAMPLE ? mask_dev + (size_t)b0 * h->graph.num_vars : mask_dev;
        rc = einet_em_accumulate(h, x_dev + (size_t)b0 * sample, m, mask_mode, nb, logp_dev ? logp_dev + b0 : nullptr,
                                 stream);
        if (rc != EINET_OK) return rc;
        rc = einet_em_update(h, step, min_var, max_var, w_floor, stream);
        if (rc != EINET_OK) return rc;
    }
    return EINET_OK;
}

int einet_sample(einet_t* h, int B, const float* x_dev, const uint8_t* mask_dev, int mask_mode, const float* u_dev,
                 const float* noise_dev, float* out_dev, void* stream) {
    if (!h) return EINET_ERR_INVALID_ARG;
    if (!h->bound) return fail(h, EINET_ERR_NOT_BOUND, "einet_bind has not been called");
    if (B < 1) return fail(h, EINET_ERR_INVALID_ARG, "B must be at least 1");
    if (B > h->spec.max_batch) return fail(h, EINET_ERR_BATCH_TOO_LARGE, "B exceeds max_batch given to einet_create");
    if (B > 65535) return fail(h, EINET_ERR_BATCH_TOO_LARGE, "einet_sample draws at most 65535 samples per call");
    if (!u_dev || !out_dev) return fail(h, EINET_ERR_INVALID_ARG, "u_dev or out_dev is NULL");
    const bool evidence = mask_mode != EINET_MASK_NONE;
    if (evidence) {
        int rc = check_batch_args(h, x_dev, mask_dev, mask_mode, B);
        if (rc != EINET_OK) return rc;
    } else if (x_dev || mask_dev) {
        return fail(h, EINET_ERR_INVALID_ARG, "without evidence (EINET_MASK_NONE) x_dev and mask_dev must be NULL");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dims d = dims_of(h, B);
    const Plan& p = h->plan;
    if (evidence) forward(h, workspace_arena(h), x_dev, mask_dev, mask_mode, nullptr, d, s);
    const float* A = reinterpret_cast<const float*>(h->ws + h->off_A);
    const double* Off = reinterpret_cast<const double*>(h->ws + h->off_Off);
    const float* amax = reinterpret_cast<const float*>(h->ws + h->off_amax);
    // the chosen entries live where the posterior arena of the EM pass lives (one int32 per node and sample)
    int32_t* sel = reinterpret_cast<int32_t*>(h->ws + h->off_G);
    h->root_ones_batch = 0;
    const int n_part = (int)h->graph.partition.size();
    run(h, KC_SAMPLE, s, [&] {
        launch_sample_init(sel, p.num_nodes, B, s);
        for (int l = p.num_layers - 1; l >= 0; --l)
            launch_sample_regions(h->dt, p.sr_layer_ptr[l], p.sr_layer_ptr[l + 1] - p.sr_layer_ptr[l], evidence,
                                  h->params, A, Off, amax, u_dev, n_part, sel, d, s);
        launch_sample_leaves(h->dt, (int)p.lv_leaf.size(), x_dev, mask_dev, mask_mode, h->params + p.phi_offset,
                             noise_dev, sel, out_dev, d, s);
    });
    return check_hip(h, "einet_sample");
}

int einet_mixture_logp(const float* logp_dev, const float* log_coef_dev, int n_components, int B, float* out_dev,
                       void* stream) {
    if (!logp_dev || !log_coef_dev || !out_dev)
        return fail(nullptr, EINET_ERR_INVALID_ARG, "einet_mixture_logp: NULL pointer");
    if (n_components < 1 || B < 1)
        return fail(nullptr, EINET_ERR_INVALID_ARG, "einet_mixture_logp: n_components and B must be at least 1");
    launch_mixture_logp(logp_dev, log_coef_dev, n_components, B, out_dev, static_cast<hipStream_t>(stream));
    return check_hip(nullptr, "einet_mixture_logp");
}

int einet_profile_enable(einet_t* h, int enable) {
    if (!h) return EINET_ERR_INVALID_ARG;
    h->profiling = enable != 0;
    return EINET_OK;
}

int einet_profile_read(einet_t* h, int capacity, int* n_classes, const char** names, double* total_ms,
                       int64_t* launches) {
    if (!h || capacity < 0 || !n_classes) return EINET_ERR_INVALID_ARG;
    double ms[KC_COUNT] = {0};
    int64_t cnt[KC_COUNT] = {0};
    int rc = EINET_OK;
    h->last_launches.clear();
    for (auto& t : h->timed) {
        float el = 0.f;
        hipError_t e = hipEventSynchronize(t.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&el, t.start, t.stop);
        if (e != hipSuccess) rc = fail(h, EINET_ERR_HIP, std::string("reading profile events: ") + hipGetErrorString(e));
        ms[t.cls] += el;
        cnt[t.cls] += 1;
        h->last_launches.push_back({t.cls, el, t.work});
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    h->timed.clear();
    if (h->profile_dropped > 0) {
        rc = fail(h, EINET_ERR_HIP, std::to_string(h->profile_dropped) + " launches were not timed (event creation failed)");
        h->profile_dropped = 0;
    }
    *n_classes = KC_COUNT;
    for (int i = 0; i < KC_COUNT && i < capacity; ++i) {
        if (names) names[i] = kKernelClassNames[i];
        if (total_ms) total_ms[i] = ms[i];
        if (launches) launches[i] = cnt[i];
    }
    return rc;
}

int einet_profile_launches(einet_t* h, int64_t capacity, int64_t* n_launches, int32_t* cls, float* ms, int64_t* work) {
    if (!h || capacity < 0 || !n_launches) return EINET_ERR_INVALID_ARG;
    *n_launches = (int64_t)h->last_launches.size();
    for (int64_t i = 0; i < *n_launches && i < capacity; ++i) {
        if (cls) cls[i] = h->last_launches[i].cls;
        if (ms) ms[i] = h->last_launches[i].ms;
        if (work) work[i] = h->last_launches[i].work;
    }
    return EINET_OK;
}

int einet_measure_peaks(const void* src_dev, void* dst_dev, int64_t bytes, int reps, double* out4, void* stream) {
    if (!src_dev || !dst_dev || !out4 || reps < 1 || bytes < (int64_t)EINET_PEAKS_MIN_BYTES || bytes % 16 != 0)
        return fail(nullptr, EINET_ERR_INVALID_ARG,
                    "einet_measure_peaks: buffers of at least EINET_PEAKS_MIN_BYTES bytes, a multiple of 16, and reps >= 1");
    if (measure_peaks(src_dev, dst_dev, (size_t)bytes, reps, out4, static_cast<hipStream_t>(stream)) != hipSuccess)
        return fail(nullptr, EINET_ERR_HIP, "einet_measure_peaks: a timed launch failed");
    return check_hip(nullptr, "einet_measure_peaks");
}

}  // extern "C"
