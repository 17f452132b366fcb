// Host-side structure compiler: region graph -> layered execution plan.
//
// A vectorised circuit (Sec. 3.1) is kept as regions (sum or leaf vectors) and
// partitions (binary product nodes, one parent region each).  The plan turns it
// into the flat tables the kernels walk: one arena slot ("node") per region and
// per simple sum (App. B), einsum layers bottom-up (Algorithm 1), mixing items,
// and per region the list of partitions that feed its posterior top-down.
#pragma once
#include <array>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/einet.h"
#include "kernels.hpp"

namespace einet_impl {

struct RegionGraph {
    int num_vars = 0;
    int num_replica = 0;
    std::vector<std::vector<int32_t>> scope;        // region -> ascending variables
    std::vector<std::array<int32_t, 3>> partition;  // parent, left, right
    std::vector<std::vector<int32_t>> parts_of;     // region -> its partitions, ascending
    std::vector<int32_t> replica;                   // leaf region -> replica, else -1
    bool is_leaf(int s) const { return parts_of[s].empty(); }
};

// Generators; return false and fill err when the structure cannot be built.
bool build_rat(int D, int depth, int R, uint64_t seed, RegionGraph& g, std::string& err);
bool build_pd(int H, int W, const int32_t* deltas, int n_deltas, int axes, RegionGraph& g, std::string& err);

// Everything the device needs, as host vectors (uploaded verbatim by einet_bind).
struct Plan {
    int K = 0, C = 0, T = 0, TD = 0, family = 0;
    int leaf_param = 1;     // trials of a binomial leaf (1 for Bernoulli), values of a categorical leaf
    int num_nodes = 0;      // regions + simple sums
    int num_layers = 0;
    int max_mix_children = 0;
    int max_leaf_scope = 0;
    int n_weight_rows = 0;  // rows of row_off/row_len that belong to einsum weights (the rest: mixing weights)

    // Index tables (see EINET_TABLES): einsum items in execution order (bottom layer first); mixing items
    // grouped by the layer whose einsum they follow; leaves; top-down items (sum layers from the root
    // down, then the leaves) with, per region, the runs of posterior blocks its parents write; M-step rows;
    // sampling items: every sum region with the einsum items of its partitions (sr_item[sr_pptr[r] ..], in the
    // order of the region's mixing weights) and its mixing item (sr_mix, -1 for a single partition).
#define X(name) std::vector<int32_t> name;
    EINET_TABLES(X)
#undef X
    std::vector<int32_t> ein_layer_ptr;             // [num_layers+1]
    std::vector<uint8_t> ein_layer_full;            // [num_layers]: every item of the layer has K output entries
    std::vector<uint8_t> ein_layer_direct;          // [num_layers]: the layer's top-down kernel reads its regions'
                                                    // posteriors from the parents' blocks (ein_gsrc), G is not assembled
    bool leaves_direct = false;                     // the leaf statistics read the leaves' posteriors from the
                                                    // parents' blocks (leaf_gsrc); G of the leaves is not assembled
    std::vector<int32_t> mix_layer_ptr;             // [num_layers+1]
    std::vector<int32_t> rb_layer_ptr;              // [num_layers+2]
    std::vector<int32_t> sr_layer_ptr;              // [num_layers+1]: sampling items (sum regions) per layer, bottom-up

    // ABI view data
    std::vector<int32_t> scope_ptr, scope_var, layer_partition, layer_ptr, partition_flat;
    std::vector<int64_t> w_offset, v_offset;
    int64_t phi_offset = 0, den_offset = 0, tot_offset = 0;
    int64_t n_params = 0, n_stats = 0;
};

bool compile_plan(const RegionGraph& g, int K, int C, int family, int leaf_param, Plan& plan, std::string& err);

}  // namespace einet_impl
