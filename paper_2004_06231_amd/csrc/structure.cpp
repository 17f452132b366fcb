// Structure generators and the layered plan (host only).
#include "structure.hpp"

#include <cmath>
#include <cstring>

#include <algorithm>
#include <map>
#include <numeric>

namespace einet_impl {

namespace {

// SplitMix64 (Steele, Lea, Flood 2014), the stream that drives the random splits.
struct SplitMix64 {
    uint64_t state;
    uint64_t next() {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

int add_region(RegionGraph& g, std::vector<int32_t> scope) {
    g.scope.push_back(std::move(scope));
    g.parts_of.emplace_back();
    g.replica.push_back(-1);
    return (int)g.scope.size() - 1;
}

void add_partition(RegionGraph& g, int parent, int left, int right) {
    g.partition.push_back({parent, left, right});
    g.parts_of[parent].push_back((int)g.partition.size() - 1);
}

}  // namespace

// Random binary trees (Sec. 4.1): the scope is halved at random down to the
// given depth, R times; region/partition numbers follow the heap index so that
// the numbering does not depend on traversal order.
bool build_rat(int D, int depth, int R, uint64_t seed, RegionGraph& g, std::string& err) {
    g = RegionGraph();
    g.num_vars = D;
    g.num_replica = R;
    const int64_t per_tree = (int64_t(1) << (depth + 1)) - 2;
    const int64_t splits = (int64_t(1) << depth) - 1;
    std::vector<int32_t> all(D);
    std::iota(all.begin(), all.end(), 0);
    add_region(g, all);
    for (int64_t i = 0; i < R * per_tree; ++i) add_region(g, {});
    g.partition.assign(R * splits, {0, 0, 0});
    for (int r = 0; r < R; ++r) {
        auto region_of = [&](int64_t h) { return h == 1 ? 0 : int(1 + r * per_tree + (h - 2)); };
        for (int64_t h = 1; h <= splits; ++h) {
            std::vector<int32_t> a = g.scope[region_of(h)];
            const int n = (int)a.size();
            if (n < 2) {
                err = "random binary tree: a scope of one variable would have to be split (depth too large for D)";
                return false;
            }
            SplitMix64 rng{seed ^ (0xD1B54A32D192ED03ull * uint64_t(r + 1)) ^ (0x8CB92BA72F3D8DD7ull * uint64_t(h))};
            for (int t = n - 1; t >= 1; --t) std::swap(a[t], a[rng.next() % uint64_t(t + 1)]);
            std::vector<int32_t> left(a.begin(), a.begin() + n / 2), right(a.begin() + n / 2, a.end());
            std::sort(left.begin(), left.end());
            std::sort(right.begin(), right.end());
            const int l = region_of(2 * h), rr = region_of(2 * h + 1);
            g.scope[l] = std::move(left);
            g.scope[rr] = std::move(right);
            g.partition[r * splits + (h - 1)] = {region_of(h), l, rr};
        }
        for (int64_t h = splits + 1; h <= 2 * splits + 1; ++h) g.replica[region_of(h)] = r;
    }
    for (size_t n = 0; n < g.partition.size(); ++n) g.parts_of[g.partition[n][0]].push_back((int)n);
    for (auto& v : g.parts_of) std::sort(v.begin(), v.end());
    return true;
}

// Poon-Domingos (Sec. 4.2): every rectangle is cut along the grid given by the
// first step that cuts it; identical rectangles are one region.
bool build_pd(int H, int W, const int32_t* deltas, int n_deltas, int axes, RegionGraph& g, std::string& err) {
    g = RegionGraph();
    g.num_vars = H * W;
    struct Rect { int y0, y1, x0, x1; };
    std::vector<Rect> rects;
    std::map<std::array<int, 4>, int> seen;
    auto region_for = [&](Rect r) {
        std::array<int, 4> key{r.y0, r.y1, r.x0, r.x1};
        auto it = seen.find(key);
        if (it != seen.end()) return it->second;
        std::vector<int32_t> sc;
        sc.reserve(size_t(r.y1 - r.y0) * (r.x1 - r.x0));
        for (int y = r.y0; y < r.y1; ++y)
            for (int x = r.x0; x < r.x1; ++x) sc.push_back(y * W + x);
        int id = add_region(g, std::move(sc));
        rects.push_back(r);
        seen[key] = id;
        return id;
    };
    region_for({0, H, 0, W});
    for (size_t s = 0; s < rects.size(); ++s) {
        const Rect r = rects[s];
        for (int di = 0; di < n_deltas; ++di) {
            const int d = deltas[di];
            const bool cut_y = (axes & EINET_AXIS_Y) && r.y0 + d < r.y1;
            const bool cut_x = (axes & EINET_AXIS_X) && r.x0 + d < r.x1;
            if (!cut_y && !cut_x) continue;
            if (cut_y)
                for (int c = r.y0 + d; c < r.y1; c += d) {
                    int l = region_for({r.y0, c, r.x0, r.x1});
                    int rr = region_for({c, r.y1, r.x0, r.x1});
                    add_partition(g, (int)s, l, rr);
                }
            if (cut_x)
                for (int c = r.x0 + d; c < r.x1; c += d) {
                    int l = region_for({r.y0, r.y1, r.x0, c});
                    int rr = region_for({r.y0, r.y1, c, r.x1});
                    add_partition(g, (int)s, l, rr);
                }
            break;
        }
    }
    if (g.is_leaf(0)) {
        err = "Poon-Domingos: no step in deltas cuts the image";
        return false;
    }
    // replicas: leaves that share one must not overlap (Sec. 3.4); first fit in region order
    std::vector<std::vector<char>> covered;
    for (int s = 0; s < (int)g.scope.size(); ++s) {
        if (!g.is_leaf(s)) continue;
        int chosen = -1;
        for (int r = 0; r < (int)covered.size() && chosen < 0; ++r) {
            bool clash = false;
            for (int v : g.scope[s]) clash = clash || covered[r][v];
            if (!clash) chosen = r;
        }
        if (chosen < 0) {
            covered.emplace_back(g.num_vars, 0);
            chosen = (int)covered.size() - 1;
        }
        for (int v : g.scope[s]) covered[chosen][v] = 1;
        g.replica[s] = chosen;
    }
    g.num_replica = (int)covered.size();
    return true;
}

bool compile_plan(const RegionGraph& g, int K, int C, int family, int leaf_param, Plan& p, std::string& err) {
    p = Plan();
    p.K = K;
    p.C = C;
    p.family = family;
    // sufficient statistics per leaf entry (Sec. 3.4) and constants the kernels derive from them
    p.T = family == EINET_LEAF_GAUSSIAN ? 2 : (family == EINET_LEAF_CATEGORICAL ? leaf_param : 1);
    p.TD = family == EINET_LEAF_GAUSSIAN ? 3 : (family == EINET_LEAF_CATEGORICAL ? leaf_param : 2);
    p.leaf_param = family == EINET_LEAF_BINOMIAL || family == EINET_LEAF_CATEGORICAL ? leaf_param : 1;
    if (family == EINET_LEAF_BINOMIAL)
        for (int v = 0; v <= leaf_param; ++v) {
            const float lc = (float)(std::lgamma(leaf_param + 1.0) - std::lgamma(v + 1.0) - std::lgamma(leaf_param - v + 1.0));
            int32_t bits;
            std::memcpy(&bits, &lc, sizeof bits);
            p.leaf_logc.push_back(bits);
        }
    else
        p.leaf_logc.push_back(0);                      // log C(1, v) = 0
    const int nr = (int)g.scope.size(), np = (int)g.partition.size();
    auto kout = [&](int s) { return s == 0 ? 1 : K; };

    // ---- parameter layout
    int64_t off = 0;
    p.w_offset.resize(np);
    for (int n = 0; n < np; ++n) {
        p.w_offset[n] = off;
        off += int64_t(kout(g.partition[n][0])) * K * K;
    }
    p.v_offset.assign(nr, -1);
    for (int s = 0; s < nr; ++s)
        if (g.parts_of[s].size() > 1) {
            p.v_offset[s] = off;
            off += int64_t(kout(s)) * (int64_t)g.parts_of[s].size();
        }
    p.phi_offset = off;
    off += int64_t(g.num_vars) * C * g.num_replica * p.T * K;
    p.n_params = off;
    p.den_offset = off;
    p.tot_offset = p.den_offset + int64_t(g.num_vars) * g.num_replica * K;
    p.n_stats = p.tot_offset + int64_t(g.num_vars) * g.num_replica * K;
    if (p.n_stats >= (int64_t(1) << 31)) {
        err = "model too large: parameter offsets must fit in 31 bits";
        return false;
    }

    // ---- Algorithm 1: a sum enters the layer below the last of its parents.
    // pending[s] counts parent partitions not yet placed.
    std::vector<int> pending(nr, 0);
    for (auto& pt : g.partition) {
        pending[pt[1]]++;
        pending[pt[2]]++;
    }
    std::vector<std::vector<int>> sum_layers, prod_layers;   // top-down
    std::vector<int> frontier{0};
    int placed = 0;
    while (!frontier.empty()) {
        std::sort(frontier.begin(), frontier.end());
        std::vector<int> prods, next;
        for (int s : frontier)
            for (int n : g.parts_of[s]) prods.push_back(n);
        std::sort(prods.begin(), prods.end());
        for (int n : prods)
            for (int side = 1; side <= 2; ++side) {
                int c = g.partition[n][side];
                if (--pending[c] == 0 && !g.is_leaf(c)) next.push_back(c);
            }
        placed += (int)prods.size();
        sum_layers.push_back(frontier);
        prod_layers.push_back(prods);
        frontier.swap(next);
    }
    if (placed != np) {
        err = "structure is not a rooted graph of alternating sums and products";
        return false;
    }
    std::reverse(sum_layers.begin(), sum_layers.end());
    std::reverse(prod_layers.begin(), prod_layers.end());
    p.num_layers = (int)prod_layers.size();

    // ---- arena nodes: regions first, then one simple sum per partition of a multi-partition region
    std::vector<int> simple_node(np, -1);
    int nodes = nr;
    for (int n = 0; n < np; ++n)
        if (g.parts_of[g.partition[n][0]].size() > 1) simple_node[n] = nodes++;
    p.num_nodes = nodes;

    // ---- einsum items, bottom-up; remember each partition's item for the posterior slots
    std::vector<int> item_of(np, -1);
    p.ein_layer_ptr.push_back(0);
    p.layer_ptr.push_back(0);
    for (auto& layer : prod_layers) {
        for (int n : layer) {
            item_of[n] = (int)p.ein_left.size();
            int parent = g.partition[n][0];
            p.ein_left.push_back(g.partition[n][1]);
            p.ein_right.push_back(g.partition[n][2]);
            p.ein_out.push_back(simple_node[n] >= 0 ? simple_node[n] : parent);
            p.ein_reg.push_back(parent);
            p.ein_kout.push_back(kout(parent));
            p.ein_woff.push_back((int32_t)p.w_offset[n]);
            // mixing weight v[parent][k][c] of this partition sits at ein_voff + k * ein_vstr (App. B)
            const auto& sib = g.parts_of[parent];
            if (sib.size() > 1) {
                int c = int(std::find(sib.begin(), sib.end(), n) - sib.begin());
                p.ein_voff.push_back((int32_t)(p.v_offset[parent] + c));
                p.ein_vstr.push_back((int32_t)sib.size());
            } else {
                p.ein_voff.push_back(-1);
                p.ein_vstr.push_back(0);
            }
            p.layer_partition.push_back(n);
            p.ein_part.push_back(n);
        }
        bool full = true;
        for (size_t e = (size_t)p.ein_layer_ptr.back(); e < p.ein_kout.size(); ++e) full = full && p.ein_kout[e] == K;
        p.ein_layer_full.push_back(full ? 1 : 0);
        p.ein_layer_ptr.push_back((int32_t)p.ein_left.size());
        p.layer_ptr.push_back((int32_t)p.layer_partition.size());
    }

    // ---- mixing items per layer
    p.mix_layer_ptr.push_back(0);
    p.mix_cptr.push_back(0);
    for (auto& layer : sum_layers) {
        for (int s : layer) {
            if (g.parts_of[s].size() < 2) continue;
            p.mix_node.push_back(s);
            p.mix_kout.push_back(kout(s));
            p.mix_voff.push_back((int32_t)p.v_offset[s]);
            for (int n : g.parts_of[s]) p.mix_child.push_back(simple_node[n]);
            p.max_mix_children = std::max(p.max_mix_children, (int)g.parts_of[s].size());
            p.mix_cptr.push_back((int32_t)p.mix_child.size());
        }
        p.mix_layer_ptr.push_back((int32_t)p.mix_node.size());
    }

    // ---- one record per mixing item (see MIX_REC_INTS)
    p.mix_rec.assign(p.mix_node.size() * MIX_REC_INTS, -1);
    for (size_t i = 0; i < p.mix_node.size(); ++i) {
        int32_t* rec = p.mix_rec.data() + i * MIX_REC_INTS;
        const int nc = p.mix_cptr[i + 1] - p.mix_cptr[i];
        rec[0] = p.mix_node[i];
        rec[1] = p.mix_kout[i];
        rec[2] = p.mix_voff[i];
        rec[3] = nc;
        for (int c = 0; c < nc && c < MIX_REC_CHILDREN; ++c) rec[4 + c] = p.mix_child[p.mix_cptr[i] + c];
    }

    // ---- the root's partitions (see ROOT_REC_STRIDE): the items of the top einsum layer
    if (p.num_layers > 0) {
        const int e0 = p.ein_layer_ptr[p.num_layers - 1], e1 = p.ein_layer_ptr[p.num_layers];
        const auto& sib = g.parts_of[0];
        p.root_rec.assign(4 + (size_t)(e1 - e0) * ROOT_REC_STRIDE, 0);
        p.root_rec[0] = e1 - e0;
        p.root_rec[1] = 0;
        p.root_rec[2] = (int32_t)p.v_offset[0];
        for (int e = e0; e < e1; ++e) {
            int32_t* q = p.root_rec.data() + 4 + (size_t)(e - e0) * ROOT_REC_STRIDE;
            q[0] = e;
            q[1] = p.ein_left[e];
            q[2] = p.ein_right[e];
            q[3] = p.ein_out[e];
            q[4] = p.ein_woff[e];
            q[5] = int(std::find(sib.begin(), sib.end(), p.ein_part[e]) - sib.begin());
        }
    } else {
        p.root_rec.assign(4, 0);
    }

    // ---- sampling items: the sum regions layer by layer, each with the einsum items of its partitions
    {
        std::vector<int> mix_of(nr, -1);
        for (size_t i = 0; i < p.mix_node.size(); ++i) mix_of[p.mix_node[i]] = (int)i;
        p.sr_layer_ptr.push_back(0);
        p.sr_pptr.push_back(0);
        for (auto& layer : sum_layers) {
            for (int s : layer) {
                p.sr_node.push_back(s);
                p.sr_mix.push_back(mix_of[s]);
                for (int n : g.parts_of[s]) p.sr_item.push_back(item_of[n]);
                p.sr_pptr.push_back((int32_t)p.sr_item.size());
            }
            p.sr_layer_ptr.push_back((int32_t)p.sr_node.size());
        }
    }

    // ---- one record per sampling item (see SR_REC_INTS)
    p.sr_rec.assign(p.sr_node.size() * SR_REC_INTS, -1);
    for (size_t i = 0; i < p.sr_node.size(); ++i) {
        int32_t* rec = p.sr_rec.data() + i * SR_REC_INTS;
        const int np_i = p.sr_pptr[i + 1] - p.sr_pptr[i];
        rec[0] = p.sr_node[i];
        rec[1] = np_i;
        rec[2] = p.sr_mix[i] >= 0 ? p.mix_voff[p.sr_mix[i]] : -1;
        if (np_i > SR_REC_PARTS) continue;
        for (int c = 0; c < np_i; ++c) {
            const int e = p.sr_item[p.sr_pptr[i] + c];
            int32_t* q = rec + 4 + c * SR_REC_STRIDE;
            q[0] = e;
            q[1] = p.ein_left[e];
            q[2] = p.ein_right[e];
            q[3] = p.ein_woff[e];
            q[4] = p.ein_part[e];
            q[5] = p.ein_out[e] == p.sr_node[i] ? -1 : p.ein_out[e];
        }
    }

    // ---- leaves
    p.leaf_sptr.push_back(0);
    for (int s = 0; s < nr; ++s) {
        if (!g.is_leaf(s)) continue;
        int li = (int)p.leaf_node.size();
        p.leaf_node.push_back(s);
        p.leaf_replica.push_back(g.replica[s]);
        p.max_leaf_scope = std::max(p.max_leaf_scope, (int)g.scope[s].size());
        for (int v : g.scope[s]) {
            p.leaf_var.push_back(v);
            p.lv_leaf.push_back(li);
            p.lv_var.push_back(v);
        }
        p.leaf_sptr.push_back((int32_t)p.leaf_var.size());
    }

    // ---- top-down items: which posterior blocks flow into each region.  Item e owns blocks
    // e*nb .. e*nb+nb-1 of Gp: block 0 for its left child, blocks 1.. (one per workgroup of the top-down
    // einsum kernel) for its right child.
    const int nb = gp_blocks_per_item(K);
    std::vector<std::vector<std::pair<int, int>>> runs(nr);
    std::vector<int> layer_of_item(np, 0);
    for (int l = 0; l < p.num_layers; ++l)
        for (int e = p.ein_layer_ptr[l]; e < p.ein_layer_ptr[l + 1]; ++e) layer_of_item[e] = l;
    for (int n = 0; n < np; ++n) {
        const int e = item_of[n], l = layer_of_item[e];
        const int groups = bwd_blocks_of_item(p.ein_layer_ptr[l + 1] - p.ein_layer_ptr[l], K, p.ein_layer_full[l] != 0,
                                              e - p.ein_layer_ptr[l]);
        runs[g.partition[n][1]].push_back({e * nb, 1});
        runs[g.partition[n][2]].push_back({e * nb + 1, groups});
    }
    // ---- layers whose regions need no assembled posterior (see GSRC_MAX_BLOCKS)
    p.ein_gsrc.assign(np, 0);
    p.ein_layer_direct.assign(p.num_layers, 0);
    for (int l = 0; l + 1 < p.num_layers; ++l) {       // (the root's layer has a kernel of its own)
        bool all = !bwd_uses_split_kernel(K, p.ein_layer_full[l] != 0);
        for (int e = p.ein_layer_ptr[l]; e < p.ein_layer_ptr[l + 1]; ++e) {
            const int s = g.partition[p.ein_part[e]][0];
            if (g.parts_of[s].size() == 1 && runs[s].size() == 1 && runs[s][0].second <= GSRC_MAX_BLOCKS)
                p.ein_gsrc[e] = (runs[s][0].first << 3) | runs[s][0].second;
            else
                all = false;
        }
        p.ein_layer_direct[l] = all ? 1 : 0;
        if (!all)
            for (int e = p.ein_layer_ptr[l]; e < p.ein_layer_ptr[l + 1]; ++e) p.ein_gsrc[e] = 0;
    }
    // the same for the leaves (element-wise statistics kernels only: no categorical leaves, scopes below the 512
    // pairs from which the matrix-pipe kernel may be chosen)
    p.leaf_gsrc.assign(p.leaf_node.size(), 0);
    p.leaves_direct = family != EINET_LEAF_CATEGORICAL && p.max_leaf_scope * C < 512 && !p.leaf_node.empty();
    for (size_t i = 0; i < p.leaf_node.size() && p.leaves_direct; ++i) {
        const int s = p.leaf_node[i];
        if (runs[s].size() == 1 && runs[s][0].second <= GSRC_MAX_BLOCKS)
            p.leaf_gsrc[i] = (runs[s][0].first << 3) | runs[s][0].second;
        else
            p.leaves_direct = false;
    }
    if (!p.leaves_direct) p.leaf_gsrc.assign(p.leaf_node.size(), 0);
    p.rb_layer_ptr.push_back(0);
    p.rb_pptr.push_back(0);
    auto push_region = [&](int s) {
        p.rb_node.push_back(s);
        p.rb_kout.push_back(kout(s));
        std::sort(runs[s].begin(), runs[s].end());
        for (auto& r : runs[s])
            for (int q = 0; q < r.second; ++q) p.rb_pblk.push_back(r.first + q);
        p.rb_pptr.push_back((int32_t)p.rb_pblk.size());
    };
    for (int l = p.num_layers - 1; l >= 0; --l) {
        for (int s : sum_layers[l]) push_region(s);
        p.rb_layer_ptr.push_back((int32_t)p.rb_node.size());
    }
    for (int s : p.leaf_node) push_region(s);
    p.rb_layer_ptr.push_back((int32_t)p.rb_node.size());

    // ---- one record per top-down region (see RB_REC_INTS)
    p.rb_rec.assign(p.rb_node.size() * RB_REC_INTS, 0);
    for (size_t i = 0; i < p.rb_node.size(); ++i) {
        int32_t* rec = p.rb_rec.data() + i * RB_REC_INTS;
        const int cnt = p.rb_pptr[i + 1] - p.rb_pptr[i];
        rec[0] = p.rb_node[i];
        rec[1] = p.rb_kout[i];
        rec[2] = cnt;
        rec[3] = p.rb_pptr[i];
        for (int q = 0; q < cnt && q < RB_REC_BLOCKS; ++q) rec[4 + q] = p.rb_pblk[p.rb_pptr[i] + q];
    }

    // ---- M-step rows
    for (int n = 0; n < np; ++n)
        for (int k = 0; k < kout(g.partition[n][0]); ++k) {
            p.row_off.push_back((int32_t)(p.w_offset[n] + int64_t(k) * K * K));
            p.row_len.push_back(K * K);
        }
    p.n_weight_rows = (int)p.row_off.size();
    for (int s = 0; s < nr; ++s)
        if (p.v_offset[s] >= 0) {
            int c = (int)g.parts_of[s].size();
            for (int k = 0; k < kout(s); ++k) {
                p.row_off.push_back((int32_t)(p.v_offset[s] + int64_t(k) * c));
                p.row_len.push_back(c);
            }
        }

    // ---- ABI view
    p.scope_ptr.push_back(0);
    for (int s = 0; s < nr; ++s) {
        for (int v : g.scope[s]) p.scope_var.push_back(v);
        p.scope_ptr.push_back((int32_t)p.scope_var.size());
    }
    for (auto& pt : g.partition) {
        p.partition_flat.push_back(pt[0]);
        p.partition_flat.push_back(pt[1]);
        p.partition_flat.push_back(pt[2]);
    }
    return true;
}

}  // namespace einet_impl
