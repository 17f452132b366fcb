// Launchers of the HIP kernels (device code: leaf_forward, einsum_forward, einsum_backward, statistics, update and
// sampling .hip).  All pointers
// are device pointers; every launcher only enqueues work on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "../../include/einet.h"

namespace einet_impl {

// Index tables of the plan: one int32 vector each on the host (Plan) and one
// pointer each into the bound workspace on the device (DevTables).  leaf_logc holds
// the float32 bit patterns of log C(N, v), v = 0..N, for binomial leaves.
#define EINET_TABLES(X)                                                                                    \
    X(ein_left) X(ein_right) X(ein_out) X(ein_reg) X(ein_kout) X(ein_woff) X(ein_voff) X(ein_vstr) X(ein_part) \
    X(ein_gsrc) X(leaf_gsrc)                                                                               \
    X(mix_node) X(mix_kout) X(mix_cptr) X(mix_child) X(mix_voff) X(mix_rec)                                \
    X(leaf_node) X(leaf_replica) X(leaf_sptr) X(leaf_var) X(lv_leaf) X(lv_var)                             \
    X(rb_node) X(rb_kout) X(rb_pptr) X(rb_pblk) X(row_off) X(row_len) X(leaf_logc)                         \
    X(sr_node) X(sr_pptr) X(sr_item) X(sr_mix) X(rb_rec) X(sr_rec) X(root_rec)

struct DevTables {
#define X(name) const int32_t* name;
    EINET_TABLES(X)
#undef X
};

struct Dims {
    int B, D, C, R, K, T, TD, family;
    int P;   // leaf parameter: trials of a binomial leaf (1 for Bernoulli), values of a categorical leaf
};

void launch_leaf_derive(const float* phi, float* theta, const Dims& d, hipStream_t s);
// A [node][B][K] float32 holds residuals, Off [node][B] float64 the offsets: log-density = Off + A
void launch_leaf_forward(const DevTables& t, int n_leaves, int max_scope, const float* x, const uint8_t* mask,
                         int mask_mode, const float* theta, float* A, double* Off, const Dims& d, hipStream_t s);
// logp (may be NULL): the launch that produces the root value also writes it there.  full_k: every item of the
// launch has K output entries (all layers but the root's).
void launch_einsum_forward(const DevTables& t, int first, int count, bool full_k, const float* params, float* A,
                           double* Off, float* amax, float* logp, const Dims& d, hipStream_t s);
// A mixing item with at most MIX_REC_CHILDREN partitions also has a record of MIX_REC_INTS ints in mix_rec:
// node, entries, offset of its weights, number of partitions, then the nodes of the partitions.  The kernel gets
// all of it with one request instead of walking three tables one after the other.
constexpr int MIX_REC_CHILDREN = 8, MIX_REC_INTS = 16;
// max_children: the largest number of partitions of a region of these items
void launch_mixing_forward(const DevTables& t, int first, int count, int max_children, const float* params, float* A,
                           double* Off, float* logp, const Dims& d, hipStream_t s);

// The top of the circuit in one launch each way.  The top einsum layer holds exactly the partitions of the root (a
// single output entry each); root_rec lists them: number of partitions, the root's node, the offset of its mixing
// weights (-1: one partition), unused, then ROOT_REC_STRIDE ints per partition: einsum item, left node, right node,
// node of the partition's own output (the root's node when it is the only one), offset of W, position among the
// root's mixing weights.
constexpr int ROOT_REC_STRIDE = 6;
// Row stride (floats) of the LDS copies of these kernels: a multiple of 4 whose quarter is odd, so that 16-byte reads
// of eight consecutive rows fall into different banks.
#if defined(__HIPCC__)
__host__ __device__
#endif
inline int root_row_stride(int K) {
    const int k4 = (K + 3) & ~3;
    return ((k4 >> 2) & 1) ? k4 : k4 + 4;
}
// LDS of the bottom-up kernel: per wave a copy of W [K][stride] and of eR [samples][stride], then offset (float64) and
// residual of every partition for the workgroup's samples, and the mixing weight of every partition.
constexpr int ROOT_FWD_WAVES = 8, ROOT_FWD_SAMPLES = 4;
inline size_t root_forward_lds_bytes(int K, int n_partitions) {
    const size_t ks = (size_t)root_row_stride(K);
    return sizeof(float) * ROOT_FWD_WAVES * (K * ks + ROOT_FWD_SAMPLES * ks) +
           (sizeof(double) + sizeof(float)) * (size_t)n_partitions * ROOT_FWD_SAMPLES + sizeof(float) * (size_t)n_partitions;
}
// The kernel serves the top layer whenever it fits the 160 KB of LDS of a compute unit (a few
// hundred partitions at K = 64); beyond that the general einsum and mixing kernels run.
inline bool root_kernels_apply(int n_partitions, int K) {
    return n_partitions > 0 && root_forward_lds_bytes(K, n_partitions) <= 160 * 1024;
}
// Bottom-up: S~, shifts and offsets of every partition (Eq. 3-5), then the root's mixture (App. B) and log P.
void launch_root_forward(const DevTables& t, int n_partitions, const float* params, float* A, double* Off, float* amax,
                         float* logp, const Dims& d, hipStream_t s);
struct PartialSumList;   // sums of statistics blocks left for the end of a top-down pass (below)
// Top-down: weight statistics (Eq. 6) and child posteriors of the root's partitions; the root's posterior is 1 and its
// mixing step is folded in.  Writes the posterior blocks that launch_einsum_backward writes for a layer of
// n_partitions items with one output entry each (bwd_groups_per_item workgroups and right-child blocks per item).
// e_woff: the weight offsets of the layer's items in order (for the sum of the virtual items' blocks); part, jobs as
// for launch_einsum_backward (root_bwd_partial_bound floats), or null.
void launch_root_backward(const DevTables& t, int n_partitions, const int32_t* e_woff, float* part, PartialSumList* jobs,
                          bool accumulate, const float* params, float* stats,
                          const float* A, const double* Off, const float* amax, float* Gp, const Dims& d, hipStream_t s);

// Every top-down region also has a record of RB_REC_INTS ints in rb_rec: node, entries, number of parent blocks,
// position of its list in rb_pblk, then the first RB_REC_BLOCKS block numbers (the rest, if any, only in the list).
constexpr int RB_REC_INTS = 32, RB_REC_BLOCKS = 28;
void launch_region_assemble(const DevTables& t, int first, int count, bool is_root_layer, float* G, const float* Gp,
                            const Dims& d, hipStream_t s);
// accumulate = false: the weight statistics of these items are known to be zero and are overwritten.
// direct: the posterior of every item's region is not in G; the kernel adds up the parent's blocks itself, as
// ein_gsrc says (only layers with Plan::ein_layer_direct set; then no launch_region_assemble for their regions).
// full_k: every item of the launch has K output entries (all layers but the root's).
// part: bwd_partial_bound floats of scratch for the blocks of virtual items, or null (then the chunks of an item are
// always walked in turn); with virtual items the sum of the blocks is appended to *jobs, not launched.
void launch_einsum_backward(const DevTables& t, int first, int count, bool full_k, bool accumulate,
                            const float* params, float* stats, const float* A, const double* Off, const float* amax,
                            const float* G, float* Gp, float* part, PartialSumList* jobs, bool direct, const Dims& d,
                            hipStream_t s);
// A region with one partition and one parent partition (every inner region of a random binary tree) has its
// posterior in at most GSRC_MAX_BLOCKS consecutive blocks of Gp, written by that parent.  The top-down einsum kernel
// of its partition can add them up while it stages its operands, which saves the launch that would assemble G for
// the layer.  ein_gsrc[item] = (first block << 3) | number of blocks, 0 when the region does not qualify.
constexpr int GSRC_MAX_BLOCKS = 6;
// posterior blocks ([B][K] floats each) reserved per einsum item in Gp: one for its left child, then up to
// one per slice of four left entries for its right child
inline int gp_blocks_per_item(int K) { return 1 + (K + 3) / 4; }
// Workgroups per item of the top-down einsum kernel for a layer of `count` items: the slices of an item are
// spread over as many workgroups as keeps the launch within one round of the 256 compute units of the
// MI355X (one workgroup per unit).  Workgroup grp takes slices grp*KQ/groups .. (grp+1)*KQ/groups - 1 and
// writes right-child block 1+grp of the item.
inline int bwd_groups_per_item(int count, int K) {
    const int kq = (K + 3) / 4;
    const int g = 256 / (count > 0 ? count : 1);
    return g < 1 ? 1 : (g > kq ? kq : g);
}
// Layers whose items all have K output entries, K a multiple of 8 up to 40, take the top-down kernel with
// specialised waves: one workgroup per compute unit, the layer's count * K/4 (item, slice) pairs split evenly
// over the workgroups in order, so that a workgroup's pairs touch one or two items.  Workgroup g owns the pairs
// g * P / G .. (g + 1) * P / G - 1 and writes right-child block 1 + (g - first workgroup of the item).
inline bool bwd_uses_split_kernel(int K, bool full_k) { return full_k && (K & 7) == 0 && K <= 40; }
inline int bwd_split_grid(int count, int K) {
    const int pairs = count * (K / 4);
    return pairs < 256 ? pairs : 256;
}
// A layer of so few items that its pairs leave more than half of the compute units idle, with a batch of several
// chunks of 128 samples: every item is launched as this many virtual items, each with a share of the chunks, one
// workgroup per (virtual item, slice), at most 256 in all.  The virtual items of an item write their statistics to
// blocks of their own (bwd_partial_bound floats together), which a later launch adds up in a fixed order.
// That launch costs about 4 us (one for all layers of a pass), so the split is taken only where the chunks a workgroup
// no longer walks are worth twice that: a workgroup spends roughly bwd_unit_us(K) on one chunk of one slice (10 us at K = 40, measured; the
// work grows with K^2), half of that in the root's layer.
constexpr float BWD_SPLIT_PAYS_US = 8.f;
inline float bwd_unit_us(int K) { return 1.f + 9.f * (float)(K * K) / 1600.f; }
inline int bwd_virtual_items(int count, int K, int B) {
    const int pairs = count * (K / 4), nchunks = (B + 127) / 128;
    if (pairs <= 0 || pairs > 128 || nchunks < 2) return 1;
    int v = 256 / pairs;
    if (v > nchunks) v = nchunks;
    const int cpv = (nchunks + v - 1) / v;
    if ((float)(nchunks - cpv) * bwd_unit_us(K) < BWD_SPLIT_PAYS_US) return 1;
    return (nchunks + cpv - 1) / cpv;
}
// The sums of the blocks are not needed before the M-step, so the launches of a top-down pass only note them down
// and one launch at the end of the pass does them all: per job,
//   stats[e_woff[item] + r] (+)= sum over v < vper of part[(v * count + item) * block + r], r < block.
constexpr int PARTIAL_SUM_JOBS = 8;
struct PartialSumJob {
    const int32_t* e_woff;
    const float* part;
    int count, vper, block;
};
struct PartialSumList {
    int n = 0;
    PartialSumJob job[PARTIAL_SUM_JOBS];
};
void launch_sum_partial_stats(const PartialSumList& jobs, float* stats, bool accumulate, hipStream_t s);
// floats of scratch that a layer's launch needs for its blocks with any batch up to max_B (0: never virtual items)
inline size_t bwd_partial_bound(int count, int K, int max_B, bool full_k);
inline size_t root_bwd_partial_bound(int n_partitions, int K, int max_B);
// The same for the root's layer (n_partitions items of K^2 weights, bwd_groups_per_item workgroups each): shares of
// the chunks of 128 samples per workgroup when the launch would leave half of the compute units idle.
inline int root_bwd_virtual_items(int n_partitions, int K, int B) {
    const int groups = bwd_groups_per_item(n_partitions, K), wgs = n_partitions * groups, nchunks = (B + 127) / 128;
    if (wgs <= 0 || wgs > 128 || nchunks < 2) return 1;
    int v = 256 / wgs;
    if (v > nchunks) v = nchunks;
    const int cpv = (nchunks + v - 1) / v;
    const int slices = ((K + 3) / 4 + groups - 1) / groups;      // per workgroup
    if ((float)((nchunks - cpv) * slices) * 0.5f * bwd_unit_us(K) < BWD_SPLIT_PAYS_US) return 1;
    return (nchunks + cpv - 1) / cpv;
}
// workgroup that owns pair x of P pairs split over G workgroups
#if defined(__HIPCC__)
__host__ __device__
#endif
inline int bwds_wg_of_pair(long long x, long long P, long long G) { return (int)(((x + 1) * G - 1) / P); }
// right-child blocks that item li of a layer of `count` items writes (the workgroups that touch it)
inline int bwd_blocks_of_item(int count, int K, bool full_k, int li) {
    if (!bwd_uses_split_kernel(K, full_k)) return bwd_groups_per_item(count, K);
    const long long ns = K / 4, P = (long long)count * ns, G = bwd_split_grid(count, K);
    return bwds_wg_of_pair((li + 1) * ns - 1, P, G) - bwds_wg_of_pair(li * ns, P, G) + 1;
}
inline size_t bwd_partial_bound(int count, int K, int max_B, bool full_k) {
    const int pairs = count * (K / 4), nchunks = (max_B + 127) / 128;
    if (!bwd_uses_split_kernel(K, full_k) || pairs <= 0 || pairs > 128 || nchunks < 2) return 0;
    const int v = 256 / pairs < nchunks ? 256 / pairs : nchunks;
    return (size_t)v * count * K * K * K;
}
inline size_t root_bwd_partial_bound(int n_partitions, int K, int max_B) {
    const int wgs = n_partitions * bwd_groups_per_item(n_partitions, K), nchunks = (max_B + 127) / 128;
    if (wgs <= 0 || wgs > 128 || nchunks < 2) return 0;
    const int v = 256 / wgs < nchunks ? 256 / wgs : nchunks;
    return (size_t)v * n_partitions * K * K;
}
// Leaf statistics on the matrix pipe (nothing marginalised, scopes of at least 512 (variable, channel) pairs): with
// so few leaves that the workgroups of the launch (one per leaf and 64 or 128 pairs) leave half of the compute units
// idle, the batch is split into this many groups of passes of 64 samples (at least two passes each), every group
// with workgroups of its own that write to a block of their own; a second launch adds the blocks to the statistics.
inline int leaf_stats_pairs_per_group(int K) { return K > 32 ? 64 : 128; }
// (most groups any batch of up to B samples is split into)
inline int leaf_stats_groups_max(int n_leaves, int max_scope, int C, int K, int B) {
    const int pc = leaf_stats_pairs_per_group(K), wgs = n_leaves * ((max_scope * C + pc - 1) / pc), passes = (B + 63) / 64;
    if (max_scope * C < 512 || wgs > 128 || passes < 4) return 1;
    const int v = 256 / wgs;
    return v > passes / 2 ? passes / 2 : v;
}
inline int leaf_stats_groups(int n_leaves, int max_scope, int C, int K, int B) {
    const int v = leaf_stats_groups_max(n_leaves, max_scope, C, K, B), passes = (B + 63) / 64;
    if (v <= 1) return 1;
    const int ppv = (passes + v - 1) / v;
    return (passes + ppv - 1) / ppv;
}
// leaf statistics and mixing statistics (independent of each other) in one launch
// part: part_floats floats of scratch for the blocks of the batch groups above, or null; n_stats: length of stats.
// direct: the leaves' posteriors are not in G; the element-wise forms of the leaf statistics add up the parents'
// blocks of Gp themselves, as leaf_gsrc says (only with Plan::leaves_direct, which also keeps the scopes below the
// 512 pairs from which the matrix-pipe form, which reads G, can be chosen).
void launch_tail_backward(const DevTables& t, int n_lv, int n_leaves, int max_scope, int n_mix, int max_children,
                          const float* x, const uint8_t* mask, int mask_mode, const float* params, const float* A,
                          const double* Off, const float* G, const float* Gp, bool direct, float* stats,
                          int64_t phi_off, int64_t den_off, int64_t tot_off, int64_t n_stats, float* part,
                          size_t part_floats, const Dims& d, hipStream_t s);
// the whole M-step in one launch; the statistics of the first n_lazy_rows weight rows are left as they
// are (the next E-step overwrites them); when no E-step has run since they were last consumed
// (lazy_rows_are_zero) those rows count as zero and their weights are kept
void launch_em_update(const DevTables& t, int n_rows, int n_lazy_rows, bool lazy_rows_are_zero, float* params,
                      float* stats, float* theta,
                      int64_t phi_off, int64_t den_off, int64_t tot_off, float step, float min_var, float max_var,
                      float w_floor, const Dims& d, hipStream_t s);
void launch_fill(float* p, float value, int64_t n, hipStream_t s);
void launch_init_params(const DevTables& t, int n_rows, float* params, int64_t phi_off, uint64_t seed, float lo,
                        float hi, const Dims& d, hipStream_t s);

// ---- top-down sampling.  sel[node][B] (int32) holds the entry each sample uses at a node, -1 where the
// sample does not visit it.  u [num_partitions + num_regions][B]: the uniforms of the choices.
// evidence = false: no forward pass has run, the choices follow the weights alone.
void launch_sample_init(int32_t* sel, int num_nodes, int B, hipStream_t s);
// A sampling item (sum region) with at most SR_REC_PARTS partitions also has a record of SR_REC_INTS ints in
// sr_rec: node, number of partitions, offset of its mixing weights (-1: one partition), unused, then per partition
// SR_REC_STRIDE ints: einsum item, left node, right node, offset of W, partition number, node of the partition's
// own output (-1: the region itself), unused.  Regions with more partitions have nparts only (the kernel then walks
// the tables).
constexpr int SR_REC_INTS = 64, SR_REC_PARTS = 8, SR_REC_STRIDE = 7;
// One launch per sum layer: for every region of the layer that a sample reaches, the choice of a partition
// (regions with several) and then of a pair of child entries.  Items first .. first+count-1 of the sr_* tables.
void launch_sample_regions(const DevTables& t, int first, int count, bool evidence, const float* params,
                           const float* A, const double* Off, const float* amax, const float* u, int num_partitions,
                           int32_t* sel, const Dims& d, hipStream_t s);
void launch_sample_leaves(const DevTables& t, int n_lv, const float* x, const uint8_t* mask, int mask_mode,
                          const float* phi, const float* noise, const int32_t* sel, float* out, const Dims& d,
                          hipStream_t s);
// Device address, on the current device, of the library's fixed arena of EINET_STATIC_SCRATCH_BYTES bytes
// (256-byte aligned).  No allocation: the arena is part of the loaded code object.
hipError_t static_scratch_address(void** ptr);

// Streaming-copy rate (GB/s, read + written) and register-resident fp32 MFMA rates (TFLOP/s: 32x32x2; 16x16x4 with one
// and with four waves per SIMD) of the current device, best of `reps` launches each; dst also receives the loops'
// results (it needs at least EINET_PEAKS_MIN_BYTES bytes).
hipError_t measure_peaks(const void* src, void* dst, size_t bytes, int reps, double* out, hipStream_t s);

void launch_mixture_logp(const float* lp, const float* log_coef, int n_components, int B, float* out, hipStream_t s);

}  // namespace einet_impl
