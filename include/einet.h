/*
 * einet.h - C ABI of libeinet: Einsum Networks (arxiv 2004.06231) on one MI355X.
 *
 * The library evaluates a vectorised probabilistic circuit layer by layer in
 * the log domain (Sec. 3.2-3.4 of the paper) and accumulates the expected
 * sufficient statistics of EM (Sec. 3.5).  Every step runs in hand-written
 * HIP kernels for gfx950; the library allocates no device memory: the caller
 * asks for the sizes, allocates, and binds the buffers.
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP
 *     device memory on the current device; the comment of every argument
 *     says which.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Compute calls only enqueue work on it and return; they never
 *     synchronise.  Calls on one handle must be issued in order on one
 *     stream (they share the handle's workspace).
 *   - Every function returning int returns EINET_OK (0) or a negative
 *     EINET_ERR_* code; nothing throws or aborts across the boundary.
 *     einet_last_error() gives a human-readable reason.
 *   - Vector length: every region holds K entries, except the root region,
 *     which holds one (K_out = 1).
 *
 * Structure numbering (fixed so that an independent implementation builds the
 * identical graph from the same arguments):
 *   Random binary trees (Sec. 4.1): region 0 is the root over variables
 *   0..D-1.  Replica r is a complete binary tree of split depth `depth`; its
 *   node with heap index h (root 1, children 2h, 2h+1), h >= 2, is region
 *   1 + r*(2^(depth+1)-2) + (h-2); the split of heap node h < 2^depth is
 *   partition r*(2^depth-1) + (h-1).  A scope (sorted ascending, n entries) is
 *   shuffled by Fisher-Yates, t = n-1..1: swap a[t], a[u mod (t+1)], u drawn
 *   from SplitMix64 started at state seed ^ (0xD1B54A32D192ED03*(r+1)) ^
 *   (0x8CB92BA72F3D8DD7*h) (64-bit wrap); the first n/2 entries (sorted) form
 *   the left child, the others the right child.  Leaves of replica r use leaf
 *   parameter replica r.
 *   Poon-Domingos (Sec. 4.2): variable y*width + x is pixel (y, x); regions
 *   are rectangles, region 0 the image; rectangles are processed in creation
 *   order; the step of a rectangle is the first entry of `deltas` that cuts
 *   it on an allowed axis; cuts along y (ascending) come before cuts along x;
 *   each cut is one partition (top or left part = left child); a rectangle
 *   gets the next region number when first seen (left before right).  Leaf
 *   regions take, in region order, the smallest replica index whose earlier
 *   leaves do not overlap them (Sec. 3.4).
 *
 * Flat parameter buffer (float32, n_params entries), in this order:
 *   W   for each partition n in order: [K_out(parent)][K][K], last index (the
 *       right child's entry j) fastest; non-negative, each [K][K] block sums
 *       to one (Eq. 2)
 *   v   for each region with C_s > 1 partitions, in region order:
 *       [K_out][C_s] mixing weights, private per entry k (App. B)
 *   phi [D][channels][R][T][K] expectation parameters of the leaves
 *       (Sec. 3.4): Bernoulli T=1: p; Gaussian T=2: (E[x], E[x^2]); binomial
 *       with N = leaf_param trials T=1: E[x] = N p, x in {0..N}; categorical
 *       over V = leaf_param values T=V: the probabilities, x in {0..V-1}
 *       (discrete values are passed as float32 like all data)
 * Flat statistics buffer (float32, n_stats entries):
 *   Nw, Nv, num with the shapes of W, v, phi, then den [D][R][K] and
 *   tot [D][R][K]  (posterior mass of a leaf entry over observed samples /
 *   over all samples).
 */
#ifndef EINET_H
#define EINET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct einet einet_t;

enum {
    EINET_OK = 0,
    EINET_ERR_INVALID_ARG = -1,
    EINET_ERR_BAD_STRUCTURE = -2,
    EINET_ERR_NOT_BOUND = -3,
    EINET_ERR_BATCH_TOO_LARGE = -4,
    EINET_ERR_HIP = -5
};

enum { EINET_STRUCTURE_RAT = 0, EINET_STRUCTURE_PD = 1 };
enum { EINET_LEAF_BERNOULLI = 0, EINET_LEAF_GAUSSIAN = 1, EINET_LEAF_BINOMIAL = 2, EINET_LEAF_CATEGORICAL = 3 };
enum { EINET_MASK_NONE = 0, EINET_MASK_SHARED = 1, EINET_MASK_PER_SAMPLE = 2 };
enum { EINET_AXIS_Y = 1, EINET_AXIS_X = 2 };
#define EINET_MAX_DELTAS 8

/* Description of a model; plain data, read only during einet_create. */
typedef struct einet_spec {
    int32_t structure;     /* EINET_STRUCTURE_* */
    int32_t K;             /* entries per sum / leaf vector (Sec. 3.1), 1..64 */
    int32_t channels;      /* values per variable; the leaf factorises over them (Sec. 4.2) */
    int32_t leaf_family;   /* EINET_LEAF_* */
    int32_t max_batch;     /* largest B any later call will pass */
    /* random binary trees */
    int32_t num_vars;      /* D */
    int32_t depth;         /* split depth, 2^depth leaves per replica */
    int32_t num_replica;   /* R trees mixed at the root */
    uint64_t seed;
    /* Poon-Domingos */
    int32_t height, width;
    int32_t num_deltas;    /* 1..EINET_MAX_DELTAS */
    int32_t deltas[EINET_MAX_DELTAS];
    int32_t axes;          /* EINET_AXIS_Y | EINET_AXIS_X; X alone = vertical cuts only */
    /* leaves */
    int32_t leaf_param;    /* binomial: trials N, 1..4095; categorical: values V, 2..256; else ignored */
} einet_spec;

/* Read-only view of the compiled structure; all pointers are host memory
 * owned by the handle and valid until einet_destroy. */
typedef struct einet_structure_view {
    int32_t num_vars, num_regions, num_partitions, num_replica;
    int32_t num_layers;               /* einsum layers (= product layers of Algorithm 1) */
    int32_t K, channels, num_suff_stats;
    const int32_t* scope_ptr;         /* [num_regions+1] CSR into scope_var */
    const int32_t* scope_var;         /* variables of each region, ascending */
    const int32_t* region_replica;    /* [num_regions] replica of a leaf region, -1 otherwise */
    const int32_t* partition;         /* [num_partitions][3] = parent region, left region, right region */
    const int32_t* layer_ptr;         /* [num_layers+1] CSR into layer_partition, bottom layer first */
    const int32_t* layer_partition;   /* partitions of each einsum layer, ascending */
    const int64_t* w_offset;          /* [num_partitions] offset (floats) of W[n] in the parameter buffer */
    const int64_t* v_offset;          /* [num_regions] offset of v[s], -1 if the region has < 2 partitions */
    int64_t phi_offset;               /* offset of phi in the parameter buffer (= of num in the statistics) */
    int64_t den_offset, tot_offset;   /* offsets in the statistics buffer */
} einet_structure_view;

/* Builds the region graph (Sec. 3.1; generators of Sec. 4.1 / 4.2), assigns
 * leaf replicas (Sec. 3.4), orders it in topological layers (Algorithm 1) and
 * splits sums with several children into simple sums plus a mixing layer
 * (App. B).  Host work only.  spec: host.  *out receives a handle owned by the
 * library (release with einet_destroy).  Errors: EINET_ERR_INVALID_ARG for
 * out-of-range fields, EINET_ERR_BAD_STRUCTURE when the structure cannot be
 * built (a one-variable scope would have to split; no delta cuts the image). */
int einet_create(const einet_spec* spec, einet_t** out);

/* Frees the handle and its host tables.  Never touches caller buffers. */
void einet_destroy(einet_t* h);

/* Reason of the last error on this handle (or of the last failed
 * einet_create when h is NULL).  Host string owned by the library. */
const char* einet_last_error(const einet_t* h);

/* Sizes the caller must allocate on the device: n_params and n_stats in
 * float32 elements, workspace in bytes (index tables, derived leaf constants,
 * activation arena with its per-sample offsets and posterior arenas for
 * max_batch samples and, for models with so few einsum items or leaves that
 * the chunks of a large batch are processed side by side, blocks for their
 * partial statistics).  All outputs: host. */
int einet_sizes(const einet_t* h, size_t* n_params, size_t* n_stats, size_t* workspace_bytes);

/* Fills *view (host) with pointers into the handle's host tables. */
int einet_structure(const einet_t* h, einet_structure_view* view);

/* Registers the caller's device buffers (params: n_params floats, stats:
 * n_stats floats, both 16-byte aligned: the kernels read whole groups of four
 * weights; workspace: workspace_bytes, 256-byte aligned; a misaligned buffer is
 * EINET_ERR_INVALID_ARG) and uploads
 * the index tables into the workspace on `stream`, synchronising once.  The
 * buffers stay owned by the caller and must outlive every later call.  The
 * parameter buffer may be uninitialised at this point; call einet_refresh
 * after writing it.  The statistics buffer is taken as it is (statistics to be
 * continued), with one exception: binding again the very buffer that an
 * einet_em_update on this handle has consumed keeps it logically zero.  A copy
 * of such a buffer holds unspecified einsum-weight statistics (see
 * einet_em_update): call einet_em_reset after binding it. */
int einet_bind(einet_t* h, float* params_dev, float* stats_dev, void* workspace_dev, void* stream);

/* Recomputes what the kernels derive from the parameters (per leaf entry:
 * log p, log(1-p), or mean, -1/(2 var), -log(2 pi var)/2, or the logarithms
 * of a categorical table; Sec. 3.4) after the caller has written the parameter
 * buffer.  einet_em_update and einet_init_params do it themselves. */
int einet_refresh(einet_t* h, void* stream);

/* Random initial parameters, written into the bound parameter buffer (the
 * paper prescribes no initialisation; this is the customary one): every weight
 * row (the K*K weights of a sum entry, the C_s mixing weights of an entry) is a
 * draw from the flat Dirichlet distribution, formed as normalised unit
 * exponentials e = -log u; Bernoulli p, Gaussian mean and binomial E[x]/N are
 * leaf_lo + (leaf_hi - leaf_lo) u, Gaussian variance 1; categorical tables as
 * the weight rows.  u of the parameter at position p of the flat buffer is
 * (top 23 bits of output p+1 of the SplitMix64 stream started at `seed`, plus
 * 1/2) / 2^23, so an independent implementation reproduces the numbers.  Also
 * refreshes the derived leaf constants.  Errors: EINET_ERR_NOT_BOUND,
 * EINET_ERR_INVALID_ARG (leaf_lo > leaf_hi; probabilities outside (0,1)). */
int einet_init_params(einet_t* h, uint64_t seed, float leaf_lo, float leaf_hi, void* stream);

/* log P(x) per sample: leaf layer (Sec. 3.4), einsum layers with the
 * log-einsum-exp stabilisation (Eq. 4-5), mixing layers (App. B).
 *   x_dev     device, [B][D][channels] float32 (Bernoulli: 0.0 / 1.0)
 *   mask_dev  device uint8, 1 = observed, 0 = integrated out (a marginalised
 *             variable's leaf factor is 1; Sec. 2): NULL with EINET_MASK_NONE,
 *             [D] with EINET_MASK_SHARED, [B][D] with EINET_MASK_PER_SAMPLE
 *   logp_dev  device, [B] float32, written
 * The conditional of Eq. 1 is einet_logp(mask = q|e) - einet_logp(mask = e).
 * Errors: EINET_ERR_NOT_BOUND, EINET_ERR_BATCH_TOO_LARGE (B > max_batch),
 * EINET_ERR_INVALID_ARG (B < 1, bad mask_mode, NULL pointers), EINET_ERR_HIP. */
int einet_logp(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B,
               float* logp_dev, void* stream);

/* einet_logp for callers that cannot allocate device memory for a batch (code
 * under HIP graph capture, serving loops, harnesses that forbid hipMalloc):
 * same arguments, same kernels and the same result as einet_logp, but the
 * activations of the forward pass (the per-node log-densities, their
 * per-sample offsets and the shifts of Eq. 4) live in an arena of
 * EINET_STATIC_SCRATCH_BYTES bytes that is part of the library's code object
 * on every GPU, not in the bound workspace.  The call allocates nothing and
 * frees nothing.  The handle must be bound (parameters, index tables and
 * derived leaf constants are read from the caller's buffers); besides
 * B <= max_batch the batch is limited by the arena:
 *   4*nodes*B*K + 8*nodes*B + 8*partitions*B bytes, each term rounded up to
 *   a multiple of 256 (nodes = regions + one per partition of a region with
 *   several),
 * must fit, else EINET_ERR_BATCH_TOO_LARGE and nothing is launched.  All calls on one
 * GPU, from any handle, share that GPU's arena: calls that overlap in time on
 * one GPU (different streams or threads) race; calls on one stream are safe.
 * Nothing in the arena has to be zero at entry; its contents after the call are
 * unspecified.  einet_em_accumulate and einet_sample do not use it. */
#define EINET_STATIC_SCRATCH_BYTES (16u << 20)
int einet_logp_static(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B,
                      float* logp_dev, void* stream);

/* E-step on one batch (Eq. 6): forward pass as einet_logp, then the top-down
 * pass that yields n = w * dlogP/dw for every sum weight and the posterior
 * p = dlogP/dlogL of every leaf entry, summed over the batch and ADDED to the
 * bound statistics buffer (p*T(x) into num, p over observed samples into den,
 * p over all samples into tot).  Batch reductions use no atomics: results are
 * bit-reproducible.  logp_dev may be NULL. */
int einet_em_accumulate(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int B,
                        float* logp_dev, void* stream);

/* M-step (Eq. 7) blended with step size `step` in (0,1] (Eq. 8-9):
 *   weights: hat = Nw / sum_ij Nw per (n,k) (kept if the sum is 0), floored at
 *            w_floor and renormalised, w <- (1-step) w + step hat; v likewise;
 *   leaves : hat = (num + (tot-den) phi) / tot (kept if tot is 0; equals
 *            num/den when nothing was masked), phi <- (1-step) phi + step hat;
 *            Bernoulli p clipped to [1e-6, 1-1e-6] (binomial: E[x]/N);
 *            categorical probabilities raised to at least 1e-6 and
 *            renormalised; Gaussian variance E[x^2]-E[x]^2 projected to
 *            [min_var, max_var] (Sec. 4.2).
 * Afterwards the statistics are zero for every later call: the mixing and leaf
 * statistics are cleared in memory; the einsum-weight statistics Nw are left
 * as they are and the next einet_em_accumulate overwrites them instead of
 * adding (saves one pass over the largest buffer), so the Nw part of the
 * caller's buffer is unspecified between this call and that one (a second
 * einet_em_update in that interval keeps the einsum weights, as for zero
 * statistics); use einet_em_reset to have zeros in memory.  Also refreshes the
 * derived leaf constants. */
int einet_em_update(einet_t* h, float step, float min_var, float max_var, float w_floor, void* stream);

/* Zeroes the whole statistics buffer in memory. */
int einet_em_reset(einet_t* h, void* stream);

/* Stochastic EM over one pass of the data (Eq. 8-9 with the schedule of
 * Sec. 4.2): the N samples are visited in consecutive mini-batches of `batch`
 * samples (the last one may be shorter); for each, einet_em_accumulate on that
 * slice followed by einet_em_update(step, min_var, max_var, w_floor).  The
 * result is exactly that of making those calls one by one; the loop runs in
 * the library, enqueues everything on `stream` and never synchronises.
 *   x_dev     device, [N][D][C] float32
 *   mask_dev  device, as in einet_logp; EINET_MASK_PER_SAMPLE: [N][D]
 *   batch     1 <= batch <= max_batch
 *   logp_dev  device, [N] float32 or NULL: log-density of every sample under
 *             the parameters in force when its mini-batch was visited
 * Statistics present in the buffer at entry are consumed by the first update;
 * the buffer is logically zero on return.  Errors as einet_em_accumulate and
 * einet_em_update, plus EINET_ERR_INVALID_ARG for N < 1. */
int einet_em_epoch(einet_t* h, const float* x_dev, const uint8_t* mask_dev, int mask_mode, int64_t N, int batch,
                   float step, float min_var, float max_var, float w_floor, float* logp_dev, void* stream);

/* Top-down sampling (Sec. 2: the latent-variable reading of a smooth and
 * decomposable circuit; Sec. 4.2: samples and inpainting; App. D: leaf means).
 * Starting from the root entry, a region with several partitions chooses one
 * with probability v[k][c] S^c[k] / S[k], a partition chooses the pair (i, j)
 * of entries of its children with probability W[k][i][j] L[i] R[j] / S[k], and
 * a leaf reached with entry k keeps its observed variables and fills the others
 * from its k-th distribution.  With evidence a forward pass as in einet_logp
 * (unobserved variables integrated out) provides the node values, so the draw
 * is from the conditional of Eq. 1; without evidence the choices follow the
 * weights alone (ancestral sampling) and no forward pass runs.
 * A choice from weights w_0.. with a uniform u is the first index whose running
 * sum exceeds u times the total; pairs are numbered i*K + j.  All random numbers
 * are inputs:
 *   u_dev      device, [num_partitions + num_regions][B] float32 uniforms in
 *              [0,1): row n decides the pair of partition n, row
 *              num_partitions + s the partition of region s (rows of decisions a
 *              sample does not meet are not read)
 *   noise_dev  device, [B][D][C] float32, or NULL for the leaf means (App. D).
 *              Gaussian leaves: standard normal numbers, x = mean + sd * noise;
 *              Bernoulli leaves: uniforms, x = 1 if noise < p else 0; binomial
 *              and categorical leaves: uniforms, x = the first value whose
 *              running probability sum exceeds noise * (sum of all of them)
 *   x_dev, mask_dev, mask_mode   evidence as in einet_logp (1 = observed);
 *              EINET_MASK_NONE means no evidence: both pointers must be NULL
 *   out_dev    device, [B][D][C] float32, written completely: observed entries
 *              are copied from x_dev
 * The evidence must have non-zero density.  Uses the workspace (overwrites the
 * activations and the posterior arena; the statistics buffer is not touched).
 * Errors: as einet_logp; B above 65535: EINET_ERR_BATCH_TOO_LARGE. */
int einet_sample(einet_t* h, int B, const float* x_dev, const uint8_t* mask_dev, int mask_mode, const float* u_dev,
                 const float* noise_dev, float* out_dev, void* stream);

/* Mixture of several EiNets (Sec. 4.2: one EiNet per cluster, the cluster
 * proportions as coefficients):
 *   out[b] = log sum_c exp(log_coef[c] + logp[c][b]),
 * evaluated with a shift by the largest term; -inf when every term is -inf.
 *   logp_dev      device, [n_components][B] float32: row c is the output of
 *                 einet_logp of component c on the same batch
 *   log_coef_dev  device, [n_components] float32
 *   out_dev       device, [B] float32, written
 * Needs no handle; asynchronous on `stream`.  Errors: EINET_ERR_INVALID_ARG
 * (NULL pointers, n_components < 1, B < 1), EINET_ERR_HIP; the reason is read
 * with einet_last_error(NULL). */
int einet_mixture_logp(const float* logp_dev, const float* log_coef_dev, int n_components, int B, float* out_dev,
                       void* stream);

/* Per-kernel timing for benchmarks (no passage of the paper: measurement aid).
 * While enabled, every kernel launch of the compute calls above is bracketed
 * by two HIP events recorded on the call's stream.  einet_profile_read
 * synchronises those events, adds the elapsed times per kernel class, clears
 * the record, and writes up to `capacity` classes: names[i] (host strings
 * owned by the library), total_ms[i], launches[i]; *n_classes receives the
 * number of classes.  All outputs: host.  Disabled by default; recording costs
 * host time per launch, so throughput is measured with it off. */
int einet_profile_enable(einet_t* h, int enable);
int einet_profile_read(einet_t* h, int capacity, int* n_classes, const char** names, double* total_ms,
                       int64_t* launches);
/* The launches that the last einet_profile_read summed, one by one and in the order
 * they were enqueued: cls[i] (index into the names of einet_profile_read),
 * ms[i], and work[i]: for the launches of an einsum layer o * 2^24 + p, with p
 * the layer's partitions and o their output entries summed (K per partition,
 * 1 for a partition of the root), so that the launch's algorithmic flop are
 * 2 B K^2 o bottom-up and 4 B K^2 o top-down (Eq. 5, Eq. 6); 0 for the other
 * classes.  Writes up to `capacity` entries; *n_launches receives their
 * number.  All outputs: host. */
int einet_profile_launches(einet_t* h, int64_t capacity, int64_t* n_launches, int32_t* cls, float* ms, int64_t* work);

/* Achievable peaks of the current device, measured with plain kernels (no
 * passage of the paper: measurement aid, needs no handle): out4[0] the rate
 * of a streaming copy of `bytes` bytes from src_dev to dst_dev in GB/s (read
 * plus written), out4[1] the rate of a register-resident loop of
 * v_mfma_f32_32x32x2_f32 in TFLOP/s, out4[2] and out4[3] the same for
 * v_mfma_f32_16x16x4_f32 with one and with four waves per SIMD; each the best
 * of `reps` launches.  src_dev, dst_dev: device buffers of `bytes` bytes owned
 * by the caller (bytes a multiple of 16, at least EINET_PEAKS_MIN_BYTES;
 * dst_dev is overwritten); out4: host.  Synchronises `stream`.  Errors:
 * EINET_ERR_INVALID_ARG, EINET_ERR_HIP (reason via einet_last_error(NULL)). */
#define EINET_PEAKS_MIN_BYTES (4 * 1024 * 1024)
int einet_measure_peaks(const void* src_dev, void* dst_dev, int64_t bytes, int reps, double* out4, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EINET_H */
