// Leaf layer (Sec. 3.4): constants derived from the expectation parameters, log-densities of the leaves.
#include "device_common.hpp"

#include <mutex>
#include <type_traits>

namespace einet_impl {

namespace {

// ------------------------------------------------------------------ leaves
// Per leaf entry, what the log-density needs besides x (Sec. 3.4):
//   Gaussian  phi = (E x, E x^2): mean, -1/(2 var), -log(2 pi var)/2
//   Bernoulli phi = p           : log p, log(1-p)
__global__ void k_leaf_derive(const float* __restrict__ phi, float* __restrict__ theta, int n_entries, int K,
                              int family, int P) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_entries * K) return;
    int e = idx / K, k = idx - e * K;
    if (family == EINET_LEAF_GAUSSIAN) {
        float m = phi[(e * 2 + 0) * K + k], s = phi[(e * 2 + 1) * K + k];
        float var = fmaxf(fmaf(-m, m, s), 1e-30f);
        theta[(e * 3 + 0) * K + k] = m;
        theta[(e * 3 + 1) * K + k] = -0.5f / var;
        theta[(e * 3 + 2) * K + k] = -0.5f * logf(6.283185307179586f * var);
    } else if (family == EINET_LEAF_CATEGORICAL) {
        for (int v = 0; v < P; ++v) theta[((size_t)e * P + v) * K + k] = logf(phi[((size_t)e * P + v) * K + k]);
    } else {
        float p = phi[e * K + k] / (float)P;         // Bernoulli: P = 1; binomial: phi = P p
        theta[(e * 2 + 0) * K + k] = logf(p);
        theta[(e * 2 + 1) * K + k] = log1pf(-p);
    }
}

// Log-density of one value under one leaf entry, without the part that does not depend on the entry
// (Sec. 3.4; th points at the entry's derived constants, which are K floats apart):
//   Gaussian      -1/(2 var) (x - mean)^2 - log(2 pi var)/2
//   Bernoulli, binomial with P trials   x log p + (P - x) log(1 - p); the binomial coefficient goes to the offset
//   categorical   log p[x]
// Bernoulli / binomial term x log p + (P - x) log(1 - p).  A count of zero contributes log 1 = 0 also when the
// probability is 0 or 1 (the density p^x (1-p)^(P-x) at the boundary); 0 * -inf would be NaN.
__device__ __forceinline__ float count_term(float xv, float lp, float l1p, float nf) {
    const float a = xv != 0.f ? xv * lp : 0.f;
    const float b = nf != xv ? (nf - xv) * l1p : 0.f;
    return a + b;
}

// A marginalised variable contributes 0 whatever its term is (also -inf).
__device__ __forceinline__ float observed_term(float o, float term) { return o != 0.f ? term : 0.f; }

template <int FAMILY>
__device__ __forceinline__ float leaf_term(float xv, const float* __restrict__ th, int K, int P) {
    if constexpr (FAMILY == EINET_LEAF_GAUSSIAN) {
        const float diff = xv - th[0];
        return fmaf(th[K] * diff, diff, th[2 * K]);
    } else if constexpr (FAMILY == EINET_LEAF_CATEGORICAL) {
        return th[(size_t)min(max((int)xv, 0), P - 1) * K];
    } else {
        return count_term(xv, th[0], th[K], (float)P);
    }
}

__device__ __forceinline__ float leaf_base(const int32_t* __restrict__ logc, float xv, int P) {
    return __int_as_float(logc[min(max((int)xv, 0), P)]);
}

// Leaf layer: value[b][k] = sum over the leaf's scope and the channels of the
// log-density of x under entry k; a marginalised variable contributes 0.  Stored
// as Off[leaf][b] = max_k value (0 if every entry is -inf) and A = value - Off.
// A workgroup of TPB threads serves one leaf: thread (part, sample slot, k) computes entry k of RB samples
// (slot, slot + rows, ...), its part taking every NCH-th variable of the scope; the partial sums (float64:
// a scope of thousands of variables sums to 1e4 and more) meet in LDS.  Several samples per thread because
// the kernel is bound by the chain index -> value/constants of every thread, not by arithmetic: the
// constants are loaded once for RB samples and there are RB times fewer threads to wait for.  The family
// is a template parameter: with a run-time switch inside the loop over the scope the loads of consecutive
// variables are no longer issued together and the kernel takes twice as long.
template <int NCH, int FAMILY, int TPB, int RB>
__global__ __launch_bounds__(TPB) void k_leaf_forward(const int32_t* __restrict__ leaf_node,
                                                      const int32_t* __restrict__ leaf_replica,
                                                      const int32_t* __restrict__ leaf_sptr,
                                                      const int32_t* __restrict__ leaf_var,
                                                      const float* __restrict__ x, const uint8_t* __restrict__ mask,
                                                      int mask_mode, const float* __restrict__ theta,
                                                      const int32_t* __restrict__ logc, float* __restrict__ A,
                                                      double* __restrict__ Off, Dims d) {
    constexpr int NO = TPB / NCH;
    __shared__ double red[NCH][RB][NO];
    const int leaf = blockIdx.x, lo = threadIdx.x % NO, part_id = threadIdx.x / NO;
    const int rows = NO / d.K;                       // sample slots per workgroup (K <= 64 <= NO)
    const int bl = lo / d.K, k = lo - bl * d.K;
    int bs[RB];                                      // this thread's samples (clamped; `valid` says which exist)
    bool valid[RB];
#pragma unroll
    for (int q = 0; q < RB; ++q) {
        const int brow = (blockIdx.y * RB + q) * rows + bl;
        valid[q] = bl < rows && brow < d.B;
        bs[q] = valid[q] ? brow : 0;
    }
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0;
    const size_t tstride = (size_t)d.TD * d.K;
    const bool base = FAMILY == EINET_LEAF_BINOMIAL && k == 0;   // this thread also sums the binomial coefficients
    double acc[RB], hacc[RB];
#pragma unroll
    for (int q = 0; q < RB; ++q) acc[q] = hacc[q] = 0.0;
    constexpr int U = RB > 1 ? 2 : 4;                // variables per round, their loads issued together
    for (int v0 = part_id; v0 < nv; v0 += NCH * U) {
        int var[U];
        bool in[U];                                  // the variable exists (the last round may be short)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + u * NCH;
            in[u] = v < nv;
            var[u] = in[u] ? leaf_var[s0 + v] : 0;
        }
        float obs[U][RB];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < RB; ++q) {
                bool o = in[u];
                if (in[u] && mask_mode == EINET_MASK_SHARED) o = mask[var[u]] != 0;
                if (in[u] && mask_mode == EINET_MASK_PER_SAMPLE) o = mask[(size_t)bs[q] * d.D + var[u]] != 0;
                obs[u][q] = o ? 1.f : 0.f;
            }
        for (int c = 0; c < d.C; ++c) {
            float t[U][RB], h[U][RB];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float* th = theta + ((size_t)(var[u] * d.C + c) * d.R + r) * tstride + k;
#pragma unroll
                for (int q = 0; q < RB; ++q) {
                    t[u][q] = h[u][q] = 0.f;
                    if (in[u]) {
                        const float xv = x[((size_t)bs[q] * d.D + var[u]) * d.C + c];
                        t[u][q] = leaf_term<FAMILY>(xv, th, d.K, d.P);
                        if constexpr (FAMILY == EINET_LEAF_BINOMIAL)
                            if (base) h[u][q] = leaf_base(logc, xv, d.P);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int q = 0; q < RB; ++q) {
                    acc[q] += obs[u][q] != 0.f ? (double)t[u][q] : 0.0;
                    if constexpr (FAMILY == EINET_LEAF_BINOMIAL) hacc[q] += obs[u][q] != 0.f ? (double)h[u][q] : 0.0;
                }
        }
    }
    if constexpr (NCH > 1) {
#pragma unroll
        for (int q = 0; q < RB; ++q) red[part_id][q][lo] = acc[q];
        __syncthreads();
        if (part_id == 0) {
#pragma unroll
            for (int q = 0; q < RB; ++q)
#pragma unroll
                for (int p = 1; p < NCH; ++p) acc[q] += red[p][q][lo];
        }
        if constexpr (FAMILY == EINET_LEAF_BINOMIAL) {   // a second round for the base measure
            __syncthreads();
#pragma unroll
            for (int q = 0; q < RB; ++q) red[part_id][q][lo] = hacc[q];
            __syncthreads();
            if (part_id == 0)
                for (int q = 0; q < RB; ++q)
                    for (int p = 1; p < NCH; ++p) hacc[q] += red[p][q][lo];
        }
    }
    if (part_id == 0) {                              // its own slots: nobody else has read or will write them
#pragma unroll
        for (int q = 0; q < RB; ++q) red[0][q][lo] = acc[q];
    }
    __syncthreads();
    if (part_id == 0) {
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            if (!valid[q]) continue;
            double m = -INFINITY;
            for (int kk = 0; kk < d.K; ++kk) m = fmax(m, red[0][q][bl * d.K + kk]);
            if (m == -INFINITY) m = 0.0;             // every entry excludes the sample: residuals -inf
            const size_t row = (size_t)leaf_node[leaf] * d.B + bs[q];
            A[row * d.K + k] = (float)(acc[q] - m);
            if (k == 0) Off[row] = m + hacc[q];
        }
    }
}

// Leaf layer for leaves with scopes of more than LEAF_CHUNK (variable, channel) pairs (the strips of a
// 128x128x3 image): a workgroup of 1024 threads takes one leaf and BS samples.  The scope is walked in chunks of at most LEAF_CHUNK (variable, channel) pairs: the
// samples' values of a chunk are staged in LDS with coalesced reads of x; thread (k, part) loads the constants
// of a few pairs once and applies them to all staged samples from registers.  A part sums only a handful of
// terms per chunk, so float32 is enough there; across chunks and across parts the sums (magnitude 1e2..1e5)
// are float64.  Then offset and residuals as above.
constexpr int LEAF_RED = 8;   // the partial sums of the parts are [nparts][LEAF_RED][K] float32 in LDS
constexpr int LEAF_CHUNK = 384;
constexpr int LEAF_U = 4;      // pairs whose constants a thread requests together

// variables per chunk (whole variables, so that a chunk holds all channels of each)
__host__ __device__ inline int leaf_chunk_vars(int max_scope, int C) {
    const int v = LEAF_CHUNK / C;
    return max_scope < v ? max_scope : (v < 1 ? 1 : v);
}
// bytes of LDS for BS samples per workgroup: the finished entries (float64), the partial sums of the parts
// ([nparts][LEAF_RED][K] float32, or the same bytes as [nparts][LEAF_RED/2][K] float64 for leaves of several
// chunks, reduced four samples at a time), the values, the observation flags and the chunk's variable numbers
__host__ __device__ inline size_t leaf_wide_lds_bytes(int max_scope, int C, int K, int BS) {
    return sizeof(double) * ((size_t)BS * K) +
           sizeof(float) * ((size_t)(1024 / K) * LEAF_RED * K + (size_t)(BS * (C + 1) + 1) * leaf_chunk_vars(max_scope, C));
}

// MASKED: some variables may be marginalised (else the flags are neither staged nor read).
// BS: samples per workgroup (8: with 16 there are half as many workgroups, each twice as long, and the layer
// of a 128x128x3 image, four leaves, took twice the time).
template <bool MASKED, int BS>
__global__ __launch_bounds__(1024) void k_leaf_forward_wide(const int32_t* __restrict__ leaf_node,
                                                            const int32_t* __restrict__ leaf_replica,
                                                            const int32_t* __restrict__ leaf_sptr,
                                                            const int32_t* __restrict__ leaf_var,
                                                            const float* __restrict__ x,
                                                            const uint8_t* __restrict__ mask, int mask_mode,
                                                            const float* __restrict__ theta,
                                                            const int32_t* __restrict__ logc, float* __restrict__ A,
                                                            double* __restrict__ Off, int max_scope, Dims d) {
    extern __shared__ double lds_d[];
    const int leaf = blockIdx.x, b0 = blockIdx.y * BS, tid = threadIdx.x;
    const int nbs = min(BS, d.B - b0);
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0;
    const int nparts = 1024 / d.K;
    const int vch = leaf_chunk_vars(max_scope, d.C);      // variables per chunk
    double* val = lds_d;                                  // [BS][K] finished entries
    float* red = reinterpret_cast<float*>(val + BS * d.K);   // partial sums of the parts
    double* redd = reinterpret_cast<double*>(red);        // the same memory as [nparts][LEAF_RED/2][K] float64
    float* xs = red + (size_t)nparts * LEAF_RED * d.K;    // [BS][vch*C] values of the chunk
    float* ob = xs + (size_t)BS * vch * d.C;         // [BS][vch] 1 = observed
    int* vs = reinterpret_cast<int*>(ob + (size_t)BS * vch);   // [vch] variables of the chunk
    const int k = tid % d.K, part = tid / d.K;
    const size_t tstride = (size_t)d.TD * d.K;
    const bool base = d.family == EINET_LEAF_BINOMIAL && k == 0;   // this thread also sums the binomial coefficients
    typedef double acc_t;
    acc_t acc[BS], hacc[BS];
#pragma unroll
    for (int b = 0; b < BS; ++b) acc[b] = hacc[b] = 0;
    for (int v0 = 0; v0 < nv; v0 += vch) {
        const int cv = min(vch, nv - v0), np = cv * d.C;  // variables and pairs of this chunk
        if (v0 > 0) __syncthreads();                      // readers of the previous chunk are done
        // the variable numbers of the chunk come from LDS below: one memory latency less in front of every load
        // that depends on them, chunk after chunk
        for (int v = tid; v < cv; v += 1024) vs[v] = leaf_var[s0 + v0 + v];
        __syncthreads();
        auto var_of = [&](int v) { return vs[v]; };
        for (int idx = tid; idx < BS * np; idx += 1024) {
            const int b = idx / np, p = idx - b * np, v = p / d.C, c = p - v * d.C;
            xs[idx] = b < nbs ? x[((size_t)(b0 + b) * d.D + var_of(v)) * d.C + c] : 0.f;
        }
        for (int idx = tid; MASKED && idx < BS * cv; idx += 1024) {
            const int b = idx / cv, v = idx - b * cv;
            float o = 1.f;
            if (b < nbs && mask_mode == EINET_MASK_SHARED) o = mask[var_of(v)] ? 1.f : 0.f;
            if (b < nbs && mask_mode == EINET_MASK_PER_SAMPLE)
                o = mask[(size_t)(b0 + b) * d.D + var_of(v)] ? 1.f : 0.f;
            ob[idx] = o;
        }
        __syncthreads();
        if (part < nparts) {
            // LEAF_U pairs per round: their constants are requested together (one memory latency per round, not
            // per pair), their terms are summed in float32 and the group goes to the float64 sums
            for (int p0 = part; p0 < np; p0 += LEAF_U * nparts) {
                const float* th[LEAF_U];
                int pp[LEAF_U], vv[LEAF_U];
                bool in[LEAF_U];
#pragma unroll
                for (int u = 0; u < LEAF_U; ++u) {
                    const int p = p0 + u * nparts;
                    in[u] = p < np;
                    pp[u] = in[u] ? p : part;
                    vv[u] = pp[u] / d.C;
                    const int c = pp[u] - vv[u] * d.C;
                    th[u] = theta + ((size_t)(var_of(vv[u]) * d.C + c) * d.R + r) * tstride + k;
                }
                float t[BS], ht[BS];
#pragma unroll
                for (int b = 0; b < BS; ++b) t[b] = ht[b] = 0.f;
                if (d.family == EINET_LEAF_GAUSSIAN) {
                    float mu[LEAF_U], c1[LEAF_U], c0[LEAF_U];
#pragma unroll
                    for (int u = 0; u < LEAF_U; ++u) {
                        mu[u] = th[u][0];
                        c1[u] = in[u] ? th[u][d.K] : 0.f;     // a pair that does not exist adds 0
                        c0[u] = in[u] ? th[u][2 * d.K] : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < LEAF_U; ++u)
                        if (in[u])
#pragma unroll
                        for (int b = 0; b < BS; ++b) {
                            const float diff = xs[b * np + pp[u]] - mu[u];
                            const float term = fmaf(c1[u] * diff, diff, c0[u]);
                            t[b] += MASKED ? observed_term(ob[b * cv + vv[u]], term) : term;
                        }
                } else if (d.family == EINET_LEAF_CATEGORICAL) {
#pragma unroll
                    for (int u = 0; u < LEAF_U; ++u)
                        if (in[u])
#pragma unroll
                        for (int b = 0; b < BS; ++b) {
                            const float term = leaf_term<EINET_LEAF_CATEGORICAL>(xs[b * np + pp[u]], th[u], d.K, d.P);
                            t[b] += MASKED ? observed_term(ob[b * cv + vv[u]], term) : term;
                        }
                } else {
                    float lp[LEAF_U], l1p[LEAF_U];
                    const float nf = (float)d.P;
#pragma unroll
                    for (int u = 0; u < LEAF_U; ++u) {
                        lp[u] = in[u] ? th[u][0] : 0.f;
                        l1p[u] = in[u] ? th[u][d.K] : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < LEAF_U; ++u)
                        if (in[u])
#pragma unroll
                        for (int b = 0; b < BS; ++b) {
                            const float xv = xs[b * np + pp[u]];
                            const float term = count_term(xv, lp[u], l1p[u], nf);
                            t[b] += MASKED ? observed_term(ob[b * cv + vv[u]], term) : term;
                            if (base)
                                ht[b] += MASKED ? ob[b * cv + vv[u]] * leaf_base(logc, xv, d.P) : leaf_base(logc, xv, d.P);
                        }
                }
#pragma unroll
                for (int b = 0; b < BS; ++b) {
                    acc[b] += (acc_t)t[b];
                    hacc[b] += (acc_t)ht[b];
                }
            }
        }
    }
    const bool fin = tid < BS * d.K;
    const int fb = fin ? tid / d.K : 0, kk = tid - fb * d.K;
    const int nact = min(nparts, min(nv, vch) * d.C);     // parts beyond the pairs of a chunk hold zeros
    double sum = 0.0, h = 0.0;
    {
        // float64 partial sums, half of the samples at a time (the same LDS bytes)
        constexpr int HB = LEAF_RED / 2;
#pragma unroll
        for (int half = 0; half < BS / HB; ++half) {
            __syncthreads();                              // the chunk loop, or the previous half, is done with LDS
            if (part < nparts) {
#pragma unroll
                for (int b = 0; b < HB; ++b) redd[(part * HB + b) * d.K + k] = acc[half * HB + b];
            }
            __syncthreads();
            if (fin && fb / HB == half)
                for (int q = 0; q < nact; ++q) sum += redd[(q * HB + (fb - half * HB)) * d.K + kk];
            if (d.family == EINET_LEAF_BINOMIAL) {
                __syncthreads();
                if (base && part < nparts) {
#pragma unroll
                    for (int b = 0; b < HB; ++b) redd[(part * HB + b) * d.K] = hacc[half * HB + b];
                }
                __syncthreads();
                if (fin && kk == 0 && fb / HB == half)
                    for (int q = 0; q < nact; ++q) h += redd[(q * HB + (fb - half * HB)) * d.K];
            }
        }
    }
    if (fin) val[fb * d.K + kk] = sum;
    __syncthreads();
    if (fin && fb < nbs) {
        double m = -INFINITY;
        for (int q = 0; q < d.K; ++q) m = fmax(m, val[fb * d.K + q]);
        if (m == -INFINITY) m = 0.0;
        const size_t row = (size_t)leaf_node[leaf] * d.B + b0 + fb;
        A[row * d.K + kk] = (float)(sum - m);
        if (kk == 0) Off[row] = m + h;
    }
}

// Leaves of several chunks whose entries have two or three constants (Gaussian, Bernoulli, binomial): the same
// decomposition as above (a workgroup per leaf and LL_BS samples, thread (k, part), values staged chunk by chunk),
// arranged so that no wave waits for memory in front of its arithmetic and the arithmetic waves issue little
// besides it.  The last of the sixteen waves does nothing but stage: while the others work on chunk c it gathers
// the values of chunk c+1 into the other half of a double buffer and, for chunk c+2, where each pair's constants
// are (every lane owns the same LL_SLOTS pairs of every chunk, so its divisions are done once and
// what it needs of the next chunk stays in its registers).  The other waves take U pairs per round with the
// constants of the next round, also across the end of a chunk, requested before the arithmetic of this one; values
// are pair-major in LDS and read sixteen bytes at a time.  A round may reach beyond the pairs of its chunk: such a
// slot is sent to an entry of zeros, with which every term is zero whatever finite value the slot holds, so the loop
// has no bounds check, no division and no conditional load.  One barrier per chunk.
constexpr int LL_BS = 8;                  // samples per workgroup
constexpr int LL_U = 8;                   // pairs per round (half as many for the families with count terms)
constexpr int LL_COMPUTE = 960;           // threads of the fifteen waves that do arithmetic
constexpr int LL_SLOTS = LEAF_CHUNK / 64; // pairs of a chunk per lane of the staging wave
static_assert(LEAF_CHUNK % 64 == 0 && LL_BS == 8, "a lane stages whole pairs, two 16-byte stores each");

// How a workgroup divides a chunk: parts (threads with the same k are `parts` pairs apart), rounds per chunk and
// the slots the rounds of a chunk reach (at least the pairs of a full chunk).
struct LeafLongShape {
    int vch, chp, parts, rpc, cap;
};
__host__ __device__ inline LeafLongShape leaf_long_shape(int max_scope, int C, int K, bool gauss) {
    const int U = gauss ? LL_U : LL_U / 2;
    LeafLongShape s;
    s.vch = leaf_chunk_vars(max_scope, C);
    s.chp = s.vch * C;
    const int fit = LL_COMPUTE / K, need = (s.chp + U - 1) / U;   // more parts than pairs per round would idle
    s.parts = fit < need ? fit : need;
    s.rpc = (s.chp + s.parts * U - 1) / (s.parts * U);
    s.cap = s.rpc * U * s.parts;
    return s;
}
// bytes of LDS: finished entries (float64), partial sums of the parts, two buffers of values, (two of observation
// flags), three of offsets into the table of constants
__host__ __device__ inline size_t leaf_long_lds_bytes(int max_scope, int C, int K, bool masked, bool gauss) {
    const LeafLongShape s = leaf_long_shape(max_scope, C, K, gauss);
    return sizeof(double) * ((size_t)LL_BS * K) +
           sizeof(float) * ((size_t)s.parts * LL_BS * K + (masked ? 4 : 2) * (size_t)s.cap * LL_BS) +
           sizeof(long long) * 3 * (size_t)s.cap;
}

// constants of an entry with which every term is zero (never written): what a slot beyond its chunk reads
__device__ float leaf_zero_consts[3 * 64];

template <bool MASKED, bool GAUSS>
__global__ __launch_bounds__(1024) void k_leaf_forward_long(const int32_t* __restrict__ leaf_node,
                                                            const int32_t* __restrict__ leaf_replica,
                                                            const int32_t* __restrict__ leaf_sptr,
                                                            const int32_t* __restrict__ leaf_var,
                                                            const float* __restrict__ x,
                                                            const uint8_t* __restrict__ mask, int mask_mode,
                                                            const float* __restrict__ theta,
                                                            const int32_t* __restrict__ logc, float* __restrict__ A,
                                                            double* __restrict__ Off, int max_scope, Dims d) {
    extern __shared__ double lds_d[];
    constexpr int U = GAUSS ? LL_U : LL_U / 2;                 // pairs per round
    const int leaf = blockIdx.x, b0 = blockIdx.y * LL_BS, tid = threadIdx.x;
    const int nbs = min(LL_BS, d.B - b0);
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0;
    const LeafLongShape sh = leaf_long_shape(max_scope, d.C, d.K, GAUSS);
    const int nparts = sh.parts, vch = sh.vch, chp = sh.chp, rpc = sh.rpc, cap = sh.cap;
    const int nchunks = (nv + vch - 1) / vch;
    double* val = lds_d;                                       // [LL_BS][K] finished entries
    float* red = reinterpret_cast<float*>(val + LL_BS * d.K);  // partial sums of the parts
    double* redd = reinterpret_cast<double*>(red);             // the same memory as [nparts][LL_BS/2][K] float64
    float* xs = red + (size_t)nparts * LL_BS * d.K;            // [2][cap][LL_BS] values
    float* ob = xs + (size_t)2 * cap * LL_BS;                  // [2][cap][LL_BS] 1 = observed (MASKED)
    // [3][cap] where a pair's constants are, in bytes from the table's start (as offsets from a kernel argument the
    // loads stay loads from global memory; a pointer read from LDS would make them loads from any address space)
    long long* ptrs = reinterpret_cast<long long*>(ob + (MASKED ? (size_t)2 * cap * LL_BS : 0));
    const long long zeros_at = reinterpret_cast<const char*>(leaf_zero_consts) - reinterpret_cast<const char*>(theta);
    const int k = tid % d.K, part = tid / d.K;
    const bool stager = tid >= LL_COMPUTE, comp = !stager && part < nparts;
    const bool base = !GAUSS && d.family == EINET_LEAF_BINOMIAL && k == 0;   // also sums the binomial coefficients
    auto pairs_of = [&](int c) { return min(vch, nv - c * vch) * d.C; };
    double acc[LL_BS], hacc[LL_BS];
#pragma unroll
    for (int b = 0; b < LL_BS; ++b) acc[b] = hacc[b] = 0.0;
    // every slot starts with finite values and is sent to the zeros
    for (int i = tid; i < 2 * cap * LL_BS; i += 1024) xs[i] = 0.f;
    for (int i = tid; i < 3 * cap; i += 1024) ptrs[i] = zeros_at;
    __syncthreads();
    // The two roles are two separate pieces of code, so that neither holds the other's registers; each passes the
    // same barriers, one before the first chunk and one after every chunk.  The stager's loads are never
    // conditional: an index that does not exist is replaced by one that does and the value is dropped, which keeps
    // every load a single instruction with nothing to wait for in front of it.
    if (stager) {
        const int sl = tid - LL_COMPUTE;
        int vj[LL_SLOTS], cj[LL_SLOTS];                        // variable (within a chunk) and channel of lane's pairs
        unsigned row[LL_SLOTS], var[LL_SLOTS];                 // of the chunk whose values are staged next
#pragma unroll
        for (int j = 0; j < LL_SLOTS; ++j) {
            vj[j] = (sl + 64 * j) / d.C;
            cj[j] = sl + 64 * j - vj[j] * d.C;
        }
        const float* xrow[LL_BS];                              // the samples' rows of x (the last one repeated)
        const uint8_t* mrow[LL_BS];
#pragma unroll
        for (int b = 0; b < LL_BS; ++b) {
            const size_t bb = (size_t)(b0 + min(b, nbs - 1));
            xrow[b] = x + bb * d.D * d.C;
            mrow[b] = MASKED ? (mask_mode == EINET_MASK_SHARED ? mask : mask + bb * d.D) : nullptr;
        }
        const size_t tstride = (size_t)d.TD * d.K;
        auto stage_rows = [&](int c) {
            const int np = pairs_of(c);
            const int32_t* lv = leaf_var + s0 + c * vch;
#pragma unroll
            for (int j = 0; j < LL_SLOTS; ++j) var[j] = (unsigned)lv[sl + 64 * j < np ? vj[j] : 0];
#pragma unroll
            for (int j = 0; j < LL_SLOTS; ++j) {
                const bool in = sl + 64 * j < np;
                row[j] = var[j] * d.C + (in ? cj[j] : 0);      // (always a pair that exists)
                if (sl + 64 * j < chp)
                    ptrs[(c % 3) * cap + sl + 64 * j] =
                        in ? (long long)(sizeof(float) * ((size_t)row[j] * d.R + r) * tstride) : zeros_at;
            }
        };
        auto stage_values = [&](int c) {
            const int np = pairs_of(c);
            float* xb = xs + (size_t)(c & 1) * cap * LL_BS;
            float xv[LL_SLOTS][LL_BS];
#pragma unroll
            for (int j = 0; j < LL_SLOTS; ++j)
#pragma unroll
                for (int b = 0; b < LL_BS; ++b) xv[j][b] = xrow[b][row[j]];
#pragma unroll
            for (int j = 0; j < LL_SLOTS; ++j)
                if (sl + 64 * j < np) {
                    float4* dst = reinterpret_cast<float4*>(xb + (size_t)(sl + 64 * j) * LL_BS);
                    dst[0] = make_float4(xv[j][0], xv[j][1], xv[j][2], xv[j][3]);
                    dst[1] = make_float4(xv[j][4], xv[j][5], xv[j][6], xv[j][7]);
                }
            if constexpr (MASKED) {
                float* obb = ob + (size_t)(c & 1) * cap * LL_BS;
                uint8_t mv[LL_SLOTS][LL_BS];
#pragma unroll
                for (int j = 0; j < LL_SLOTS; ++j)
#pragma unroll
                    for (int b = 0; b < LL_BS; ++b) mv[j][b] = mrow[b][var[j]];
#pragma unroll
                for (int j = 0; j < LL_SLOTS; ++j)
                    if (sl + 64 * j < np) {
                        float o[LL_BS];
#pragma unroll
                        for (int b = 0; b < LL_BS; ++b) o[b] = mv[j][b] ? 1.f : 0.f;
                        float4* dst = reinterpret_cast<float4*>(obb + (size_t)(sl + 64 * j) * LL_BS);
                        dst[0] = make_float4(o[0], o[1], o[2], o[3]);
                        dst[1] = make_float4(o[4], o[5], o[6], o[7]);
                    }
            }
        };
        stage_rows(0);
        stage_values(0);
        if (nchunks > 1) stage_rows(1);
        __syncthreads();
        for (int c = 0; c < nchunks; ++c) {
            if (c + 1 < nchunks) stage_values(c + 1);          // (with the rows of chunk c+1, still in registers)
            if (c + 2 < nchunks) stage_rows(c + 2);
            __syncthreads();
        }
    } else {
        // the constants of round rr of chunk c (nothing is done to the values here, so nothing waits for them)
        auto request = [&](int c, int rr, float (&t0)[U], float (&t1)[U], float (&t2)[U]) {
            const long long* pt = ptrs + (size_t)(c % 3) * cap + rr * U * nparts + part;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float* th = reinterpret_cast<const float*>(reinterpret_cast<const char*>(theta) + pt[u * nparts]) + k;
                t0[u] = th[0];
                t1[u] = th[d.K];
                if constexpr (GAUSS) t2[u] = th[2 * d.K];
            }
        };
        auto compute = [&](int c, int rr, const float (&t0)[U], const float (&t1)[U], const float (&t2)[U]) {
            const int np = pairs_of(c);
            const float* xb = xs + ((size_t)(c & 1) * cap + rr * U * nparts + part) * LL_BS;
            const float* obb = ob + ((size_t)(c & 1) * cap + rr * U * nparts + part) * LL_BS;
            const float nf = (float)d.P;
            float t[LL_BS];
#pragma unroll
            for (int b = 0; b < LL_BS; ++b) t[b] = 0.f;
            float csum = 0.f;                                    // Gaussian, nothing marginalised: the terms' constants
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float4 xa = *reinterpret_cast<const float4*>(xb + (size_t)u * nparts * LL_BS);
                const float4 xc = *reinterpret_cast<const float4*>(xb + (size_t)u * nparts * LL_BS + 4);
                const float xv[LL_BS] = {xa.x, xa.y, xa.z, xa.w, xc.x, xc.y, xc.z, xc.w};
                float ov[LL_BS];
                if constexpr (MASKED) {
                    const float4 oa = *reinterpret_cast<const float4*>(obb + (size_t)u * nparts * LL_BS);
                    const float4 oc = *reinterpret_cast<const float4*>(obb + (size_t)u * nparts * LL_BS + 4);
                    ov[0] = oa.x; ov[1] = oa.y; ov[2] = oa.z; ov[3] = oa.w;
                    ov[4] = oc.x; ov[5] = oc.y; ov[6] = oc.z; ov[7] = oc.w;
                }
                if constexpr (GAUSS && !MASKED) csum += t2[u];
#pragma unroll
                for (int b = 0; b < LL_BS; ++b) {
                    if constexpr (GAUSS && !MASKED) {
                        const float diff = xv[b] - t0[u];
                        t[b] = fmaf(t1[u] * diff, diff, t[b]);
                    } else if constexpr (GAUSS) {
                        const float diff = xv[b] - t0[u];
                        t[b] += observed_term(ov[b], fmaf(t1[u] * diff, diff, t2[u]));
                    } else {
                        const float term = count_term(xv[b], t0[u], t1[u], nf);
                        t[b] += MASKED ? observed_term(ov[b], term) : term;
                    }
                }
                if constexpr (!GAUSS)
                    if (base && part + (rr * U + u) * nparts < np) {     // (one thread in K: straight to float64)
#pragma unroll
                        for (int b = 0; b < LL_BS; ++b) {
                            const float hb = leaf_base(logc, xv[b], d.P);
                            hacc[b] += (double)(MASKED ? ov[b] * hb : hb);
                        }
                    }
            }
#pragma unroll
            for (int b = 0; b < LL_BS; ++b) acc[b] += (double)(t[b] + csum);
        };
        // Two sets of constants, used in turn; the loop is written out for two rounds so that each set keeps its
        // registers.  (c, rr) is the round at hand, (cn, rn) the one after it; a chunk's last round ends at the barrier.
        // The request is not conditional: with a branch around it the compiler must assume at every use of the set
        // at hand that no younger loads are in flight, and waits for the new ones too.  After the last round it
        // re-reads what the offsets of an earlier chunk (or the zeros) name, and the values are dropped.
        float a0[U], a1[U], a2[U], e0[U], e1[U], e2[U];
        __syncthreads();
        if (comp) request(0, 0, a0, a1, a2);
        int c = 0, rr = 0;
        while (c < nchunks) {
            int rn = rr + 1 == rpc ? 0 : rr + 1, cn = rn == 0 ? c + 1 : c;
            if (comp) {
                request(cn, rn, e0, e1, e2);
                compute(c, rr, a0, a1, a2);
            }
            if (cn != c) __syncthreads();
            c = cn, rr = rn;
            if (c >= nchunks) break;
            rn = rr + 1 == rpc ? 0 : rr + 1, cn = rn == 0 ? c + 1 : c;
            if (comp) {
                request(cn, rn, a0, a1, a2);
                compute(c, rr, e0, e1, e2);
            }
            if (cn != c) __syncthreads();
            c = cn, rr = rn;
        }
    }

    // ---- the parts meet: float64 partial sums, half of the samples at a time (the same LDS bytes)
    const bool fin = tid < LL_BS * d.K;
    const int fb = fin ? tid / d.K : 0, kk = tid - fb * d.K;
    const int nact = min(nparts, min(nv, vch) * d.C);             // parts beyond the pairs of a chunk hold zeros
    double sum = 0.0, h = 0.0;
    constexpr int HB = LL_BS / 2;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if (half) __syncthreads();                                // the previous half has been read
        if (comp) {
#pragma unroll
            for (int b = 0; b < HB; ++b) redd[(part * HB + b) * d.K + k] = acc[half * HB + b];
        }
        __syncthreads();
        if (fin && fb / HB == half)
            for (int qq = 0; qq < nact; ++qq) sum += redd[(qq * HB + (fb - half * HB)) * d.K + kk];
        if (!GAUSS && d.family == EINET_LEAF_BINOMIAL) {
            __syncthreads();
            if (base && comp) {
#pragma unroll
                for (int b = 0; b < HB; ++b) redd[(part * HB + b) * d.K] = hacc[half * HB + b];
            }
            __syncthreads();
            if (fin && kk == 0 && fb / HB == half)
                for (int qq = 0; qq < nact; ++qq) h += redd[(qq * HB + (fb - half * HB)) * d.K];
        }
    }
    if (fin) val[fb * d.K + kk] = sum;
    __syncthreads();
    if (fin && fb < nbs) {
        double m = -INFINITY;
        for (int qq = 0; qq < d.K; ++qq) m = fmax(m, val[fb * d.K + qq]);
        if (m == -INFINITY) m = 0.0;
        const size_t rowo = (size_t)leaf_node[leaf] * d.B + b0 + fb;
        A[rowo * d.K + kk] = (float)(sum - m);
        if (kk == 0) Off[rowo] = m + h;
    }
}

// The same for leaves whose scope fits one chunk (the image cells of the benchmark configurations): one
// staging step, float32 sums per part (a part sums only a handful of terms), float64 across the parts.  A
// workgroup of 1024 threads takes one leaf and LEAF_RED samples.  The samples' values are staged in LDS with coalesced reads of x; thread
// (k, part) loads the constants of a few (variable, channel) pairs once and applies them to all
// staged samples from registers; the parts (float64) meet in LDS, then offset and residuals as above.

// bytes of LDS: the finished entries (float64) first, then the partial sums of the parts, the values and the
// observation flags.  A part sums only a handful of terms, so float32 is enough for it; the sum over the
// parts, of magnitude 1e2..1e4, is taken in float64.
__host__ __device__ inline size_t leaf_wide1_lds_bytes(int max_scope, int C, int K) {
    return sizeof(double) * ((size_t)LEAF_RED * K) +
           sizeof(float) * ((size_t)(1024 / K) * LEAF_RED * K + (size_t)LEAF_RED * max_scope * (C + 1) + max_scope);
}

__global__ __launch_bounds__(1024) void k_leaf_forward_wide1(const int32_t* __restrict__ leaf_node,
                                                            const int32_t* __restrict__ leaf_replica,
                                                            const int32_t* __restrict__ leaf_sptr,
                                                            const int32_t* __restrict__ leaf_var,
                                                            const float* __restrict__ x,
                                                            const uint8_t* __restrict__ mask, int mask_mode,
                                                            const float* __restrict__ theta,
                                                            const int32_t* __restrict__ logc, float* __restrict__ A,
                                                            double* __restrict__ Off, int max_scope, Dims d) {
    extern __shared__ double lds_d[];
    const int leaf = blockIdx.x, b0 = blockIdx.y * LEAF_RED, tid = threadIdx.x;
    const int nbs = min(LEAF_RED, d.B - b0);
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0, np = nv * d.C;
    const int nparts = 1024 / d.K;
    double* val = lds_d;                                  // [LEAF_RED][K] finished entries
    float* red = reinterpret_cast<float*>(val + LEAF_RED * d.K);   // [nparts][LEAF_RED][K]
    // pair-major: the LEAF_RED samples of a pair (a variable) are contiguous and are read with 16-byte loads
    float* xs = red + (size_t)nparts * LEAF_RED * d.K;     // [np][LEAF_RED] values, zeros where unused
    float* ob = xs + (size_t)LEAF_RED * max_scope * d.C;   // [nv][LEAF_RED] 1 = observed
    int* vs = reinterpret_cast<int*>(ob + (size_t)LEAF_RED * max_scope);   // [nv] the leaf's variables
    for (int v = tid; v < nv; v += 1024) vs[v] = leaf_var[s0 + v];
    for (int idx = tid; idx < LEAF_RED * np; idx += 1024) {
        const int b = idx / np, p = idx - b * np, v = p / d.C, c = p - v * d.C;
        xs[p * LEAF_RED + b] = b < nbs ? x[((size_t)(b0 + b) * d.D + leaf_var[s0 + v]) * d.C + c] : 0.f;
    }
    for (int idx = tid; idx < LEAF_RED * nv; idx += 1024) {
        const int b = idx / nv, v = idx - b * nv;
        float o = 1.f;
        if (b < nbs && mask_mode == EINET_MASK_SHARED) o = mask[leaf_var[s0 + v]] ? 1.f : 0.f;
        if (b < nbs && mask_mode == EINET_MASK_PER_SAMPLE) o = mask[(size_t)(b0 + b) * d.D + leaf_var[s0 + v]] ? 1.f : 0.f;
        ob[v * LEAF_RED + b] = o;
    }
    __syncthreads();
    const int k = tid % d.K, part = tid / d.K;
    const size_t tstride = (size_t)d.TD * d.K;
    const bool base = d.family == EINET_LEAF_BINOMIAL && k == 0;   // this thread also sums the binomial coefficients
    float acc[LEAF_RED], hacc[LEAF_RED];
#pragma unroll
    for (int b = 0; b < LEAF_RED; ++b) acc[b] = hacc[b] = 0.f;
    if (part < nparts) {
        if (d.family == EINET_LEAF_CATEGORICAL) {
            for (int p = part; p < np; p += nparts) {
                const int v = p / d.C, c = p - v * d.C;
                const float* th = theta + ((size_t)(vs[v] * d.C + c) * d.R + r) * tstride + k;
#pragma unroll
                for (int b = 0; b < LEAF_RED; ++b)
                    acc[b] += observed_term(ob[v * LEAF_RED + b], leaf_term<EINET_LEAF_CATEGORICAL>(xs[p * LEAF_RED + b], th, d.K, d.P));
            }
        } else {
            // Four pairs per round: their variable numbers are requested together, then their constants, so that
            // a round waits for two memory latencies instead of eight.  The terms are added in the order of the
            // pairs, as a pair-by-pair loop would.
            const bool gauss = d.family == EINET_LEAF_GAUSSIAN;
            const float nf = (float)d.P;
            for (int p = part; p < np; p += 4 * nparts) {
                int vq[4], pq[4], var[4];
                float t0[4], t1[4], t2[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    pq[q] = min(p + q * nparts, np - 1);
                    vq[q] = pq[q] / d.C;
                    var[q] = vs[vq[q]];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    // a pair beyond the scope repeats the last one with all constants zero: its terms are zero
                    const bool in = p + q * nparts < np;
                    const float* th = theta + ((size_t)(var[q] * d.C + (pq[q] - vq[q] * d.C)) * d.R + r) * tstride + k;
                    t0[q] = in ? th[0] : 0.f;
                    t1[q] = in ? th[d.K] : 0.f;
                    t2[q] = (in && gauss) ? th[2 * d.K] : 0.f;
                }
                static_assert(LEAF_RED == 8, "two 16-byte reads per pair");
                if (gauss) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 xa = *reinterpret_cast<const float4*>(xs + pq[q] * LEAF_RED);
                        const float4 xb = *reinterpret_cast<const float4*>(xs + pq[q] * LEAF_RED + 4);
                        const float4 oa = *reinterpret_cast<const float4*>(ob + vq[q] * LEAF_RED);
                        const float4 oc = *reinterpret_cast<const float4*>(ob + vq[q] * LEAF_RED + 4);
                        const float xv[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
                        const float ov[8] = {oa.x, oa.y, oa.z, oa.w, oc.x, oc.y, oc.z, oc.w};
#pragma unroll
                        for (int b = 0; b < LEAF_RED; ++b) {
                            const float diff = xv[b] - t0[q];
                            acc[b] += ov[b] * fmaf(t1[q] * diff, diff, t2[q]);
                        }
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 xa = *reinterpret_cast<const float4*>(xs + pq[q] * LEAF_RED);
                        const float4 xb = *reinterpret_cast<const float4*>(xs + pq[q] * LEAF_RED + 4);
                        const float4 oa = *reinterpret_cast<const float4*>(ob + vq[q] * LEAF_RED);
                        const float4 oc = *reinterpret_cast<const float4*>(ob + vq[q] * LEAF_RED + 4);
                        const float xv[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
                        const float ov[8] = {oa.x, oa.y, oa.z, oa.w, oc.x, oc.y, oc.z, oc.w};
#pragma unroll
                        for (int b = 0; b < LEAF_RED; ++b) {
                            // (nf * t1 is zero for a pair beyond the scope: both logarithms were set to zero)
                            acc[b] += observed_term(ov[b], count_term(xv[b], t0[q], t1[q], nf));
                            if (base && p + q * nparts < np) hacc[b] += ov[b] * leaf_base(logc, xv[b], d.P);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int b = 0; b < LEAF_RED; ++b) red[(part * LEAF_RED + b) * d.K + k] = acc[b];
    }
    __syncthreads();
    const bool fin = tid < LEAF_RED * d.K;
    const int fb = fin ? tid / d.K : 0, kk = tid - fb * d.K;
    const int nact = min(nparts, np);                // parts beyond the number of pairs hold zeros
    double sum = 0.0;
    if (fin) {
        for (int q = 0; q < nact; ++q) sum += (double)red[(q * LEAF_RED + fb) * d.K + kk];
        val[fb * d.K + kk] = sum;
    }
    __syncthreads();
    if (base && part < nparts) {                     // (after the barrier: the sums above have been read)
#pragma unroll
        for (int b = 0; b < LEAF_RED; ++b) red[(part * LEAF_RED + b) * d.K] = hacc[b];
    }
    if (d.family == EINET_LEAF_BINOMIAL) __syncthreads();
    if (fin && fb < nbs) {
        double m = -INFINITY;
        for (int q = 0; q < d.K; ++q) m = fmax(m, val[fb * d.K + q]);
        if (m == -INFINITY) m = 0.0;
        const size_t row = (size_t)leaf_node[leaf] * d.B + b0 + fb;
        A[row * d.K + kk] = (float)(sum - m);
        if (kk == 0) {
            double h = 0.0;
            if (d.family == EINET_LEAF_BINOMIAL)
                for (int q = 0; q < nact; ++q) h += (double)red[(q * LEAF_RED + fb) * d.K];
            Off[row] = m + h;
        }
    }
}

// The same kernel in the form that needs at most 64 vector registers (values sample-major in LDS, read one by one,
// one pair at a time), so that two workgroups share a compute unit: for launches of more workgroups than the chip
// has room for at once, where occupancy counts for more than the shorter dependency chains of the kernel above.
__global__ __launch_bounds__(1024, 8) void k_leaf_forward_wide1_lean(const int32_t* __restrict__ leaf_node,
                                                            const int32_t* __restrict__ leaf_replica,
                                                            const int32_t* __restrict__ leaf_sptr,
                                                            const int32_t* __restrict__ leaf_var,
                                                            const float* __restrict__ x,
                                                            const uint8_t* __restrict__ mask, int mask_mode,
                                                            const float* __restrict__ theta,
                                                            const int32_t* __restrict__ logc, float* __restrict__ A,
                                                            double* __restrict__ Off, int max_scope, Dims d) {
    extern __shared__ double lds_d[];
    const int leaf = blockIdx.x, b0 = blockIdx.y * LEAF_RED, tid = threadIdx.x;
    const int nbs = min(LEAF_RED, d.B - b0);
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0, np = nv * d.C;
    const int nparts = 1024 / d.K;
    double* val = lds_d;                                  // [LEAF_RED][K] finished entries
    float* red = reinterpret_cast<float*>(val + LEAF_RED * d.K);   // [nparts][LEAF_RED][K]
    float* xs = red + (size_t)nparts * LEAF_RED * d.K;     // [LEAF_RED][np] values, zeros where unused
    float* ob = xs + (size_t)LEAF_RED * max_scope * d.C;   // [LEAF_RED][nv] 1 = observed
    for (int idx = tid; idx < LEAF_RED * np; idx += 1024) {
        const int b = idx / np, p = idx - b * np, v = p / d.C, c = p - v * d.C;
        xs[idx] = b < nbs ? x[((size_t)(b0 + b) * d.D + leaf_var[s0 + v]) * d.C + c] : 0.f;
    }
    for (int idx = tid; idx < LEAF_RED * nv; idx += 1024) {
        const int b = idx / nv, v = idx - b * nv;
        float o = 1.f;
        if (b < nbs && mask_mode == EINET_MASK_SHARED) o = mask[leaf_var[s0 + v]] ? 1.f : 0.f;
        if (b < nbs && mask_mode == EINET_MASK_PER_SAMPLE) o = mask[(size_t)(b0 + b) * d.D + leaf_var[s0 + v]] ? 1.f : 0.f;
        ob[idx] = o;
    }
    __syncthreads();
    const int k = tid % d.K, part = tid / d.K;
    const size_t tstride = (size_t)d.TD * d.K;
    const bool base = d.family == EINET_LEAF_BINOMIAL && k == 0;   // this thread also sums the binomial coefficients
    float acc[LEAF_RED], hacc[LEAF_RED];
#pragma unroll
    for (int b = 0; b < LEAF_RED; ++b) acc[b] = hacc[b] = 0.f;
    if (part < nparts) {
        for (int p = part; p < np; p += nparts) {
            const int v = p / d.C, c = p - v * d.C;
            const float* th = theta + ((size_t)(leaf_var[s0 + v] * d.C + c) * d.R + r) * tstride + k;
            if (d.family == EINET_LEAF_GAUSSIAN) {
                const float mu = th[0], c1 = th[d.K], c0 = th[2 * d.K];
#pragma unroll
                for (int b = 0; b < LEAF_RED; ++b) {
                    const float diff = xs[b * np + p] - mu;
                    acc[b] += ob[b * nv + v] * fmaf(c1 * diff, diff, c0);
                }
            } else if (d.family == EINET_LEAF_CATEGORICAL) {
#pragma unroll
                for (int b = 0; b < LEAF_RED; ++b)
                    acc[b] += observed_term(ob[b * nv + v], leaf_term<EINET_LEAF_CATEGORICAL>(xs[b * np + p], th, d.K, d.P));
            } else {
                const float lp = th[0], l1p = th[d.K], nf = (float)d.P;
#pragma unroll
                for (int b = 0; b < LEAF_RED; ++b) {
                    const float xv = xs[b * np + p];
                    acc[b] += observed_term(ob[b * nv + v], count_term(xv, lp, l1p, nf));
                    if (base) hacc[b] += ob[b * nv + v] * leaf_base(logc, xv, d.P);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < LEAF_RED; ++b) red[(part * LEAF_RED + b) * d.K + k] = acc[b];
    }
    __syncthreads();
    const bool fin = tid < LEAF_RED * d.K;
    const int fb = fin ? tid / d.K : 0, kk = tid - fb * d.K;
    const int nact = min(nparts, np);                // parts beyond the number of pairs hold zeros
    double sum = 0.0;
    if (fin) {
        for (int q = 0; q < nact; ++q) sum += (double)red[(q * LEAF_RED + fb) * d.K + kk];
        val[fb * d.K + kk] = sum;
    }
    __syncthreads();
    if (base && part < nparts) {                     // (after the barrier: the sums above have been read)
#pragma unroll
        for (int b = 0; b < LEAF_RED; ++b) red[(part * LEAF_RED + b) * d.K] = hacc[b];
    }
    if (d.family == EINET_LEAF_BINOMIAL) __syncthreads();
    if (fin && fb < nbs) {
        double m = -INFINITY;
        for (int q = 0; q < d.K; ++q) m = fmax(m, val[fb * d.K + q]);
        if (m == -INFINITY) m = 0.0;
        const size_t row = (size_t)leaf_node[leaf] * d.B + b0 + fb;
        A[row * d.K + kk] = (float)(sum - m);
        if (kk == 0) {
            double h = 0.0;
            if (d.family == EINET_LEAF_BINOMIAL)
                for (int q = 0; q < nact; ++q) h += (double)red[(q * LEAF_RED + fb) * d.K];
            Off[row] = m + h;
        }
    }
}

}  // namespace

void launch_leaf_derive(const float* phi, float* theta, const Dims& d, hipStream_t s) {
    const int n = d.D * d.C * d.R;
    const int total = n * d.K;
    hipLaunchKernelGGL(k_leaf_derive, dim3((total + 255) / 256), dim3(256), 0, s, phi, theta, n, d.K, d.family, d.P);
}

void launch_leaf_forward(const DevTables& t, int n_leaves, int max_scope, const float* x, const uint8_t* mask,
                         int mask_mode, const float* theta, float* A, double* Off, const Dims& d, hipStream_t s) {
    const int pairs = max_scope * d.C;
    if (pairs >= 32 && pairs * d.K >= 768 && leaf_wide_lds_bytes(max_scope, d.C, d.K, 8) <= 64 * 1024) {
        // long scopes (at least three quarters of the 1024/K parts of a workgroup get a (variable, channel) pair):
        // one workgroup per (leaf, 8 or 16 samples), values staged in LDS chunk by chunk
        const bool multi = max_scope > leaf_chunk_vars(max_scope, d.C), masked = mask_mode != EINET_MASK_NONE;
        dim3 grid(n_leaves, (d.B + LEAF_RED - 1) / LEAF_RED);
        if (!multi) {
            // the kernel with the batched loads needs 122 registers, one workgroup of 1024 threads per compute unit: it
            // serves launches of one round; beyond that the 64-register form, two workgroups per compute unit
            if ((size_t)grid.x * grid.y <= EINET_NUM_CUS)
                hipLaunchKernelGGL(k_leaf_forward_wide1, grid, dim3(1024), leaf_wide1_lds_bytes(max_scope, d.C, d.K), s,
                                   t.leaf_node, t.leaf_replica, t.leaf_sptr, t.leaf_var, x, mask, mask_mode, theta,
                                   t.leaf_logc, A, Off, max_scope, d);
            else
                hipLaunchKernelGGL(k_leaf_forward_wide1_lean, grid, dim3(1024),
                                   leaf_wide1_lds_bytes(max_scope, d.C, d.K), s, t.leaf_node, t.leaf_replica,
                                   t.leaf_sptr, t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off, max_scope,
                                   d);
            return;
        }
        if (d.family != EINET_LEAF_CATEGORICAL &&
            leaf_long_lds_bytes(max_scope, d.C, d.K, masked, d.family == EINET_LEAF_GAUSSIAN) <= 160 * 1024) {
            // two or three constants per entry: the kernel with a staging wave and constants requested a round ahead
            static std::once_flag attr_set[EINET_MAX_DEVICES];
            int dev = 0;
            (void)hipGetDevice(&dev);
            std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] {
                allow_dynamic_lds(&k_leaf_forward_long<false, false>, 160 * 1024);
                allow_dynamic_lds(&k_leaf_forward_long<false, true>, 160 * 1024);
                allow_dynamic_lds(&k_leaf_forward_long<true, false>, 160 * 1024);
                allow_dynamic_lds(&k_leaf_forward_long<true, true>, 160 * 1024);
            });
            const bool gauss = d.family == EINET_LEAF_GAUSSIAN;
            const size_t ll = leaf_long_lds_bytes(max_scope, d.C, d.K, masked, gauss);
#define EINET_LONG(M, G)                                                                                              \
    hipLaunchKernelGGL((k_leaf_forward_long<M, G>), grid, dim3(1024), ll, s, t.leaf_node, t.leaf_replica, t.leaf_sptr, \
                       t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off, max_scope, d)
            if (masked) { if (gauss) EINET_LONG(true, true); else EINET_LONG(true, false); }
            else { if (gauss) EINET_LONG(false, true); else EINET_LONG(false, false); }
#undef EINET_LONG
            return;
        }
        const size_t lds = leaf_wide_lds_bytes(max_scope, d.C, d.K, LEAF_RED);
        if (masked)
            hipLaunchKernelGGL((k_leaf_forward_wide<true, LEAF_RED>), grid, dim3(1024), lds, s, t.leaf_node,
                               t.leaf_replica, t.leaf_sptr, t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off,
                               max_scope, d);
        else
            hipLaunchKernelGGL((k_leaf_forward_wide<false, LEAF_RED>), grid, dim3(1024), lds, s, t.leaf_node,
                               t.leaf_replica, t.leaf_sptr, t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off,
                               max_scope, d);
        return;
    }
    // parts per workgroup: enough that each thread walks only a few variables of the scope
    const int nch = pairs >= 96 ? 16 : (pairs >= 24 ? 4 : 1);
    // Many outputs (enough threads to fill the chip twice over): 256 threads with four samples each.
    // Otherwise, and for long scopes with sixteen parts: 1024 threads, one sample each.
    const bool many = nch != 16 && (int64_t)n_leaves * d.B * d.K * nch >= 1000000;
    const int tpb = many ? 256 : 1024, rb = many ? 4 : 1;
    const int rows = (tpb / nch) / d.K;               // sample slots per workgroup
    dim3 grid(n_leaves, (d.B + rows * rb - 1) / (rows * rb));
#define EINET_LAUNCH(N, F, TPB, RB)                                                                                 \
    hipLaunchKernelGGL((k_leaf_forward<N, F, TPB, RB>), grid, dim3(TPB), 0, s, t.leaf_node, t.leaf_replica,           \
                       t.leaf_sptr, t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off, d)
#define EINET_LAUNCH_SHAPE(N, F) \
    if (many) EINET_LAUNCH(N, F, 256, 4); else EINET_LAUNCH(N, F, 1024, 1)
#define EINET_LAUNCH_FAMILY(N)                                                          \
    switch (d.family) {                                                                 \
    case EINET_LEAF_GAUSSIAN: EINET_LAUNCH_SHAPE(N, EINET_LEAF_GAUSSIAN); break;        \
    case EINET_LEAF_BINOMIAL: EINET_LAUNCH_SHAPE(N, EINET_LEAF_BINOMIAL); break;        \
    case EINET_LEAF_CATEGORICAL: EINET_LAUNCH_SHAPE(N, EINET_LEAF_CATEGORICAL); break;  \
    default: EINET_LAUNCH_SHAPE(N, EINET_LEAF_BERNOULLI); break;                        \
    }
    if (nch == 16) EINET_LAUNCH_FAMILY(16)
    else if (nch == 4) EINET_LAUNCH_FAMILY(4)
    else EINET_LAUNCH_FAMILY(1)
#undef EINET_LAUNCH_FAMILY
#undef EINET_LAUNCH_SHAPE
#undef EINET_LAUNCH
}

}  // namespace einet_impl
