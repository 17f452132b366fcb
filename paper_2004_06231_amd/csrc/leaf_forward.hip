// Leaf layer (Sec. 3.4): constants derived from the expectation parameters, log-densities of the leaves.
#include "device_common.hpp"

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
template <int FAMILY>
__device__ __forceinline__ float leaf_term(float xv, const float* __restrict__ th, int K, int P) {
    if constexpr (FAMILY == EINET_LEAF_GAUSSIAN) {
        const float diff = xv - th[0];
        return fmaf(th[K] * diff, diff, th[2 * K]);
    } else if constexpr (FAMILY == EINET_LEAF_CATEGORICAL) {
        return th[(size_t)min(max((int)xv, 0), P - 1) * K];
    } else {
        return xv * th[0] + ((float)P - xv) * th[K];
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

// Leaf layer for leaves with long scopes (image cells): a workgroup of 1024 threads takes one leaf
// and LEAF_BS samples.  The samples' values are staged in LDS with coalesced reads of x; thread
// (k, part) loads the constants of a few (variable, channel) pairs once and applies them to all
// staged samples from registers; the parts (float64) meet in LDS, then offset and residuals as above.
constexpr int LEAF_BS = 8;

// bytes of LDS: the finished entries (float64) first, then the partial sums of the parts, the values and the
// observation flags.  A part sums only a handful of terms, so float32 is enough for it; the sum over the
// parts, of magnitude 1e2..1e4, is taken in float64.
__host__ __device__ inline size_t leaf_wide_lds_bytes(int max_scope, int C, int K) {
    return sizeof(double) * ((size_t)LEAF_BS * K) +
           sizeof(float) * ((size_t)(1024 / K) * LEAF_BS * K + (size_t)LEAF_BS * max_scope * (C + 1));
}

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
    const int leaf = blockIdx.x, b0 = blockIdx.y * LEAF_BS, tid = threadIdx.x;
    const int nbs = min(LEAF_BS, d.B - b0);
    const int r = leaf_replica[leaf];
    const int s0 = leaf_sptr[leaf], nv = leaf_sptr[leaf + 1] - s0, np = nv * d.C;
    const int nparts = 1024 / d.K;
    double* val = lds_d;                                  // [LEAF_BS][K] finished entries
    float* red = reinterpret_cast<float*>(val + LEAF_BS * d.K);   // [nparts][LEAF_BS][K]
    float* xs = red + (size_t)nparts * LEAF_BS * d.K;     // [LEAF_BS][np] values, zeros where unused
    float* ob = xs + (size_t)LEAF_BS * max_scope * d.C;   // [LEAF_BS][nv] 1 = observed
    for (int idx = tid; idx < LEAF_BS * np; idx += 1024) {
        const int b = idx / np, p = idx - b * np, v = p / d.C, c = p - v * d.C;
        xs[idx] = b < nbs ? x[((size_t)(b0 + b) * d.D + leaf_var[s0 + v]) * d.C + c] : 0.f;
    }
    for (int idx = tid; idx < LEAF_BS * nv; idx += 1024) {
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
    float acc[LEAF_BS], hacc[LEAF_BS];
#pragma unroll
    for (int b = 0; b < LEAF_BS; ++b) acc[b] = hacc[b] = 0.f;
    if (part < nparts) {
        for (int p = part; p < np; p += nparts) {
            const int v = p / d.C, c = p - v * d.C;
            const float* th = theta + ((size_t)(leaf_var[s0 + v] * d.C + c) * d.R + r) * tstride + k;
            if (d.family == EINET_LEAF_GAUSSIAN) {
                const float mu = th[0], c1 = th[d.K], c0 = th[2 * d.K];
#pragma unroll
                for (int b = 0; b < LEAF_BS; ++b) {
                    const float diff = xs[b * np + p] - mu;
                    acc[b] += ob[b * nv + v] * fmaf(c1 * diff, diff, c0);
                }
            } else if (d.family == EINET_LEAF_CATEGORICAL) {
#pragma unroll
                for (int b = 0; b < LEAF_BS; ++b)
                    acc[b] += ob[b * nv + v] * leaf_term<EINET_LEAF_CATEGORICAL>(xs[b * np + p], th, d.K, d.P);
            } else {
                const float lp = th[0], l1p = th[d.K], nf = (float)d.P;
#pragma unroll
                for (int b = 0; b < LEAF_BS; ++b) {
                    const float xv = xs[b * np + p];
                    acc[b] += ob[b * nv + v] * (xv * lp + (nf - xv) * l1p);
                    if (base) hacc[b] += ob[b * nv + v] * leaf_base(logc, xv, d.P);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < LEAF_BS; ++b) red[(part * LEAF_BS + b) * d.K + k] = acc[b];
    }
    __syncthreads();
    const bool fin = tid < LEAF_BS * d.K;
    const int fb = fin ? tid / d.K : 0, kk = tid - fb * d.K;
    const int nact = min(nparts, np);                // parts beyond the number of pairs hold zeros
    double sum = 0.0;
    if (fin) {
        for (int q = 0; q < nact; ++q) sum += (double)red[(q * LEAF_BS + fb) * d.K + kk];
        val[fb * d.K + kk] = sum;
    }
    __syncthreads();
    if (base && part < nparts) {                     // (after the barrier: the sums above have been read)
#pragma unroll
        for (int b = 0; b < LEAF_BS; ++b) red[(part * LEAF_BS + b) * d.K] = hacc[b];
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
                for (int q = 0; q < nact; ++q) h += (double)red[(q * LEAF_BS + fb) * d.K];
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
    if (pairs >= 32 && pairs * d.K >= 768) {
        // long scopes (at least three quarters of the 1024/K parts of a workgroup get a (variable, channel) pair): one
        // workgroup per (leaf, LEAF_BS samples), values staged in LDS
        const size_t lds = leaf_wide_lds_bytes(max_scope, d.C, d.K);
        if (lds <= 64 * 1024) {
            dim3 grid(n_leaves, (d.B + LEAF_BS - 1) / LEAF_BS);
            hipLaunchKernelGGL(k_leaf_forward_wide, grid, dim3(1024), lds, s, t.leaf_node, t.leaf_replica, t.leaf_sptr,
                               t.leaf_var, x, mask, mask_mode, theta, t.leaf_logc, A, Off, max_scope, d);
            return;
        }
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
