// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts).
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
// posterior arena G has the same shape; Gp[2e+side][b][k] holds what einsum
// item e sends down to its left (side 0) or right (side 1) child, and a child
// sums the slots of its parents when it is processed: no atomics anywhere.
#include "kernels.hpp"

#include <cmath>

namespace einet_impl {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));


__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

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

// ------------------------------------------------------------------ einsum layer, forward
// With eL = exp(L - a), eR = exp(R - a') (a, a' the row maxima; Eq. 4) the layer needs
//     S~[b,k] = sum_i eL[b,i] * T[(k,i), b],   T[(k,i), b] = sum_j W[k,i,j] eR[b,j].
// T is a dense GEMM (rows (k,i), columns b, contraction j) on v_mfma_f32_16x16x4_f32;
// one MFMA tile holds 4 outputs k (one per 16-lane group) x 4 inputs i (one per
// accumulator register), so the i-reduction of Eq. 4 is four in-lane FMAs per tile
// and the K x K outer product of Sec. 3.2 is never formed.
//
// One workgroup per (einsum item, tile of 4 outputs k).  Its slice W[4 k][K][K] is
// contiguous in memory; it is staged once in LDS, zero-padded to multiples of 4,
// with row strides chosen so that the A-operand reads of a half-wave hit 32
// distinct banks (i-stride = 8 mod 16, k-stride = 2 mod 32, lane groups read
// consecutive j).  Every wave then takes tiles of 16 samples: eR (the B operand)
// lives in registers, eL in a wave-private LDS tile, and each tile costs KQ*KQ
// MFMAs (KQ = ceil(K/4)).
template <int KQ>
struct FwdLayout {
    static constexpr int KP = 4 * KQ;
    static constexpr int SJ = ((KP + 7) / 16) * 16 + 8;   // smallest value >= KP that is 8 mod 16
    static constexpr int SK = KP * SJ + 2;
    static constexpr int LDS_W = ((4 * SK + 3) / 4) * 4;  // W slice, rounded so the eL tiles stay 16-byte aligned
    static constexpr int SE = KP + 4;                     // row stride of a wave's eL tile
    static constexpr int LDS_FLOATS = LDS_W + 8 * 16 * SE;
};

template <int KQ>
__global__ __launch_bounds__(512, 4) void k_einsum_forward(const int32_t* __restrict__ e_left,
                                                        const int32_t* __restrict__ e_right,
                                                        const int32_t* __restrict__ e_out,
                                                        const int32_t* __restrict__ e_kout,
                                                        const int32_t* __restrict__ e_woff,
                                                        const float* __restrict__ params, float* __restrict__ A,
                                                        double* __restrict__ Off, float* __restrict__ amax,
                                                        float* __restrict__ logp, int item0, int B, int K, int nkt) {
    using LY = FwdLayout<KQ>;
    constexpr int KP = LY::KP, SJ = LY::SJ, SK = LY::SK;
    extern __shared__ float Wl[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int li = blockIdx.x / nkt, kt = blockIdx.x - li * nkt;
    const int item = item0 + li;
    const int kout = e_kout[li];
    if (4 * kt >= kout) return;                        // root items have a single output entry
    const float* Lp = A + (size_t)e_left[li] * B * K;
    const float* Rp = A + (size_t)e_right[li] * B * K;
    const float* W = params + e_woff[li];

    const int c = lane & 15, g = lane >> 4;          // sample column of the tile, lane group
    const int gm = c >> 2, rm = c & 3;               // as A-operand lane: row 4*gm+rm = (k = 4kt+gm, i = 4it+rm)
    const int n_btiles = (B + 15) >> 4;
    // stage W[4kt .. 4kt+3][.][.]
    if ((K & 3) == 0) {
        for (int q = tid; q < 4 * KP * KQ; q += blockDim.x) {
            const int j4 = q % KQ, i = (q / KQ) % KP, kl = q / (KQ * KP);
            const int k = 4 * kt + kl;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < kout && i < K) v = *reinterpret_cast<const float4*>(W + ((size_t)k * K + i) * K + 4 * j4);
            float* dst = Wl + kl * SK + i * SJ + 4 * j4;
            *reinterpret_cast<float2*>(dst) = make_float2(v.x, v.y);
            *reinterpret_cast<float2*>(dst + 2) = make_float2(v.z, v.w);
        }
    } else {
        for (int q = tid; q < 4 * KP * KP; q += blockDim.x) {
            const int j = q % KP, i = (q / KP) % KP, kl = q / (KP * KP);
            const int k = 4 * kt + kl;
            float v = 0.f;
            if (k < kout && i < K && j < K) v = W[((size_t)k * K + i) * K + j];
            Wl[kl * SK + i * SJ + j] = v;
        }
    }
    __syncthreads();

    const float* wl = Wl + gm * SK + rm * SJ + g;    // + it*4*SJ + 4*s : contraction index j = 4s + g
    float* elw = Wl + LY::LDS_W + wave * (16 * LY::SE);   // this wave's eL tile [16][SE]
    for (int bt0 = 0; bt0 < n_btiles; bt0 += nwaves) {
        const int bt = bt0 + wave;
        const int b = bt * 16 + c;
        const bool ok = bt < n_btiles && b < B;
        // lane (c, g) holds entries 4s+g of row b of both inputs
        float er[KQ], el[KQ];
        float mr = -INFINITY, ml = -INFINITY;
#pragma unroll
        for (int s = 0; s < KQ; ++s) {
            const int j = 4 * s + g;
            const bool in = ok && j < K;
            er[s] = in ? Rp[(size_t)b * K + j] : -INFINITY;
            el[s] = in ? Lp[(size_t)b * K + j] : -INFINITY;
            mr = fmaxf(mr, er[s]);
            ml = fmaxf(ml, el[s]);
        }
        mr = fmaxf(mr, __shfl_xor(mr, 16, 64));
        mr = fmaxf(mr, __shfl_xor(mr, 32, 64));
        ml = fmaxf(ml, __shfl_xor(ml, 16, 64));
        ml = fmaxf(ml, __shfl_xor(ml, 32, 64));
        if (mr == -INFINITY) mr = 0.f;               // an all-zero input vector: exp(-inf) = 0, no NaN
        if (ml == -INFINITY) ml = 0.f;
        __syncthreads();                             // previous tile's eL reads are done
#pragma unroll
        for (int s = 0; s < KQ; ++s) {
            er[s] = __expf(er[s] - mr);              // stays in registers: the B operand
            elw[c * LY::SE + 4 * s + g] = __expf(el[s] - ml);
        }
        __syncthreads();
        float sacc = 0.f;
#pragma unroll
        for (int it = 0; it < KQ; ++it) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KQ; ++s)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wl[it * 4 * SJ + 4 * s], er[s], acc, 0, 0, 0);
            const float4 e4 = *reinterpret_cast<const float4*>(elw + c * LY::SE + 4 * it);
            sacc += acc[0] * e4.x + acc[1] * e4.y + acc[2] * e4.z + acc[3] * e4.w;
        }
        const int k = 4 * kt + g;
        const float res = __logf(sacc);                // residual against Off[left] + Off[right] + ml + mr
        if (ok && k < kout) A[((size_t)e_out[li] * B + b) * K + k] = res;
        if (ok && kt == 0 && g == 0) {
            const double off = Off[(size_t)e_left[li] * B + b] + Off[(size_t)e_right[li] * B + b] + (double)ml + (double)mr;
            Off[(size_t)e_out[li] * B + b] = off;
            if (logp && e_out[li] == 0) logp[b] = (float)(off + (double)res);   // node 0: the root region, one entry
            amax[((size_t)item * 2) * B + b] = ml;     // the shifts, kept for the top-down pass
            amax[((size_t)item * 2 + 1) * B + b] = mr;
        }
    }
}

// ------------------------------------------------------------------ mixing layer, forward (App. B)
// Offset of the output: the largest offset of the children (their residuals are at most 0, so no term
// exceeds its weight); residual: log sum_c v[c] exp((Off[c] - Off[out]) + A[c]).
__global__ void k_mixing_forward(const int32_t* __restrict__ m_node, const int32_t* __restrict__ m_kout,
                                 const int32_t* __restrict__ m_cptr, const int32_t* __restrict__ m_child,
                                 const int32_t* __restrict__ m_voff, const float* __restrict__ params,
                                 float* __restrict__ A, double* __restrict__ Off, float* __restrict__ logp, int B,
                                 int K) {
    const int item = blockIdx.x;
    const int kout = m_kout[item];
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= B * kout) return;
    const int b = e / kout, k = e - b * kout;
    const int c0 = m_cptr[item], nc = m_cptr[item + 1] - c0;
    const float* v = params + m_voff[item] + (size_t)k * nc;
    double m = -INFINITY;
    for (int c = 0; c < nc; ++c) m = fmax(m, Off[(size_t)m_child[c0 + c] * B + b]);
    float s = 0.f;
    for (int c = 0; c < nc; ++c) {
        const size_t row = (size_t)m_child[c0 + c] * B + b;
        s += v[c] * expf((float)(Off[row] - m) + A[row * K + k]);
    }
    const float res = logf(s);
    const size_t row = (size_t)m_node[item] * B + b;
    A[row * K + k] = res;
    if (k == 0) {
        Off[row] = m;
        if (logp && m_node[item] == 0) logp[b] = (float)(m + (double)res);   // node 0: the root region, one entry
    }
}

// The same for regions with many partitions (the root over R replicas of random binary trees): one wave per
// output element, the children spread over the lanes, maximum and sum by wave reductions.
__global__ __launch_bounds__(256) void k_mixing_forward_many(
    const int32_t* __restrict__ m_node, const int32_t* __restrict__ m_kout, const int32_t* __restrict__ m_cptr,
    const int32_t* __restrict__ m_child, const int32_t* __restrict__ m_voff, const float* __restrict__ params,
    float* __restrict__ A, double* __restrict__ Off, float* __restrict__ logp, int B, int K) {
    const int item = blockIdx.x;
    const int kout = m_kout[item];
    const int lane = threadIdx.x & 63;
    const int e = blockIdx.y * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (e >= B * kout) return;                       // whole waves leave
    const int b = e / kout, k = e - b * kout;
    const int c0 = m_cptr[item], nc = m_cptr[item + 1] - c0;
    const float* v = params + m_voff[item] + (size_t)k * nc;
    double m = -INFINITY;
    for (int c = lane; c < nc; c += 64) m = fmax(m, Off[(size_t)m_child[c0 + c] * B + b]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmax(m, __shfl_xor(m, o, 64));
    float s = 0.f;
    for (int c = lane; c < nc; c += 64) {
        const size_t row = (size_t)m_child[c0 + c] * B + b;
        s += v[c] * expf((float)(Off[row] - m) + A[row * K + k]);
    }
    s = wave_sum(s);
    if (lane == 0) {
        const float res = logf(s);
        const size_t row = (size_t)m_node[item] * B + b;
        A[row * K + k] = res;
        if (k == 0) {
            Off[row] = m;
            if (logp && m_node[item] == 0) logp[b] = (float)(m + (double)res);
        }
    }
}

// ------------------------------------------------------------------ top-down pass, regions
// G[region][b][k] = sum of the posterior blocks its parent partitions wrote (1 at
// the root).  Element-wise, one thread per (region, b, k); summing here instead of
// scattering from the producers keeps the pass free of atomics.
__global__ void k_region_assemble(const int32_t* __restrict__ r_node, const int32_t* __restrict__ r_kout,
                                  const int32_t* __restrict__ r_pptr, const int32_t* __restrict__ r_pblk,
                                  int is_root, float* __restrict__ G, const float* __restrict__ Gp, int B, int K) {
    const int item = blockIdx.x;
    const int kout = r_kout[item];
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= B * kout) return;
    const int b = e / kout, k = e - b * kout;
    const size_t blk = (size_t)B * K, o = (size_t)b * K + k;
    float g = is_root ? 1.f : 0.f;
    const int p1 = r_pptr[item + 1];
#pragma unroll 8
    for (int p = r_pptr[item]; p < p1; ++p) g += Gp[(size_t)r_pblk[p] * blk + o];
    G[(size_t)r_node[item] * blk + o] = g;
}

// Statistics of the mixing weights (App. B, Eq. 6): Nv[s,k,c] += v[s,k,c] * sum_b G[s][b,k] * S^c[b,k] / S[b,k].
// One workgroup per (mixing item, child); a reduction over the batch through LDS.  Runs in the same
// launch as the leaf statistics (k_tail_backward): the two are independent.
__device__ __forceinline__ void mixing_stats_body(int item, int c, const int32_t* __restrict__ m_node,
                                                  const int32_t* __restrict__ m_kout,
                                                  const int32_t* __restrict__ m_cptr,
                                                  const int32_t* __restrict__ m_child,
                                                  const int32_t* __restrict__ m_voff, const float* __restrict__ params,
                                                  float* __restrict__ stats, const float* __restrict__ A,
                                                  const double* __restrict__ Off, const float* __restrict__ G, int B,
                                                  int K) {
    __shared__ float red[1024];
    const int tid = threadIdx.x;
    const int c0 = m_cptr[item], nc = m_cptr[item + 1] - c0;
    if (c >= nc) return;
    const int kout = m_kout[item];
    const int nbl = 1024 / kout, k = tid % kout, bl = tid / kout;
    const float* As = A + (size_t)m_node[item] * B * K;
    const float* Ac = A + (size_t)m_child[c0 + c] * B * K;
    const float* Gs = G + (size_t)m_node[item] * B * K;
    const double* Os = Off + (size_t)m_node[item] * B;
    const double* Oc = Off + (size_t)m_child[c0 + c] * B;
    float part = 0.f;
    if (bl < nbl)
        for (int b = bl; b < B; b += nbl) {
            const size_t o = (size_t)b * K + k;
            const float g = Gs[o];
            if (g != 0.f) part += g * expf((float)(Oc[b] - Os[b]) + Ac[o] - As[o]);
        }
    red[tid] = part;
    __syncthreads();
    if (tid < kout) {
        float tot = 0.f;
        for (int l = 0; l < nbl; ++l) tot += red[l * kout + tid];
        const size_t o = (size_t)m_voff[item] + (size_t)tid * nc + c;
        stats[o] += params[o] * tot;
    }
}

// ------------------------------------------------------------------ top-down pass, einsum items
// For one einsum item, with Q[b,k] = G_out[b,k] / S~[b,k] (S~ the shifted sum of Eq. 4):
//   weight statistics (Eq. 6)   Nw[k,i,j] += W[k,i,j] * sum_b Q[b,k] eL[b,i] eR[b,j]        (GEMM-1)
//   posterior of the children   U[b,i,j]   = sum_k Q[b,k] W[k,i,j]                           (GEMM-2)
//                               Gp_left[b,i]  = eL[b,i] sum_j U[b,i,j] eR[b,j]
//                               Gp_right[b,j] = eR[b,j] sum_i U[b,i,j] eL[b,i]
// G_out is the posterior of the item's region s times, for a region with several
// partitions, the mixing weight and S^c/S; S^c cancels against S~ (the residual of the
// item's own output is log S~), leaving
//   Q = G[s] * v * exp((Off[out] - Off[s]) - A[s])        (Off[out] = Off[s] for a single partition).
// A workgroup takes one item and a run of slices, a slice being four consecutive
// left entries i.  eR and Q of up to 128 samples are staged once in LDS; the
// slices W[:, 4 i, :] then stream through LDS one at a time (the next one is
// already in flight in registers while the current one is used), and each serves
// both GEMMs, so W is read once per pass.
// GEMM-1 contracts over the batch: rows (k, i) in tiles of 4x4, columns j in tiles
// of 16; the A operand Q*eL is formed on the fly; a wave owns up to MAXU tiles and
// advances them together so that consecutive MFMAs are independent.
// GEMM-2 contracts over k: rows (j, i) in tiles of 4x4, columns = 16 samples, one
// sample tile per wave, all KQ row tiles advancing together.  The sum over the
// slice's four i (right child) is in-lane; the sum over j (left child) is in-lane
// across tiles plus one exchange between the four lane groups at the end.
// Gp_left is complete for the slice's entries; Gp_right is a partial sum over the
// workgroup's slices (summed in LDS, each entry by the lane that owns it), written to
// the workgroup's own block and added up by k_region_assemble.
template <int KQ>
struct BwdLayout {
    static constexpr int KP = 4 * KQ;
    static constexpr int SI = ((KP + 7) / 16) * 16 + 8;   // stride between the slice's i rows: 8 mod 16
    static constexpr int S = 4 * SI + 4;                  // stride between k rows: 4 mod 32
    static constexpr int NJ = (KP + 15) / 16;             // column tiles of GEMM-1
    static constexpr int BC = 128;                        // samples per pass over the batch
    static constexpr int ST = BC + 4;                     // row stride of the sample-major operand copies: 4 mod 32
    static constexpr int OFF_R = KP * S;                  // eR^T [16 NJ][ST]
    static constexpr int OFF_Q = OFF_R + 16 * NJ * ST;    // Q^T  [KP][ST]
    static constexpr int OFF_L = OFF_Q + KP * ST;         // eL^T [4][ST] of the current slice
    static constexpr int OFF_G = OFF_L + 4 * ST;          // Gp_right of the workgroup's slices [BC][KP] ...
    static constexpr bool LDS_ACC = OFF_G + BC * KP <= 40960;   // ... if it fits in the 160 KB of LDS
    static constexpr int LDS_FLOATS = OFF_G + (LDS_ACC ? BC * KP : 0);
    static constexpr int MAXU = (NJ * KQ + 7) / 8;        // GEMM-1 tiles per wave
    static constexpr int NW4 = (KP * 4 * KQ + 511) / 512; // float4 per thread of one W slice
    static constexpr int NW1 = (KP * 4 * KP + 511) / 512; // floats per thread when K is not a multiple of 4
};

// GEMM-1 over one pass of the batch for NU tiles of this wave.  The operands are kept
// sample-major in LDS (eR^T, Q^T, eL^T) and lane group g contracts samples g*RG .. g*RG+RG-1,
// so that one 16-byte LDS read feeds four consecutive MFMA steps.
template <int KQ, int NU>
__device__ __forceinline__ void bwd_gemm1(floatx4* acc1, const float* const* qcol, const float* const* rcol,
                                          const float* elcol, int rg) {
#pragma unroll 2
    for (int s = 0; s < rg; s += 4) {
        const float4 e = *reinterpret_cast<const float4*>(elcol + s);
        float4 qa[NU], rb[NU];
#pragma unroll
        for (int q = 0; q < NU; ++q) {
            qa[q] = *reinterpret_cast<const float4*>(qcol[q] + s);
            rb[q] = *reinterpret_cast<const float4*>(rcol[q] + s);
        }
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].x * e.x, rb[q].x, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].y * e.y, rb[q].y, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].z * e.z, rb[q].z, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].w * e.w, rb[q].w, acc1[q], 0, 0, 0);
    }
}

template <int KQ, bool VEC, bool ACCUM>
__global__ __launch_bounds__(512, 2) void k_einsum_backward(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_reg, const int32_t* __restrict__ e_kout, const int32_t* __restrict__ e_woff,
    const int32_t* __restrict__ e_voff, const int32_t* __restrict__ e_vstr, const float* __restrict__ params,
    float* __restrict__ stats, const float* __restrict__ A, const double* __restrict__ Off,
    const float* __restrict__ amax, const float* __restrict__ G, float* __restrict__ Gp, int item0, int ngroups, int B,
    int K) {
    using LY = BwdLayout<KQ>;
    constexpr int KP = LY::KP, SI = LY::SI, S = LY::S, ST = LY::ST, BC = LY::BC, MAXU = LY::MAXU;
    extern __shared__ float lds[];
    float* Wl = lds;
    float* sR = lds + LY::OFF_R;
    float* sQ = lds + LY::OFF_Q;
    float* sL = lds + LY::OFF_L;
    float* sG = lds + LY::OFF_G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = blockIdx.x / ngroups, grp = blockIdx.x - li * ngroups;
    const int it0 = grp * KQ / ngroups, it1 = (grp + 1) * KQ / ngroups;     // this workgroup's slices
    const bool multi = it1 - it0 > 1;   // several slices: their shares of Gp_right are summed in LDS first
    const int item = item0 + li;
    const int kout = e_kout[li], nkt = (kout + 3) >> 2;
    const size_t blk = (size_t)B * K;
    const float* Lp = A + (size_t)e_left[li] * blk;
    const float* Rp = A + (size_t)e_right[li] * blk;
    const float* As = A + (size_t)e_reg[li] * blk;
    const float* Gs = G + (size_t)e_reg[li] * blk;
    const float* W = params + e_woff[li];
    const size_t wbase = (size_t)e_woff[li];
    const int voff = e_voff[li], vstr = e_vstr[li];
    const float* aL = amax + (size_t)item * 2 * B;
    const float* aR = aL + B;
    const double* Oo = Off + (size_t)e_out[li] * B;
    const double* Os = Off + (size_t)e_reg[li] * B;
    const int nblk = 1 + KQ;

    // registers that carry the next W slice
    float4 w4[VEC ? LY::NW4 : 1];
    float w1[VEC ? 1 : LY::NW1];
    auto fetch_w = [&](int it) {
        if constexpr (VEC) {
#pragma unroll
            for (int n = 0; n < LY::NW4; ++n) {
                const int q = tid + 512 * n;
                const int j4 = q % KQ, il = (q / KQ) & 3, k = q / (4 * KQ);
                w4[n] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < kout) w4[n] = *reinterpret_cast<const float4*>(W + ((size_t)k * K + 4 * it + il) * K + 4 * j4);
            }
        } else {
#pragma unroll
            for (int n = 0; n < LY::NW1; ++n) {
                const int q = tid + 512 * n;
                const int j = q % KP, il = (q / KP) & 3, k = q / (4 * KP);
                const int i = 4 * it + il;
                w1[n] = (k < kout && i < K && j < K) ? W[((size_t)k * K + i) * K + j] : 0.f;
            }
        }
    };
    auto store_w = [&]() {
        if constexpr (VEC) {
#pragma unroll
            for (int n = 0; n < LY::NW4; ++n) {
                const int q = tid + 512 * n;
                const int j4 = q % KQ, il = (q / KQ) & 3, k = q / (4 * KQ);
                if (k < KP) *reinterpret_cast<float4*>(Wl + k * S + il * SI + 4 * j4) = w4[n];
            }
        } else {
#pragma unroll
            for (int n = 0; n < LY::NW1; ++n) {
                const int q = tid + 512 * n;
                const int j = q % KP, il = (q / KP) & 3, k = q / (4 * KP);
                if (k < KP) Wl[k * S + il * SI + j] = w1[n];
            }
        }
    };
    fetch_w(it0);

    const int c = lane & 15, g = lane >> 4;
    const int gm = c >> 2, rm = c & 3;
    // GEMM-1 tiles of this wave: u = jt * nkt + kt
    const int U = LY::NJ * nkt;
    const int u0 = wave * U / 8, nu = (wave + 1) * U / 8 - u0;
    const float* qcol[MAXU];
    const float* rcol[MAXU];
    int uoff[MAXU], uwl[MAXU];        // offset of (k, i = 0, j) in W / Nw, and in the LDS slice
    bool uok[MAXU];
#pragma unroll
    for (int q = 0; q < MAXU; ++q) {
        const int u = min(u0 + q, U - 1);
        const int jt = u / nkt, ukt = u - jt * nkt;
        qcol[q] = sQ + (4 * ukt + gm) * ST;     // + g*RG + s
        rcol[q] = sR + (16 * jt + c) * ST;
        const int k = 4 * ukt + g, j = 16 * jt + c;
        uok[q] = q < nu && k < kout && j < K;
        uoff[q] = uok[q] ? (k * K) * K + j : 0;
        uwl[q] = uok[q] ? k * S + j : 0;
    }
    float* Nw = stats + wbase;

    // staging of eR and Q: thread t owns row t/4 of the pass and a quarter of its columns
    const int srow = tid >> 2, sq = tid & 3;
    float vw[KQ];
#pragma unroll
    for (int u = 0; u < KQ; ++u) {
        const int k = sq * KQ + u;
        vw[u] = (voff >= 0 && k < kout) ? params[voff + k * vstr] : 1.f;
    }

    for (int b0 = 0; b0 < B; b0 += BC) {
        const int nb = min(BC, B - b0);
        const int rg = (((nb + 3) >> 2) + 3) & ~3;         // samples per lane group in GEMM-1, multiple of 4
        const bool rok = srow < nb;
        const int ro = (b0 + min(srow, nb - 1)) * K;       // a valid row even for the idle tail threads
        const float al = aL[b0 + min(srow, nb - 1)], ar = aR[b0 + min(srow, nb - 1)];
        const float dd = (float)(Oo[b0 + min(srow, nb - 1)] - Os[b0 + min(srow, nb - 1)]);
        __syncthreads();                                   // readers of the previous pass are done
        {
            float rv[KQ], gv[KQ], av[KQ];
#pragma unroll
            for (int u = 0; u < KQ; ++u) {
                const int k = sq * KQ + u;
                const int kc = VEC ? k : min(k, K - 1);
                rv[u] = Rp[ro + kc];
                gv[u] = Gs[ro + min(kc, kout - 1)];
                av[u] = As[ro + min(kc, kout - 1)];
            }
#pragma unroll
            for (int u = 0; u < KQ; ++u) {
                const int k = sq * KQ + u;
                const float e = __expf(rv[u] - ar);
                const float q = gv[u] * vw[u] * __expf(dd - av[u]);
                sR[k * ST + srow] = (rok && (VEC || k < K)) ? e : 0.f;
                sQ[k * ST + srow] = (rok && k < kout && gv[u] != 0.f) ? q : 0.f;
            }
            for (int j = KP + sq; j < 16 * LY::NJ; j += 4) sR[j * ST + srow] = 0.f;   // rows beyond the padded K
            if (multi && LY::LDS_ACC)
                for (int u = 0; u < KQ; ++u) sG[srow * KP + sq * KQ + u] = 0.f;
        }

        for (int it = it0; it < it1; ++it) {
            if (it != it0) __syncthreads();                // readers of the previous slice are done
            store_w();
            {
                const float e = __expf(Lp[ro + min(4 * it + sq, K - 1)] - al);
                sL[sq * ST + srow] = (rok && 4 * it + sq < K) ? e : 0.f;
            }
            __syncthreads();
            // next slice of this pass, or the first slice of the next pass, goes in flight now
            if (it + 1 < it1) fetch_w(it + 1);
            else if (b0 + BC < B) fetch_w(it0);

            // statistics this wave will update, fetched early (not needed when they are known to be zero)
            float nw[MAXU][4];
#pragma unroll
            for (int q = 0; q < MAXU; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = VEC ? 4 * it + r : min(4 * it + r, K - 1);
                    // (units that are not ours read a valid dummy; later passes over the batch always add)
                    nw[q][r] = (ACCUM || b0 > 0) ? Nw[uoff[q] + i * K] : 0.f;
                }

            // ---- GEMM-1
            floatx4 acc1[MAXU];
#pragma unroll
            for (int q = 0; q < MAXU; ++q) acc1[q] = floatx4{0.f, 0.f, 0.f, 0.f};
            {
                const float* elcol = sL + rm * ST + g * rg;
                const float* qc[MAXU];
                const float* rc[MAXU];
#pragma unroll
                for (int q = 0; q < MAXU; ++q) {
                    qc[q] = qcol[q] + g * rg;
                    rc[q] = rcol[q] + g * rg;
                }
                if (nu == MAXU) bwd_gemm1<KQ, MAXU>(acc1, qc, rc, elcol, rg);
                else if (MAXU > 1 && nu == MAXU - 1)
                    bwd_gemm1<KQ, (MAXU > 1 ? MAXU - 1 : 1)>(acc1, qc, rc, elcol, rg);
                else
                    for (int q = 0; q < nu; ++q) bwd_gemm1<KQ, 1>(acc1 + q, qc + q, rc + q, elcol, rg);
            }

            // ---- GEMM-2: one tile of 16 samples per wave
            if (wave * 16 < nb) {
                const int bl = wave * 16 + c;
                const bool ok = bl < nb;
                float erg[KQ];
#pragma unroll
                for (int s = 0; s < KQ; ++s) erg[s] = sR[(4 * s + g) * ST + bl];
                const float* qrow = sQ + g * ST + bl;
                const float4 e4 = make_float4(sL[bl], sL[ST + bl], sL[2 * ST + bl], sL[3 * ST + bl]);
                const float* wl = Wl + g * S + rm * SI + gm;      // row 4*gm+rm of a tile = (j = 4jt+gm, i = 4it+rm)
                floatx4 acc[KQ];
#pragma unroll
                for (int jt = 0; jt < KQ; ++jt) acc[jt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
                for (int s = 0; s < KQ; ++s) {
                    const float qs = qrow[4 * s * ST];
#pragma unroll
                    for (int jt = 0; jt < KQ; ++jt)
                        acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl[4 * s * S + 4 * jt], qs, acc[jt], 0, 0, 0);
                }
                // acc[jt][r] = U[b][i = 4it+r][j = 4jt+g]
                float gl0 = 0.f, gl1 = 0.f, gl2 = 0.f, gl3 = 0.f;
                float* right = Gp + ((size_t)(item * nblk + 1 + grp) * B + b0 + bl) * K;
                float* racc = sG + bl * KP;
#pragma unroll
                for (int jt = 0; jt < KQ; ++jt) {
                    const float t = acc[jt][0] * e4.x + acc[jt][1] * e4.y + acc[jt][2] * e4.z + acc[jt][3] * e4.w;
                    // this lane owns the entry in every slice: no race, in LDS or (for the largest K, where the
                    // accumulator does not fit) in the block itself
                    if (multi && LY::LDS_ACC) racc[4 * jt + g] += erg[jt] * t;
                    else if (ok && 4 * jt + g < K) right[4 * jt + g] = erg[jt] * t + (it > it0 ? right[4 * jt + g] : 0.f);
                    gl0 = fmaf(acc[jt][0], erg[jt], gl0);
                    gl1 = fmaf(acc[jt][1], erg[jt], gl1);
                    gl2 = fmaf(acc[jt][2], erg[jt], gl2);
                    gl3 = fmaf(acc[jt][3], erg[jt], gl3);
                }
                gl0 += __shfl_xor(gl0, 16, 64); gl0 += __shfl_xor(gl0, 32, 64);
                gl1 += __shfl_xor(gl1, 16, 64); gl1 += __shfl_xor(gl1, 32, 64);
                gl2 += __shfl_xor(gl2, 16, 64); gl2 += __shfl_xor(gl2, 32, 64);
                gl3 += __shfl_xor(gl3, 16, 64); gl3 += __shfl_xor(gl3, 32, 64);
                const float glr = g == 0 ? gl0 * e4.x : (g == 1 ? gl1 * e4.y : (g == 2 ? gl2 * e4.z : gl3 * e4.w));
                if (ok && 4 * it + g < K) Gp[((size_t)(item * nblk) * B + b0 + bl) * K + 4 * it + g] = glr;
            }

            // ---- GEMM-1 epilogue: Nw += W * acc
#pragma unroll
            for (int q = 0; q < MAXU; ++q) {
                if (uok[q]) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i = 4 * it + r;
                        if (VEC || i < K) Nw[uoff[q] + i * K] = nw[q][r] + Wl[uwl[q] + r * SI] * acc1[q][r];
                    }
                }
            }
        }
        if (multi && LY::LDS_ACC) {                        // Gp_right of the workgroup's slices, row by row
            __syncthreads();
            float* right = Gp + ((size_t)(item * nblk + 1 + grp) * B + b0) * K;
            for (int e = tid; e < nb * K; e += 512) {
                const int b = e / K, j = e - b * K;
                right[e] = sG[b * KP + j];
            }
        }
    }
}

// ------------------------------------------------------------------ top-down pass, leaves
// Posterior-weighted sufficient statistics (Eq. 6-7).  A workgroup of 1024 threads
// owns 1024/NCH consecutive statistics entries (leaf variable, channel, k); its NCH
// parts each walk every NCH-th sample and the partial sums meet in LDS.
template <int NCH>
__device__ __forceinline__ void leaf_backward_body(
    int block, const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var, const int32_t* __restrict__ leaf_node,
    const int32_t* __restrict__ leaf_replica, int n_lv, const float* __restrict__ x,
    const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G, float* __restrict__ stats,
    int64_t phi_off, int64_t den_off, int64_t tot_off, Dims d) {
    constexpr int NO = 1024 / NCH;
    __shared__ float red[NCH][4][NO];
    const int lo = threadIdx.x % NO, part_id = threadIdx.x / NO;
    const int idx = block * NO + lo;
    const bool valid = idx < n_lv * d.C * d.K;
    const int k = valid ? idx % d.K : 0, c = valid ? (idx / d.K) % d.C : 0, e = valid ? idx / (d.K * d.C) : 0;
    const int leaf = lv_leaf[e], var = lv_var[e], r = leaf_replica[leaf];
    const float* Gl = G + (size_t)leaf_node[leaf] * d.B * d.K + k;
    const float* xp = x + (size_t)var * d.C + c;
    const bool shared_obs = mask_mode != EINET_MASK_SHARED || mask[var] != 0;
    float n1 = 0.f, n2 = 0.f, den = 0.f, tot = 0.f;
#pragma unroll 4
    for (int b = part_id; b < d.B; b += NCH) {
        const float p = Gl[(size_t)b * d.K];
        bool obs = shared_obs;
        if (mask_mode == EINET_MASK_PER_SAMPLE) obs = mask[(size_t)b * d.D + var] != 0;
        const float xv = xp[(size_t)b * d.D * d.C];
        const float pm = obs ? p : 0.f;
        tot += p;
        den += pm;
        n1 = fmaf(pm, xv, n1);
        n2 = fmaf(pm * xv, xv, n2);
    }
    red[part_id][0][lo] = n1;
    red[part_id][1][lo] = n2;
    red[part_id][2][lo] = den;
    red[part_id][3][lo] = tot;
    __syncthreads();
    if (part_id || !valid) return;
#pragma unroll
    for (int q = 1; q < NCH; ++q) {
        n1 += red[q][0][lo];
        n2 += red[q][1][lo];
        den += red[q][2][lo];
        tot += red[q][3][lo];
    }
    const size_t ph = phi_off + ((size_t)(var * d.C + c) * d.R + r) * d.T * d.K + k;
    stats[ph] += n1;
    if (d.T == 2) stats[ph + d.K] += n2;
    if (c == 0) {
        const size_t o = ((size_t)var * d.R + r) * d.K + k;
        stats[den_off + o] += den;
        stats[tot_off + o] += tot;
    }
}

// Categorical leaves: the sufficient statistic is the indicator of the value, so the posterior mass of a
// sample goes to one of V rows.  One wave per (leaf variable, channel), lane k owns column k of a V x K
// histogram in LDS and walks the samples; no two lanes touch the same cell.
__global__ __launch_bounds__(64) void k_leaf_backward_categorical(
    const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var, const int32_t* __restrict__ leaf_node,
    const int32_t* __restrict__ leaf_replica, const float* __restrict__ x, const uint8_t* __restrict__ mask,
    int mask_mode, const float* __restrict__ G, float* __restrict__ stats, int64_t phi_off, int64_t den_off,
    int64_t tot_off, Dims d) {
    extern __shared__ float hist[];                   // [V][K]
    const int e = blockIdx.x / d.C, c = blockIdx.x - e * d.C, k = threadIdx.x;
    const int leaf = lv_leaf[e], var = lv_var[e], r = leaf_replica[leaf];
    const int V = d.P;
    if (k < d.K)
        for (int v = 0; v < V; ++v) hist[v * d.K + k] = 0.f;
    const bool shared_obs = mask_mode != EINET_MASK_SHARED || mask[var] != 0;
    float den = 0.f, tot = 0.f;
    if (k < d.K) {
        const float* Gl = G + (size_t)leaf_node[leaf] * d.B * d.K + k;
        for (int b = 0; b < d.B; ++b) {
            const float p = Gl[(size_t)b * d.K];
            bool obs = shared_obs;
            if (mask_mode == EINET_MASK_PER_SAMPLE) obs = mask[(size_t)b * d.D + var] != 0;
            const int v = min(max((int)x[((size_t)b * d.D + var) * d.C + c], 0), V - 1);
            tot += p;
            if (obs) {
                den += p;
                hist[v * d.K + k] += p;
            }
        }
        const size_t ph = phi_off + ((size_t)(var * d.C + c) * d.R + r) * V * d.K + k;
        for (int v = 0; v < V; ++v) stats[ph + (size_t)v * d.K] += hist[v * d.K + k];
        if (c == 0) {
            const size_t o = ((size_t)var * d.R + r) * d.K + k;
            stats[den_off + o] += den;
            stats[tot_off + o] += tot;
        }
    }
}

// The same statistics for leaves with long scopes (image cells).  A workgroup takes one leaf and a chunk of
// its (variable, channel) pairs; per pass over 128 samples the leaf's posterior block G[leaf][b][.] (contiguous
// in memory) and the pairs' values are copied to LDS, then thread (pair, k) walks the samples out of LDS.  The
// walk of the kernel above waits a full memory latency for every few samples; here it waits for LDS.
constexpr int CELL_BC = 128;                          // samples per pass
__host__ __device__ inline int cell_pairs_per_group(int K) { return 1024 / K < 64 ? 1024 / K : 64; }
__host__ __device__ inline size_t cell_lds_bytes(int K) {
    return sizeof(float) * (size_t)CELL_BC * (K + cell_pairs_per_group(K)) + (size_t)CELL_BC * cell_pairs_per_group(K);
}

__device__ __forceinline__ void leaf_backward_cells_body(
    int block, int chunks_per_leaf, const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica,
    const int32_t* __restrict__ leaf_sptr, const int32_t* __restrict__ leaf_var, const float* __restrict__ x,
    const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G, float* __restrict__ stats,
    int64_t phi_off, int64_t den_off, int64_t tot_off, Dims d) {
    extern __shared__ float cell_lds[];
    const int pc = cell_pairs_per_group(d.K);
    float* Gs = cell_lds;                             // [CELL_BC][K]
    float* xs = Gs + CELL_BC * d.K;                   // [CELL_BC][pc]
    uint8_t* os = reinterpret_cast<uint8_t*>(xs + CELL_BC * pc);   // [CELL_BC][pc] 1 = observed
    const int leaf = block / chunks_per_leaf, chunk = block - leaf * chunks_per_leaf;
    const int s0 = leaf_sptr[leaf], npairs = (leaf_sptr[leaf + 1] - s0) * d.C;
    const int p0 = chunk * pc;
    if (p0 >= npairs) return;                         // (whole workgroup) this leaf has fewer chunks
    const int np = min(pc, npairs - p0);
    const int tid = threadIdx.x;
    const int pl = tid / d.K, k = tid - pl * d.K;     // this thread's pair and entry
    const bool mine = pl < np;
    const float* Gl = G + (size_t)leaf_node[leaf] * d.B * d.K;
    float n1 = 0.f, n2 = 0.f, den = 0.f, tot = 0.f;
    for (int b0 = 0; b0 < d.B; b0 += CELL_BC) {
        const int nb = min(CELL_BC, d.B - b0);
        if (b0 > 0) __syncthreads();                  // readers of the previous pass are done
        for (int i = tid; i < nb * d.K; i += 1024) Gs[i] = Gl[(size_t)b0 * d.K + i];
        for (int i = tid; i < nb * np; i += 1024) {
            const int bb = i / np, p = i - bb * np;
            const int pair = p0 + p, v = pair / d.C, c = pair - v * d.C;
            const int var = leaf_var[s0 + v];
            xs[bb * pc + p] = x[((size_t)(b0 + bb) * d.D + var) * d.C + c];
            uint8_t o = 1;
            if (mask_mode == EINET_MASK_SHARED) o = mask[var];
            if (mask_mode == EINET_MASK_PER_SAMPLE) o = mask[(size_t)(b0 + bb) * d.D + var];
            os[bb * pc + p] = o;
        }
        __syncthreads();
        if (mine) {
#pragma unroll 4
            for (int bb = 0; bb < nb; ++bb) {
                const float p = Gs[bb * d.K + k];
                const float xv = xs[bb * pc + pl];
                const float pm = os[bb * pc + pl] ? p : 0.f;
                tot += p;
                den += pm;
                n1 = fmaf(pm, xv, n1);
                n2 = fmaf(pm * xv, xv, n2);
            }
        }
    }
    if (!mine) return;
    const int pair = p0 + pl, v = pair / d.C, c = pair - v * d.C;
    const int var = leaf_var[s0 + v], r = leaf_replica[leaf];
    const size_t ph = phi_off + ((size_t)(var * d.C + c) * d.R + r) * d.T * d.K + k;
    stats[ph] += n1;
    if (d.T == 2) stats[ph + d.K] += n2;
    if (c == 0) {
        const size_t o = ((size_t)var * d.R + r) * d.K + k;
        stats[den_off + o] += den;
        stats[tot_off + o] += tot;
    }
}

// Last launch of the top-down pass: leaf statistics in the first n_leaf_blocks workgroups, mixing
// statistics in the others (item = idx / max_children, child = idx % max_children).  NCH = 0 selects the
// kernel body for long scopes (chunks_per_leaf workgroups per leaf).
template <int NCH>
__global__ __launch_bounds__(1024) void k_tail_backward(
    int n_leaf_blocks, int max_children, const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var,
    const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica, int n_lv,
    const float* __restrict__ x, const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G,
    float* __restrict__ stats, int64_t phi_off, int64_t den_off, int64_t tot_off, const int32_t* __restrict__ m_node,
    const int32_t* __restrict__ m_kout, const int32_t* __restrict__ m_cptr, const int32_t* __restrict__ m_child,
    const int32_t* __restrict__ m_voff, const float* __restrict__ params, const float* __restrict__ A,
    const double* __restrict__ Off, const int32_t* __restrict__ leaf_sptr, const int32_t* __restrict__ leaf_var,
    int chunks_per_leaf, Dims d) {
    const int blk = blockIdx.x;
    if (blk < n_leaf_blocks) {
        if constexpr (NCH == 0)
            leaf_backward_cells_body(blk, chunks_per_leaf, leaf_node, leaf_replica, leaf_sptr, leaf_var, x, mask,
                                     mask_mode, G, stats, phi_off, den_off, tot_off, d);
        else
            leaf_backward_body<NCH>(blk, lv_leaf, lv_var, leaf_node, leaf_replica, n_lv, x, mask, mask_mode, G, stats,
                                    phi_off, den_off, tot_off, d);
    } else {
        const int idx = blk - n_leaf_blocks;
        mixing_stats_body(idx / max_children, idx % max_children, m_node, m_kout, m_cptr, m_child, m_voff, params,
                          stats, A, Off, G, d.B, d.K);
    }
}

// ------------------------------------------------------------------ M-step (Eq. 7-9)
// One wave per weight row (the K*K children of a sum entry, or its C mixing weights).
// Rows of up to 64*NPL entries are held in registers, so statistics and parameters
// are each read once and written once; longer rows fall back to several passes.
template <int NPL>
__device__ __forceinline__ void update_rows_body(int block, const int32_t* __restrict__ row_off,
                                                 const int32_t* __restrict__ row_len, int n_rows, int n_lazy_rows,
                                                 int first_row, float* __restrict__ params,
                                                 float* __restrict__ stats, float step, float w_floor) {
    const int row = block * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const bool have = row >= first_row;      // rows below first_row count as zero statistics (memory is stale)
    const bool clear = row >= n_lazy_rows;   // the first rows are overwritten, not added to, by the next E-step
    const int off = row_off[row], len = row_len[row];
    if (len <= 64 * NPL) {
        float n[NPL], w[NPL];
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < NPL; ++t) {
            const int e = lane + 64 * t;
            n[t] = e < len && have ? stats[off + e] : 0.f;
            w[t] = e < len ? params[off + e] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < NPL; ++t) s += n[t];
        const float tot = wave_sum(s);
        // 1/tot overflows for a denormal total: such rows are first scaled by an exact power of two
        const float sc = tot < 0x1p-60f ? 0x1p+64f : 1.f;
        const float inv = 1.f / (tot * sc);
        float s2 = 0.f;
#pragma unroll
        for (int t = 0; t < NPL; ++t) {
            n[t] = tot > 0.f ? (n[t] * sc) * inv : w[t];
            if (w_floor > 0.f && lane + 64 * t < len) {
                n[t] = fmaxf(n[t], w_floor);
                s2 += n[t];
            }
        }
        const float norm = w_floor > 0.f ? 1.f / wave_sum(s2) : 1.f;
#pragma unroll
        for (int t = 0; t < NPL; ++t) {
            const int e = lane + 64 * t;
            if (e < len) {
                params[off + e] = (1.f - step) * w[t] + step * (n[t] * norm);
                if (clear) stats[off + e] = 0.f;
            }
        }
        return;
    }
    float s = 0.f;
    if (have)
        for (int e = lane; e < len; e += 64) s += stats[off + e];
    const float tot = wave_sum(s);
    const float sc = tot < 0x1p-60f ? 0x1p+64f : 1.f;
    const float inv = 1.f / (tot * sc);
    float norm = 1.f;
    if (w_floor > 0.f) {
        float s2 = 0.f;
        for (int e = lane; e < len; e += 64)
            s2 += fmaxf(tot > 0.f ? (stats[off + e] * sc) * inv : params[off + e], w_floor);
        norm = 1.f / wave_sum(s2);
    }
    for (int e = lane; e < len; e += 64) {
        const float old = params[off + e];
        float hat = tot > 0.f ? (stats[off + e] * sc) * inv : old;
        if (w_floor > 0.f) hat = fmaxf(hat, w_floor) * norm;
        params[off + e] = (1.f - step) * old + step * hat;
        if (clear) stats[off + e] = 0.f;
    }
}

// Leaf M-step (Eq. 7-9, Sec. 4.2): one thread per (variable, replica, k) updates the
// parameters of all channels, clears the statistics it owns and refreshes the
// constants the leaf layer derives from the parameters.
__device__ __forceinline__ void update_leaves_body(int block, float* __restrict__ params, float* __restrict__ stats,
                                                   float* __restrict__ theta, int64_t phi_off, int64_t den_off,
                                                   int64_t tot_off, float step, float min_var, float max_var,
                                                   Dims d) {
    const int idx = block * blockDim.x + threadIdx.x;
    if (idx >= d.D * d.R * d.K) return;
    const int k = idx % d.K, r = (idx / d.K) % d.R, var = idx / (d.K * d.R);
    const size_t o = ((size_t)var * d.R + r) * d.K + k;
    const float tot = stats[tot_off + o], den = stats[den_off + o];
    stats[tot_off + o] = 0.f;
    stats[den_off + o] = 0.f;
    if (d.family == EINET_LEAF_CATEGORICAL) {
        // blend, raise to at least 1e-6, renormalise over the V values (two passes over the column)
        for (int c = 0; c < d.C; ++c) {
            const size_t e = (size_t)(var * d.C + c) * d.R + r;
            float sum = 0.f;
            for (int v = 0; v < d.P; ++v) {
                const size_t ph = phi_off + (e * d.P + v) * d.K + k;
                const float old = params[ph];
                const float hat = tot > 0.f ? (stats[ph] + (tot - den) * old) / tot : old;
                const float nw = fmaxf((1.f - step) * old + step * hat, 1e-6f);
                stats[ph] = 0.f;
                params[ph] = nw;
                sum += nw;
            }
            const float inv = 1.f / sum;
            for (int v = 0; v < d.P; ++v) {
                const size_t ph = phi_off + (e * d.P + v) * d.K + k;
                const float p = params[ph] * inv;
                params[ph] = p;
                theta[(e * d.P + v) * d.K + k] = logf(p);
            }
        }
        return;
    }
    for (int c = 0; c < d.C; ++c) {
        const size_t e = (size_t)(var * d.C + c) * d.R + r;
        float nw[2];
        for (int t = 0; t < d.T; ++t) {
            const size_t ph = phi_off + (e * d.T + t) * d.K + k;
            const float old = params[ph];
            const float hat = tot > 0.f ? (stats[ph] + (tot - den) * old) / tot : old;
            nw[t] = (1.f - step) * old + step * hat;
            stats[ph] = 0.f;
        }
        const size_t ph0 = phi_off + e * d.T * d.K + k;
        float* th = theta + e * d.TD * d.K + k;
        if (d.family == EINET_LEAF_GAUSSIAN) {
            const float mu = nw[0];
            const float var2 = fminf(fmaxf(fmaf(-mu, mu, nw[1]), min_var), max_var);
            const float m2 = fmaf(mu, mu, var2);
            params[ph0] = mu;
            params[ph0 + d.K] = m2;
            const float vd = fmaxf(fmaf(-mu, mu, m2), 1e-30f);   // as k_leaf_derive sees the stored pair
            th[0] = mu;
            th[d.K] = -0.5f / vd;
            th[2 * d.K] = -0.5f * logf(6.283185307179586f * vd);
        } else {
            const float nf = (float)d.P;               // Bernoulli: 1; binomial: phi = nf * p
            const float p = fminf(fmaxf(nw[0] / nf, 1e-6f), 1.f - 1e-6f);
            params[ph0] = nf * p;
            th[0] = logf(p);
            th[d.K] = log1pf(-p);
        }
    }
}

// The whole M-step in one launch: weight rows in the first n_row_blocks workgroups, leaves in the others.
template <int NPL>
__global__ __launch_bounds__(256) void k_em_update(int n_row_blocks, const int32_t* __restrict__ row_off,
                                                   const int32_t* __restrict__ row_len, int n_rows, int n_lazy_rows,
                                                   int first_row, float* __restrict__ params,
                                                   float* __restrict__ stats, float* __restrict__ theta, int64_t phi_off, int64_t den_off,
                                                   int64_t tot_off, float step, float min_var, float max_var,
                                                   float w_floor, Dims d) {
    if ((int)blockIdx.x < n_row_blocks)
        update_rows_body<NPL>(blockIdx.x, row_off, row_len, n_rows, n_lazy_rows, first_row, params, stats, step,
                              w_floor);
    else
        update_leaves_body(blockIdx.x - n_row_blocks, params, stats, theta, phi_off, den_off, tot_off, step, min_var,
                           max_var, d);
}

// ------------------------------------------------------------------ top-down sampling (Sec. 2, Sec. 4.2, App. D)
// sel[node][b]: entry of the node that sample b uses, -1 if the sample does not reach the node.  In a
// decomposable circuit a sample reaches a region at most once (two paths to it would sit under two children
// of one product, whose scopes are disjoint), so the writes below never collide.
__global__ void k_sample_init(int32_t* __restrict__ sel, int64_t n, int B) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) sel[i] = i < B ? 0 : -1;              // node 0 is the root region: its single entry
}

// A choice from unnormalised weights w_0..w_{n-1} with a uniform u is the first index whose running sum
// exceeds u times the total.
//
// Region with several partitions: partition c has weight v[k][c] * S^c[k] / S[k] given the evidence
// (App. B), v[k][c] without.  One thread per (region, sample).
__global__ void k_sample_mixing(const int32_t* __restrict__ m_node, const int32_t* __restrict__ m_cptr,
                                const int32_t* __restrict__ m_child, const int32_t* __restrict__ m_voff,
                                int evidence, const float* __restrict__ params, const float* __restrict__ A,
                                const double* __restrict__ Off, const float* __restrict__ u, int num_partitions,
                                int32_t* __restrict__ sel, int B, int K) {
    const int item = blockIdx.x, b = blockIdx.y * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int s = m_node[item];
    const int k = sel[(size_t)s * B + b];
    if (k < 0) return;
    const int c0 = m_cptr[item], nc = m_cptr[item + 1] - c0;
    const float* v = params + m_voff[item] + (size_t)k * nc;
    const size_t srow = (size_t)s * B + b;
    float total = 0.f;
    for (int c = 0; c < nc; ++c) {
        const size_t row = (size_t)m_child[c0 + c] * B + b;
        total += evidence ? v[c] * expf((float)(Off[row] - Off[srow]) + A[row * K + k] - A[srow * K + k]) : v[c];
    }
    const float tau = u[(size_t)(num_partitions + s) * B + b] * total;
    float run = 0.f;
    int pick = -1, last = 0;
    for (int c = 0; c < nc; ++c) {
        const size_t row = (size_t)m_child[c0 + c] * B + b;
        const float w = evidence ? v[c] * expf((float)(Off[row] - Off[srow]) + A[row * K + k] - A[srow * K + k]) : v[c];
        run += w;
        if (w > 0.f) last = c;
        if (pick < 0 && run > tau) pick = c;
    }
    if (pick < 0) pick = last;                       // u so close to 1 that rounding ate the last interval
    sel[(size_t)m_child[c0 + pick] * B + b] = k;
}

// Partition: the pair (i, j) has weight W[k][i][j] * eL[i] * eR[j] given the evidence (the posterior of
// Eq. 6 for the chosen output entry k), W[k][i][j] without; pairs are numbered i * K + j.  One wave per
// (item, sample): the K*K weights go to LDS, every lane sums a run of consecutive pairs, a wave scan of
// the run sums finds the run that holds the threshold and its lane walks it.
constexpr int SAMPLE_WAVES = 4;
__device__ __forceinline__ int sample_pos(int t) { return t + (t >> 5); }   // padded: runs start in different banks

__global__ __launch_bounds__(64 * SAMPLE_WAVES) void k_sample_einsum(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_woff, const int32_t* __restrict__ e_part, int evidence,
    const float* __restrict__ params, const float* __restrict__ A, const float* __restrict__ amax,
    const float* __restrict__ u, int32_t* __restrict__ sel, int item0, int B, int K) {
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = blockIdx.x, b = blockIdx.y * SAMPLE_WAVES + wave;
    if (b >= B) return;                              // whole waves leave: no barrier below
    const int k = sel[(size_t)e_out[li] * B + b];
    if (k < 0) return;
    const int KK = K * K;
    float* wl = lds + wave * (sample_pos(KK) + 1 + 128);
    float* el = wl + sample_pos(KK) + 1;
    float* er = el + 64;
    const int item = item0 + li;
    if (evidence) {
        const float al = amax[(size_t)item * 2 * B + b], ar = amax[((size_t)item * 2 + 1) * B + b];
        el[lane] = lane < K ? __expf(A[((size_t)e_left[li] * B + b) * K + lane] - al) : 0.f;
        er[lane] = lane < K ? __expf(A[((size_t)e_right[li] * B + b) * K + lane] - ar) : 0.f;
        __builtin_amdgcn_wave_barrier();
    }
    const float* row = params + e_woff[li] + (size_t)k * KK;
    for (int t = lane; t < KK; t += 64) {
        float w = row[t];
        if (evidence) {
            const int i = t / K, j = t - i * K;
            w *= el[i] * er[j];
        }
        wl[sample_pos(t)] = w;
    }
    __builtin_amdgcn_wave_barrier();                 // a wave reads back only its own part of LDS
    const int chunk = (KK + 63) >> 6;
    const int t0 = min(lane * chunk, KK), t1 = min(t0 + chunk, KK);
    float part = 0.f;
    for (int t = t0; t < t1; ++t) part += wl[sample_pos(t)];
    float incl = part;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    const float total = __shfl(incl, 63, 64);
    const float tau = u[(size_t)e_part[li] * B + b] * total;
    const unsigned long long hit = __ballot(incl > tau && t1 > t0);
    int pick = -1;
    if (hit != 0ull) {
        const int owner = __ffsll((long long)hit) - 1;
        if (lane == owner) {
            float run = incl - part;
            int last = t0;
            for (int t = t0; t < t1; ++t) {
                const float w = wl[sample_pos(t)];
                run += w;
                if (w > 0.f) last = t;
                if (pick < 0 && run > tau) pick = t;
            }
            if (pick < 0) pick = last;               // the run's own sum exceeded tau, its walk did not: rounding
        }
        pick = __shfl(pick, owner, 64);
    } else {
        // u so close to 1 that rounding ate the last interval: the last pair of non-zero weight
        int last = -1;
        for (int t = t0; t < t1; ++t)
            if (wl[sample_pos(t)] > 0.f) last = t;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) last = max(last, __shfl_xor(last, o, 64));
        pick = max(last, 0);
    }
    if (lane == 0) {
        const int i = pick / K;
        sel[(size_t)e_left[li] * B + b] = i;
        sel[(size_t)e_right[li] * B + b] = pick - i * K;
    }
}

// Leaves: one thread per (leaf variable, sample).  An observed variable keeps its value; the others take the
// mean of the chosen entry (noise == NULL), mean + sd * noise (Gaussian, noise standard normal) or
// noise < p (Bernoulli, noise uniform).
__global__ void k_sample_leaves(const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var,
                                const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica,
                                int n_lv, const float* __restrict__ x, const uint8_t* __restrict__ mask, int mask_mode,
                                const float* __restrict__ phi, const float* __restrict__ noise,
                                const int32_t* __restrict__ logc, const int32_t* __restrict__ sel,
                                float* __restrict__ out, Dims d) {
    const int lv = blockIdx.x * blockDim.x + threadIdx.x, b = blockIdx.y;
    if (lv >= n_lv) return;
    const int leaf = lv_leaf[lv], var = lv_var[lv];
    const int k = sel[(size_t)leaf_node[leaf] * d.B + b];
    if (k < 0) return;
    bool obs = false;
    if (mask_mode == EINET_MASK_SHARED) obs = mask[var] != 0;
    if (mask_mode == EINET_MASK_PER_SAMPLE) obs = mask[(size_t)b * d.D + var] != 0;
    const int r = leaf_replica[leaf];
    for (int c = 0; c < d.C; ++c) {
        const size_t o = ((size_t)b * d.D + var) * d.C + c;
        if (obs) {
            out[o] = x[o];
            continue;
        }
        const float* ph = phi + (((size_t)var * d.C + c) * d.R + r) * d.T * d.K + k;
        const float mean = ph[0];
        float val = mean;
        if (d.family == EINET_LEAF_CATEGORICAL) {
            float total = 0.f, ev = 0.f;
            for (int v = 0; v < d.P; ++v) {
                total += ph[(size_t)v * d.K];
                ev = fmaf((float)v, ph[(size_t)v * d.K], ev);
            }
            val = ev;                                                    // E[x]
            if (noise) {
                const float tau = noise[o] * total;
                float run = 0.f;
                int pick = -1, last = 0;
                for (int v = 0; v < d.P; ++v) {
                    const float w = ph[(size_t)v * d.K];
                    run += w;
                    if (w > 0.f) last = v;
                    if (pick < 0 && run > tau) pick = v;
                }
                val = (float)(pick < 0 ? last : pick);
            }
        } else if (d.family == EINET_LEAF_BINOMIAL) {
            if (noise) {
                const float p = mean / (float)d.P;
                const float lp = logf(p), l1p = log1pf(-p);
                float total = 0.f;
                for (int v = 0; v <= d.P; ++v)
                    total += expf(__int_as_float(logc[v]) + (float)v * lp + (float)(d.P - v) * l1p);
                const float tau = noise[o] * total;
                float run = 0.f;
                int pick = -1, last = 0;
                for (int v = 0; v <= d.P; ++v) {
                    const float w = expf(__int_as_float(logc[v]) + (float)v * lp + (float)(d.P - v) * l1p);
                    run += w;
                    if (w > 0.f) last = v;
                    if (pick < 0 && run > tau) pick = v;
                }
                val = (float)(pick < 0 ? last : pick);
            }
        } else if (noise) {
            if (d.family == EINET_LEAF_GAUSSIAN) val = mean + sqrtf(fmaxf(ph[d.K] - mean * mean, 0.f)) * noise[o];
            else val = noise[o] < mean ? 1.f : 0.f;
        }
        out[o] = val;
    }
}

// ------------------------------------------------------------------ random initial parameters
// Counter-based: parameter number p of the flat buffer uses output p + 1 of the SplitMix64 stream started at
// `seed`; its top 23 bits plus one half, over 2^23, are a uniform in (0, 1) that float32 holds exactly.
__device__ __forceinline__ float init_uniform(uint64_t seed, uint64_t p) {
    uint64_t z = seed + (p + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return ((float)(z >> 41) + 0.5f) * 0x1p-23f;
}

// Weight rows (one wave each): normalised unit exponentials, i.e. a draw from the flat Dirichlet distribution.
// Leaves (one thread per (variable, replica, entry) in the remaining workgroups): uniform in [lo, hi] for the
// Bernoulli p, the Gaussian mean (variance 1) and the binomial E[x] / N; categorical tables as the weight rows.
__global__ __launch_bounds__(256) void k_init_params(int n_row_blocks, const int32_t* __restrict__ row_off,
                                                     const int32_t* __restrict__ row_len, int n_rows,
                                                     float* __restrict__ params, int64_t phi_off, uint64_t seed,
                                                     float lo, float hi, Dims d) {
    if ((int)blockIdx.x < n_row_blocks) {
        const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
        if (row >= n_rows) return;
        const int off = row_off[row], len = row_len[row];
        float s = 0.f;
        for (int e = lane; e < len; e += 64) s += -logf(init_uniform(seed, (uint64_t)(off + e)));
        const float inv = 1.f / wave_sum(s);
        for (int e = lane; e < len; e += 64) params[off + e] = -logf(init_uniform(seed, (uint64_t)(off + e))) * inv;
        return;
    }
    const int idx = (blockIdx.x - n_row_blocks) * blockDim.x + threadIdx.x;
    if (idx >= d.D * d.R * d.K) return;
    const int k = idx % d.K, r = (idx / d.K) % d.R, var = idx / (d.K * d.R);
    for (int c = 0; c < d.C; ++c) {
        const size_t e = (size_t)(var * d.C + c) * d.R + r;
        const size_t ph = (size_t)phi_off + e * d.T * d.K + k;
        if (d.family == EINET_LEAF_CATEGORICAL) {
            float s = 0.f;
            for (int v = 0; v < d.P; ++v) s += -logf(init_uniform(seed, ph + (size_t)v * d.K));
            const float inv = 1.f / s;
            for (int v = 0; v < d.P; ++v)
                params[ph + (size_t)v * d.K] = -logf(init_uniform(seed, ph + (size_t)v * d.K)) * inv;
        } else {
            const float first = lo + (hi - lo) * init_uniform(seed, ph);
            params[ph] = d.family == EINET_LEAF_BINOMIAL ? (float)d.P * first : first;
            if (d.family == EINET_LEAF_GAUSSIAN) params[ph + d.K] = fmaf(first, first, 1.f);
        }
    }
}

// Mixture of circuits (Sec. 4.2): out[b] = log sum_c exp(log_coef[c] + lp[c][b]); thread per sample, the
// component rows are read coalesced across samples.
__global__ void k_mixture_logp(const float* __restrict__ lp, const float* __restrict__ log_coef, int n_components,
                               int B, float* __restrict__ out) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    float m = -INFINITY;
    for (int c = 0; c < n_components; ++c) m = fmaxf(m, log_coef[c] + lp[(size_t)c * B + b]);
    if (m == -INFINITY) {
        out[b] = -INFINITY;
        return;
    }
    float sum = 0.f;
    for (int c = 0; c < n_components; ++c) sum += expf(log_coef[c] + lp[(size_t)c * B + b] - m);
    out[b] = m + logf(sum);
}

__global__ void k_fill(float* __restrict__ p, float value, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = value;
}

}  // namespace

// ====================================================================== launchers
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

template <int KQ>
static void launch_einsum_forward_kq(const DevTables& t, int first, int count, const float* params, float* A,
                                     double* Off, float* amax, float* logp, const Dims& d, hipStream_t s) {
    const int nkt = (d.K + 3) / 4;
    const int n_btiles = (d.B + 15) / 16;
    const int nw = n_btiles < 8 ? n_btiles : 8;
    const size_t lds = sizeof(float) * FwdLayout<KQ>::LDS_FLOATS;
    static bool attr_set = false;
    if (lds > 64 * 1024 && !attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_einsum_forward<KQ>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    hipLaunchKernelGGL(k_einsum_forward<KQ>, dim3(count * nkt), dim3(64 * nw), lds, s, t.ein_left + first,
                       t.ein_right + first, t.ein_out + first, t.ein_kout + first, t.ein_woff + first, params, A, Off,
                       amax, logp, first, d.B, d.K, nkt);
}

void launch_einsum_forward(const DevTables& t, int first, int count, const float* params, float* A, double* Off,
                           float* amax, float* logp, const Dims& d, hipStream_t s) {
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_einsum_forward_kq<J>(t, first, count, params, A, Off, amax, logp, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

void launch_mixing_forward(const DevTables& t, int first, int count, int max_children, const float* params, float* A,
                           double* Off, float* logp, const Dims& d, hipStream_t s) {
    if (count == 0) return;
    if (max_children >= 8) {                         // a wave per output element, children over the lanes
        dim3 grid(count, (d.B * d.K + 3) / 4);
        hipLaunchKernelGGL(k_mixing_forward_many, grid, dim3(256), 0, s, t.mix_node + first, t.mix_kout + first,
                           t.mix_cptr + first, t.mix_child, t.mix_voff + first, params, A, Off, logp, d.B, d.K);
        return;
    }
    dim3 grid(count, (d.B * d.K + 255) / 256);
    hipLaunchKernelGGL(k_mixing_forward, grid, dim3(256), 0, s, t.mix_node + first, t.mix_kout + first,
                       t.mix_cptr + first, t.mix_child, t.mix_voff + first, params, A, Off, logp, d.B, d.K);
}

void launch_region_assemble(const DevTables& t, int first, int count, bool is_root_layer, float* G, const float* Gp,
                            const Dims& d, hipStream_t s) {
    if (count == 0) return;
    dim3 grid(count, (d.B * d.K + 255) / 256);
    hipLaunchKernelGGL(k_region_assemble, grid, dim3(256), 0, s, t.rb_node + first, t.rb_kout + first,
                       t.rb_pptr + first, t.rb_pblk, is_root_layer ? 1 : 0, G, Gp, d.B, d.K);
}

template <int KQ>
static void launch_einsum_backward_kq(const DevTables& t, int first, int count, bool accumulate,
                                      const float* params, float* stats, const float* A, const double* Off,
                                      const float* amax, const float* G, float* Gp, const Dims& d, hipStream_t s) {
    const size_t lds = sizeof(float) * BwdLayout<KQ>::LDS_FLOATS;
    static bool attr_set = false;
    if (lds > 64 * 1024 && !attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_einsum_backward<KQ, true, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_einsum_backward<KQ, false, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_einsum_backward<KQ, true, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_einsum_backward<KQ, false, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const int ngroups = bwd_groups_per_item(count, d.K);
#define EINET_LAUNCH(V, ACC)                                                                                      \
    hipLaunchKernelGGL((k_einsum_backward<KQ, V, ACC>), dim3(count * ngroups), dim3(512), lds, s, t.ein_left + first,  \
                       t.ein_right + first, t.ein_out + first, t.ein_reg + first, t.ein_kout + first,                 \
                       t.ein_woff + first, t.ein_voff + first, t.ein_vstr + first, params, stats, A, Off, amax, G, Gp,  \
                       first, ngroups, d.B, d.K)
    if ((d.K & 3) == 0) {
        if (accumulate) EINET_LAUNCH(true, true);
        else EINET_LAUNCH(true, false);
    } else {
        if (accumulate) EINET_LAUNCH(false, true);
        else EINET_LAUNCH(false, false);
    }
#undef EINET_LAUNCH
}

void launch_einsum_backward(const DevTables& t, int first, int count, bool accumulate, const float* params,
                            float* stats, const float* A, const double* Off, const float* amax, const float* G,
                            float* Gp, const Dims& d, hipStream_t s) {
    if (count == 0) return;
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_einsum_backward_kq<J>(t, first, count, accumulate, params, stats, A, Off, amax, G, Gp, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

void launch_tail_backward(const DevTables& t, int n_lv, int n_leaves, int max_scope, int n_mix, int max_children,
                          const float* x, const uint8_t* mask, int mask_mode, const float* params, const float* A,
                          const double* Off, const float* G, float* stats, int64_t phi_off, int64_t den_off,
                          int64_t tot_off, const Dims& d, hipStream_t s) {
    const int total = n_lv * d.C * d.K;
    const bool categorical = d.family == EINET_LEAF_CATEGORICAL;
    if (categorical)     // indicator statistics: a histogram kernel of its own (at most 256 x 64 floats of LDS)
        hipLaunchKernelGGL(k_leaf_backward_categorical, dim3(n_lv * d.C), dim3(64), sizeof(float) * d.P * d.K, s,
                           t.lv_leaf, t.lv_var, t.leaf_node, t.leaf_replica, x, mask, mask_mode, G, stats, phi_off,
                           den_off, tot_off, d);
    // long scopes: posterior block and values through LDS; short ones: straight from memory
    const int cell_chunks = (max_scope * d.C + cell_pairs_per_group(d.K) - 1) / cell_pairs_per_group(d.K);
    // (with fewer than 64 such workgroups the chip is better filled by the element-wise kernel)
    const bool cells = !categorical && max_scope * d.C >= 32 && n_leaves * cell_chunks >= 64;
    const int nch = cells ? 0 : (d.B >= 16 ? 4 : 1);
    const int chunks_per_leaf = cells ? cell_chunks : 1;
    const int n_leaf_blocks = categorical ? 0 : (cells ? n_leaves * chunks_per_leaf : (total + 1024 / nch - 1) / (1024 / nch));
    const int blocks = n_leaf_blocks + n_mix * max_children;
    if (blocks == 0) return;
    const size_t lds = cells ? cell_lds_bytes(d.K) : 0;
    static bool attr_set = false;
    if (cells && !attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tail_backward<0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        attr_set = true;
    }
#define EINET_LAUNCH(N)                                                                                              \
    hipLaunchKernelGGL(k_tail_backward<N>, dim3(blocks), dim3(1024), lds, s, n_leaf_blocks,                           \
                       max_children > 0 ? max_children : 1, t.lv_leaf, t.lv_var, t.leaf_node, t.leaf_replica, n_lv, x, \
                       mask, mask_mode, G, stats, phi_off, den_off, tot_off, t.mix_node, t.mix_kout, t.mix_cptr,      \
                       t.mix_child, t.mix_voff, params, A, Off, t.leaf_sptr, t.leaf_var, chunks_per_leaf, d)
    if (nch == 0) EINET_LAUNCH(0);
    else if (nch == 4) EINET_LAUNCH(4);
    else EINET_LAUNCH(1);
#undef EINET_LAUNCH
}

void launch_em_update(const DevTables& t, int n_rows, int n_lazy_rows, bool lazy_rows_are_zero, float* params,
                      float* stats, float* theta,
                      int64_t phi_off, int64_t den_off, int64_t tot_off, float step, float min_var, float max_var,
                      float w_floor, const Dims& d, hipStream_t s) {
    const int n_row_blocks = (n_rows + 3) / 4;
    const int n_leaf_blocks = (d.D * d.R * d.K + 255) / 256;
    // registers per lane for a weight row of K*K entries (mixing rows are shorter)
    const int per_lane = (d.K * d.K + 63) / 64;
#define EINET_LAUNCH(N)                                                                                             \
    hipLaunchKernelGGL(k_em_update<N>, dim3(n_row_blocks + n_leaf_blocks), dim3(256), 0, s, n_row_blocks, t.row_off, \
                       t.row_len, n_rows, n_lazy_rows, lazy_rows_are_zero ? n_lazy_rows : 0, params, stats, theta,    \
                       phi_off, den_off, tot_off, step, min_var, max_var, w_floor, d)
    if (per_lane <= 2) EINET_LAUNCH(2);
    else if (per_lane <= 8) EINET_LAUNCH(8);
    else EINET_LAUNCH(32);
#undef EINET_LAUNCH
}

void launch_mixture_logp(const float* lp, const float* log_coef, int n_components, int B, float* out, hipStream_t s) {
    hipLaunchKernelGGL(k_mixture_logp, dim3((B + 255) / 256), dim3(256), 0, s, lp, log_coef, n_components, B, out);
}

void launch_sample_init(int32_t* sel, int num_nodes, int B, hipStream_t s) {
    const int64_t n = (int64_t)num_nodes * B;
    hipLaunchKernelGGL(k_sample_init, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, sel, n, B);
}

void launch_sample_mixing(const DevTables& t, int first, int count, bool evidence, const float* params,
                          const float* A, const double* Off, const float* u, int num_partitions, int32_t* sel,
                          const Dims& d, hipStream_t s) {
    if (count == 0) return;
    hipLaunchKernelGGL(k_sample_mixing, dim3(count, (d.B + 63) / 64), dim3(64), 0, s, t.mix_node + first,
                       t.mix_cptr + first, t.mix_child, t.mix_voff + first, evidence ? 1 : 0, params, A, Off, u,
                       num_partitions, sel, d.B, d.K);
}

void launch_sample_einsum(const DevTables& t, int first, int count, bool evidence, const float* params,
                          const float* A, const float* amax, const float* u, int32_t* sel, const Dims& d,
                          hipStream_t s) {
    if (count == 0) return;
    const int KK = d.K * d.K;
    const size_t lds = sizeof(float) * SAMPLE_WAVES * (size_t)(KK + (KK >> 5) + 1 + 128);   // at most 68 KB (K = 64)
    static bool attr_set = false;
    if (lds > 64 * 1024 && !attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_sample_einsum),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024);
        attr_set = true;
    }
    hipLaunchKernelGGL(k_sample_einsum, dim3(count, (d.B + SAMPLE_WAVES - 1) / SAMPLE_WAVES), dim3(64 * SAMPLE_WAVES),
                       lds, s, t.ein_left + first, t.ein_right + first, t.ein_out + first, t.ein_woff + first,
                       t.ein_part + first, evidence ? 1 : 0, params, A, amax, u, sel, first, d.B, d.K);
}

void launch_sample_leaves(const DevTables& t, int n_lv, const float* x, const uint8_t* mask, int mask_mode,
                          const float* phi, const float* noise, const int32_t* sel, float* out, const Dims& d,
                          hipStream_t s) {
    hipLaunchKernelGGL(k_sample_leaves, dim3((n_lv + 255) / 256, d.B), dim3(256), 0, s, t.lv_leaf, t.lv_var,
                       t.leaf_node, t.leaf_replica, n_lv, x, mask, mask_mode, phi, noise, t.leaf_logc, sel, out, d);
}

void launch_init_params(const DevTables& t, int n_rows, float* params, int64_t phi_off, uint64_t seed, float lo,
                        float hi, const Dims& d, hipStream_t s) {
    const int n_row_blocks = (n_rows + 3) / 4;
    const int n_leaf_blocks = (d.D * d.R * d.K + 255) / 256;
    hipLaunchKernelGGL(k_init_params, dim3(n_row_blocks + n_leaf_blocks), dim3(256), 0, s, n_row_blocks, t.row_off,
                       t.row_len, n_rows, params, phi_off, seed, lo, hi, d);
}

void launch_fill(float* p, float value, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_fill, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, p, value, n);
}

}  // namespace einet_impl
