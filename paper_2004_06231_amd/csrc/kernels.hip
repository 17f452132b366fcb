// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts).
//
// Activations live in a node-major arena A[node][b][k] (float32, log domain):
// every region and every simple sum owns one dense [B][K] block, so a layer's
// "gather" of left and right inputs (Sec. 3.3) is an index lookup.  The
// posterior arena G has the same shape; Gp[2e+side][b][k] holds what einsum
// item e sends down to its left (side 0) or right (side 1) child, and a child
// sums the slots of its parents when it is processed: no atomics anywhere.
#include "kernels.hpp"

#include <cmath>

namespace einet_impl {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KMAX = 64;  // largest vector length K

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
                              int family) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_entries * K) return;
    int e = idx / K, k = idx - e * K;
    if (family == EINET_LEAF_GAUSSIAN) {
        float m = phi[(e * 2 + 0) * K + k], s = phi[(e * 2 + 1) * K + k];
        float var = fmaxf(fmaf(-m, m, s), 1e-30f);
        theta[(e * 3 + 0) * K + k] = m;
        theta[(e * 3 + 1) * K + k] = -0.5f / var;
        theta[(e * 3 + 2) * K + k] = -0.5f * logf(6.283185307179586f * var);
    } else {
        float p = phi[e * K + k];
        theta[(e * 2 + 0) * K + k] = logf(p);
        theta[(e * 2 + 1) * K + k] = log1pf(-p);
    }
}

// Leaf layer: A[leaf][b][k] = sum over the leaf's scope and the channels of the
// log-density of x under entry k; a marginalised variable contributes 0.
__global__ void k_leaf_forward(const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica,
                               const int32_t* __restrict__ leaf_sptr, const int32_t* __restrict__ leaf_var,
                               const float* __restrict__ x, const uint8_t* __restrict__ mask, int mask_mode,
                               const float* __restrict__ theta, float* __restrict__ A, Dims d) {
    const int leaf = blockIdx.x;
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= d.B * d.K) return;
    const int b = e / d.K, k = e - b * d.K;
    const int r = leaf_replica[leaf];
    float acc = 0.f;
    for (int v = leaf_sptr[leaf]; v < leaf_sptr[leaf + 1]; ++v) {
        const int var = leaf_var[v];
        if (mask_mode == EINET_MASK_SHARED && !mask[var]) continue;
        if (mask_mode == EINET_MASK_PER_SAMPLE && !mask[(size_t)b * d.D + var]) continue;
        for (int c = 0; c < d.C; ++c) {
            const float xv = x[((size_t)b * d.D + var) * d.C + c];
            const float* th = theta + ((size_t)(var * d.C + c) * d.R + r) * d.TD * d.K + k;
            if (d.family == EINET_LEAF_GAUSSIAN) {
                const float diff = xv - th[0];
                acc += fmaf(th[d.K] * diff, diff, th[2 * d.K]);
            } else {
                acc += xv * th[0] + (1.f - xv) * th[d.K];
            }
        }
    }
    A[((size_t)leaf_node[leaf] * d.B + b) * d.K + k] = acc;
}

// ------------------------------------------------------------------ einsum layer, forward
// One workgroup per (einsum item, tile of 16 samples).  With eL = exp(L - a),
// eR = exp(R - a') (a, a' the row maxima; Eq. 4) the layer needs
//     S[b,k] = sum_i eL[b,i] * T[(k,i), b],   T[(k,i), b] = sum_j W[k,i,j] eR[b,j].
// T is a dense GEMM (rows (k,i), columns b, contraction j) done with
// v_mfma_f32_16x16x4_f32: a wave takes 4 outputs k (one per 16-lane group) and
// 4 inputs i (one per accumulator register) at a time, so the i-reduction of
// Eq. 4 is four in-lane FMAs per tile and the outer product of Sec. 3.2 is
// never formed.  The contraction index is split in four contiguous chunks of
// JC = ceil(K/4), one per lane group; the order of a sum's terms is free.
template <int JC>
__global__ __launch_bounds__(512) void k_einsum_forward(const int32_t* __restrict__ e_left,
                                                        const int32_t* __restrict__ e_right,
                                                        const int32_t* __restrict__ e_out,
                                                        const int32_t* __restrict__ e_kout,
                                                        const int32_t* __restrict__ e_woff,
                                                        const float* __restrict__ params, float* __restrict__ A,
                                                        int B, int K, int n_btiles) {
    constexpr int KP = 4 * JC;
    __shared__ float sL[16 * KP];
    __shared__ float sR[16 * KP];
    __shared__ float sM[32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int item = blockIdx.x / n_btiles, bt = blockIdx.x - item * n_btiles;
    const int kout = e_kout[item];
    const float* Lp = A + (size_t)e_left[item] * B * K;
    const float* Rp = A + (size_t)e_right[item] * B * K;
    const float* W = params + e_woff[item];

    for (int idx = tid; idx < 16 * KP; idx += blockDim.x) {
        const int row = idx / KP, col = idx - row * KP, b = bt * 16 + row;
        float vl = -INFINITY, vr = -INFINITY;
        if (b < B && col < K) {
            vl = Lp[(size_t)b * K + col];
            vr = Rp[(size_t)b * K + col];
        }
        sL[idx] = vl;
        sR[idx] = vr;
    }
    __syncthreads();
    if (tid < 32) {
        const float* src = (tid < 16) ? sL : sR;
        const int row = tid & 15;
        float m = -INFINITY;
        for (int col = 0; col < K; ++col) m = fmaxf(m, src[row * KP + col]);
        sM[tid] = (m == -INFINITY) ? 0.f : m;   // an all-zero input vector: keep exp(-inf) = 0, no NaN
    }
    __syncthreads();
    for (int idx = tid; idx < 16 * KP; idx += blockDim.x) {
        const int row = idx / KP;
        sL[idx] = expf(sL[idx] - sM[row]);
        sR[idx] = expf(sR[idx] - sM[16 + row]);
    }
    __syncthreads();

    const int c = lane & 15, g = lane >> 4;          // sample column, lane group
    const int gm = c >> 2, rm = c & 3;               // as A-operand lane: row 4*gm+rm -> (k = 4kt+gm, i = 4it+rm)
    float er[JC];
#pragma unroll
    for (int s = 0; s < JC; ++s) er[s] = sR[c * KP + g * JC + s];
    const int b = bt * 16 + c;
    const int nkt = (kout + 3) >> 2;
    for (int kt = wave; kt < nkt; kt += nwaves) {
        const int ka = 4 * kt + gm;
        float sacc = 0.f;
        for (int it = 0; it < JC; ++it) {
            const int ia = 4 * it + rm;
            const bool row_ok = (ka < kout) && (ia < K);
            const float* wrow = W + ((size_t)ka * K + ia) * K + g * JC;
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < JC; ++s) {
                const float w = (row_ok && (g * JC + s < K)) ? wrow[s] : 0.f;
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w, er[s], acc, 0, 0, 0);
            }
            const float* el = sL + c * KP + 4 * it;
            sacc += acc[0] * el[0] + acc[1] * el[1] + acc[2] * el[2] + acc[3] * el[3];
        }
        const int k = 4 * kt + g;
        if (b < B && k < kout) A[((size_t)e_out[item] * B + b) * K + k] = sM[c] + sM[16 + c] + logf(sacc);
    }
}

// ------------------------------------------------------------------ mixing layer, forward (App. B)
__global__ void k_mixing_forward(const int32_t* __restrict__ m_node, const int32_t* __restrict__ m_kout,
                                 const int32_t* __restrict__ m_cptr, const int32_t* __restrict__ m_child,
                                 const int32_t* __restrict__ m_voff, const float* __restrict__ params,
                                 float* __restrict__ A, int B, int K) {
    const int item = blockIdx.x;
    const int kout = m_kout[item];
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= B * kout) return;
    const int b = e / kout, k = e - b * kout;
    const int c0 = m_cptr[item], nc = m_cptr[item + 1] - c0;
    const float* v = params + m_voff[item] + (size_t)k * nc;
    float m = -INFINITY;
    for (int c = 0; c < nc; ++c) m = fmaxf(m, A[((size_t)m_child[c0 + c] * B + b) * K + k]);
    if (m == -INFINITY) m = 0.f;
    float s = 0.f;
    for (int c = 0; c < nc; ++c) s += v[c] * expf(A[((size_t)m_child[c0 + c] * B + b) * K + k] - m);
    A[((size_t)m_node[item] * B + b) * K + k] = m + logf(s);
}

__global__ void k_copy_root(const float* __restrict__ A, float* __restrict__ logp, int B, int K) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) logp[b] = A[(size_t)b * K];   // node 0 is the root region, entry 0
}

// ------------------------------------------------------------------ top-down pass, regions
// One workgroup per region of the layer.  G[region] = sum of the slots its
// parent partitions wrote (1 at the root).  A region with several partitions
// also splits its posterior among its simple sums, rho = v * S^c / S (derivative
// of the mixture of App. B), and adds sum_b G*rho to the mixing statistics.
__global__ __launch_bounds__(256) void k_region_backward(
    const int32_t* __restrict__ r_node, const int32_t* __restrict__ r_kout, const int32_t* __restrict__ r_mix,
    const int32_t* __restrict__ r_pptr, const int32_t* __restrict__ r_pslot, const int32_t* __restrict__ m_cptr,
    const int32_t* __restrict__ m_child, const int32_t* __restrict__ m_voff, int is_root,
    const float* __restrict__ params, float* __restrict__ stats, const float* __restrict__ A, float* __restrict__ G,
    const float* __restrict__ Gp, int B, int K) {
    __shared__ float red[256];
    const int item = blockIdx.x, tid = threadIdx.x;
    const int node = r_node[item], kout = r_kout[item];
    const int nbl = 256 / kout;                      // sample lanes per entry
    const int k = tid % kout, bl = tid / kout;
    const bool active = bl < nbl;
    const int p0 = r_pptr[item], p1 = r_pptr[item + 1];
    if (active)
        for (int b = bl; b < B; b += nbl) {
            float g = is_root ? 1.f : 0.f;
            for (int p = p0; p < p1; ++p) g += Gp[((size_t)r_pslot[p] * B + b) * K + k];
            G[((size_t)node * B + b) * K + k] = g;
        }
    const int mix = r_mix[item];
    if (mix < 0) return;
    const int c0 = m_cptr[mix], nc = m_cptr[mix + 1] - c0;
    for (int c = 0; c < nc; ++c) {
        const int child = m_child[c0 + c];
        float part = 0.f;
        if (active) {
            const float vkc = params[m_voff[mix] + (size_t)k * nc + c];
            for (int b = bl; b < B; b += nbl) {
                const size_t o = (size_t)b * K + k;
                const float g = G[(size_t)node * B * K + o];     // written by this thread above
                float gr = 0.f;
                if (g != 0.f) gr = g * vkc * expf(A[(size_t)child * B * K + o] - A[(size_t)node * B * K + o]);
                G[(size_t)child * B * K + o] = gr;
                part += gr;
            }
        }
        red[tid] = part;
        __syncthreads();
        if (active && bl == 0) {
            float tot = 0.f;
            for (int l = 0; l < nbl; ++l) tot += red[l * kout + k];
            stats[m_voff[mix] + (size_t)k * nc + c] += tot;
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ top-down pass, einsum items
// Weight statistics (Eq. 6): Nw[k,i,j] += W[k,i,j] * sum_b Q[b,k] eL[b,i] eR[b,j],
// Q = G_out / S~ with S~ = exp(A_out - a - a') the shifted sum of Eq. 4.
// One workgroup per (item, k); the batch is walked in chunks staged in LDS.
constexpr int BW_CHUNK = 32;
__global__ __launch_bounds__(256) void k_einsum_backward_w(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_kout, const int32_t* __restrict__ e_woff, const float* __restrict__ params,
    float* __restrict__ stats, const float* __restrict__ A, const float* __restrict__ G, int B, int K) {
    __shared__ float sL[BW_CHUNK * KMAX];
    __shared__ float sR[BW_CHUNK * KMAX];
    __shared__ float sM[2 * BW_CHUNK];
    __shared__ float sQ[BW_CHUNK];
    const int item = blockIdx.x, k = blockIdx.y, tid = threadIdx.x;
    if (k >= e_kout[item]) return;
    const float* Lp = A + (size_t)e_left[item] * B * K;
    const float* Rp = A + (size_t)e_right[item] * B * K;
    const float* Op = A + (size_t)e_out[item] * B * K;
    const float* Gout = G + (size_t)e_out[item] * B * K;
    const int KK = K * K;
    float acc[KMAX * KMAX / 256];
#pragma unroll
    for (int m = 0; m < KMAX * KMAX / 256; ++m) acc[m] = 0.f;
    for (int b0 = 0; b0 < B; b0 += BW_CHUNK) {
        const int nb = min(BW_CHUNK, B - b0);
        for (int idx = tid; idx < nb * K; idx += 256) {
            sL[idx] = Lp[(size_t)b0 * K + idx];
            sR[idx] = Rp[(size_t)b0 * K + idx];
        }
        __syncthreads();
        if (tid < 2 * nb) {
            const float* src = (tid < nb) ? sL : sR;
            const int row = (tid < nb) ? tid : tid - nb;
            float m = -INFINITY;
            for (int col = 0; col < K; ++col) m = fmaxf(m, src[row * K + col]);
            sM[tid] = (m == -INFINITY) ? 0.f : m;
        }
        __syncthreads();
        for (int idx = tid; idx < nb * K; idx += 256) {
            const int row = idx / K;
            sL[idx] = expf(sL[idx] - sM[row]);
            sR[idx] = expf(sR[idx] - sM[nb + row]);
        }
        if (tid < nb) {
            const float g = Gout[(size_t)(b0 + tid) * K + k];
            sQ[tid] = (g != 0.f) ? g * expf(sM[tid] + sM[nb + tid] - Op[(size_t)(b0 + tid) * K + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < KMAX * KMAX / 256; ++m) {
            const int ij = tid + m * 256;
            if (ij < KK) {
                const int i = ij / K, j = ij - i * K;
                float a = 0.f;
                for (int b = 0; b < nb; ++b) a = fmaf(sQ[b] * sL[b * K + i], sR[b * K + j], a);
                acc[m] += a;
            }
        }
        __syncthreads();
    }
    const size_t base = (size_t)e_woff[item] + (size_t)k * KK;
#pragma unroll
    for (int m = 0; m < KMAX * KMAX / 256; ++m) {
        const int ij = tid + m * 256;
        if (ij < KK) stats[base + ij] += params[base + ij] * acc[m];
    }
}

// Posterior sent to the children (chain rule through Eq. 4):
//   U[b,i,j] = sum_k Q[b,k] W[k,i,j];  Gp_left[b,i] = eL[b,i] sum_j U eR[b,j];
//   Gp_right[b,j] = eR[b,j] sum_i U eL[b,i].
// One workgroup per (item, 16 samples); a wave takes 4 samples, lanes are j.
constexpr int BG_SAMPLES = 4;
__global__ __launch_bounds__(256) void k_einsum_backward_g(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_kout, const int32_t* __restrict__ e_woff, const float* __restrict__ params,
    const float* __restrict__ A, const float* __restrict__ G, float* __restrict__ Gp, int item0, int B, int K) {
    constexpr int NB = 4 * BG_SAMPLES;
    __shared__ float sL[NB * KMAX];
    __shared__ float sR[NB * KMAX];
    __shared__ float sQ[NB * KMAX];
    __shared__ float sM[2 * NB];
    const int item = item0 + blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.y * NB;
    const int nb = min(NB, B - b0);
    const int kout = e_kout[item];
    const float* Lp = A + (size_t)e_left[item] * B * K;
    const float* Rp = A + (size_t)e_right[item] * B * K;
    const float* Op = A + (size_t)e_out[item] * B * K;
    const float* Gout = G + (size_t)e_out[item] * B * K;
    const float* W = params + e_woff[item];
    for (int idx = tid; idx < NB * K; idx += 256) {
        const bool ok = idx < nb * K;
        sL[idx] = ok ? Lp[(size_t)b0 * K + idx] : -INFINITY;
        sR[idx] = ok ? Rp[(size_t)b0 * K + idx] : -INFINITY;
    }
    __syncthreads();
    if (tid < 2 * NB) {
        const float* src = (tid < NB) ? sL : sR;
        const int row = (tid < NB) ? tid : tid - NB;
        float m = -INFINITY;
        for (int col = 0; col < K; ++col) m = fmaxf(m, src[row * K + col]);
        sM[tid] = (m == -INFINITY) ? 0.f : m;
    }
    __syncthreads();
    for (int idx = tid; idx < NB * K; idx += 256) {
        const int row = idx / K, col = idx - row * K;
        sL[idx] = expf(sL[idx] - sM[row]);
        sR[idx] = expf(sR[idx] - sM[NB + row]);
        float q = 0.f;
        if (row < nb && col < kout) {
            const float g = Gout[(size_t)(b0 + row) * K + col];
            if (g != 0.f) q = g * expf(sM[row] + sM[NB + row] - Op[(size_t)(b0 + row) * K + col]);
        }
        sQ[idx] = q;
    }
    __syncthreads();
    const int j = lane;
    const bool jok = j < K;
    float accR[BG_SAMPLES], gl[BG_SAMPLES], erj[BG_SAMPLES];
#pragma unroll
    for (int s = 0; s < BG_SAMPLES; ++s) {
        accR[s] = 0.f;
        gl[s] = 0.f;
        erj[s] = jok ? sR[(wave * BG_SAMPLES + s) * K + j] : 0.f;
    }
    for (int i = 0; i < K; ++i) {
        float U[BG_SAMPLES];
#pragma unroll
        for (int s = 0; s < BG_SAMPLES; ++s) U[s] = 0.f;
        for (int k = 0; k < kout; ++k) {
            const float w = jok ? W[((size_t)k * K + i) * K + j] : 0.f;
#pragma unroll
            for (int s = 0; s < BG_SAMPLES; ++s) U[s] = fmaf(sQ[(wave * BG_SAMPLES + s) * K + k], w, U[s]);
        }
#pragma unroll
        for (int s = 0; s < BG_SAMPLES; ++s) {
            accR[s] = fmaf(U[s], sL[(wave * BG_SAMPLES + s) * K + i], accR[s]);
            const float t = wave_sum(U[s] * erj[s]);
            if (lane == i) gl[s] = t;
        }
    }
#pragma unroll
    for (int s = 0; s < BG_SAMPLES; ++s) {
        const int row = wave * BG_SAMPLES + s;
        if (row < nb && jok) {
            const size_t o = (size_t)(b0 + row) * K + j;
            Gp[(size_t)(2 * item) * B * K + o] = sL[row * K + j] * gl[s];
            Gp[(size_t)(2 * item + 1) * B * K + o] = erj[s] * accR[s];
        }
    }
}

// ------------------------------------------------------------------ top-down pass, leaves
// Posterior-weighted sufficient statistics (Eq. 6-7): one thread per
// (leaf, variable of its scope, channel, entry k) walks the batch.
__global__ void k_leaf_backward(const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var,
                                const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica,
                                int n_lv, const float* __restrict__ x, const uint8_t* __restrict__ mask,
                                int mask_mode, const float* __restrict__ G, float* __restrict__ stats,
                                int64_t phi_off, int64_t den_off, int64_t tot_off, Dims d) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_lv * d.C * d.K) return;
    const int k = idx % d.K, c = (idx / d.K) % d.C, e = idx / (d.K * d.C);
    const int leaf = lv_leaf[e], var = lv_var[e], r = leaf_replica[leaf];
    const float* Gl = G + (size_t)leaf_node[leaf] * d.B * d.K + k;
    float n1 = 0.f, n2 = 0.f, den = 0.f, tot = 0.f;
    for (int b = 0; b < d.B; ++b) {
        const float p = Gl[(size_t)b * d.K];
        float m = 1.f;
        if (mask_mode == EINET_MASK_SHARED) m = mask[var] ? 1.f : 0.f;
        if (mask_mode == EINET_MASK_PER_SAMPLE) m = mask[(size_t)b * d.D + var] ? 1.f : 0.f;
        const float xv = x[((size_t)b * d.D + var) * d.C + c];
        const float pm = p * m;
        tot += p;
        den += pm;
        n1 = fmaf(pm, xv, n1);
        n2 = fmaf(pm * xv, xv, n2);
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

// ------------------------------------------------------------------ M-step (Eq. 7-9)
// One wave per weight row (the K*K children of a sum entry, or its C mixing weights).
__global__ __launch_bounds__(256) void k_update_rows(const int32_t* __restrict__ row_off,
                                                     const int32_t* __restrict__ row_len, int n_rows,
                                                     float* __restrict__ params, float* __restrict__ stats,
                                                     float step, float w_floor) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const int off = row_off[row], len = row_len[row];
    float s = 0.f;
    for (int e = lane; e < len; e += 64) s += stats[off + e];
    const float tot = wave_sum(s);
    const float inv = tot > 0.f ? 1.f / tot : 0.f;
    float norm = 1.f;
    if (w_floor > 0.f) {
        float s2 = 0.f;
        for (int e = lane; e < len; e += 64)
            s2 += fmaxf(tot > 0.f ? stats[off + e] * inv : params[off + e], w_floor);
        norm = 1.f / wave_sum(s2);
    }
    for (int e = lane; e < len; e += 64) {
        const float old = params[off + e];
        float hat = tot > 0.f ? stats[off + e] * inv : old;
        if (w_floor > 0.f) hat = fmaxf(hat, w_floor) * norm;
        params[off + e] = (1.f - step) * old + step * hat;
        stats[off + e] = 0.f;
    }
}

__global__ void k_update_leaves(float* __restrict__ params, float* __restrict__ stats, int64_t phi_off,
                                int64_t den_off, int64_t tot_off, float step, float min_var, float max_var, Dims d) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = d.D * d.C * d.R * d.K;
    if (idx >= n) return;
    const int k = idx % d.K, e = idx / d.K;          // e = (var*C + c)*R + r
    const int r = e % d.R, var = e / (d.R * d.C);
    const size_t o = ((size_t)var * d.R + r) * d.K + k;
    const float tot = stats[tot_off + o], den = stats[den_off + o];
    float nw[2];
    for (int t = 0; t < d.T; ++t) {
        const size_t ph = phi_off + ((size_t)e * d.T + t) * d.K + k;
        const float old = params[ph];
        const float hat = tot > 0.f ? (stats[ph] + (tot - den) * old) / tot : old;
        nw[t] = (1.f - step) * old + step * hat;
        stats[ph] = 0.f;
    }
    const size_t ph0 = phi_off + (size_t)e * d.T * d.K + k;
    if (d.family == EINET_LEAF_GAUSSIAN) {
        const float mu = nw[0];
        const float var2 = fminf(fmaxf(fmaf(-mu, mu, nw[1]), min_var), max_var);
        params[ph0] = mu;
        params[ph0 + d.K] = fmaf(mu, mu, var2);
    } else {
        params[ph0] = fminf(fmaxf(nw[0], 1e-6f), 1.f - 1e-6f);
    }
}

__global__ void k_fill(float* __restrict__ p, float value, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = value;
}

int pick_waves(int nkt) {
    // waves per workgroup: the largest count up to 8 that splits the k-tiles evenly, else 4
    for (int w = 8; w >= 2; --w)
        if (nkt % w == 0) return w;
    return nkt < 4 ? nkt : 4;
}

}  // namespace

// ====================================================================== launchers
void launch_leaf_derive(const float* phi, float* theta, const Dims& d, hipStream_t s) {
    const int n = d.D * d.C * d.R;
    const int total = n * d.K;
    hipLaunchKernelGGL(k_leaf_derive, dim3((total + 255) / 256), dim3(256), 0, s, phi, theta, n, d.K, d.family);
}

void launch_leaf_forward(const DevTables& t, int n_leaves, const float* x, const uint8_t* mask, int mask_mode,
                         const float* theta, float* A, const Dims& d, hipStream_t s) {
    dim3 grid(n_leaves, (d.B * d.K + 255) / 256);
    hipLaunchKernelGGL(k_leaf_forward, grid, dim3(256), 0, s, t.leaf_node, t.leaf_replica, t.leaf_sptr, t.leaf_var, x,
                       mask, mask_mode, theta, A, d);
}

template <int JC>
static void launch_einsum_forward_jc(const DevTables& t, int first, int count, const float* params, float* A,
                                     const Dims& d, hipStream_t s) {
    const int n_btiles = (d.B + 15) / 16;
    const int nw = pick_waves((d.K + 3) / 4);
    hipLaunchKernelGGL(k_einsum_forward<JC>, dim3(count * n_btiles), dim3(64 * nw), 0, s, t.ein_left + first,
                       t.ein_right + first, t.ein_out + first, t.ein_kout + first, t.ein_woff + first, params, A, d.B,
                       d.K, n_btiles);
}

void launch_einsum_forward(const DevTables& t, int first, int count, const float* params, float* A, const Dims& d,
                           hipStream_t s) {
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_einsum_forward_jc<J>(t, first, count, params, A, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

void launch_mixing_forward(const DevTables& t, int first, int count, const float* params, float* A, const Dims& d,
                           hipStream_t s) {
    if (count == 0) return;
    dim3 grid(count, (d.B * d.K + 255) / 256);
    hipLaunchKernelGGL(k_mixing_forward, grid, dim3(256), 0, s, t.mix_node + first, t.mix_kout + first,
                       t.mix_cptr + first, t.mix_child, t.mix_voff + first, params, A, d.B, d.K);
}

void launch_copy_root(const float* A, float* logp, const Dims& d, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_root, dim3((d.B + 255) / 256), dim3(256), 0, s, A, logp, d.B, d.K);
}

void launch_region_backward(const DevTables& t, int first, int count, bool is_root_layer, const float* params,
                            float* stats, const float* A, float* G, const float* Gp, const Dims& d, hipStream_t s) {
    if (count == 0) return;
    hipLaunchKernelGGL(k_region_backward, dim3(count), dim3(256), 0, s, t.rb_node + first, t.rb_kout + first,
                       t.rb_mix + first, t.rb_pptr + first, t.rb_pslot, t.mix_cptr, t.mix_child, t.mix_voff,
                       is_root_layer ? 1 : 0, params, stats, A, G, Gp, d.B, d.K);
}

void launch_einsum_backward(const DevTables& t, int first, int count, const float* params, float* stats,
                            const float* A, const float* G, float* Gp, const Dims& d, hipStream_t s) {
    if (count == 0) return;
    hipLaunchKernelGGL(k_einsum_backward_w, dim3(count, d.K), dim3(256), 0, s, t.ein_left + first, t.ein_right + first,
                       t.ein_out + first, t.ein_kout + first, t.ein_woff + first, params, stats, A, G, d.B, d.K);
    hipLaunchKernelGGL(k_einsum_backward_g, dim3(count, (d.B + 15) / 16), dim3(256), 0, s, t.ein_left, t.ein_right,
                       t.ein_out, t.ein_kout, t.ein_woff, params, A, G, Gp, first, d.B, d.K);
}

void launch_leaf_backward(const DevTables& t, int n_lv, const float* x, const uint8_t* mask, int mask_mode,
                          const float* G, float* stats, int64_t phi_off, int64_t den_off, int64_t tot_off,
                          const Dims& d, hipStream_t s) {
    const int total = n_lv * d.C * d.K;
    hipLaunchKernelGGL(k_leaf_backward, dim3((total + 255) / 256), dim3(256), 0, s, t.lv_leaf, t.lv_var, t.leaf_node,
                       t.leaf_replica, n_lv, x, mask, mask_mode, G, stats, phi_off, den_off, tot_off, d);
}

void launch_update_rows(const DevTables& t, int n_rows, float* params, float* stats, float step, float w_floor,
                        hipStream_t s) {
    hipLaunchKernelGGL(k_update_rows, dim3((n_rows + 3) / 4), dim3(256), 0, s, t.row_off, t.row_len, n_rows, params,
                       stats, step, w_floor);
}

void launch_update_leaves(float* params, float* stats, int64_t phi_off, int64_t den_off, int64_t tot_off, float step,
                          float min_var, float max_var, const Dims& d, hipStream_t s) {
    const int total = d.D * d.C * d.R * d.K;
    hipLaunchKernelGGL(k_update_leaves, dim3((total + 255) / 256), dim3(256), 0, s, params, stats, phi_off, den_off,
                       tot_off, step, min_var, max_var, d);
}

void launch_fill(float* p, float value, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_fill, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, p, value, n);
}

}  // namespace einet_impl
