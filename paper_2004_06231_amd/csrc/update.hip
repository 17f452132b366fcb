// M-step (Eq. 7-9, Sec. 4.2), random initial parameters, mixture of circuits (Sec. 4.2), fill.
#include "device_common.hpp"

namespace einet_impl {

namespace {

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
    if constexpr (NPL >= 4) {
        // rows of whole 16-byte groups (K even): the same with four entries per load
        if (len <= 64 * NPL && ((off | len) & 3) == 0) {
            constexpr int NV = NPL / 4;
            const int len4 = len >> 2;
            const float4* st4 = reinterpret_cast<const float4*>(stats + off);
            float4* pa4 = reinterpret_cast<float4*>(params + off);
            float n[NV][4], w[NV][4];
            float s = 0.f;
#pragma unroll
            for (int t = 0; t < NV; ++t) {
                const int e = lane + 64 * t;
                const float4 nv = e < len4 && have ? st4[e] : make_float4(0.f, 0.f, 0.f, 0.f);
                const float4 wv = e < len4 ? pa4[e] : make_float4(0.f, 0.f, 0.f, 0.f);
                n[t][0] = nv.x, n[t][1] = nv.y, n[t][2] = nv.z, n[t][3] = nv.w;
                w[t][0] = wv.x, w[t][1] = wv.y, w[t][2] = wv.z, w[t][3] = wv.w;
            }
#pragma unroll
            for (int t = 0; t < NV; ++t) s += (n[t][0] + n[t][1]) + (n[t][2] + n[t][3]);
            const float tot = wave_sum(s);
            const float sc = tot < 0x1p-60f ? 0x1p+64f : 1.f;
            const float inv = 1.f / (tot * sc);
            float s2 = 0.f;
#pragma unroll
            for (int t = 0; t < NV; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    n[t][c] = tot > 0.f ? (n[t][c] * sc) * inv : w[t][c];
                    if (w_floor > 0.f && lane + 64 * t < len4) {
                        n[t][c] = fmaxf(n[t][c], w_floor);
                        s2 += n[t][c];
                    }
                }
            const float norm = w_floor > 0.f ? 1.f / wave_sum(s2) : 1.f;
#pragma unroll
            for (int t = 0; t < NV; ++t) {
                const int e = lane + 64 * t;
                if (e < len4) {
                    pa4[e] = make_float4((1.f - step) * w[t][0] + step * (n[t][0] * norm),
                                         (1.f - step) * w[t][1] + step * (n[t][1] * norm),
                                         (1.f - step) * w[t][2] + step * (n[t][2] * norm),
                                         (1.f - step) * w[t][3] + step * (n[t][3] * norm));
                    if (clear) reinterpret_cast<float4*>(stats + off)[e] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            return;
        }
    }
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

void launch_init_params(const DevTables& t, int n_rows, float* params, int64_t phi_off, uint64_t seed, float lo,
                        float hi, const Dims& d, hipStream_t s) {
    const int n_row_blocks = (n_rows + 3) / 4;
    const int n_leaf_blocks = (d.D * d.R * d.K + 255) / 256;
    hipLaunchKernelGGL(k_init_params, dim3(n_row_blocks + n_leaf_blocks), dim3(256), 0, s, n_row_blocks, t.row_off,
                       t.row_len, n_rows, params, phi_off, seed, lo, hi, d);
}

void launch_mixture_logp(const float* lp, const float* log_coef, int n_components, int B, float* out, hipStream_t s) {
    hipLaunchKernelGGL(k_mixture_logp, dim3((B + 255) / 256), dim3(256), 0, s, lp, log_coef, n_components, B, out);
}

void launch_fill(float* p, float value, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_fill, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, p, value, n);
}

}  // namespace einet_impl
