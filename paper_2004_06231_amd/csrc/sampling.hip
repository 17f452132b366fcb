// Top-down sampling (Sec. 2, Sec. 4.2, App. D).
#include "device_common.hpp"

#include <mutex>

namespace einet_impl {

namespace {

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
// (App. B), v[k][c] without.  Every lane of the wave walks the few partitions; all get the same answer.
__device__ __forceinline__ int sample_partition(int mi, int s, int k, int b, const int32_t* __restrict__ m_cptr,
                                                const int32_t* __restrict__ m_child,
                                                const int32_t* __restrict__ m_voff, int evidence,
                                                const float* __restrict__ params, const float* __restrict__ A,
                                                const double* __restrict__ Off, const float* __restrict__ u,
                                                int num_partitions, int B, int K) {
    const int c0 = m_cptr[mi], nc = m_cptr[mi + 1] - c0;
    const float* v = params + m_voff[mi] + (size_t)k * nc;
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
    return pick < 0 ? last : pick;                   // u so close to 1 that rounding ate the last interval
}

// Partition: the pair (i, j) has weight W[k][i][j] * eL[i] * eR[j] given the evidence (the posterior of
// Eq. 6 for the chosen output entry k), W[k][i][j] without; pairs are numbered i * K + j.  One wave per
// (region, sample): it first chooses the partition (above), then the K*K weights of that partition go to LDS,
// every lane sums a run of consecutive pairs, a wave scan of the run sums finds the run that holds the
// threshold and its lane walks it.
constexpr int SAMPLE_WAVES = 4;
__device__ __forceinline__ int sample_pos(int t) { return t + (t >> 5); }   // padded: runs start in different banks

__global__ __launch_bounds__(64 * SAMPLE_WAVES) void k_sample_regions(
    const int32_t* __restrict__ sr_rec, const int32_t* __restrict__ sr_pptr, const int32_t* __restrict__ sr_item,
    const int32_t* __restrict__ sr_mix, const int32_t* __restrict__ m_cptr, const int32_t* __restrict__ m_child,
    const int32_t* __restrict__ m_voff, const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right,
    const int32_t* __restrict__ e_woff, const int32_t* __restrict__ e_part, int evidence,
    const float* __restrict__ params, const float* __restrict__ A, const double* __restrict__ Off,
    const float* __restrict__ amax, const float* __restrict__ u, int num_partitions, int32_t* __restrict__ sel, int B,
    int K) {
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ri = blockIdx.x, b = blockIdx.y * SAMPLE_WAVES + wave;
    if (b >= B) return;                              // whole waves leave: no barrier below
    // the region's record: node, partitions, mixing weights, and per partition its einsum item and nodes
    const int32_t* rec = sr_rec + (size_t)ri * SR_REC_INTS;
    const int s = rec[0], nparts = rec[1];
    const int k = sel[(size_t)s * B + b];
    if (k < 0) return;
    int item, left, right, woff, upart;
    if (nparts <= SR_REC_PARTS) {
        int c = 0;
        if (nparts > 1) {
            // partition c has weight v[k][c] * S^c[k] / S[k] given the evidence (App. B), v[k][c] without; every
            // lane walks the few partitions and gets the same answer
            const float* v = params + rec[2] + (size_t)k * nparts;
            const size_t srow = (size_t)s * B + b;
            float w[SR_REC_PARTS];
#pragma unroll
            for (int q = 0; q < SR_REC_PARTS; ++q) {
                w[q] = 0.f;
                if (q < nparts) {
                    w[q] = v[q];
                    if (evidence) {
                        const size_t crow = (size_t)rec[4 + q * SR_REC_STRIDE + 5] * B + b;
                        w[q] *= expf((float)(Off[crow] - Off[srow]) + A[crow * K + k] - A[srow * K + k]);
                    }
                }
            }
            float total = 0.f;
#pragma unroll
            for (int q = 0; q < SR_REC_PARTS; ++q)
                if (q < nparts) total += w[q];
            const float tau = u[(size_t)(num_partitions + s) * B + b] * total;
            float run = 0.f;
            int pick = -1, last = 0;
#pragma unroll
            for (int q = 0; q < SR_REC_PARTS; ++q)
                if (q < nparts) {
                    run += w[q];
                    if (w[q] > 0.f) last = q;
                    if (pick < 0 && run > tau) pick = q;
                }
            c = pick < 0 ? last : pick;                  // u so close to 1 that rounding ate the last interval
            if (lane == 0) sel[(size_t)rec[4 + c * SR_REC_STRIDE + 5] * B + b] = k;
        }
        const int32_t* q = rec + 4 + c * SR_REC_STRIDE;
        item = q[0], left = q[1], right = q[2], woff = q[3], upart = q[4];
    } else {
        const int mi = sr_mix[ri];
        const int c = sample_partition(mi, s, k, b, m_cptr, m_child, m_voff, evidence, params, A, Off, u, num_partitions,
                                       B, K);
        if (lane == 0) sel[(size_t)m_child[m_cptr[mi] + c] * B + b] = k;
        item = sr_item[sr_pptr[ri] + c];
        left = e_left[item], right = e_right[item], woff = e_woff[item], upart = e_part[item];
    }
    const int KK = K * K;
    float* wl = lds + wave * (sample_pos(KK) + 1 + 128);
    float* el = wl + sample_pos(KK) + 1;
    float* er = el + 64;
    if (evidence) {
        const float al = amax[(size_t)item * 2 * B + b], ar = amax[((size_t)item * 2 + 1) * B + b];
        el[lane] = lane < K ? __expf(A[((size_t)left * B + b) * K + lane] - al) : 0.f;
        er[lane] = lane < K ? __expf(A[((size_t)right * B + b) * K + lane] - ar) : 0.f;
        __builtin_amdgcn_wave_barrier();
    }
    const float* row = params + woff + (size_t)k * KK;
    for (int t0 = lane; t0 < KK; t0 += 8 * 64) {      // eight loads in flight per lane
        float w[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) w[q] = t0 + 64 * q < KK ? row[t0 + 64 * q] : 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int t = t0 + 64 * q;
            if (t < KK) {
                if (evidence) {
                    const int i = t / K, j = t - i * K;
                    w[q] *= el[i] * er[j];
                }
                wl[sample_pos(t)] = w[q];
            }
        }
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
    const float tau = u[(size_t)upart * B + b] * total;
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
        sel[(size_t)left * B + b] = i;
        sel[(size_t)right * B + b] = pick - i * K;
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

}  // namespace

void launch_sample_init(int32_t* sel, int num_nodes, int B, hipStream_t s) {
    const int64_t n = (int64_t)num_nodes * B;
    hipLaunchKernelGGL(k_sample_init, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, sel, n, B);
}

void launch_sample_regions(const DevTables& t, int first, int count, bool evidence, const float* params,
                           const float* A, const double* Off, const float* amax, const float* u, int num_partitions,
                           int32_t* sel, const Dims& d, hipStream_t s) {
    if (count == 0) return;
    const int KK = d.K * d.K;
    const size_t lds = sizeof(float) * SAMPLE_WAVES * (size_t)(KK + (KK >> 5) + 1 + 128);   // at most 68 KB (K = 64)
    if (lds > 64 * 1024) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] { allow_dynamic_lds(&k_sample_regions, 72 * 1024); });
    }
    hipLaunchKernelGGL(k_sample_regions, dim3(count, (d.B + SAMPLE_WAVES - 1) / SAMPLE_WAVES), dim3(64 * SAMPLE_WAVES),
                       lds, s, t.sr_rec + (size_t)first * SR_REC_INTS, t.sr_pptr + first, t.sr_item, t.sr_mix + first, t.mix_cptr,
                       t.mix_child, t.mix_voff, t.ein_left, t.ein_right, t.ein_woff, t.ein_part, evidence ? 1 : 0,
                       params, A, Off, amax, u, num_partitions, sel, d.B, d.K);
}

void launch_sample_leaves(const DevTables& t, int n_lv, const float* x, const uint8_t* mask, int mask_mode,
                          const float* phi, const float* noise, const int32_t* sel, float* out, const Dims& d,
                          hipStream_t s) {
    hipLaunchKernelGGL(k_sample_leaves, dim3((n_lv + 255) / 256, d.B), dim3(256), 0, s, t.lv_leaf, t.lv_var,
                       t.leaf_node, t.leaf_replica, n_lv, x, mask, mask_mode, phi, noise, t.leaf_logc, sel, out, d);
}

}  // namespace einet_impl
