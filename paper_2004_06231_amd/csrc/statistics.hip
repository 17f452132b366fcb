// End of the top-down pass: statistics of the mixing weights and of the leaves (Eq. 6-7).
#include "device_common.hpp"

#include <mutex>

namespace einet_impl {

namespace {

// Statistics of the mixing weights (App. B, Eq. 6): Nv[s,k,c] += v[s,k,c] * sum_b G[s][b,k] * S^c[b,k] / S[b,k].
// One workgroup per (mixing item, child); a reduction over the batch through LDS.  Runs in the same
// launch as the leaf statistics (k_tail_backward): the two are independent.  The workgroup is a chain of memory
// requests: the item's record (node, entries, weight offset, partitions: one request instead of four tables one after the
// other), then the rows of four samples per thread at once together with the weight and its old statistic.
template <int TPB>
__device__ __forceinline__ void mixing_stats_body(int item, int c, const int32_t* __restrict__ m_rec,
                                                  const int32_t* __restrict__ m_cptr,
                                                  const int32_t* __restrict__ m_child, const float* __restrict__ params,
                                                  float* __restrict__ stats, const float* __restrict__ A,
                                                  const double* __restrict__ Off, const float* __restrict__ G, int B,
                                                  int K) {
    __shared__ float red[TPB];
    const int tid = threadIdx.x;
    const int32_t* rec = m_rec + (size_t)item * MIX_REC_INTS;
    const int node = rec[0], kout = rec[1], voff = rec[2], nc = rec[3];
    if (c >= nc) return;
    const int child = c < MIX_REC_CHILDREN ? rec[4 + c] : m_child[m_cptr[item] + c];
    const int nbl = TPB / kout, k = tid % kout, bl = tid / kout;
    const float* As = A + (size_t)node * B * K;
    const float* Ac = A + (size_t)child * B * K;
    const float* Gs = G + (size_t)node * B * K;
    const double* Os = Off + (size_t)node * B;
    const double* Oc = Off + (size_t)child * B;
    const size_t so = (size_t)voff + (size_t)min(tid, kout - 1) * nc + c;
    const float pv = params[so], sv = stats[so];       // (used by the first kout threads at the end)
    float part = 0.f;
    if (bl < nbl)
        for (int b0 = bl; b0 < B; b0 += 4 * nbl) {
            float g[4], ac[4], as[4];
            double dd[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = min(b0 + u * nbl, B - 1);
                const size_t o = (size_t)b * K + k;
                g[u] = Gs[o];
                ac[u] = Ac[o];
                as[u] = As[o];
                dd[u] = Oc[b] - Os[b];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (b0 + u * nbl < B && g[u] != 0.f) part += g[u] * expf((float)dd[u] + ac[u] - as[u]);
        }
    red[tid] = part;
    __syncthreads();
    // A sum with few entries (the root has one) has hundreds of sample groups: 32 threads per entry first add every 32nd
    // group, so that no thread walks more than a few dozen values.
    int ngr = nbl;
    if (nbl > 64) {
        constexpr int J = 32;
        float t = 0.f;
        const int kk = tid % kout, j = tid / kout;
        if (j < J)
            for (int l = j; l < nbl; l += J) t += red[l * kout + kk];
        __syncthreads();
        if (j < J) red[j * kout + kk] = t;
        __syncthreads();
        ngr = J;
    }
    if (tid < kout) {
        float t4[4] = {0.f, 0.f, 0.f, 0.f};
        int l = 0;
        for (; l + 4 <= ngr; l += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) t4[u] += red[(l + u) * kout + tid];
        }
        for (; l < ngr; ++l) t4[0] += red[l * kout + tid];
        stats[so] = sv + pv * ((t4[0] + t4[1]) + (t4[2] + t4[3]));
    }
}

// ------------------------------------------------------------------ top-down pass, leaves
// Posterior-weighted sufficient statistics (Eq. 6-7).  A workgroup of 1024 threads
// owns 1024/NCH consecutive statistics entries (leaf variable, channel, k); its NCH
// parts each walk every NCH-th sample and the partial sums meet in LDS.
// DIRECT: the leaf's posterior is not in G; it is the sum of the blocks of Gp that leaf_gsrc names (first block << 3 |
// number of blocks, see GSRC_MAX_BLOCKS), added up in the order the assembly launch would take.
template <int NCH, bool DIRECT>
__device__ __forceinline__ void leaf_backward_body(
    int block, const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var, const int32_t* __restrict__ leaf_node,
    const int32_t* __restrict__ leaf_replica, int n_lv, const float* __restrict__ x,
    const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G, const float* __restrict__ Gp,
    const int32_t* __restrict__ leaf_gsrc, float* __restrict__ stats,
    int64_t phi_off, int64_t den_off, int64_t tot_off, Dims d) {
    constexpr int NO = 1024 / NCH;
    __shared__ float red[NCH][4][NO];
    const int lo = threadIdx.x % NO, part_id = threadIdx.x / NO;
    const int idx = block * NO + lo;
    const bool valid = idx < n_lv * d.C * d.K;
    const int k = valid ? idx % d.K : 0, c = valid ? (idx / d.K) % d.C : 0, e = valid ? idx / (d.K * d.C) : 0;
    const int leaf = lv_leaf[e], var = lv_var[e], r = leaf_replica[leaf];
    const size_t gblk = (size_t)d.B * d.K;
    const int gsrc = DIRECT ? leaf_gsrc[leaf] : 0, gcnt = gsrc & 7;
    const float* Gl = (DIRECT ? Gp + (size_t)(gsrc >> 3) * gblk : G + (size_t)leaf_node[leaf] * gblk) + k;
    const float* xp = x + (size_t)var * d.C + c;
    const bool shared_obs = mask_mode != EINET_MASK_SHARED || mask[var] != 0;
    float n1 = 0.f, n2 = 0.f, den = 0.f, tot = 0.f;
#pragma unroll 4
    for (int b = part_id; b < d.B; b += NCH) {
        float p = Gl[(size_t)b * d.K];
        if (DIRECT && gcnt > 1) {
            float px[GSRC_MAX_BLOCKS - 1];
#pragma unroll
            for (int q = 1; q < GSRC_MAX_BLOCKS; ++q) px[q - 1] = q < gcnt ? Gl[q * gblk + (size_t)b * d.K] : 0.f;
#pragma unroll
            for (int q = 1; q < GSRC_MAX_BLOCKS; ++q)
                if (q < gcnt) p += px[q - 1];
        }
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
// PPT: pairs per thread.  With four, a workgroup covers four times the pairs (for image rows of three channels
// 400 contiguous bytes of x per sample instead of 100) and the posterior block is copied a quarter as often.
__host__ __device__ inline size_t cell_lds_bytes(int K, int PPT) {
    return sizeof(float) * ((size_t)CELL_BC * (K + cell_pairs_per_group(K) * PPT) + cell_pairs_per_group(K) * PPT + 2) +
           (size_t)CELL_BC * cell_pairs_per_group(K) * PPT;
}

template <int PPT, bool DIRECT>
__device__ __forceinline__ void leaf_backward_cells_body(
    int block, int chunks_per_leaf, const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica,
    const int32_t* __restrict__ leaf_sptr, const int32_t* __restrict__ leaf_var, const float* __restrict__ x,
    const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G, const float* __restrict__ Gp,
    const int32_t* __restrict__ leaf_gsrc, float* __restrict__ stats,
    int64_t phi_off, int64_t den_off, int64_t tot_off, Dims d) {
    extern __shared__ float cell_lds[];
    const int pc = cell_pairs_per_group(d.K) * PPT;   // pairs per workgroup
    float* Gs = cell_lds;                             // [CELL_BC][K]
    float* xs = Gs + CELL_BC * d.K;                   // [CELL_BC][pc]
    int* vsl = reinterpret_cast<int*>(xs + CELL_BC * pc);          // [pc + 2] variables the chunk's pairs belong to
    uint8_t* os = reinterpret_cast<uint8_t*>(vsl + pc + 2);        // [CELL_BC][pc] 1 = observed
    const int leaf = block / chunks_per_leaf, chunk = block - leaf * chunks_per_leaf;
    const int s0 = leaf_sptr[leaf], npairs = (leaf_sptr[leaf + 1] - s0) * d.C;
    const int p0 = chunk * pc;
    if (p0 >= npairs) return;                         // (whole workgroup) this leaf has fewer chunks
    const int np = min(pc, npairs - p0);
    const int tid = threadIdx.x;
    const int pl = (tid / d.K) * PPT, k = tid % d.K;  // this thread's first pair and its entry
    const size_t gblk = (size_t)d.B * d.K;
    const int gsrc = DIRECT ? leaf_gsrc[leaf] : 0, gcnt = gsrc & 7;
    const float* Gl = DIRECT ? Gp + (size_t)(gsrc >> 3) * gblk : G + (size_t)leaf_node[leaf] * gblk;
    // the variable numbers go to LDS once, so that the loads of the values do not each wait for one
    const int vfirst = p0 / d.C, vcount = (p0 + np - 1) / d.C - vfirst + 1;
    for (int j = tid; j < vcount; j += 1024) vsl[j] = leaf_var[s0 + vfirst + j];
    __syncthreads();
    float n1[PPT], n2[PPT], den[PPT], tot = 0.f;
#pragma unroll
    for (int q = 0; q < PPT; ++q) n1[q] = n2[q] = den[q] = 0.f;
    for (int b0 = 0; b0 < d.B; b0 += CELL_BC) {
        const int nb = min(CELL_BC, d.B - b0);
        if (b0 > 0) __syncthreads();                  // readers of the previous pass are done
        for (int i0 = tid; i0 < nb * d.K; i0 += 4 * 1024) {      // four loads in flight per thread
            float gq[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) gq[q] = i0 + q * 1024 < nb * d.K ? Gl[(size_t)b0 * d.K + i0 + q * 1024] : 0.f;
            if (DIRECT && gcnt > 1) {
                for (int y = 1; y < gcnt; ++y) {       // (the same element of the next block, all four together)
                    float gy[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        gy[q] = i0 + q * 1024 < nb * d.K ? Gl[y * gblk + (size_t)b0 * d.K + i0 + q * 1024] : 0.f;
#pragma unroll
                    for (int q = 0; q < 4; ++q) gq[q] += gy[q];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (i0 + q * 1024 < nb * d.K) Gs[i0 + q * 1024] = gq[q];
        }
#pragma unroll 4
        for (int i = tid; i < nb * np; i += 1024) {
            const int bb = i / np, p = i - bb * np;
            const int pair = p0 + p, v = pair / d.C, c = pair - v * d.C;
            const int var = vsl[v - vfirst];
            xs[bb * pc + p] = x[((size_t)(b0 + bb) * d.D + var) * d.C + c];
            if (mask_mode == EINET_MASK_SHARED) os[bb * pc + p] = mask[var];
            if (mask_mode == EINET_MASK_PER_SAMPLE) os[bb * pc + p] = mask[(size_t)(b0 + bb) * d.D + var];
        }
        __syncthreads();
        // (pairs beyond np read stale LDS values; their sums are never written)
        if (pl < np && mask_mode != EINET_MASK_NONE) {
#pragma unroll 4
            for (int bb = 0; bb < nb; ++bb) {
                const float p = Gs[bb * d.K + k];
                tot += p;
#pragma unroll
                for (int q = 0; q < PPT; ++q) {
                    const float xv = xs[bb * pc + pl + q];
                    const float pm = os[bb * pc + pl + q] ? p : 0.f;
                    den[q] += pm;
                    n1[q] = fmaf(pm, xv, n1[q]);
                    n2[q] = fmaf(pm * xv, xv, n2[q]);
                }
            }
        } else if (pl < np) {                         // everything observed: no flags to read, den = tot
#pragma unroll 4
            for (int bb = 0; bb < nb; ++bb) {
                const float p = Gs[bb * d.K + k];
                tot += p;
#pragma unroll
                for (int q = 0; q < PPT; ++q) {
                    const float xv = xs[bb * pc + pl + q];
                    n1[q] = fmaf(p, xv, n1[q]);
                    n2[q] = fmaf(p * xv, xv, n2[q]);
                }
            }
        }
    }
    if (mask_mode == EINET_MASK_NONE) {
#pragma unroll
        for (int q = 0; q < PPT; ++q) den[q] = tot;
    }
    const int r = leaf_replica[leaf];
#pragma unroll
    for (int q = 0; q < PPT; ++q) {
        if (pl + q >= np) continue;
        const int pair = p0 + pl + q, v = pair / d.C, c = pair - v * d.C;
        const int var = vsl[v - vfirst];
        const size_t ph = phi_off + ((size_t)(var * d.C + c) * d.R + r) * d.T * d.K + k;
        stats[ph] += n1[q];
        if (d.T == 2) stats[ph + d.K] += n2[q];
        if (c == 0) {
            const size_t o = ((size_t)var * d.R + r) * d.K + k;
            stats[den_off + o] += den[q];
            stats[tot_off + o] += tot;
        }
    }
}

// The same statistics for very long scopes (strips of a large image: thousands of (variable, channel) pairs per leaf)
// when nothing is marginalised: num[pair][k] = sum_b x[b][pair] p[b][k] (and the same with x^2) is a GEMM with the
// batch as contraction, here on v_mfma_f32_32x32x2_f32: rows = 32 pairs (A operand: the values, staged per pass of 64
// samples in LDS exactly as above), columns = 32 entries k (B operand: the leaf's posterior block, zero beyond K).
// A workgroup of four waves takes one leaf and 128 / NCT of its pairs, NCT being the number of column tiles (K <= 32:
// one); a wave takes one tile of 32 pairs x 32 entries, so that every wave of a launch carries the same number of
// MFMAs whatever K is.  Three workgroups share a compute unit (one stages while another multiplies); SQ adds the
// x^2 rows (Gaussian leaves).  tot = den = sum_b p[b][k] is summed on the side.
typedef float floatx16s __attribute__((ext_vector_type(16)));
constexpr int LSM_BC = 64;                             // samples per pass
template <int NCT>
struct LsmLayout {
    static constexpr int PC = 128 / NCT;               // pairs per workgroup
    static constexpr int XS = PC + 8;                  // row stride of the values
    static constexpr int PH = 256 / PC;                // threads per pair while staging: thread takes every PH-th sample
    static constexpr size_t LDS_BYTES = sizeof(float) * ((size_t)LSM_BC * 64 + (size_t)LSM_BC * XS + 64) + sizeof(int) * (PC + 2);
};

template <bool SQ, int NCT>
__global__ __launch_bounds__(256, NCT == 2 ? 3 : 2) void k_leaf_stats_mfma(
    const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica, const int32_t* __restrict__ leaf_sptr,
    const int32_t* __restrict__ leaf_var, const float* __restrict__ x, const float* __restrict__ G,
    float* __restrict__ stats, int64_t phi_off, int64_t den_off, int64_t tot_off, int chunks_per_leaf, int groups,
    int group_samples, float* __restrict__ part, int64_t part_stride, Dims d) {
    using LY = LsmLayout<NCT>;
    constexpr int PC = LY::PC, XS = LY::XS, PH = LY::PH, NX = LSM_BC / PH;
    extern __shared__ float lsm_lds[];
    float* Gs = lsm_lds;                               // [LSM_BC][64], columns beyond K are zero
    float* xs = Gs + LSM_BC * 64;                      // [LSM_BC][XS]
    float* tots = xs + LSM_BC * XS;                    // [64]
    int* vsl = reinterpret_cast<int*>(tots + 64);      // variables of the chunk's pairs
    // groups > 1: workgroup (leaf, chunk, group) takes the samples [bfirst, bend) and writes (not adds) its sums to
    // block `group` of part, which is laid out like the leaf part of the statistics (from phi_off on)
    const int lc = blockIdx.x / groups, group = blockIdx.x - lc * groups;
    const int leaf = lc / chunks_per_leaf, chunk = lc - leaf * chunks_per_leaf;
    const int bfirst = group * group_samples, bend = min(d.B, bfirst + group_samples);
    float* dst = groups > 1 ? part + (size_t)group * part_stride - phi_off : stats;
    const bool adds = groups == 1;
    const int s0 = leaf_sptr[leaf], npairs = (leaf_sptr[leaf + 1] - s0) * d.C;
    const int p0 = chunk * PC;
    if (p0 >= npairs) return;                          // (whole workgroup) this leaf has fewer chunks
    const int np = min(PC, npairs - p0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rt = wave % (4 / NCT), ct = wave / (4 / NCT);   // this wave's tile: pairs 32 rt .., entries 32 ct ..
    const int n = lane & 31, h = lane >> 5;
    const float* Gl = G + (size_t)leaf_node[leaf] * d.B * d.K;
    const int vfirst = p0 / d.C, vcount = (p0 + np - 1) / d.C - vfirst + 1;
    for (int j = tid; j < vcount; j += 256) vsl[j] = leaf_var[s0 + vfirst + j];
    floatx16s acc[SQ ? 2 : 1];
#pragma unroll
    for (int q = 0; q < (SQ ? 2 : 1); ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
    float tot = 0.f;                                   // thread (k, quarter): its share of sum_b p[b][k]
    __syncthreads();
    // thread (pair = tid % PC, phase = tid / PC) stages every PH-th sample of its pair (part of a column of xs) and 16
    // entries of the posterior block per pass; the values of the next pass are requested before the MFMAs of the current
    // one and go to LDS after them
    size_t xoff = 0;
    const int sp = tid & (PC - 1), sh = tid / PC;
    const bool pin = sp < np;
    if (pin) {
        const int pair = p0 + sp, vv = pair / d.C, c = pair - vv * d.C;
        xoff = (size_t)vsl[vv - vfirst] * d.C + c;
    }
    const size_t xstride = (size_t)d.D * d.C;
    float xr[NX], gq[LSM_BC * 64 / 256];
    auto fetch = [&](int b0) {
        const int nb = min(LSM_BC, bend - b0);
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int bb = PH * q + sh;
            xr[q] = (pin && bb < nb) ? x[(size_t)(b0 + bb) * xstride + xoff] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < LSM_BC * 64 / 256; ++q) {
            const int i = tid + 256 * q, bb = i >> 6, k = i & 63;
            gq[q] = (bb < nb && k < d.K) ? Gl[(size_t)(b0 + bb) * d.K + k] : 0.f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int q = 0; q < NX; ++q) xs[(PH * q + sh) * XS + sp] = xr[q];
#pragma unroll
        for (int q = 0; q < LSM_BC * 64 / 256; ++q) Gs[tid + 256 * q] = gq[q];
    };
    fetch(bfirst);
    for (int b0 = bfirst; b0 < bend; b0 += LSM_BC) {
        if (b0 > bfirst) __syncthreads();              // readers of the previous pass are done
        stage();
        __syncthreads();
        if (b0 + LSM_BC < bend) fetch(b0 + LSM_BC);
        __builtin_amdgcn_sched_barrier(0);             // (the requests stay ahead of the MFMA loop)
        {
            // thread (k = tid % 64, quarter = tid / 64) sums a quarter of the pass (rows beyond the batch are zero)
            float t4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int bb = 0; bb < LSM_BC / 4; ++bb) t4[bb & 3] += Gs[(16 * wave + bb) * 64 + lane];
            tot += (t4[0] + t4[1]) + (t4[2] + t4[3]);
        }
        const float* xa = xs + h * XS + 32 * rt + n;   // + 2 s XS
        const float* pb = Gs + h * 64 + 32 * ct + n;   // + 2 s 64
        // operands of the next step are requested before the MFMAs of the current one; the squares are formed ahead of
        // the MFMAs, not between them
        float a[2], b[2];
        a[0] = xa[0];
        b[0] = pb[0];
#pragma unroll
        for (int s = 0; s < LSM_BC / 2; ++s) {
            const int cur = s & 1, nxt = cur ^ 1;
            if (s + 1 < LSM_BC / 2) {
                a[nxt] = xa[2 * (s + 1) * XS];
                b[nxt] = pb[2 * (s + 1) * 64];
            }
            const float a2 = a[cur] * a[cur];
            __builtin_amdgcn_sched_barrier(0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur], b[cur], acc[0], 0, 0, 0);
            if (SQ) acc[SQ ? 1 : 0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2, b[cur], acc[SQ ? 1 : 0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // acc[q][v]: pair = 32 rt + 8 (v / 4) + 4 h + v % 4 of the chunk, entry k = 32 ct + n
    const int r = leaf_replica[leaf];
    const int k = 32 * ct + n;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int p = 32 * rt + 8 * (v >> 2) + 4 * h + (v & 3);
        if (p < np && k < d.K) {
            const int pair = p0 + p, vv = pair / d.C, c = pair - vv * d.C;
            const size_t ph = phi_off + ((size_t)(vsl[vv - vfirst] * d.C + c) * d.R + r) * d.T * d.K;
            dst[ph + k] = (adds ? dst[ph + k] : 0.f) + acc[0][v];
            if (SQ) dst[ph + d.K + k] = (adds ? dst[ph + d.K + k] : 0.f) + acc[SQ ? 1 : 0][v];
        }
    }
    // den = tot for every variable whose first channel lies in this chunk
    __syncthreads();                                   // (the last pass has been read: Gs is free)
    Gs[tid] = tot;
    __syncthreads();
    if (tid < 64) tots[tid] = tid < d.K ? (Gs[tid] + Gs[64 + tid]) + (Gs[128 + tid] + Gs[192 + tid]) : 0.f;
    __syncthreads();
    const int vlo = (p0 + d.C - 1) / d.C, vhi = (p0 + np - 1) / d.C;      // variables with pair (v, 0) in [p0, p0 + np)
    for (int i = tid; i < (vhi - vlo + 1) * d.K; i += 256) {
        const int vv = vlo + i / d.K, kk = i % d.K;
        const size_t o = ((size_t)vsl[vv - vfirst] * d.R + r) * d.K + kk;
        dst[den_off + o] = (adds ? dst[den_off + o] : 0.f) + tots[kk];
        dst[tot_off + o] = (adds ? dst[tot_off + o] : 0.f) + tots[kk];
    }
}

// stats[i] += sum over the blocks of part[.][i], i over the n floats of the leaf part of the statistics (what follows
// k_leaf_stats_mfma with several batch groups): workgroup blk of n_blocks, in the launch of the mixing statistics
__device__ __forceinline__ void sum_leaf_blocks_body(int blk, int n_blocks, const float* __restrict__ part,
                                                     float* __restrict__ stats, int64_t n, int groups) {
    for (int64_t i = (int64_t)blk * blockDim.x + threadIdx.x; i < n; i += (int64_t)n_blocks * blockDim.x) {
        float sum = stats[i];
        for (int v = 0; v < groups; ++v) sum += part[v * n + i];
        stats[i] = sum;
    }
}

// Last launch of the top-down pass: leaf statistics in the first n_leaf_blocks workgroups, mixing
// statistics in the others (item = idx / max_children, child = idx % max_children).  NCH = 0 selects the
// kernel body for long scopes (chunks_per_leaf workgroups per leaf, PPT pairs per thread), NCH = TAIL_SUMS the sum of
// the blocks that the batch groups of k_leaf_stats_mfma left in part.
constexpr int TAIL_SUMS = 64;
template <int NCH, int PPT, bool DIRECT>
__global__ __launch_bounds__(1024) void k_tail_backward(
    int n_leaf_blocks, int max_children, const int32_t* __restrict__ lv_leaf, const int32_t* __restrict__ lv_var,
    const int32_t* __restrict__ leaf_node, const int32_t* __restrict__ leaf_replica, int n_lv,
    const float* __restrict__ x, const uint8_t* __restrict__ mask, int mask_mode, const float* __restrict__ G,
    const float* __restrict__ Gp, const int32_t* __restrict__ leaf_gsrc,
    float* __restrict__ stats, int64_t phi_off, int64_t den_off, int64_t tot_off, const int32_t* __restrict__ m_rec,
    const int32_t* __restrict__ m_cptr, const int32_t* __restrict__ m_child, const float* __restrict__ params,
    const float* __restrict__ A, const double* __restrict__ Off, const int32_t* __restrict__ leaf_sptr,
    const int32_t* __restrict__ leaf_var, int chunks_per_leaf, const float* __restrict__ part, int64_t part_n,
    int groups, Dims d) {
    const int blk = blockIdx.x;
    if (blk < n_leaf_blocks) {
        if constexpr (NCH == TAIL_SUMS)
            sum_leaf_blocks_body(blk, n_leaf_blocks, part, stats + phi_off, part_n, groups);
        else if constexpr (NCH == 0)
            leaf_backward_cells_body<PPT, DIRECT>(blk, chunks_per_leaf, leaf_node, leaf_replica, leaf_sptr, leaf_var, x,
                                                  mask, mask_mode, G, Gp, leaf_gsrc, stats, phi_off, den_off, tot_off, d);
        else
            leaf_backward_body<NCH, DIRECT>(blk, lv_leaf, lv_var, leaf_node, leaf_replica, n_lv, x, mask, mask_mode, G, Gp,
                                            leaf_gsrc, stats, phi_off, den_off, tot_off, d);
    } else {
        const int idx = blk - n_leaf_blocks;
        mixing_stats_body<1024>(idx / max_children, idx % max_children, m_rec, m_cptr, m_child, params, stats, A, Off, G,
                                d.B, d.K);
    }
}

}  // namespace

void launch_tail_backward(const DevTables& t, int n_lv, int n_leaves, int max_scope, int n_mix, int max_children,
                          const float* x, const uint8_t* mask, int mask_mode, const float* params, const float* A,
                          const double* Off, const float* G, const float* Gp, bool direct, float* stats,
                          int64_t phi_off, int64_t den_off, int64_t tot_off, int64_t n_stats, float* part,
                          size_t part_floats, const Dims& d, hipStream_t s) {
    const int total = n_lv * d.C * d.K;
    const bool categorical = d.family == EINET_LEAF_CATEGORICAL;
    if (categorical)     // indicator statistics: a histogram kernel of its own (at most 256 x 64 floats of LDS)
        hipLaunchKernelGGL(k_leaf_backward_categorical, dim3(n_lv * d.C), dim3(64), sizeof(float) * d.P * d.K, s,
                           t.lv_leaf, t.lv_var, t.leaf_node, t.leaf_replica, x, mask, mask_mode, G, stats, phi_off,
                           den_off, tot_off, d);
    // very long scopes, nothing marginalised: the statistics as a GEMM over the batch on the matrix pipe, the mixing
    // statistics in a launch of their own
    bool leaves_done = categorical;
    const int64_t n_leaf_stats = n_stats - phi_off;
    int groups = part ? leaf_stats_groups(n_leaves, max_scope, d.C, d.K, d.B) : 1;
    if ((size_t)groups * (size_t)n_leaf_stats > part_floats) groups = 1;
    if (!categorical && mask_mode == EINET_MASK_NONE && (max_scope * d.C >= 1024 || groups > 1) && d.K <= 64) {
        static std::once_flag attr_m[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_m[dev % EINET_MAX_DEVICES], [&] {
            allow_dynamic_lds(&k_leaf_stats_mfma<true, 1>, LsmLayout<1>::LDS_BYTES);
            allow_dynamic_lds(&k_leaf_stats_mfma<true, 2>, LsmLayout<2>::LDS_BYTES);
            allow_dynamic_lds(&k_leaf_stats_mfma<false, 1>, LsmLayout<1>::LDS_BYTES);
            allow_dynamic_lds(&k_leaf_stats_mfma<false, 2>, LsmLayout<2>::LDS_BYTES);
        });
#define EINET_LSM(SQ, NCT)                                                                                       \
    {                                                                                                            \
        static_assert(LsmLayout<NCT>::PC == (NCT == 2 ? 64 : 128), "leaf_stats_pairs_per_group");                \
        const int cpl = (max_scope * d.C + LsmLayout<NCT>::PC - 1) / LsmLayout<NCT>::PC;                         \
        hipLaunchKernelGGL((k_leaf_stats_mfma<SQ, NCT>), dim3(n_leaves * cpl * groups), dim3(256),               \
                           LsmLayout<NCT>::LDS_BYTES, s, t.leaf_node, t.leaf_replica, t.leaf_sptr, t.leaf_var, x, G, \
                           stats, phi_off, den_off, tot_off, cpl, groups, group_samples, part, n_leaf_stats, d);   \
    }
        const int passes = (d.B + LSM_BC - 1) / LSM_BC;
        const int group_samples = groups > 1 ? LSM_BC * ((passes + groups - 1) / groups) : d.B;
        if (d.T == 2 && d.K > 32) EINET_LSM(true, 2)
        else if (d.T == 2) EINET_LSM(true, 1)
        else if (d.K > 32) EINET_LSM(false, 2)
        else EINET_LSM(false, 1)
#undef EINET_LSM
        leaves_done = true;
    }
    // long scopes: posterior block and values through LDS; short ones: straight from memory
    const int pc1 = cell_pairs_per_group(d.K);
    const int chunks1 = (max_scope * d.C + pc1 - 1) / pc1;
    // (with fewer than 64 such workgroups the chip is better filled by the element-wise kernel)
    const bool cells = !categorical && max_scope * d.C >= 32 && n_leaves * chunks1 >= 64;
    // four pairs per thread when there would be more than a thousand workgroups (and the values still fit LDS)
    const int ppt = cells && n_leaves * chunks1 >= 1024 && pc1 * 4 <= 128 ? 4 : 1;
    // (eight parts from 64 samples on: 17.4 -> 15.5 us for 2560 leaves of three variables and 100 samples; sixteen: 21.6 us)
    const int nch = cells ? 0 : (d.B >= 64 ? 8 : d.B >= 16 ? 4 : 1);
    const int chunks_per_leaf = cells ? (max_scope * d.C + pc1 * ppt - 1) / (pc1 * ppt) : 1;
    // (after the matrix kernel with batch groups: the leaf workgroups of this launch add the groups' blocks up)
    const bool sums = leaves_done && !categorical && groups > 1;
    const int sum_blocks = (int)((n_leaf_stats + 4095) / 4096 < 256 ? (n_leaf_stats + 4095) / 4096 : 256);
    const int n_leaf_blocks = sums ? sum_blocks
                              : leaves_done ? 0 : (cells ? n_leaves * chunks_per_leaf : (total + 1024 / nch - 1) / (1024 / nch));
    const int blocks = n_leaf_blocks + n_mix * max_children;
    if (blocks == 0) return;
    const size_t lds = cells && !sums ? cell_lds_bytes(d.K, ppt) : 0;
    if (cells && !sums) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] {
            allow_dynamic_lds(&k_tail_backward<0, 1, false>, 64 * 1024);
            allow_dynamic_lds(&k_tail_backward<0, 4, false>, 128 * 1024);
            allow_dynamic_lds(&k_tail_backward<0, 1, true>, 64 * 1024);
            allow_dynamic_lds(&k_tail_backward<0, 4, true>, 128 * 1024);
        });
    }
#define EINET_LAUNCH_D(N, P, DIR)                                                                                    \
    hipLaunchKernelGGL((k_tail_backward<N, P, DIR>), dim3(blocks), dim3(1024), lds, s, n_leaf_blocks,                 \
                       max_children > 0 ? max_children : 1, t.lv_leaf, t.lv_var, t.leaf_node, t.leaf_replica, n_lv, x, \
                       mask, mask_mode, G, Gp, t.leaf_gsrc, stats, phi_off, den_off, tot_off, t.mix_rec, t.mix_cptr,  \
                       t.mix_child, params, A, Off, t.leaf_sptr, t.leaf_var, chunks_per_leaf, part, n_leaf_stats,     \
                       groups, d)
#define EINET_LAUNCH(N, P)                       \
    do {                                         \
        if (direct) EINET_LAUNCH_D(N, P, true);  \
        else EINET_LAUNCH_D(N, P, false);        \
    } while (0)
    if (sums) EINET_LAUNCH_D(TAIL_SUMS, 1, false);
    else if (nch == 0 && ppt == 4) EINET_LAUNCH(0, 4);
    else if (nch == 0) EINET_LAUNCH(0, 1);
    else if (nch == 8) EINET_LAUNCH(8, 1);
    else if (nch == 4) EINET_LAUNCH(4, 1);
    else EINET_LAUNCH(1, 1);
#undef EINET_LAUNCH
#undef EINET_LAUNCH_D
}

}  // namespace einet_impl
