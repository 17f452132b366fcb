// The top of the circuit, one launch each way.  The partitions of the root are einsum items with a single output
// entry (Eq. 3-5): K^2 multiply-adds per sample, far too little for the matrix pipe to matter, so these launches are
// chains of dependent memory requests.  Both kernels read one record (all indices of all partitions), request rows,
// offsets and weights together, and work on the vector ALU; bottom-up the root's mixture (App. B) and log P are formed
// in the same launch, top-down the mixing step of the root is folded into the posterior weight (Eq. 6).
#include "device_common.hpp"

#include <mutex>

namespace einet_impl {

namespace {

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A workgroup takes RF_SB samples and all partitions, one partition per wave at a time; 16 lanes share a sample:
// lane t holds the entries t, t + 16, .. of both child rows, finds the shifts with its 15 neighbours, and takes the
// left entries i = t, t + 16, .. of  S~ = sum_i eL[i] sum_j W[i][j] eR[j]  (W and eR through a wave-private LDS
// tile; eR is read back once, all reads of a W row are requested together).  Written per partition: residual
// log S~, offset, the two shifts; then, by the first wave, the mixture.  KQ = ceil(K / 4).
constexpr int RF_WAVES = ROOT_FWD_WAVES, RF_SB = ROOT_FWD_SAMPLES;

template <int KQ>
__global__ __launch_bounds__(64 * RF_WAVES) void k_root_forward(const int32_t* __restrict__ rec,
                                                               const float* __restrict__ params, float* __restrict__ A,
                                                               double* __restrict__ Off, float* __restrict__ amax,
                                                               float* __restrict__ logp, int B, int K) {
    constexpr int K4 = 4 * KQ, KS = (KQ & 1) ? K4 : K4 + 4;     // row stride, see root_row_stride
    constexpr int NR = (K4 + 15) / 16;                          // entries of a row per lane
    constexpr int NW = (K4 * KQ + 63) / 64;                     // 16-byte pieces of W per lane
    extern __shared__ float lds[];
    const int P = rec[0], root = rec[1], voff = rec[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bl = lane >> 4, t = lane & 15;
    const int b = blockIdx.x * RF_SB + bl;
    const bool valid = b < B;
    const int bc = valid ? b : B - 1;                  // (lanes beyond the batch read a valid row and store nothing)
    float* Wl = lds + (size_t)wave * (K * KS + RF_SB * KS);
    float* eRs = Wl + K * KS;
    double* poff = reinterpret_cast<double*>(lds + (size_t)RF_WAVES * (K * KS + RF_SB * KS));   // [P][RF_SB]
    float* pres = reinterpret_cast<float*>(poff + (size_t)P * RF_SB);                           // [P][RF_SB]
    float* pv = pres + (size_t)P * RF_SB;                                                       // [P]: mixing weights
    const size_t blk = (size_t)B * K;
    for (int p = wave; p < P; p += RF_WAVES) {
        const int32_t* q = rec + 4 + p * ROOT_REC_STRIDE;
        const int item = q[0], left = q[1], right = q[2], out = q[3];
        const float* W = params + q[4];
        // everything is requested before anything is used: offsets, rows, weights
        double offc = 0.0;
        float vmix = 1.f;
        if (t == 0) {
            offc = Off[(size_t)left * B + bc] + Off[(size_t)right * B + bc];
            if (voff >= 0) vmix = params[voff + q[5]];
        }
        float l[NR], r[NR];
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int i = t + 16 * u;
            l[u] = i < K ? A[(size_t)left * blk + (size_t)bc * K + i] : -INFINITY;
            r[u] = i < K ? A[(size_t)right * blk + (size_t)bc * K + i] : -INFINITY;
        }
        if ((K & 3) == 0) {
            float4 w[NW];
#pragma unroll
            for (int u = 0; u < NW; ++u) w[u] = *reinterpret_cast<const float4*>(W + 4 * (size_t)min(lane + 64 * u, K4 * KQ - 1));
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                const int f = lane + 64 * u;
                if (f < K4 * KQ) *reinterpret_cast<float4*>(Wl + (f / KQ) * KS + 4 * (f % KQ)) = w[u];
            }
        } else {
            for (int f0 = lane; f0 < K * K4; f0 += 64 * 8) {
                float w[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int f = f0 + 64 * u, row = f / K4, j = f - row * K4;
                    w[u] = (f < K * K4 && j < K) ? W[(size_t)row * K + j] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int f = f0 + 64 * u, row = f / K4, j = f - row * K4;
                    if (f < K * K4) Wl[row * KS + j] = w[u];
                }
            }
        }
        float xl = -INFINITY, xr = -INFINITY;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            xl = fmaxf(xl, l[u]);
            xr = fmaxf(xr, r[u]);
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            xl = fmaxf(xl, __shfl_xor(xl, o, 64));
            xr = fmaxf(xr, __shfl_xor(xr, o, 64));
        }
        if (xl == -INFINITY) xl = 0.f;                 // an all-zero input vector: exp(-inf) = 0, no NaN
        if (xr == -INFINITY) xr = 0.f;
        float el[NR];
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int i = t + 16 * u;
            el[u] = __expf(l[u] - xl);
            if (i < K4) eRs[bl * KS + i] = __expf(r[u] - xr);      // (entries K .. K4 - 1: exp(-inf) = 0)
        }
        wave_lds_fence();
        float4 er[KQ];
#pragma unroll
        for (int j = 0; j < KQ; ++j) er[j] = *reinterpret_cast<const float4*>(eRs + bl * KS + 4 * j);
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < NR; ++u) {
            const int i = min(t + 16 * u, K - 1);      // (a lane without an entry reads a valid row; its eL is 0)
            float4 w[KQ];
#pragma unroll
            for (int j = 0; j < KQ; ++j) w[j] = *reinterpret_cast<const float4*>(Wl + i * KS + 4 * j);
            float d0 = 0.f, d1 = 0.f;
#pragma unroll
            for (int j = 0; j < KQ; ++j) {
                d0 = fmaf(w[j].x, er[j].x, d0);
                d1 = fmaf(w[j].y, er[j].y, d1);
                d0 = fmaf(w[j].z, er[j].z, d0);
                d1 = fmaf(w[j].w, er[j].w, d1);
            }
            acc = fmaf(t + 16 * u < K ? el[u] : 0.f, d0 + d1, acc);
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) acc += __shfl_xor(acc, o, 64);
        if (t == 0) {
            const float res = __logf(acc);             // residual against the children's offsets plus the shifts
            const double off = offc + (double)xl + (double)xr;
            if (valid) {
                A[(size_t)out * blk + (size_t)b * K] = res;
                Off[(size_t)out * B + b] = off;
                amax[((size_t)item * 2) * B + b] = xl; // the shifts, kept for the top-down pass
                amax[((size_t)item * 2 + 1) * B + b] = xr;
                if (P == 1 && logp) logp[b] = (float)(off + (double)res);   // the only partition writes the root itself
            }
            poff[p * RF_SB + bl] = off;
            pres[p * RF_SB + bl] = res;
            if (bl == 0) pv[p] = vmix;
        }
        wave_lds_fence();                              // the tile is free for the wave's next partition
    }
    if (P == 1) return;
    __syncthreads();
    if (wave == 0) {
        // mixture of the partitions: offset = the largest of theirs, residual = log sum_c v[c] exp((Off[c] - offset) + A[c])
        double m = -INFINITY;
        for (int p = t; p < P; p += 16) m = fmax(m, poff[p * RF_SB + bl]);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) m = fmax(m, __shfl_xor(m, o, 64));
        float s = 0.f;
        for (int p = t; p < P; p += 16) s += pv[p] * expf((float)(poff[p * RF_SB + bl] - m) + pres[p * RF_SB + bl]);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
        if (t == 0 && valid) {
            const float res = logf(s);
            A[(size_t)root * blk + (size_t)b * K] = res;
            Off[(size_t)root * B + b] = m;
            if (logp) logp[b] = (float)(m + (double)res);
        }
    }
}

// ------------------------------------------------------------------ top-down
// With one output entry the posterior weight of a sample is a scalar,
//     q[b] = v exp((Off[out][b] - Off[root][b]) - A[root][b])            (v = 1, Off[out] = Off[root] for one partition;
// the root's own posterior is 1), and with QL[b][i] = q[b] eL[b][i]:
//     Nw[i][j]      += W[i][j] sum_b QL[b][i] eR[b][j]
//     Gp_left[b][i]  = QL[b][i] sum_j W[i][j] eR[b][j]
//     Gp_right[b][j] = eR[b][j] sum_i W[i][j] QL[b][i].
// A workgroup takes one partition and a run of slices (four consecutive left entries i each), the same split and the
// same posterior blocks as the general top-down kernel: the left block is complete per slice, the right block of the
// workgroup holds the sum over its slices.  Per slice and pass of RB_BC samples everything is requested at once (the
// right rows, the slice's four left entries, offsets, shifts, the four W rows) and staged in LDS: eR both sample-major
// (statistics and left posterior: lanes along the batch) and row-major (right posterior: lanes along j, stores
// coalesced), QL likewise, W transposed [j][4].
constexpr int RB_BC = 128, RB_ST = RB_BC + 4, RB_THREADS = 512;

template <int KQ>
struct RootBwdLayout {
    static constexpr int K4 = 4 * KQ, KS = (KQ & 1) ? K4 : K4 + 4;
    static constexpr int OFF_RT = 0;                         // eR^T [K4][RB_ST]
    static constexpr int OFF_R = OFF_RT + K4 * RB_ST;        // eR   [RB_BC][KS]
    static constexpr int OFF_QT = OFF_R + RB_BC * KS;        // QL^T [4][RB_ST]
    static constexpr int OFF_Q = OFF_QT + 4 * RB_ST;         // QL   [RB_BC][4]
    static constexpr int OFF_WT = OFF_Q + 4 * RB_BC;         // W^T  [K4][4] of the slice
    static constexpr int LDS_FLOATS = OFF_WT + 4 * K4;
};

template <int KQ>
__global__ __launch_bounds__(RB_THREADS) void k_root_backward(const int32_t* __restrict__ rec, const float* __restrict__ params,
                                                       float* __restrict__ stats, const float* __restrict__ A,
                                                       const double* __restrict__ Off, const float* __restrict__ amax,
                                                       float* __restrict__ Gp, int ngroups, int accumulate, int B, int K,
                                                       int vper, int cpv, float* __restrict__ part, int n_partitions) {
    using LY = RootBwdLayout<KQ>;
    constexpr int K4 = LY::K4, KS = LY::KS;
    extern __shared__ float lds[];
    float* sRT = lds + LY::OFF_RT;
    float* sR = lds + LY::OFF_R;
    float* sQT = lds + LY::OFF_QT;
    float* sQ = lds + LY::OFF_Q;
    float* sWT = lds + LY::OFF_WT;
    const int root = rec[1], voff = rec[2];
    // vper > 1: workgroup (partition, group of slices, share vg of the chunks) takes the samples [bfirst, bend) and
    // writes its statistics to block (vg, partition) of part; a launch that follows adds the blocks up
    const int pg = blockIdx.x / vper, vg = blockIdx.x - pg * vper;
    const int p = pg / ngroups, grp = pg - p * ngroups;
    const int bfirst = vg * cpv * RB_BC, bend = min(B, bfirst + cpv * RB_BC);
    const int32_t* q = rec + 4 + p * ROOT_REC_STRIDE;
    const int item = q[0], left = q[1], right = q[2], out = q[3], woff = q[4];
    const int it0 = grp * KQ / ngroups, it1 = (grp + 1) * KQ / ngroups;
    const int tid = threadIdx.x;
    const size_t blk = (size_t)B * K;
    const float* Lp = A + (size_t)left * blk;
    const float* Rp = A + (size_t)right * blk;
    const float* As = A + (size_t)root * blk;
    const double* Oo = Off + (size_t)out * B;
    const double* Os = Off + (size_t)root * B;
    const float* aL = amax + (size_t)item * 2 * B;
    const float* aR = aL + B;
    const float* W = params + woff;
    float* Nw = vper > 1 ? part + ((size_t)vg * n_partitions + p) * ((size_t)K * K) : stats + woff;
    const int nblk = 1 + KQ;
    float* gleft = Gp + (size_t)item * nblk * blk;
    float* gright = Gp + ((size_t)item * nblk + 1 + grp) * blk;
    const bool vec = (K & 3) == 0;
    // Roles within a pass (they run side by side): threads 0 .. 127 stage QL and take the left child (one sample each),
    // threads 128 .. 128 + 4K - 1 take the statistics (entry (il, j) each; the first K4 of them also bring the W rows in),
    // everybody stages eR and shares the right child.
    const int st = tid - 128;
    const int sil = st >= 0 ? st / K : 0, sj = st - sil * K;
    for (int it = it0; it < it1; ++it) {
        const bool sact = st >= 0 && st < 4 * K && 4 * it + sil < K;
        float acc = 0.f;
        // (this thread's weight and old statistic are requested with the first pass, not after the last)
        const size_t sidx = sact ? (size_t)(4 * it + sil) * K + sj : 0;
        const float wown = sact ? W[sidx] : 0.f;
        const float nold = sact && accumulate ? Nw[sidx] : 0.f;
        for (int b0 = bfirst; b0 < bend; b0 += RB_BC) {
            const int nb = min(RB_BC, bend - b0), nb4 = (nb + 3) & ~3;
            // ---- requests: everything this pass needs, before the first value is used
            float vq = 1.f, lq[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}, alq = 0.f, asq = 0.f;
            double ddq = 0.0;
            if (tid < nb) {
                const int b = b0 + tid;
                if (voff >= 0) vq = params[voff + q[5]];
                ddq = Oo[b] - Os[b];
                asq = As[(size_t)b * K];
                alq = aL[b];
                if (vec) {
                    const float4 l4 = *reinterpret_cast<const float4*>(Lp + (size_t)b * K + 4 * it);
                    lq[0] = l4.x, lq[1] = l4.y, lq[2] = l4.z, lq[3] = l4.w;
                } else {
#pragma unroll
                    for (int il = 0; il < 4; ++il)
                        if (4 * it + il < K) lq[il] = Lp[(size_t)b * K + 4 * it + il];
                }
            }
            float wq[4] = {0.f, 0.f, 0.f, 0.f};            // thread j < K4: column j of the slice's four W rows
            if (tid >= 128 && tid < 128 + K4) {
                const int j = tid - 128;
#pragma unroll
                for (int il = 0; il < 4; ++il)
                    if (4 * it + il < K && j < K) wq[il] = W[(size_t)(4 * it + il) * K + j];
            }
            constexpr int NF = (RB_BC * KQ + RB_THREADS - 1) / RB_THREADS;   // 16-byte pieces of the right rows per thread
            float4 r4[NF];
            float ar[NF];
#pragma unroll
            for (int n = 0; n < NF; ++n) {
                const int f = min(tid + RB_THREADS * n, nb * KQ - 1), row = f / KQ, k4 = f - row * KQ;
                ar[n] = aR[b0 + row];
                if (vec) {
                    r4[n] = *reinterpret_cast<const float4*>(Rp + (size_t)(b0 + row) * K + 4 * k4);
                } else {
                    const float* src = Rp + (size_t)(b0 + row) * K + 4 * k4;
                    r4[n].x = 4 * k4 + 0 < K ? src[0] : -INFINITY;
                    r4[n].y = 4 * k4 + 1 < K ? src[1] : -INFINITY;
                    r4[n].z = 4 * k4 + 2 < K ? src[2] : -INFINITY;
                    r4[n].w = 4 * k4 + 3 < K ? src[3] : -INFINITY;
                }
            }
            __syncthreads();                               // the previous pass (or slice) has been read
            // ---- staging
            if (tid < nb4) {
                const float qv = tid < nb ? vq * __expf((float)ddq - asq) : 0.f;
                float4 ql;
                ql.x = tid < nb ? qv * __expf(lq[0] - alq) : 0.f;     // (entries beyond K: exp(-inf) = 0)
                ql.y = tid < nb ? qv * __expf(lq[1] - alq) : 0.f;
                ql.z = tid < nb ? qv * __expf(lq[2] - alq) : 0.f;
                ql.w = tid < nb ? qv * __expf(lq[3] - alq) : 0.f;
                *reinterpret_cast<float4*>(sQ + 4 * tid) = ql;
                sQT[tid] = ql.x, sQT[RB_ST + tid] = ql.y, sQT[2 * RB_ST + tid] = ql.z, sQT[3 * RB_ST + tid] = ql.w;
            }
            if (tid >= 128 && tid < 128 + K4)
                *reinterpret_cast<float4*>(sWT + 4 * (tid - 128)) = make_float4(wq[0], wq[1], wq[2], wq[3]);
#pragma unroll
            for (int n = 0; n < NF; ++n) {
                const int f = tid + RB_THREADS * n, row = f / KQ, k4 = f - row * KQ;
                if (f < nb4 * KQ) {
                    const bool in = row < nb;              // rows nb .. nb4 - 1 are zeros: the loops below run over whole fours
                    float4 e;
                    e.x = in ? __expf(r4[n].x - ar[n]) : 0.f;
                    e.y = in ? __expf(r4[n].y - ar[n]) : 0.f;
                    e.z = in ? __expf(r4[n].z - ar[n]) : 0.f;
                    e.w = in ? __expf(r4[n].w - ar[n]) : 0.f;
                    *reinterpret_cast<float4*>(sR + row * KS + 4 * k4) = e;
                    sRT[(4 * k4 + 0) * RB_ST + row] = e.x;
                    sRT[(4 * k4 + 1) * RB_ST + row] = e.y;
                    sRT[(4 * k4 + 2) * RB_ST + row] = e.z;
                    sRT[(4 * k4 + 3) * RB_ST + row] = e.w;
                }
            }
            __syncthreads();
            // ---- statistics: thread (il, j) contracts the batch, four samples per 16-byte read
            if (sact) {
                const float* qp = sQT + sil * RB_ST;
                const float* rp = sRT + sj * RB_ST;
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
                for (int m = 0; m < nb4; m += 4) {
                    const float4 qq = *reinterpret_cast<const float4*>(qp + m);
                    const float4 rr = *reinterpret_cast<const float4*>(rp + m);
                    a0 = fmaf(qq.x, rr.x, a0);
                    a1 = fmaf(qq.y, rr.y, a1);
                    a2 = fmaf(qq.z, rr.z, a2);
                    a3 = fmaf(qq.w, rr.w, a3);
                }
                acc += (a0 + a1) + (a2 + a3);
            }
            // ---- left child: thread b takes the four entries of the slice
            if (tid < nb) {
                float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll 4
                for (int j = 0; j < K4; ++j) {
                    const float4 w = *reinterpret_cast<const float4*>(sWT + 4 * j);
                    const float r = sRT[j * RB_ST + tid];
                    d0 = fmaf(w.x, r, d0);
                    d1 = fmaf(w.y, r, d1);
                    d2 = fmaf(w.z, r, d2);
                    d3 = fmaf(w.w, r, d3);
                }
                const float4 ql = *reinterpret_cast<const float4*>(sQ + 4 * tid);
                float* dst = gleft + (size_t)(b0 + tid) * K + 4 * it;
                if (vec) {
                    *reinterpret_cast<float4*>(dst) = make_float4(ql.x * d0, ql.y * d1, ql.z * d2, ql.w * d3);
                } else {
                    if (4 * it + 0 < K) dst[0] = ql.x * d0;
                    if (4 * it + 1 < K) dst[1] = ql.y * d1;
                    if (4 * it + 2 < K) dst[2] = ql.z * d2;
                    if (4 * it + 3 < K) dst[3] = ql.w * d3;
                }
            }
            // ---- right child: lanes along j, the workgroup's slices summed in place (the same thread owns an entry in
            // every slice)
#pragma unroll 4
            for (int e = tid; e < nb * K4; e += RB_THREADS) {
                const int bl = e / K4, j = e - bl * K4;    // (K4 is a constant: no division)
                const float4 ql = *reinterpret_cast<const float4*>(sQ + 4 * bl);
                const float4 w = *reinterpret_cast<const float4*>(sWT + 4 * j);
                const float tsum = fmaf(w.x, ql.x, fmaf(w.y, ql.y, fmaf(w.z, ql.z, w.w * ql.w)));
                if (j < K) {
                    float* dst = gright + (size_t)(b0 + bl) * K + j;
                    *dst = sR[bl * KS + j] * tsum + (it > it0 ? *dst : 0.f);
                }
            }
        }
        if (sact) Nw[sidx] = wown * acc + nold;
    }
}

template <int KQ>
void launch_root_forward_kq(const DevTables& t, int n_partitions, const float* params, float* A, double* Off, float* amax,
                            float* logp, const Dims& d, hipStream_t s) {
    const size_t lds = root_forward_lds_bytes(d.K, n_partitions);
    if (lds > 64 * 1024) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] { allow_dynamic_lds(&k_root_forward<KQ>, 160 * 1024); });
    }
    hipLaunchKernelGGL(k_root_forward<KQ>, dim3((d.B + RF_SB - 1) / RF_SB), dim3(64 * RF_WAVES), lds, s, t.root_rec, params,
                       A, Off, amax, logp, d.B, d.K);
}

template <int KQ>
void launch_root_backward_kq(const DevTables& t, int n_partitions, const int32_t* e_woff, float* part,
                             PartialSumList* jobs, bool accumulate, const float* params, float* stats, const float* A,
                             const double* Off, const float* amax, float* Gp, const Dims& d, hipStream_t s) {
    const size_t lds = sizeof(float) * RootBwdLayout<KQ>::LDS_FLOATS;
    if (lds > 64 * 1024) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] { allow_dynamic_lds(&k_root_backward<KQ>, lds); });
    }
    const int ngroups = bwd_groups_per_item(n_partitions, d.K);
    const int vper = part && jobs && jobs->n < PARTIAL_SUM_JOBS ? root_bwd_virtual_items(n_partitions, d.K, d.B) : 1;
    const int nchunks = (d.B + RB_BC - 1) / RB_BC, cpv = (nchunks + vper - 1) / vper;
    // (with virtual items the blocks are written, never added to; their sum, later, adds to the statistics or overwrites them)
    hipLaunchKernelGGL(k_root_backward<KQ>, dim3(n_partitions * ngroups * vper), dim3(RB_THREADS), lds, s, t.root_rec, params,
                       stats, A, Off, amax, Gp, ngroups, vper > 1 ? 0 : (accumulate ? 1 : 0), d.B, d.K, vper, cpv, part,
                       n_partitions);
    if (vper > 1) jobs->job[jobs->n++] = PartialSumJob{e_woff, part, n_partitions, vper, d.K * d.K};
}

}  // namespace

void launch_root_forward(const DevTables& t, int n_partitions, const float* params, float* A, double* Off, float* amax,
                         float* logp, const Dims& d, hipStream_t s) {
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_root_forward_kq<J>(t, n_partitions, params, A, Off, amax, logp, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

void launch_root_backward(const DevTables& t, int n_partitions, const int32_t* e_woff, float* part, PartialSumList* jobs,
                          bool accumulate, const float* params, float* stats,
                          const float* A, const double* Off, const float* amax, float* Gp, const Dims& d, hipStream_t s) {
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_root_backward_kq<J>(t, n_partitions, e_woff, part, jobs, accumulate, params, stats, A, Off, amax, Gp, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

}  // namespace einet_impl
