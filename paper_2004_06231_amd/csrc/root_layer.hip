// The top of the circuit bottom-up, in one launch.  The partitions of the root are einsum items with a single output
// entry (Eq. 3-5): K^2 multiply-adds per sample, far too little for the matrix pipe to matter, so this launch is a
// chain of dependent memory requests.  The kernel reads one record (all indices of all partitions), requests rows,
// offsets and weights together, works on the vector ALU, and forms the root's mixture (App. B) and log P itself.
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

}  // namespace einet_impl
