// Bottom-up pass: einsum layers (Eq. 3-5) and mixing layers (App. B).
#include "device_common.hpp"

#include <mutex>

namespace einet_impl {

namespace {

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

// Orders the LDS traffic of one wave: what its lanes wrote before is visible to all its lanes after (the LDS
// serves the requests of a wave in order; this keeps the compiler from moving accesses across).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int KQ>
__global__ __launch_bounds__(512, KQ >= 14 ? 2 : 4) void k_einsum_forward(const int32_t* __restrict__ e_left,
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
    const int vb = xcd_contiguous_block();
    const int li = vb / nkt, kt = vb - li * nkt;
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
        // four 16-byte loads per thread in flight before the first goes to LDS
        for (int q0 = tid; q0 < 4 * KP * KQ; q0 += 4 * blockDim.x) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * blockDim.x;
                const int j4 = q % KQ, i = (q / KQ) % KP, kl = q / (KQ * KP);
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (q < 4 * KP * KQ && 4 * kt + kl < kout && i < K)
                    v[u] = *reinterpret_cast<const float4*>(W + ((size_t)(4 * kt + kl) * K + i) * K + 4 * j4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * blockDim.x;
                if (q < 4 * KP * KQ) {
                    const int j4 = q % KQ, i = (q / KQ) % KP, kl = q / (KQ * KP);
                    float* dst = Wl + kl * SK + i * SJ + 4 * j4;
                    *reinterpret_cast<float2*>(dst) = make_float2(v[u].x, v[u].y);
                    *reinterpret_cast<float2*>(dst + 2) = make_float2(v[u].z, v[u].w);
                }
            }
        }
    } else {
        for (int q0 = tid; q0 < 4 * KP * KP; q0 += 8 * blockDim.x) {     // eight loads in flight, as above
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * blockDim.x;
                const int j = q % KP, i = (q / KP) % KP, kl = q / (KP * KP);
                v[u] = 0.f;
                if (q < 4 * KP * KP && 4 * kt + kl < kout && i < K && j < K) v[u] = W[((size_t)(4 * kt + kl) * K + i) * K + j];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * blockDim.x;
                if (q < 4 * KP * KP) Wl[(q / (KP * KP)) * SK + ((q / KP) % KP) * SJ + q % KP] = v[u];
            }
        }
    }
    __syncthreads();

    const float* wl = Wl + gm * SK + rm * SJ + g;    // + it*4*SJ + 4*s : contraction index j = 4s + g
    float* elw = Wl + LY::LDS_W + wave * (16 * LY::SE);   // this wave's eL tile [16][SE]
    for (int bt0 = 0; bt0 < n_btiles; bt0 += nwaves) {
        const int bt = bt0 + wave;
        const int b = bt * 16 + c;
        const bool ok = bt < n_btiles && b < B;
        // offsets of the children, needed only when the result is stored: requested now, used at the end
        double off_children = 0.0;
        if (ok && kt == 0 && g == 0)
            off_children = Off[(size_t)e_left[li] * B + b] + Off[(size_t)e_right[li] * B + b];
        // lane (c, g) holds entries 4s+g of row b of both inputs
        float er[KQ], el[KQ];
        float mr = -INFINITY, ml = -INFINITY;
        if ((K & 3) == 0) {
            // The 16 rows of the tile are contiguous in memory: they are fetched with 16-byte loads, consecutive
            // lanes consecutive addresses, and reach the operand layout through the wave's LDS tile.
            constexpr int NFW = (16 * KQ + 63) / 64;
            const int rows = bt < n_btiles ? min(16, B - 16 * bt) : 0;
            float4 rawR[NFW], rawL[NFW];
#pragma unroll
            for (int n = 0; n < NFW; ++n) {
                const int f = min(lane + 64 * n, max(rows, 1) * KQ - 1);
                rawR[n] = rawL[n] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (rows > 0) {
                    rawR[n] = *reinterpret_cast<const float4*>(Rp + (size_t)16 * bt * K + 4 * f);
                    rawL[n] = *reinterpret_cast<const float4*>(Lp + (size_t)16 * bt * K + 4 * f);
                }
            }
            wave_lds_sync();                         // the previous tile's reads of eL are done
#pragma unroll
            for (int n = 0; n < NFW; ++n) {
                const int f = lane + 64 * n;
                if (f < 16 * KQ) *reinterpret_cast<float4*>(elw + (f / KQ) * LY::SE + 4 * (f % KQ)) = rawR[n];
            }
            wave_lds_sync();
#pragma unroll
            for (int s = 0; s < KQ; ++s) er[s] = ok ? elw[c * LY::SE + 4 * s + g] : -INFINITY;
            wave_lds_sync();
#pragma unroll
            for (int n = 0; n < NFW; ++n) {
                const int f = lane + 64 * n;
                if (f < 16 * KQ) *reinterpret_cast<float4*>(elw + (f / KQ) * LY::SE + 4 * (f % KQ)) = rawL[n];
            }
            wave_lds_sync();
#pragma unroll
            for (int s = 0; s < KQ; ++s) el[s] = ok ? elw[c * LY::SE + 4 * s + g] : -INFINITY;
        } else {
#pragma unroll
            for (int s = 0; s < KQ; ++s) {
                const int j = 4 * s + g;
                const bool in = ok && j < K;
                er[s] = in ? Rp[(size_t)b * K + j] : -INFINITY;
                el[s] = in ? Lp[(size_t)b * K + j] : -INFINITY;
            }
            wave_lds_sync();                         // the previous tile's reads of eL are done
        }
#pragma unroll
        for (int s = 0; s < KQ; ++s) {
            mr = fmaxf(mr, er[s]);
            ml = fmaxf(ml, el[s]);
        }
        mr = fmaxf(mr, __shfl_xor(mr, 16, 64));
        mr = fmaxf(mr, __shfl_xor(mr, 32, 64));
        ml = fmaxf(ml, __shfl_xor(ml, 16, 64));
        ml = fmaxf(ml, __shfl_xor(ml, 32, 64));
        if (mr == -INFINITY) mr = 0.f;               // an all-zero input vector: exp(-inf) = 0, no NaN
        if (ml == -INFINITY) ml = 0.f;
        // (the tile is private to the wave, and every lane overwrites the entries it has read itself)
#pragma unroll
        for (int s = 0; s < KQ; ++s) {
            er[s] = __expf(er[s] - mr);              // stays in registers: the B operand
            elw[c * LY::SE + 4 * s + g] = __expf(el[s] - ml);
        }
        wave_lds_sync();
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
            const double off = off_children + (double)ml + (double)mr;
            Off[(size_t)e_out[li] * B + b] = off;
            if (logp && e_out[li] == 0) logp[b] = (float)(off + (double)res);   // node 0: the root region, one entry
            amax[((size_t)item * 2) * B + b] = ml;     // the shifts, kept for the top-down pass
            amax[((size_t)item * 2 + 1) * B + b] = mr;
        }
    }
}

// ------------------------------------------------------------------ einsum layer, forward, K a multiple of 8
// The same factorisation on v_mfma_f32_32x32x2_f32 (the fp32 shape that issues at the full rate of the matrix
// pipe), as one workgroup per compute unit that walks a run of work units.  A tile of the product T has 32 rows
// (k, i) and 32 samples; with i fastest, groups of 8 rows stay inside one k, and a lane holds four consecutive i of
// four such groups, so the i-reduction is again in-lane: 16 FMAs per tile.  K / 8 tiles hold exactly four k.
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int K8>
struct FwdSLayout {
    static constexpr int K = 8 * K8;
    static constexpr int RS = K + 4;                 // row stride (floats): RS/4 odd -> 16-byte operand reads of 8 lanes hit 32 banks
    static constexpr int SLICE = 4 * K * RS;         // W[4 k][K i][RS]
    static constexpr int OFF_E = 2 * SLICE;          // eR, eL of the four sample tiles: [tile][2][K8][64 lanes][4]
    static constexpr int OFF_S = OFF_E + 4 * 2 * K8 * 256;   // sums of a unit: [2 slots][tile][64 lanes][4]
    static constexpr int LDS_FLOATS = OFF_S + 2 * 4 * 256;
    static constexpr int NQ4 = 4 * K * (K / 4);      // float4 of a slice
    static constexpr int NL = (NQ4 + 255) / 256;     // per producer thread
};

// A workgroup owns a run of units; a unit is (item, batch chunk of 128 samples, 4 outputs k) = K8 tiles of 32 rows
// (k, i) of the product W[(k,i), j] eR[j, b].  Waves 0-3 only run the matrix pipe: wave w owns samples 32 w .. 32 w + 31
// of the chunk, reads its operands from LDS and leaves four sums per lane in LDS.  Waves 4-7 do everything else: they
// bring the W slices and the child rows in, form exp(x - max), and turn the sums of the previous unit into log values.
template <int K8>
__global__ __launch_bounds__(512, 1) void k_einsum_forward_s(const int32_t* __restrict__ e_left,
                                                           const int32_t* __restrict__ e_right,
                                                           const int32_t* __restrict__ e_out,
                                                           const int32_t* __restrict__ e_woff,
                                                           const float* __restrict__ params, float* __restrict__ A,
                                                           double* __restrict__ Off, float* __restrict__ amax,
                                                           int item0, int count, int B) {
    using LY = FwdSLayout<K8>;
    constexpr int K = LY::K, RS = LY::RS, NQ = K / 4, NL = LY::NL;
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int nt = wave & 3;                          // sample tile of this wave (both roles)
    const int nchunks = (B + 127) >> 7;
    const int U = count * nchunks * NQ;              // unit = (item, chunk, quad), quad fastest
    const int g = xcd_contiguous_block();
    const int u0 = (int)((long long)g * U / gridDim.x), u1 = (int)((long long)(g + 1) * U / gridDim.x);
    if (u0 >= u1) return;
    // position of the first unit
    int quad = u0 % NQ, chunk = (u0 / NQ) % nchunks, li = u0 / (NQ * nchunks);
    float* erl = lds + LY::OFF_E + nt * (2 * K8 * 256) + lane * 4;       // + (2 * which + t) * 256 ... see below

    if (wave >= 4) {
        // ------------------------------------------------------------ producer waves
        const int pt = tid - 256;
        floatx4 wv[NL];
#define FETCH_W(li_, quad_)                                                                \
    {                                                                                      \
        const float* W_ = params + e_woff[li_] + (size_t)(quad_) * 4 * K * K;              \
        _Pragma("unroll") for (int q = 0; q < NL; ++q) {                                   \
            const int f = min(pt + 256 * q, LY::NQ4 - 1);                                  \
            wv[q] = *reinterpret_cast<const floatx4*>(W_ + (size_t)4 * f);                 \
        }                                                                                  \
    }
#define STORE_W(buf_)                                                                      \
    {                                                                                      \
        _Pragma("unroll") for (int q = 0; q < NL; ++q) {                                   \
            const int f = pt + 256 * q;                                                    \
            const int row = f / (K / 4), c4 = f - row * (K / 4);                           \
            if (f < LY::NQ4) *reinterpret_cast<floatx4*>((buf_) + row * RS + 4 * c4) = wv[q]; \
        }                                                                                  \
    }
        // rows of (item, chunk): lane (n, h) of tile nt takes entries 8 t + 4 h .. + 3 of sample 32 nt + n; exp(x - max)
        // goes to LDS for the matrix wave of the same tile; the item's first unit also owns the offsets and shifts
        auto rows = [&](int rli, int rchunk, bool owner) {
            const int b = rchunk * 128 + nt * 32 + n;
            const int bc = min(b, B - 1);              // rows beyond the batch read the last one again
            const int left = e_left[rli], right = e_right[rli];
            const float* Lp = A + ((size_t)left * B + bc) * K + 4 * h;
            const float* Rp = A + ((size_t)right * B + bc) * K + 4 * h;
            floatx4 rawR[K8], rawL[K8];
#pragma unroll
            for (int t = 0; t < K8; ++t) {
                rawR[t] = *reinterpret_cast<const floatx4*>(Rp + 8 * t);
                rawL[t] = *reinterpret_cast<const floatx4*>(Lp + 8 * t);
            }
            double off_children = 0.0;
            if (owner && h == 0) off_children = Off[(size_t)left * B + bc] + Off[(size_t)right * B + bc];
            float xr = -INFINITY, xl = -INFINITY;
#pragma unroll
            for (int t = 0; t < K8; ++t) {
                xr = fmaxf(fmaxf(xr, fmaxf(rawR[t][0], rawR[t][1])), fmaxf(rawR[t][2], rawR[t][3]));
                xl = fmaxf(fmaxf(xl, fmaxf(rawL[t][0], rawL[t][1])), fmaxf(rawL[t][2], rawL[t][3]));
            }
            xr = fmaxf(xr, __shfl_xor(xr, 32, 64));
            xl = fmaxf(xl, __shfl_xor(xl, 32, 64));
            if (xr == -INFINITY) xr = 0.f;             // an all-zero input vector: exp(-inf) = 0, no NaN
            if (xl == -INFINITY) xl = 0.f;
#pragma unroll
            for (int t = 0; t < K8; ++t) {
                floatx4 er, el;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    er[c] = __expf(rawR[t][c] - xr);
                    el[c] = __expf(rawL[t][c] - xl);
                }
                *reinterpret_cast<floatx4*>(erl + t * 256) = er;
                *reinterpret_cast<floatx4*>(erl + (K8 + t) * 256) = el;
            }
            if (owner && h == 0 && b < B) {
                const int out = e_out[rli];
                Off[(size_t)out * B + b] = off_children + (double)xl + (double)xr;
                amax[((size_t)(item0 + rli) * 2) * B + b] = xl;
                amax[((size_t)(item0 + rli) * 2 + 1) * B + b] = xr;
            }
        };
        // sums of a finished unit -> residuals log S~
        auto finish = [&](int fli, int fchunk, int fquad, int slot) {
            const float* sp = lds + LY::OFF_S + (slot * 4 + nt) * 256 + n * 4;
            const floatx4 s0 = *reinterpret_cast<const floatx4*>(sp);
            const floatx4 s1 = *reinterpret_cast<const floatx4*>(sp + 128);
            const int b = fchunk * 128 + nt * 32 + n;
            if (h == 0 && b < B) {
                floatx4 r;
#pragma unroll
                for (int c = 0; c < 4; ++c) r[c] = __logf(s0[c] + s1[c]);
                *reinterpret_cast<floatx4*>(A + ((size_t)e_out[fli] * B + b) * K + 4 * fquad) = r;
            }
        };
        rows(li, chunk, quad == 0);                     // (the matrix waves bring the first slice in)
        // position of the unit whose slice is in flight
        int lq = quad, lc = chunk, lli = li;
        auto advance = [&](int& q_, int& c_, int& i_) {
            if (++q_ == NQ) { q_ = 0; if (++c_ == nchunks) { c_ = 0; ++i_; } }
        };
        advance(lq, lc, lli);
        if (u0 + 1 < u1) FETCH_W(lli, lq)
        __syncthreads();                                // B0: slice u0 and the first rows are in LDS
        __syncthreads();                                // X: the matrix waves hold the rows in registers
        int pq = quad, pc = chunk, pli = li;            // previous unit
        for (int u = u0; u < u1; ++u) {
            // the matrix waves work on unit u = (li, chunk, quad)
            if (u + 1 < u1) {
                STORE_W(lds + ((u + 1 - u0) & 1) * LY::SLICE)
                int q2 = lq, c2 = lc, i2 = lli;
                advance(q2, c2, i2);
                if (u + 2 < u1) FETCH_W(i2, q2)
            }
            if (u > u0) finish(pli, pc, pq, (u - 1 - u0) & 1);
            const bool new_rows = u + 1 < u1 && quad == NQ - 1;
            if (new_rows) rows(lli, lc, true);
            pq = quad; pc = chunk; pli = li;
            quad = lq; chunk = lc; li = lli;
            advance(lq, lc, lli);
            __syncthreads();                            // B(u+1)
            if (new_rows) __syncthreads();              // X
        }
        finish(pli, pc, pq, (u1 - 1 - u0) & 1);
    } else {
        // ------------------------------------------------------------ matrix waves
        float er[4 * K8], el[K8][4];
        const bool active = chunk * 128 + nt * 32 < B || nchunks > 1;     // (a tile beyond a short batch does nothing)
        {
            // the first W slice, while the producer waves fetch and shift the first rows
            const float* W_ = params + e_woff[li] + (size_t)quad * 4 * K * K;
            floatx4 w0[NL];
#pragma unroll
            for (int q = 0; q < NL; ++q) w0[q] = *reinterpret_cast<const floatx4*>(W_ + (size_t)4 * min(tid + 256 * q, LY::NQ4 - 1));
#pragma unroll
            for (int q = 0; q < NL; ++q) {
                const int f = tid + 256 * q;
                const int row = f / (K / 4), c4 = f - row * (K / 4);
                if (f < LY::NQ4) *reinterpret_cast<floatx4*>(lds + row * RS + 4 * c4) = w0[q];
            }
        }
        __syncthreads();                                // B0
        bool load_rows = true;
        for (int u = u0; u < u1; ++u) {
            if (load_rows) {
#pragma unroll
                for (int t = 0; t < K8; ++t) {
                    const floatx4 r = *reinterpret_cast<const floatx4*>(erl + t * 256);
                    const floatx4 l = *reinterpret_cast<const floatx4*>(erl + (K8 + t) * 256);
#pragma unroll
                    for (int c = 0; c < 4; ++c) { er[4 * t + c] = r[c]; el[t][c] = l[c]; }
                }
                __syncthreads();                        // X
            }
            const float* wrow = lds + ((u - u0) & 1) * LY::SLICE + n * RS + 4 * h;
            float sk[4] = {0.f, 0.f, 0.f, 0.f};
            if (active) {
                floatx4 a[2][K8];
                floatx16 acc[2];
#pragma unroll
                for (int t = 0; t < K8; ++t) a[0][t] = *reinterpret_cast<const floatx4*>(wrow + 8 * t);
#pragma unroll
                for (int m = 0; m <= K8; ++m) {
                    if (m + 1 < K8) {
#pragma unroll
                        for (int t = 0; t < K8; ++t)
                            a[(m + 1) & 1][t] = *reinterpret_cast<const floatx4*>(wrow + 32 * (m + 1) * RS + 8 * t);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (m < K8) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[m & 1][r] = 0.f;
#pragma unroll
                        for (int t = 0; t < K8; ++t) {
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                acc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m & 1][t][c], er[4 * t + c], acc[m & 1], 0, 0, 0);
                        }
                    }
                    if (m > 0) {
                        // acc[4 a + c]: row 8 a + 4 h + c of tile m - 1; group g = 4 (m - 1) + a: k = g / K8, i = 8 (g % K8) + 4 h + c
#pragma unroll
                        for (int a4 = 0; a4 < 4; ++a4) {
                            const int gg = 4 * (m - 1) + a4, kq = gg / K8, uu = gg % K8;
#pragma unroll
                            for (int c = 0; c < 4; ++c) sk[kq] = fmaf(acc[(m - 1) & 1][4 * a4 + c], el[uu][c], sk[kq]);
                        }
                    }
                }
            }
            floatx4 sv = {sk[0], sk[1], sk[2], sk[3]};
            *reinterpret_cast<floatx4*>(lds + LY::OFF_S + (((u - u0) & 1) * 4 + nt) * 256 + lane * 4) = sv;
            load_rows = u + 1 < u1 && quad == NQ - 1;
            if (++quad == NQ) quad = 0;
            __syncthreads();                            // B(u+1)
        }
    }
#undef FETCH_W
#undef STORE_W
}

// ------------------------------------------------------------------ mixing layer, forward (App. B)
// Offset of the output: the largest offset of the children (their residuals are at most 0, so no term
// exceeds its weight); residual: log sum_c v[c] exp((Off[c] - Off[out]) + A[c]).
constexpr int MIX_UNROLL = MIX_REC_CHILDREN;
__global__ void k_mixing_forward(const int32_t* __restrict__ m_rec, const float* __restrict__ params,
                                 float* __restrict__ A, double* __restrict__ Off, float* __restrict__ logp, int B,
                                 int K) {
    // the item's record: node, entries, weight offset, number of partitions, partition nodes
    const int32_t* rec = m_rec + (size_t)blockIdx.x * MIX_REC_INTS;
    const int node = rec[0], kout = rec[1], nc = rec[3];
    int child[MIX_UNROLL];
#pragma unroll
    for (int c = 0; c < MIX_UNROLL; ++c) child[c] = rec[4 + c];
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= B * kout) return;
    const int b = e / kout, k = e - b * kout;
    const float* v = params + rec[2] + (size_t)k * nc;
    double m = -INFINITY;
    float s = 0.f;
    {
        // offsets, residuals and weights of all children are requested together: one memory latency, not two
        double off[MIX_UNROLL];
        float a[MIX_UNROLL], w[MIX_UNROLL];
#pragma unroll
        for (int c = 0; c < MIX_UNROLL; ++c) {
            off[c] = 0.0;
            a[c] = w[c] = 0.f;
            if (c < nc) {
                const size_t row = (size_t)child[c] * B + b;
                off[c] = Off[row];
                a[c] = A[row * K + k];
                w[c] = v[c];
            }
        }
#pragma unroll
        for (int c = 0; c < MIX_UNROLL; ++c)
            if (c < nc) m = fmax(m, off[c]);
#pragma unroll
        for (int c = 0; c < MIX_UNROLL; ++c)
            if (c < nc) s += w[c] * expf((float)(off[c] - m) + a[c]);
    }
    const float res = logf(s);
    const size_t row = (size_t)node * B + b;
    A[row * K + k] = res;
    if (k == 0) {
        Off[row] = m;
        if (logp && node == 0) logp[b] = (float)(m + (double)res);   // node 0: the root region, one entry
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

}  // namespace

template <int KQ>
static void launch_einsum_forward_kq(const DevTables& t, int first, int count, const float* params, float* A,
                                     double* Off, float* amax, float* logp, const Dims& d, hipStream_t s) {
    const int nkt = (d.K + 3) / 4;
    const int n_btiles = (d.B + 15) / 16;
    const int nw_max = count * nkt >= 1024 ? 4 : 8;    // many small workgroups: more of them per compute unit
    const int nw = n_btiles < nw_max ? n_btiles : nw_max;
    const size_t lds = sizeof(float) * FwdLayout<KQ>::LDS_FLOATS;
    if (lds > 64 * 1024) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] { allow_dynamic_lds(&k_einsum_forward<KQ>, lds); });
    }
    hipLaunchKernelGGL(k_einsum_forward<KQ>, dim3(count * nkt), dim3(64 * nw), lds, s, t.ein_left + first,
                       t.ein_right + first, t.ein_out + first, t.ein_kout + first, t.ein_woff + first, params, A, Off,
                       amax, logp, first, d.B, d.K, nkt);
}

template <int K8>
static void launch_einsum_forward_k8(const DevTables& t, int first, int count, const float* params, float* A,
                                     double* Off, float* amax, const Dims& d, hipStream_t s) {
    using LY = FwdSLayout<K8>;
    const size_t lds = sizeof(float) * LY::LDS_FLOATS;
    static std::once_flag attr_set[EINET_MAX_DEVICES];
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] { allow_dynamic_lds(&k_einsum_forward_s<K8>, lds); });
    const int units = count * ((d.B + 127) / 128) * (LY::K / 4);
    hipLaunchKernelGGL(k_einsum_forward_s<K8>, dim3(units < EINET_NUM_CUS ? units : EINET_NUM_CUS), dim3(512), lds, s,
                       t.ein_left + first, t.ein_right + first, t.ein_out + first, t.ein_woff + first, params, A, Off,
                       amax, first, count, d.B);
}

void launch_einsum_forward(const DevTables& t, int first, int count, bool full_k, const float* params, float* A,
                           double* Off, float* amax, float* logp, const Dims& d, hipStream_t s) {
    if (full_k && (d.K & 7) == 0 && d.K <= 48) {
        switch (d.K / 8) {
#define EINET_CASE(J) \
        case J: launch_einsum_forward_k8<J>(t, first, count, params, A, Off, amax, d, s); return;
            EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6)
#undef EINET_CASE
        }
    }
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
    hipLaunchKernelGGL(k_mixing_forward, grid, dim3(256), 0, s, t.mix_rec + (size_t)first * MIX_REC_INTS, params, A,
                       Off, logp, d.B, d.K);
}

}  // namespace einet_impl
