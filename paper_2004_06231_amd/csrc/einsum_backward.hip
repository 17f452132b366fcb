// Top-down pass: posterior of the regions and the fused einsum kernel (weight statistics of Eq. 6 and the
// posteriors of the children).
#include "device_common.hpp"

#include <mutex>

namespace einet_impl {

namespace {

// ------------------------------------------------------------------ top-down pass, regions
// G[region][b][k] = sum of the posterior blocks its parent partitions wrote (1 at
// the root).  Element-wise, one thread per (region, b, k); summing here instead of
// scattering from the producers keeps the pass free of atomics.
__global__ void k_region_assemble(const int32_t* __restrict__ r_rec, const int32_t* __restrict__ r_pblk, int is_root,
                                  float* __restrict__ G, const float* __restrict__ Gp, int B, int K) {
    // the region's record: node, entries, number of parent blocks, start of its block list, first block numbers
    const int32_t* rec = r_rec + (size_t)blockIdx.x * RB_REC_INTS;
    const int node = rec[0], kout = rec[1], cnt = rec[2];
    const int e = blockIdx.y * blockDim.x + threadIdx.x;
    if (e >= B * kout) return;
    const int b = e / kout, k = e - b * kout;
    const size_t blk = (size_t)B * K, o = (size_t)b * K + k;
    float g = is_root ? 1.f : 0.f;
    // Fourteen blocks per round, all requested before the first is added: a region of a Poon-Domingos structure
    // has a few dozen parent blocks, and one memory latency per block would be the whole kernel.  The numbers of
    // the first 28 blocks come with the record, so that the blocks are the second request, not the third.
    constexpr int RND = RB_REC_BLOCKS / 2;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (r * RND < cnt) {
            float v[RND];
#pragma unroll
            for (int q = 0; q < RND; ++q) v[q] = r * RND + q < cnt ? Gp[(size_t)rec[4 + r * RND + q] * blk + o] : 0.f;
#pragma unroll
            for (int q = 0; q < RND; ++q)
                if (r * RND + q < cnt) g += v[q];
        }
    }
    for (int p0 = RB_REC_BLOCKS; p0 < cnt; p0 += 16) {   // the rest of a very long list
        const int32_t* list = r_pblk + rec[3];
        float v[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) v[q] = p0 + q < cnt ? Gp[(size_t)list[p0 + q] * blk + o] : 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (p0 + q < cnt) g += v[q];
    }
    G[(size_t)node * blk + o] = g;
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
    // operands of the next four samples are requested before the MFMAs of the current four are issued
    float4 e = *reinterpret_cast<const float4*>(elcol);
    float4 qa[NU], rb[NU];
#pragma unroll
    for (int q = 0; q < NU; ++q) {
        qa[q] = *reinterpret_cast<const float4*>(qcol[q]);
        rb[q] = *reinterpret_cast<const float4*>(rcol[q]);
    }
    for (int s = 0; s < rg; s += 4) {
        const int sn = min(s + 4, rg - 4);           // the last round reads its own operands again
        const float4 en = *reinterpret_cast<const float4*>(elcol + sn);
        float4 qn[NU], rn[NU];
#pragma unroll
        for (int q = 0; q < NU; ++q) {
            qn[q] = *reinterpret_cast<const float4*>(qcol[q] + sn);
            rn[q] = *reinterpret_cast<const float4*>(rcol[q] + sn);
        }
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].x * e.x, rb[q].x, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].y * e.y, rb[q].y, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].z * e.z, rb[q].z, acc1[q], 0, 0, 0);
#pragma unroll
        for (int q = 0; q < NU; ++q) acc1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[q].w * e.w, rb[q].w, acc1[q], 0, 0, 0);
        e = en;
#pragma unroll
        for (int q = 0; q < NU; ++q) {
            qa[q] = qn[q];
            rb[q] = rn[q];
        }
    }
}

template <int KQ, bool VEC, bool ACCUM, bool DIRECT>
__global__ __launch_bounds__(512, 2) void k_einsum_backward(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_reg, const int32_t* __restrict__ e_kout, const int32_t* __restrict__ e_woff,
    const int32_t* __restrict__ e_voff, const int32_t* __restrict__ e_vstr, const int32_t* __restrict__ e_gsrc,
    const float* __restrict__ params, float* __restrict__ stats, const float* __restrict__ A,
    const double* __restrict__ Off, const float* __restrict__ amax, const float* __restrict__ G, float* __restrict__ Gp,
    int item0, int ngroups, int B, int K) {
    using LY = BwdLayout<KQ>;
    constexpr int KP = LY::KP, SI = LY::SI, S = LY::S, ST = LY::ST, BC = LY::BC, MAXU = LY::MAXU;
    extern __shared__ float lds[];
    float* Wl = lds;
    float* sR = lds + LY::OFF_R;
    float* sQ = lds + LY::OFF_Q;
    float* sL = lds + LY::OFF_L;
    float* sG = lds + LY::OFF_G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int vb = xcd_contiguous_block();
    const int li = vb / ngroups, grp = vb - li * ngroups;
    const int it0 = grp * KQ / ngroups, it1 = (grp + 1) * KQ / ngroups;     // this workgroup's slices
    const bool multi = it1 - it0 > 1;   // several slices: their shares of Gp_right are summed in LDS first
    const int item = item0 + li;
    const int kout = e_kout[li], nkt = (kout + 3) >> 2;
    const size_t blk = (size_t)B * K;
    const float* Lp = A + (size_t)e_left[li] * blk;
    const float* Rp = A + (size_t)e_right[li] * blk;
    const float* As = A + (size_t)e_reg[li] * blk;
    // posterior of the item's region: assembled in G, or (DIRECT) the sum of gcnt consecutive blocks that the
    // region's only parent wrote to Gp, added up in the order the assembly launch would take
    const int gsrc = DIRECT ? e_gsrc[li] : 0, gcnt = gsrc & 7;
    const float* Gs = DIRECT ? Gp + (size_t)(gsrc >> 3) * blk : G + (size_t)e_reg[li] * blk;
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

    // staging of eR and Q
    const int srow = tid >> 2, sq = tid & 3;
    constexpr int NF = (BC * KQ + 511) / 512;      // float4 of a [BC][K] block per thread

    for (int b0 = 0; b0 < B; b0 += BC) {
        const int nb = min(BC, B - b0);
        const int rg = (((nb + 3) >> 2) + 3) & ~3;         // samples per lane group in GEMM-1, multiple of 4
        const bool rok = srow < nb;
        const int ro = (b0 + min(srow, nb - 1)) * K;       // a valid row even for the idle tail threads
        const float al = aL[b0 + min(srow, nb - 1)];
        __syncthreads();                                   // readers of the previous pass are done
        if constexpr (VEC) {
            // the [nb][K] blocks are contiguous: 16-byte loads, consecutive threads consecutive addresses
            float4 r4[NF], g4[NF], a4[NF], v4[NF];
            float arn[NF], ddn[NF];
#pragma unroll
            for (int n = 0; n < NF; ++n) {
                const int f = min(tid + 512 * n, nb * KQ - 1);
                const int row = f / KQ, k4 = f - row * KQ;
                r4[n] = *reinterpret_cast<const float4*>(Rp + (size_t)(b0 + row) * K + 4 * k4);
                g4[n] = *reinterpret_cast<const float4*>(Gs + (size_t)(b0 + row) * K + 4 * k4);
                if (DIRECT && gcnt > 1) {
                    float4 gx[GSRC_MAX_BLOCKS - 1];
#pragma unroll
                    for (int x = 1; x < GSRC_MAX_BLOCKS; ++x)
                        gx[x - 1] = x < gcnt ? *reinterpret_cast<const float4*>(Gs + x * blk + (size_t)(b0 + row) * K + 4 * k4)
                                             : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int x = 1; x < GSRC_MAX_BLOCKS; ++x)
                        if (x < gcnt) {
                            g4[n].x += gx[x - 1].x;
                            g4[n].y += gx[x - 1].y;
                            g4[n].z += gx[x - 1].z;
                            g4[n].w += gx[x - 1].w;
                        }
                }
                a4[n] = *reinterpret_cast<const float4*>(As + (size_t)(b0 + row) * K + 4 * k4);
                arn[n] = aR[b0 + row];
                ddn[n] = (float)(Oo[b0 + row] - Os[b0 + row]);
                v4[n] = make_float4(1.f, 1.f, 1.f, 1.f);
                if (voff >= 0) {
                    v4[n].x = params[voff + min(4 * k4 + 0, kout - 1) * vstr];
                    v4[n].y = params[voff + min(4 * k4 + 1, kout - 1) * vstr];
                    v4[n].z = params[voff + min(4 * k4 + 2, kout - 1) * vstr];
                    v4[n].w = params[voff + min(4 * k4 + 3, kout - 1) * vstr];
                }
            }
#pragma unroll
            for (int n = 0; n < NF; ++n) {
                const int f = tid + 512 * n;
                if (f < BC * KQ) {
                    const int row = f / KQ, k4 = f - row * KQ;
                    const bool in = row < nb;
                    const float rr[4] = {r4[n].x, r4[n].y, r4[n].z, r4[n].w};
                    const float gg[4] = {g4[n].x, g4[n].y, g4[n].z, g4[n].w};
                    const float aa[4] = {a4[n].x, a4[n].y, a4[n].z, a4[n].w};
                    const float vv[4] = {v4[n].x, v4[n].y, v4[n].z, v4[n].w};
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        const int k = 4 * k4 + c4;
                        const float e = __expf(rr[c4] - arn[n]);
                        const float q = gg[c4] * vv[c4] * __expf(ddn[n] - aa[c4]);
                        sR[k * ST + row] = in ? e : 0.f;
                        sQ[k * ST + row] = (in && k < kout && gg[c4] != 0.f) ? q : 0.f;
                    }
                }
            }
            for (int j = KP + sq; j < 16 * LY::NJ; j += 4) sR[j * ST + srow] = 0.f;   // rows beyond the padded K
            if (multi && LY::LDS_ACC)
                for (int u = 0; u < KQ; ++u) sG[srow * KP + sq * KQ + u] = 0.f;
        } else {
            const float ar = aR[b0 + min(srow, nb - 1)];
            const float dd = (float)(Oo[b0 + min(srow, nb - 1)] - Os[b0 + min(srow, nb - 1)]);
            float rv[KQ], gv[KQ], av[KQ];
#pragma unroll
            for (int u = 0; u < KQ; ++u) {
                const int k = sq * KQ + u;
                const int kc = min(k, K - 1);
                rv[u] = Rp[ro + kc];
                gv[u] = Gs[ro + min(kc, kout - 1)];
                if (DIRECT && gcnt > 1) {
                    float gx[GSRC_MAX_BLOCKS - 1];
#pragma unroll
                    for (int x = 1; x < GSRC_MAX_BLOCKS; ++x) gx[x - 1] = x < gcnt ? Gs[x * blk + ro + min(kc, kout - 1)] : 0.f;
#pragma unroll
                    for (int x = 1; x < GSRC_MAX_BLOCKS; ++x)
                        if (x < gcnt) gv[u] += gx[x - 1];
                }
                av[u] = As[ro + min(kc, kout - 1)];
            }
#pragma unroll
            for (int u = 0; u < KQ; ++u) {
                const int k = sq * KQ + u;
                const float vw = (voff >= 0 && k < kout) ? params[voff + k * vstr] : 1.f;
                const float e = __expf(rv[u] - ar);
                const float q = gv[u] * vw * __expf(dd - av[u]);
                sR[k * ST + srow] = (rok && k < K) ? e : 0.f;
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
                if (nkt == KQ) {
#pragma unroll 2
                    for (int s = 0; s < KQ; ++s) {
                        const float qs = qrow[4 * s * ST];
#pragma unroll
                        for (int jt = 0; jt < KQ; ++jt)
                            acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl[4 * s * S + 4 * jt], qs, acc[jt], 0, 0, 0);
                    }
                } else {
                    // an item of the root has one output entry: the other contraction steps would add zeros
                    for (int s = 0; s < nkt; ++s) {
                        const float qs = qrow[4 * s * ST];
#pragma unroll
                        for (int jt = 0; jt < KQ; ++jt)
                            acc[jt] = __builtin_amdgcn_mfma_f32_16x16x4f32(wl[4 * s * S + 4 * jt], qs, acc[jt], 0, 0, 0);
                    }
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

// ------------------------------------------------------------------ top-down pass, einsum items, K a multiple of 8 up to 40
// The same two GEMMs on v_mfma_f32_32x32x2_f32 (the fp32 shape that issues at the full rate of the matrix pipe), as
// one workgroup per compute unit that walks a run of (item, slice) pairs, a slice being four consecutive left
// entries i.  Waves 0-3 only run the matrix pipe, waves 4-7 do everything else:
//   producers   bring the W slice in (transposed on the way: four consecutive k of a row (il, j) in 16 bytes, rows
//               swizzled so that neither their 16-byte stores nor the operand reads collide), stage eR^T, eL^T and
//               Q^T of up to 128 samples per (item, chunk), and finish the tiles that the four matrix waves share;
//   statistics  rows (k, il) in tiles of 32, columns j: one 32-column tile (K >= 32) on 32x32x2, the remaining
//               columns on 16x16x4; a wave owns whole tiles (all samples) and takes its 32 samples of the tiles that
//               are left over, whose shares meet in LDS;
//   posteriors  rows (il, j) in K/8 tiles of 32, columns = this wave's 32 samples, contraction over k; both
//               reductions are in-lane: the left child's entries are complete per slice, the right child's are kept
//               in registers over the workgroup's slices of the item and written once, as a block of their own.
// A vector instruction between two MFMAs of a wave stalls the matrix pipe for about 15 cycles, so operand products
// are formed in batches ahead of the MFMAs that use them.
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int K8>
struct BwdSLayout {
    static constexpr int K = 8 * K8;
    static constexpr int NS = K / 4;                   // slices (four consecutive left entries i) per item
    static constexpr int ST = 128 + 4;                 // row stride of the sample-major operand copies
    static constexpr int SLICE = 4 * K * K;            // W[:, 4 it .. 4 it + 3, :] as [K/4 kq][4K rows (il, j), swizzled][4 kr]
    static constexpr int OFF_R = 2 * SLICE;            // eR^T [K][ST]
    static constexpr int OFF_Q = OFF_R + K * ST;       // Q^T  [K][ST]
    static constexpr int OFF_L = OFF_Q + K * ST;       // eL^T [K][ST]
    static constexpr int N32 = K / 32;                 // 32-column tiles of the statistics GEMM (K <= 40: 0 or 1)
    static constexpr int N16C = (K % 32 + 15) / 16;    // 16-column tiles for the remaining columns
    static constexpr int T32 = K8 * N32;               // 32x32 tiles of a slice (K8 row tiles of 32 rows (k, il))
    static constexpr int O32 = T32 / 4, S32 = T32 % 4; // owned per matrix wave; shared (contraction split over the four waves)
    static constexpr int T16 = (K / 4) * N16C;         // 16x16 tiles of a slice
    static constexpr int O16 = T16 / 4, S16 = T16 % 4;
    static constexpr int NPART = 16 * S32 + 4 * S16;   // registers per lane of a matrix wave that hold shared tiles
    static constexpr int OFF_P = OFF_L + K * ST;       // [4 waves][NPART][64 lanes]
    static constexpr int LDS_FLOATS = OFF_P + 4 * NPART * 64;
    static constexpr int WITEMS = K * K / 4;           // work items of the slice copy: (kq, il, j4) -> 4 x 16 bytes
    static constexpr int NWI = (WITEMS + 255) / 256;
};

template <int K8, bool ACCUM>
__global__ __launch_bounds__(512, 1) void k_einsum_backward_s(
    const int32_t* __restrict__ e_left, const int32_t* __restrict__ e_right, const int32_t* __restrict__ e_out,
    const int32_t* __restrict__ e_reg, const int32_t* __restrict__ e_woff, const int32_t* __restrict__ e_voff,
    const int32_t* __restrict__ e_vstr, const float* __restrict__ params, float* __restrict__ stats,
    const float* __restrict__ A, const double* __restrict__ Off, const float* __restrict__ amax,
    const float* __restrict__ G, float* __restrict__ Gp, int item0, int count, int B, int vper, int cpv,
    float* __restrict__ part) {
    using LY = BwdSLayout<K8>;
    constexpr int K = LY::K, NS = LY::NS, ST = LY::ST, NB = 1 + NS;
    extern __shared__ float lds[];
    float* sR = lds + LY::OFF_R;
    float* sQ = lds + LY::OFF_Q;
    float* sL = lds + LY::OFF_L;
    float* sP = lds + LY::OFF_P;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nchunks = (B + 127) >> 7;
    // A layer of few items and several chunks is launched with every item as vper virtual items, each with cpv of the
    // chunks: their statistics go to blocks of their own in `part` ([vper][count][K^3], summed into the statistics by
    // the launch that follows), so that the chunks of an item run side by side.  vper = 1: the items as they are.
    const long long P = (long long)count * vper * NS;
    const int g = xcd_contiguous_block();
    const int p0 = (int)((long long)g * P / gridDim.x), p1 = (int)((long long)(g + 1) * P / gridDim.x);
    if (p0 >= p1) return;
    const size_t blk = (size_t)B * K;

    // position of a unit: virtual item vi = item li with chunks [c0, c1), chunk, slice it; [s0, s1) are this
    // workgroup's slices of the virtual item
    struct Pos { int vi, li, c0, c1, chunk, it, s0, s1; };
    auto seg = [&](Pos& q) {
        q.s0 = max(p0 - q.vi * NS, 0);
        q.s1 = min(p1 - q.vi * NS, NS);
        q.li = q.vi / vper;
        q.c0 = (q.vi - q.li * vper) * cpv;
        q.c1 = min(q.c0 + cpv, nchunks);
        q.chunk = q.c0;
    };
    auto advance = [&](Pos& q) {          // -> false past the end
        if (++q.it < q.s1) return true;
        if (++q.chunk < q.c1) { q.it = q.s0; return true; }
        ++q.vi;
        if (q.vi * NS >= p1) return false;
        seg(q); q.it = q.s0;
        return true;
    };
    Pos pos;
    pos.vi = p0 / NS; seg(pos); pos.it = pos.s0;
    // where the statistics of a unit's item are, and whether the unit adds to them
    auto stat_base = [&](const Pos& q) -> float* {
        return vper > 1 ? part + ((size_t)(q.vi - q.li * vper) * count + q.li) * ((size_t)K * K * K)
                        : stats + (size_t)e_woff[q.li];
    };
    auto stat_adds = [&](const Pos& q) { return ACCUM || q.chunk > q.c0; };

    if (wave >= 4) {
        // ============================================================ producer waves
        const int pt = tid - 256;
        // ---- W slice of (li, it): 16 bytes at four consecutive k per work item, transposed in registers
        floatx4 wv[LY::NWI][4];
        auto fetch_w = [&](const Pos& q) {
            const float* W = params + e_woff[q.li];
#pragma unroll
            for (int x = 0; x < LY::NWI; ++x) {
                const int wi = min(pt + 256 * x, LY::WITEMS - 1);
                const int j4 = wi % (K / 4), il = (wi / (K / 4)) & 3, kq = wi / K;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    wv[x][kk] = *reinterpret_cast<const floatx4*>(W + ((size_t)(4 * kq + kk) * K + 4 * q.it + il) * K + 4 * j4);
            }
        };
        auto store_w = [&](float* buf) {
#pragma unroll
            for (int x = 0; x < LY::NWI; ++x) {
                const int wi = pt + 256 * x;
                const int j4 = wi % (K / 4), il = (wi / (K / 4)) & 3, kq = wi / K;
                if (wi < LY::WITEMS) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int rho = il * K + 4 * j4 + c;
                        const int ps = rho ^ ((rho >> 3) & 7);
                        floatx4 o = {wv[x][0][c], wv[x][1][c], wv[x][2][c], wv[x][3][c]};
                        *reinterpret_cast<floatx4*>(buf + ((size_t)kq * 4 * K + ps) * 4) = o;
                    }
                }
            }
        };
        // ---- operands of (li, chunk): thread (b = pt / 2, half hh = pt % 2) holds K/2 entries of row b of R, L, G, A[s]
        const int rb_ = pt >> 1, hh = pt & 1;
        floatx4 r4[K8], l4[K8], g4[K8], a4[K8], v4[K8];
        float arow = 0.f, alrow = 0.f, ddrow = 0.f;
        bool rin = false;
        auto fetch_rows = [&](const Pos& q, bool with_q) {
            const int bg = q.chunk * 128 + rb_;
            rin = bg < B;
            const int bc = min(bg, B - 1);
            const int item = item0 + q.li;
            const size_t ro = (size_t)bc * K + 4 * hh * K8;
            const float* Rp = A + (size_t)e_right[q.li] * blk + ro;
            const float* Lp = A + (size_t)e_left[q.li] * blk + ro;
            const float* Gs = G + (size_t)e_reg[q.li] * blk + ro;
            const float* As = A + (size_t)e_reg[q.li] * blk + ro;
#pragma unroll
            for (int x = 0; x < K8; ++x) {
                r4[x] = *reinterpret_cast<const floatx4*>(Rp + 4 * x);
                l4[x] = *reinterpret_cast<const floatx4*>(Lp + 4 * x);
                if (with_q) {
                    g4[x] = *reinterpret_cast<const floatx4*>(Gs + 4 * x);
                    a4[x] = *reinterpret_cast<const floatx4*>(As + 4 * x);
                }
            }
            alrow = amax[(size_t)item * 2 * B + bc];
            arow = amax[((size_t)item * 2 + 1) * B + bc];
            if (with_q) {
                ddrow = (float)(Off[(size_t)e_out[q.li] * B + bc] - Off[(size_t)e_reg[q.li] * B + bc]);
                const int voff = e_voff[q.li], vstr = e_vstr[q.li];
#pragma unroll
                for (int x = 0; x < K8; ++x)
#pragma unroll
                    for (int c = 0; c < 4; ++c) v4[x][c] = voff >= 0 ? params[voff + (4 * (hh * K8 + x) + c) * vstr] : 1.f;
            }
        };
        auto stage_rows = [&](bool with_q) {
#pragma unroll
            for (int x = 0; x < K8; ++x)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int k = 4 * (hh * K8 + x) + c;
                    const float e = __expf(r4[x][c] - arow);
                    const float l = __expf(l4[x][c] - alrow);
                    sR[k * ST + rb_] = rin ? e : 0.f;
                    sL[k * ST + rb_] = rin ? l : 0.f;
                    if (with_q) {
                        const float qv = g4[x][c] * v4[x][c] * __expf(ddrow - a4[x][c]);
                        sQ[k * ST + rb_] = (rin && g4[x][c] != 0.f) ? qv : 0.f;
                    }
                }
        };
        // ---- shared tiles of a finished unit: sum the four waves' shares, then Nw (+)= W * sum.  The W entries (and the old
        // statistics, when they are added to) are requested while the unit is still being computed.
        float wred[LY::NPART / 4 > 0 ? LY::NPART / 4 : 1], nred[LY::NPART / 4 > 0 ? LY::NPART / 4 : 1];
        auto shared_index = [&](int x, int& k, int& il, int& j) {
            const int e = pt + 256 * x;
            const int reg = e >> 6, ln = e & 63;
            if (reg < 16 * LY::S32) {
                const int m1 = 4 * LY::O32 + (reg >> 4), rr = reg & 15;
                k = 8 * m1 + 2 * (rr >> 2) + (ln >> 5); il = rr & 3; j = ln & 31;
            } else {
                const int r2 = reg - 16 * LY::S32;
                const int ptile = 4 * LY::O16 + (r2 >> 2);
                const int rt = ptile / (LY::N16C > 0 ? LY::N16C : 1), ct = ptile % (LY::N16C > 0 ? LY::N16C : 1);
                k = 4 * rt + (ln >> 4); il = r2 & 3; j = 32 * LY::N32 + 16 * ct + (ln & 15);
            }
        };
        auto fetch_shared = [&](const Pos& q) {
            if constexpr (LY::NPART > 0) {
                const size_t wbase = (size_t)e_woff[q.li];
#pragma unroll
                for (int x = 0; x < LY::NPART / 4; ++x) {
                    int k, il, j;
                    shared_index(x, k, il, j);
                    const size_t idx = ((size_t)k * K + 4 * q.it + il) * K + min(j, K - 1);
                    wred[x] = params[wbase + idx];
                    nred[x] = stat_adds(q) ? stat_base(q)[idx] : 0.f;
                }
            }
        };
        auto reduce_shared = [&](const Pos& q) {
            if constexpr (LY::NPART > 0) {
                float* Nw = stat_base(q);
#pragma unroll
                for (int x = 0; x < LY::NPART / 4; ++x) {
                    const int e = pt + 256 * x;
                    const int reg = e >> 6, ln = e & 63;
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) s += sP[(w * LY::NPART + reg) * 64 + ln];
                    int k, il, j;
                    shared_index(x, k, il, j);
                    if (j < K) Nw[((size_t)k * K + 4 * q.it + il) * K + j] = nred[x] + wred[x] * s;
                }
            }
        };

        fetch_w(pos);
        fetch_rows(pos, false);             // (the matrix waves stage Q^T of the first operands themselves)
        store_w(lds);
        stage_rows(false);
        Pos npos = pos;
        bool nvalid = advance(npos);
        if (nvalid) fetch_w(npos);
        __syncthreads();                                  // B0
        Pos prev = pos;
        int u = 0;
        bool have_prev = false;
        for (;;) {
            // the matrix waves work on unit u = pos; slice npos is in registers
            if (have_prev) reduce_shared(prev);
            if (nvalid) store_w(lds + ((u + 1) & 1) * LY::SLICE);
            if constexpr (LY::NPART > 0) __syncthreads();  // M(u)
            fetch_shared(pos);
            if (nvalid) {
                Pos nn = npos;
                if (advance(nn)) fetch_w(nn);
            }
            const bool new_ops = nvalid && (npos.li != pos.li || npos.chunk != pos.chunk);
            if (new_ops) fetch_rows(npos, true);
            __syncthreads();                              // B(u+1)
            prev = pos; have_prev = true;
            if (!nvalid) break;
            pos = npos;
            nvalid = advance(npos);
            ++u;
            if (new_ops) {
                stage_rows(true);
                __syncthreads();                          // X(u)
            }
        }
        reduce_shared(prev);
    } else {
        // ============================================================ matrix waves
        const int n = lane & 31, h = lane >> 5;
        const int c16 = lane & 15, kg = lane >> 4;
        const int bl = 32 * wave + n;                     // sample of this lane within the chunk (posterior GEMM)
        float q[4 * K8], er[4 * K8], gr[4 * K8];
#pragma unroll
        for (int x = 0; x < 4 * K8; ++x) gr[x] = 0.f;
        // swizzled rows of the K8 tiles of the slice
        int prow[K8];
#pragma unroll
        for (int m = 0; m < K8; ++m) {
            const int rho = 32 * m + n;
            prow[m] = (rho ^ ((rho >> 3) & 7)) * 4;
        }
        {
            // Q^T of the first operands: thread (b = tid / 2, half = tid % 2), as the producers do it for the later ones
            const int rb_ = tid >> 1, hh = tid & 1;
            const int bgq = pos.chunk * 128 + rb_;
            const bool rin = bgq < B;
            const int bc = min(bgq, B - 1);
            const size_t ro = (size_t)bc * K + 4 * hh * K8;
            const float* Gs = G + (size_t)e_reg[pos.li] * blk + ro;
            const float* As = A + (size_t)e_reg[pos.li] * blk + ro;
            floatx4 g4[K8], a4[K8];
#pragma unroll
            for (int x = 0; x < K8; ++x) {
                g4[x] = *reinterpret_cast<const floatx4*>(Gs + 4 * x);
                a4[x] = *reinterpret_cast<const floatx4*>(As + 4 * x);
            }
            const float ddrow = (float)(Off[(size_t)e_out[pos.li] * B + bc] - Off[(size_t)e_reg[pos.li] * B + bc]);
            const int voff = e_voff[pos.li], vstr = e_vstr[pos.li];
#pragma unroll
            for (int x = 0; x < K8; ++x)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int k = 4 * (hh * K8 + x) + c;
                    const float vw = voff >= 0 ? params[voff + k * vstr] : 1.f;
                    const float qv = g4[x][c] * vw * __expf(ddrow - a4[x][c]);
                    sQ[k * ST + rb_] = (rin && g4[x][c] != 0.f) ? qv : 0.f;
                }
        }
        __syncthreads();                                  // B0
        bool new_ops = true;
        int u = 0;
        for (;;) {
            const int item = item0 + pos.li;
            const int bg = pos.chunk * 128 + bl;
            if (new_ops) {
#pragma unroll
                for (int t = 0; t < K8; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        q[4 * t + c] = sQ[(8 * t + 4 * h + c) * ST + bl];
                        er[4 * t + c] = sR[(8 * t + 4 * h + c) * ST + bl];
                    }
            }
            float el4[4];
#pragma unroll
            for (int il = 0; il < 4; ++il) el4[il] = sL[(4 * pos.it + il) * ST + bl];
            const size_t wbase = (size_t)e_woff[pos.li];
            float* Nw = stat_base(pos);
            const bool accum = stat_adds(pos);

            // ---- statistics GEMM: P[(k, il), j] = sum_b Q[b,k] eL[b, 4 it + il] eR[b,j] over the 128 staged samples
            const float* wcur = lds + (u & 1) * LY::SLICE;      // W of the slice, for Nw (+)= W * P
            // 32x32 tiles: lane (n, h) is row n of the tile as A operand: (k = 8 m1 + n / 4, il = n % 4); as B operand column j = n;
            // group t contracts the samples 8 t + 4 h .. + 3.  Owned tiles first (all samples), then the shared ones (this wave's
            // 32 samples); a tile's registers are free again before the next one starts.
#pragma unroll
            for (int o = 0; o < LY::O32 + LY::S32; ++o) {
                const bool own = o < LY::O32;
                const int m1 = own ? wave + 4 * o : 4 * LY::O32 + (o - LY::O32);
                const int t0 = own ? 0 : 4 * wave;
                const int nt = own ? 16 : 4;
                float nold[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) nold[v] = 0.f;
                if (own && accum) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        nold[v] = Nw[((size_t)(8 * m1 + 2 * (v >> 2) + h) * K + 4 * pos.it + (v & 3)) * K + n];
                }
                if constexpr (LY::NPART > 0) {
                    if (o == LY::O32) __syncthreads();    // M(u): the shares of the previous unit have been read
                }
                const float* qp = sQ + (8 * m1 + (n >> 2)) * ST + 4 * h + 8 * t0;
                const float* lp = sL + (4 * pos.it + (n & 3)) * ST + 4 * h + 8 * t0;
                const float* rp = sR + n * ST + 4 * h + 8 * t0;
                floatx16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
                // Batches of two groups (eight MFMAs): the products of a batch are formed before its first MFMA, because a vector
                // instruction between two MFMAs of a wave costs about 15 cycles of the matrix pipe; operands are requested two
                // batches ahead.
                floatx4 qa[3][2], ea[3][2], rb[3][2];
                constexpr int NBAT32 = 8;
                const int nbat = nt / 2;
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int y = 0; y < 2; ++y) {
                        qa[x][y] = *reinterpret_cast<const floatx4*>(qp + 8 * (2 * x + y));
                        ea[x][y] = *reinterpret_cast<const floatx4*>(lp + 8 * (2 * x + y));
                        rb[x][y] = *reinterpret_cast<const floatx4*>(rp + 8 * (2 * x + y));
                    }
#pragma unroll
                for (int x = 0; x < NBAT32; ++x) {
                    if (x < nbat) {
                        if (x + 2 < nbat) {
#pragma unroll
                            for (int y = 0; y < 2; ++y) {
                                qa[(x + 2) % 3][y] = *reinterpret_cast<const floatx4*>(qp + 8 * (2 * (x + 2) + y));
                                ea[(x + 2) % 3][y] = *reinterpret_cast<const floatx4*>(lp + 8 * (2 * (x + 2) + y));
                                rb[(x + 2) % 3][y] = *reinterpret_cast<const floatx4*>(rp + 8 * (2 * (x + 2) + y));
                            }
                        }
                        float pr[8];
#pragma unroll
                        for (int y = 0; y < 2; ++y)
#pragma unroll
                            for (int c = 0; c < 4; ++c) pr[4 * y + c] = qa[x % 3][y][c] * ea[x % 3][y][c];
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int y = 0; y < 2; ++y)
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pr[4 * y + c], rb[x % 3][y][c], acc, 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (own) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int k = 8 * m1 + 2 * (v >> 2) + h, rho = (v & 3) * K + n;
                        const float wv_ = wcur[((k >> 2) * 4 * K + (rho ^ ((rho >> 3) & 7))) * 4 + (k & 3)];
                        Nw[((size_t)k * K + 4 * pos.it + (v & 3)) * K + n] = nold[v] + wv_ * acc[v];
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) sP[(wave * LY::NPART + 16 * (o - LY::O32) + v) * 64 + lane] = acc[v];
                }
            }
            if constexpr (LY::NPART > 0 && LY::S32 == 0) __syncthreads();   // M(u) when no 32x32 tile is shared
            // 16x16 tiles: lane (c16, kg): A row c16 = (k = 4 rt + c16 / 4, il = c16 % 4), B column j = jb + c16; group t contracts
            // the samples 16 t + 4 kg .. + 3
            // (two tiles advance together where possible: a single chain of this shape does not keep the matrix pipe busy)
#pragma unroll
            for (int part = 0; part < 2; ++part)
#pragma unroll
            for (int o0 = 0; o0 < (part == 0 ? LY::O16 : LY::S16); o0 += 2) {
                const bool own = part == 0;                 // owned tiles, then shared ones; a pair never mixes them
                const int np = o0 + 1 < (own ? LY::O16 : LY::S16) ? 2 : 1;
                const int t0 = own ? 0 : 2 * wave;
                const int nt = own ? 8 : 2;
                int rt[2], jj[2];
                const float* qp[2];
                const float* rp[2];
                const float* lp = sL + (4 * pos.it + (c16 & 3)) * ST + 4 * kg + 16 * t0;
                float nold[2][4];
#pragma unroll
                for (int z = 0; z < 2; ++z) {
                    const int o = o0 + (z < np ? z : 0);
                    const int ptile = own ? wave + 4 * o : 4 * LY::O16 + o;
                    rt[z] = ptile / (LY::N16C > 0 ? LY::N16C : 1);
                    jj[z] = 32 * LY::N32 + 16 * (ptile % (LY::N16C > 0 ? LY::N16C : 1)) + c16;
                    qp[z] = sQ + (4 * rt[z] + (c16 >> 2)) * ST + 4 * kg + 16 * t0;
                    rp[z] = sR + min(jj[z], K - 1) * ST + 4 * kg + 16 * t0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) nold[z][c] = 0.f;
                    if (own && accum && z < np) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) nold[z][c] = Nw[((size_t)(4 * rt[z] + kg) * K + 4 * pos.it + c) * K + min(jj[z], K - 1)];
                    }
                }
                // (a dependent chain of this shape issues every 42 cycles, four independent ones every 32: each tile keeps two
                // accumulators, for the even and the odd groups)
                floatx4 acc2[2][2] = {{{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}};
                floatx4 qa[3][2], ea[3], rb[3][2];
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    ea[x] = *reinterpret_cast<const floatx4*>(lp + 16 * x);
#pragma unroll
                    for (int z = 0; z < 2; ++z) {
                        if (z < np) {
                            qa[x][z] = *reinterpret_cast<const floatx4*>(qp[z] + 16 * x);
                            rb[x][z] = *reinterpret_cast<const floatx4*>(rp[z] + 16 * x);
                        }
                    }
                }
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    if (x < nt) {
                        if (x + 2 < nt) {
                            ea[(x + 2) % 3] = *reinterpret_cast<const floatx4*>(lp + 16 * (x + 2));
#pragma unroll
                            for (int z = 0; z < 2; ++z) {
                                if (z < np) {
                                    qa[(x + 2) % 3][z] = *reinterpret_cast<const floatx4*>(qp[z] + 16 * (x + 2));
                                    rb[(x + 2) % 3][z] = *reinterpret_cast<const floatx4*>(rp[z] + 16 * (x + 2));
                                }
                            }
                        }
                        float pr[2][4];
#pragma unroll
                        for (int z = 0; z < 2; ++z)
#pragma unroll
                            for (int c = 0; c < 4; ++c) pr[z][c] = z < np ? qa[x % 3][z][c] * ea[x % 3][c] : 0.f;
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int c = 0; c < 4; ++c)
#pragma unroll
                            for (int z = 0; z < 2; ++z)
                                if (z < np)
                                    acc2[z][x & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(pr[z][c], rb[x % 3][z][c], acc2[z][x & 1], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                floatx4 acc[2];
#pragma unroll
                for (int z = 0; z < 2; ++z) acc[z] = acc2[z][0] + acc2[z][1];
#pragma unroll
                for (int z = 0; z < 2; ++z) {
                    if (z < np) {
                        if (own) {
                            if (jj[z] < K) {
#pragma unroll
                                for (int c = 0; c < 4; ++c) {
                                    const int k = 4 * rt[z] + kg, rho = c * K + jj[z];
                                    const float wv_ = wcur[((k >> 2) * 4 * K + (rho ^ ((rho >> 3) & 7))) * 4 + (k & 3)];
                                    Nw[((size_t)k * K + 4 * pos.it + c) * K + jj[z]] = nold[z][c] + wv_ * acc[z][c];
                                }
                            }
                        } else {
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                sP[(wave * LY::NPART + 16 * LY::S32 + 4 * (o0 + z) + c) * 64 + lane] = acc[z][c];
                        }
                    }
                }
            }
            // ---- posterior GEMM: U[(il, j), b] = sum_k W[k, 4 it + il, j] Q[b, k]; tile m holds rows 32 m .. 32 m + 31 of (il, j)
            const float* wsl = lds + (u & 1) * LY::SLICE + h * (4 * K * 4);
            float gl[4] = {0.f, 0.f, 0.f, 0.f};
            {
                floatx4 a[2][K8];
                floatx16 acc[2];
#pragma unroll
                for (int t = 0; t < K8; ++t) a[0][t] = *reinterpret_cast<const floatx4*>(wsl + 2 * t * (4 * K * 4) + prow[0]);
#pragma unroll
                for (int m = 0; m <= K8; ++m) {
                    if (m + 1 < K8) {
#pragma unroll
                        for (int t = 0; t < K8; ++t)
                            a[(m + 1) & 1][t] = *reinterpret_cast<const floatx4*>(wsl + 2 * t * (4 * K * 4) + prow[m + 1 < K8 ? m + 1 : 0]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (m < K8) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[m & 1][v] = 0.f;
#pragma unroll
                        for (int t = 0; t < K8; ++t)
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                acc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m & 1][t][c], q[4 * t + c], acc[m & 1], 0, 0, 0);
                    }
                    if (m > 0) {
                        // acc[4 a + c]: row 8 a + 4 h + c of tile m - 1; group gg = 4 (m - 1) + a: il = gg / K8, j = 8 (gg % K8) + 4 h + c
#pragma unroll
                        for (int a4 = 0; a4 < 4; ++a4) {
                            const int gg = 4 * (m - 1) + a4, il = gg / K8, uu = gg % K8;
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const float v = acc[(m - 1) & 1][4 * a4 + c];
                                gl[il] = fmaf(v, er[4 * uu + c], gl[il]);
                                gr[4 * uu + c] = fmaf(v, el4[il], gr[4 * uu + c]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int il = 0; il < 4; ++il) gl[il] += __shfl_xor(gl[il], 32, 64);
            if (h == 0 && bg < B) {
                floatx4 o = {gl[0] * el4[0], gl[1] * el4[1], gl[2] * el4[2], gl[3] * el4[3]};
                *reinterpret_cast<floatx4*>(Gp + ((size_t)item * NB * B + bg) * K + 4 * pos.it) = o;
            }
            // next unit
            Pos npos = pos;
            const bool nvalid = advance(npos);
            new_ops = !nvalid || npos.li != pos.li || npos.chunk != pos.chunk;
            if (new_ops) {
                // the right child's share of this workgroup's slices of (item, chunk)
                const int grp = g - bwds_wg_of_pair((long long)pos.vi * NS, P, gridDim.x);
                if (bg < B) {
                    float* right = Gp + ((size_t)(item * NB + 1 + grp) * B + bg) * K + 4 * h;
#pragma unroll
                    for (int t = 0; t < K8; ++t) {
                        floatx4 o = {gr[4 * t] * er[4 * t], gr[4 * t + 1] * er[4 * t + 1], gr[4 * t + 2] * er[4 * t + 2], gr[4 * t + 3] * er[4 * t + 3]};
                        *reinterpret_cast<floatx4*>(right + 8 * t) = o;
                    }
                }
#pragma unroll
                for (int x = 0; x < 4 * K8; ++x) gr[x] = 0.f;
            }
            __syncthreads();                              // B(u+1)
            if (!nvalid) break;
            pos = npos;
            ++u;
            if (new_ops) __syncthreads();                 // X(u): the next operands are staged
        }
    }
}

}  // namespace

void launch_region_assemble(const DevTables& t, int first, int count, bool is_root_layer, float* G, const float* Gp,
                            const Dims& d, hipStream_t s) {
    if (count == 0) return;
    dim3 grid(count, (d.B * d.K + 255) / 256);
    hipLaunchKernelGGL(k_region_assemble, grid, dim3(256), 0, s, t.rb_rec + (size_t)first * RB_REC_INTS, t.rb_pblk,
                       is_root_layer ? 1 : 0, G, Gp, d.B, d.K);
}

template <int KQ>
static void launch_einsum_backward_kq(const DevTables& t, int first, int count, bool accumulate,
                                      const float* params, float* stats, const float* A, const double* Off,
                                      const float* amax, const float* G, float* Gp, bool direct, const Dims& d,
                                      hipStream_t s) {
    const size_t lds = sizeof(float) * BwdLayout<KQ>::LDS_FLOATS;
    if (lds > 64 * 1024) {
        static std::once_flag attr_set[EINET_MAX_DEVICES];
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] {
            allow_dynamic_lds(&k_einsum_backward<KQ, true, true, false>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, false, true, false>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, true, false, false>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, false, false, false>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, true, true, true>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, false, true, true>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, true, false, true>, lds);
            allow_dynamic_lds(&k_einsum_backward<KQ, false, false, true>, lds);
        });
    }
    const int ngroups = bwd_groups_per_item(count, d.K);
#define EINET_LAUNCH_D(V, ACC, DIR)                                                                               \
    hipLaunchKernelGGL((k_einsum_backward<KQ, V, ACC, DIR>), dim3(count * ngroups), dim3(512), lds, s, t.ein_left + first,  \
                       t.ein_right + first, t.ein_out + first, t.ein_reg + first, t.ein_kout + first,                 \
                       t.ein_woff + first, t.ein_voff + first, t.ein_vstr + first,                                    \
                       t.ein_gsrc + first, params, stats, A, Off, amax, G, Gp, first, ngroups, d.B, d.K)
#define EINET_LAUNCH(V, ACC)                   \
    do {                                       \
        if (direct) EINET_LAUNCH_D(V, ACC, true); \
        else EINET_LAUNCH_D(V, ACC, false);    \
    } while (0)
    if ((d.K & 3) == 0) {
        if (accumulate) EINET_LAUNCH(true, true);
        else EINET_LAUNCH(true, false);
    } else {
        if (accumulate) EINET_LAUNCH(false, true);
        else EINET_LAUNCH(false, false);
    }
#undef EINET_LAUNCH
#undef EINET_LAUNCH_D
}

// stats[item][r] (+)= sum over the vper blocks of part[.][item][r], job blockIdx.y of the list: the launch at the end of
// a top-down pass whose launches ran virtual items
namespace {
__global__ void k_sum_partial_stats(PartialSumList jobs, float* __restrict__ stats, int accumulate) {
    const PartialSumJob& j = jobs.job[blockIdx.y];
    const size_t n = (size_t)j.count * j.block;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int li = (int)(i / j.block);
        float* dst = stats + (size_t)j.e_woff[li] + (i - (size_t)li * j.block);
        float sum = accumulate ? *dst : 0.f;
        for (int v = 0; v < j.vper; ++v) sum += j.part[(size_t)v * n + i];
        *dst = sum;
    }
}
}  // namespace

void launch_sum_partial_stats(const PartialSumList& jobs, float* stats, bool accumulate, hipStream_t s) {
    if (jobs.n == 0) return;
    size_t most = 0;
    for (int i = 0; i < jobs.n; ++i) most = std::max(most, (size_t)jobs.job[i].count * jobs.job[i].block);
    const unsigned bx = (unsigned)std::min<size_t>((most + 255) / 256, 1024);
    hipLaunchKernelGGL(k_sum_partial_stats, dim3(bx, jobs.n), dim3(256), 0, s, jobs, stats, accumulate ? 1 : 0);
}

template <int K8>
static void launch_einsum_backward_k8(const DevTables& t, int first, int count, bool accumulate, const float* params,
                                      float* stats, const float* A, const double* Off, const float* amax,
                                      const float* G, float* Gp, float* part, PartialSumList* jobs, const Dims& d,
                                      hipStream_t s) {
    using LY = BwdSLayout<K8>;
    const size_t lds = sizeof(float) * LY::LDS_FLOATS;
    static std::once_flag attr_set[EINET_MAX_DEVICES];
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::call_once(attr_set[dev % EINET_MAX_DEVICES], [&] {
        allow_dynamic_lds(&k_einsum_backward_s<K8, true>, lds);
        allow_dynamic_lds(&k_einsum_backward_s<K8, false>, lds);
    });
    const int vper = part && jobs && jobs->n < PARTIAL_SUM_JOBS ? bwd_virtual_items(count, d.K, d.B) : 1;
    const int nchunks = (d.B + 127) / 128, cpv = (nchunks + vper - 1) / vper;
    const int grid = vper > 1 ? count * vper * (d.K / 4) : bwd_split_grid(count, d.K);
#define EINET_LAUNCH(ACC)                                                                                         \
    hipLaunchKernelGGL((k_einsum_backward_s<K8, ACC>), dim3(grid), dim3(512), lds, s, t.ein_left + first,          \
                       t.ein_right + first, t.ein_out + first, t.ein_reg + first, t.ein_woff + first,             \
                       t.ein_voff + first, t.ein_vstr + first, params, stats, A, Off, amax, G, Gp, first, count, d.B, \
                       vper, cpv, part)
    if (vper > 1) {
        // (the blocks are written, not added to; their sum, later, adds to the statistics or overwrites them)
        EINET_LAUNCH(false);
        jobs->job[jobs->n++] = PartialSumJob{t.ein_woff + first, part, count, vper, d.K * d.K * d.K};
    } else if (accumulate) EINET_LAUNCH(true);
    else EINET_LAUNCH(false);
#undef EINET_LAUNCH
}

void launch_einsum_backward(const DevTables& t, int first, int count, bool full_k, bool accumulate,
                            const float* params, float* stats, const float* A, const double* Off, const float* amax,
                            const float* G, float* Gp, float* part, PartialSumList* jobs, bool direct, const Dims& d,
                            hipStream_t s) {
    if (count == 0) return;
    if (bwd_uses_split_kernel(d.K, full_k)) {
        switch (d.K / 8) {
#define EINET_CASE(J) \
        case J: launch_einsum_backward_k8<J>(t, first, count, accumulate, params, stats, A, Off, amax, G, Gp, part, jobs, d, s); return;
            EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5)
#undef EINET_CASE
        }
    }
    switch ((d.K + 3) / 4) {
#define EINET_CASE(J) \
    case J: launch_einsum_backward_kq<J>(t, first, count, accumulate, params, stats, A, Off, amax, G, Gp, direct, d, s); break;
        EINET_CASE(1) EINET_CASE(2) EINET_CASE(3) EINET_CASE(4) EINET_CASE(5) EINET_CASE(6) EINET_CASE(7) EINET_CASE(8)
        EINET_CASE(9) EINET_CASE(10) EINET_CASE(11) EINET_CASE(12) EINET_CASE(13) EINET_CASE(14) EINET_CASE(15)
        EINET_CASE(16)
#undef EINET_CASE
    }
}

}  // namespace einet_impl
