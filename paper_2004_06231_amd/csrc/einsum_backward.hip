// Top-down pass: posterior of the regions and the fused einsum kernel (weight statistics of Eq. 6 and the
// posteriors of the children).
#include "device_common.hpp"

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
                                      const float* amax, const float* G, float* Gp, const Dims& d, hipStream_t s) {
    const size_t lds = sizeof(float) * BwdLayout<KQ>::LDS_FLOATS;
    static bool attr_set = false;
    if (lds > 64 * 1024 && !attr_set) {
        allow_dynamic_lds(&k_einsum_backward<KQ, true, true>, lds);
        allow_dynamic_lds(&k_einsum_backward<KQ, false, true>, lds);
        allow_dynamic_lds(&k_einsum_backward<KQ, true, false>, lds);
        allow_dynamic_lds(&k_einsum_backward<KQ, false, false>, lds);
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

}  // namespace einet_impl
