// FlexAttention backward kernels for gfx950 (backward template of paper section 4.1, walking the
// BlockMask in both orientations, section 4.2).  The paper gives no formulas; with P recomputed
// from the saved LSE this is the usual softmax-attention calculus:
//     dV = P^T dO,  dP = dO V^T,  dS' = P * (dP - delta),  delta = rowsum(dO * O),
//     dS = dS' * d score_mod / d s,  dQ = scale * dS K,  dK = scale * dS^T Q.
// Three kernels, no floating-point atomics (results are deterministic):
//   bwd_delta_kernel   delta and LSE * log2(e) per query row.
//   bwd_dkdv_kernel    one workgroup per 64 keys of one (b, hkv); walks the q-blocks listed for
//                      that column of blocks (transposed BlockMask) for every query head of the
//                      group; score tile in S = Q K^T orientation so that P and dS are the B
//                      operands of dV^T += dO^T P and dK^T += Q^T dS.
//   bwd_dq_kernel      one workgroup per row of blocks of one (b, hq); walks the kv-blocks listed
//                      for it; score tile transposed (S^T = K Q^T) so that dS^T is the B operand of
//                      dQ^T += K^T dS^T and LSE / delta are per-lane scalars.
#pragma once

#include "flex_common.h"

namespace flexattn {

struct BwdArgs {
    const bf16* Q;
    const bf16* K;
    const bf16* V;
    const bf16* O;
    const bf16* dO;
    const float* LSE;
    bf16* dQ;
    bf16* dK;
    bf16* dV;
    float* delta;   // [B, Hq, q_len]
    float* lse2;    // [B, Hq, q_len]  LSE * log2(e); +inf for rows with every key masked
    int64_t q_sb, q_sh, q_ss, k_sb, k_sh, k_ss, v_sb, v_sh, v_ss, o_sb, o_sh, o_ss, do_sb, do_sh, do_ss;
    int64_t dq_sb, dq_sh, dq_ss, dk_sb, dk_sh, dk_ss, dv_sb, dv_sh, dv_ss;
    int B, Hq, Hkv, G, q_len, kv_len;
    int NR, NC, Bq, Bk;
    int bm_Bm, bm_Hm;
    const int32_t* kv_num;
    const int32_t* kv_idx;
    const int32_t* full_kv_num;
    const int32_t* full_kv_idx;
    const int32_t* q_num;
    const int32_t* q_idx;
    const int32_t* full_q_num;
    const int32_t* full_q_idx;
    float scale;
    flexattn_mod_params p;
};

// Position of element t (0..15) inside a 16-wide chunk of a transposed LDS tile; see fwd_kernel.h.
__device__ __forceinline__ constexpr int tr_pos16(int t) { return 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3); }

// Writes a 4-row x 8-column unit (rows r..r+3 of a row-major tile, held as four 16-byte registers)
// into a transposed tile T[col][row-position] with row stride TS elements.
__device__ __forceinline__ void store_unit_transposed(bf16* T, int TS, int col0, int pos, const u32x4 (&u)[4]) {
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) {
        const uint32_t r0 = u[0][wd], r1 = u[1][wd], r2 = u[2][wd], r3 = u[3][wd];
        u32x2 lo, hi;
        lo[0] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
        lo[1] = __builtin_amdgcn_perm(r3, r2, 0x05040100u);
        hi[0] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
        hi[1] = __builtin_amdgcn_perm(r3, r2, 0x07060302u);
        *(u32x2*)(&T[(col0 + 2 * wd) * TS + pos]) = lo;
        *(u32x2*)(&T[(col0 + 2 * wd + 1) * TS + pos]) = hi;
    }
}

// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const BwdArgs a) {
    // 8 lanes per row (D = 64) or 16 lanes per row (D = 128): each lane owns 8 consecutive dims.
    constexpr int LPR = D / 8;
    constexpr int RPB = 256 / LPR;
    const int64_t rows = (int64_t)a.B * a.Hq * a.q_len;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
    const int c = threadIdx.x % LPR;
    if (row >= rows) return;
    const int q = (int)(row % a.q_len);
    const int h = (int)((row / a.q_len) % a.Hq);
    const int b = (int)(row / ((int64_t)a.q_len * a.Hq));
    const bf16x8 o = *(const bf16x8*)(a.O + b * a.o_sb + h * a.o_sh + (int64_t)q * a.o_ss + c * 8);
    const bf16x8 g = *(const bf16x8*)(a.dO + b * a.do_sb + h * a.do_sh + (int64_t)q * a.do_ss + c * 8);
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (float)o[i] * (float)g[i];
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (c == 0) {
        a.delta[row] = s;
        const float l = a.LSE[row];
        a.lse2[row] = (l == -INFINITY) ? INFINITY : l * kLog2e;
    }
}

// ------------------------------------------------------------------------------------------
// dK, dV.  256 threads = 4 waves; wave w owns keys 32 * (w & 1) .. +32 of the 64-key tile and
// query rows 32 * (w >> 1) .. +32 of every 64-row query tile; the two waves that share keys add
// their accumulators through LDS at the end.
template <int D, uint32_t MASK, uint32_t SCORE>
__global__ __launch_bounds__(256, 1) void bwd_dkdv_kernel(const BwdArgs a) {
    constexpr int DC = D / 8;
    constexpr int NS = D + 8;           // natural tiles: [64 rows][D] padded
    constexpr int TS = 64 + 8;          // transposed tiles: [D][64 rows] padded
    constexpr int NU = 16 * DC;         // 4-row x 8-col units per 64 x D tile
    constexpr int UPT = (NU + 255) / 256;
    constexpr int TQ = 64;              // query rows per step

    // one LDS block: natural Q and dO tiles, their transposes; reused for the final reduction
    constexpr int kTileElems = 2 * TQ * NS + 2 * D * TS;
    static_assert(sizeof(bf16) * kTileElems >= sizeof(float) * 4 * D * 32, "reduction buffer must fit");
    __shared__ __attribute__((aligned(16))) bf16 smem[kTileElems];
    __shared__ float s_lse[TQ], s_delta[TQ];
    bf16* const Qn = smem;
    bf16* const dOn = Qn + TQ * NS;
    bf16* const Qt = dOn + TQ * NS;
    bf16* const dOt = Qt + D * TS;

    // workgroup -> (b, hkv, 64-key tile); all tiles of one (b, hkv) on one XCD
    const int units = a.B * a.Hkv;
    const int tiles = a.kv_len / 64;
    const int id = blockIdx.x, xcd = id & 7, kk = id >> 3;
    const int unit = (kk / tiles) * 8 + xcd;
    if (unit >= units) return;
    const int tile = kk % tiles;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv;
    const int kv0 = tile * 64;
    const int col = kv0 / a.Bk;         // column of BlockMask blocks this tile lies in

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int kb = w & 1, qh = w >> 1;
    const int kv_lane = kv0 + 32 * kb + l32;

    // K, V fragments of this wave's 32 keys: B operands (column = key, k-slots = dims)
    bf16x8 kf[D / 16], vf[D / 16];
    {
        const bf16* kp = a.K + b * a.k_sb + hkv * a.k_sh + (int64_t)kv_lane * a.k_ss + half * 8;
        const bf16* vp = a.V + b * a.v_sb + hkv * a.v_sh + (int64_t)kv_lane * a.v_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            kf[ks] = *(const bf16x8*)(kp + ks * 16);
            vf[ks] = *(const bf16x8*)(vp + ks * 16);
        }
    }

    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dk[db][r] = 0.0f;
            dv[db][r] = 0.0f;
        }

    const int sub = a.Bq / TQ;          // query tiles per BlockMask row block
    u32x4 qreg[UPT][4], doreg[UPT][4];
    float lse_reg = 0.0f, delta_reg = 0.0f;

    for (int g = 0; g < a.G; ++g) {
        const int hq = hkv * a.G + g;
        const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NC + col;
        const int n_full = a.full_q_num[line], n_part = a.q_num[line];
        const int32_t* full_idx = a.full_q_idx + line * a.NR;
        const int32_t* part_idx = a.q_idx + line * a.NR;
        const int T = (n_full + n_part) * sub;
        if (T == 0) continue;
        const bf16* q_base = a.Q + b * a.q_sb + hq * a.q_sh;
        const bf16* do_base = a.dO + b * a.do_sb + hq * a.do_sh;
        const float* lse_base = a.lse2 + ((int64_t)b * a.Hq + hq) * a.q_len;
        const float* delta_base = a.delta + ((int64_t)b * a.Hq + hq) * a.q_len;
        const ScoreMod<SCORE> smod(a.p, hq, a.scale);

        auto tile_q0 = [&](int t) {
            const int pos = t / sub, s = t - pos * sub;
            const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
            return blk * a.Bq + s * TQ;
        };
        auto gload = [&](int q0) {
#pragma unroll
            for (int i = 0; i < UPT; ++i) {
                const int u = tid + i * 256;
                if (NU % 256 == 0 || u < NU) {
                    const int gq = u / DC, cc = u % DC;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        qreg[i][r4] = *(const u32x4*)(q_base + (int64_t)(q0 + 4 * gq + r4) * a.q_ss + cc * 8);
                        doreg[i][r4] = *(const u32x4*)(do_base + (int64_t)(q0 + 4 * gq + r4) * a.do_ss + cc * 8);
                    }
                }
            }
            if (tid < TQ) {
                lse_reg = lse_base[q0 + tid];
                delta_reg = delta_base[q0 + tid];
            }
        };
        auto sstore = [&]() {
#pragma unroll
            for (int i = 0; i < UPT; ++i) {
                const int u = tid + i * 256;
                if (NU % 256 == 0 || u < NU) {
                    const int gq = u / DC, cc = u % DC;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        *(u32x4*)(&Qn[(4 * gq + r4) * NS + cc * 8]) = qreg[i][r4];
                        *(u32x4*)(&dOn[(4 * gq + r4) * NS + cc * 8]) = doreg[i][r4];
                    }
                    const int pos = 16 * (gq >> 2) + tr_pos16(4 * (gq & 3));
                    store_unit_transposed(Qt, TS, cc * 8, pos, qreg[i]);
                    store_unit_transposed(dOt, TS, cc * 8, pos, doreg[i]);
                }
            }
            if (tid < TQ) {
                s_lse[tid] = lse_reg;
                s_delta[tid] = delta_reg;
            }
        };

        int q0 = tile_q0(0);
        gload(q0);
        for (int t = 0; t < T; ++t) {
            __syncthreads();            // previous step's readers are done with the LDS tiles
            sstore();
            __syncthreads();
            const int q0_cur = q0;
            if (t + 1 < T) {
                q0 = tile_q0(t + 1);
                gload(q0);
            }
            const bool partial = (t / sub) >= n_full;

            // S = Q K^T and dP = dO V^T for this wave's 32 x 32 piece
            f32x16 sacc, dpacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sacc[r] = 0.0f;
                dpacc[r] = 0.0f;
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 qa = *(const bf16x8*)(&Qn[(32 * qh + l32) * NS + ks * 16 + half * 8]);
                sacc = mfma32(qa, kf[ks], sacc);
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 da = *(const bf16x8*)(&dOn[(32 * qh + l32) * NS + ks * 16 + half * 8]);
                dpacc = mfma32(da, vf[ks], dpacc);
            }

            // P = exp2(x - lse2), dS = P * (dP - delta) * dscore; row q = 32 qh + crow(r, half)
            u32x4 pk[2], dsk[2];
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    float pv[2], dsv[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int r = 8 * c + 2 * jj + e;
                        const int ql = 32 * qh + crow(r, half);
                        const int qi = q0_cur + ql;
                        const float x = smod.apply(sacc[r], qi - kv_lane);
                        float pe = fast_exp2(x - s_lse[ql]);
                        if (partial) {
                            const MaskRow<MASK> mrow(a.p, b, hq, qi);
                            pe = mrow(kv_lane) ? pe : 0.0f;
                        }
                        pv[e] = pe;
                        dsv[e] = pe * (dpacc[r] - s_delta[ql]) * smod.dscore(x);
                    }
                    pk[c][jj] = pack_bf16(pv[0], pv[1]);
                    dsk[c][jj] = pack_bf16(dsv[0], dsv[1]);
                }

            // dV^T += dO^T P, dK^T += Q^T dS  (contraction over this wave's 32 query rows)
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int off = (db * 32 + l32) * TS + (2 * qh + c) * 16 + half * 8;
                    const bf16x8 dot = *(const bf16x8*)(&dOt[off]);
                    const bf16x8 qt = *(const bf16x8*)(&Qt[off]);
                    dv[db] = mfma32(dot, __builtin_bit_cast(bf16x8, pk[c]), dv[db]);
                    dk[db] = mfma32(qt, __builtin_bit_cast(bf16x8, dsk[c]), dk[db]);
                }
        }
        __syncthreads();                // before the next head overwrites the tiles
    }

    // ---- add the two query-halves through LDS and write dK, dV (bf16)
    float* red = (float*)smem;          // [key block][dK | dV][D][32 keys] floats
    __syncthreads();
    if (qh == 1) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                red[((kb * 2 + 0) * D + db * 32 + crow(r, half)) * 32 + l32] = dk[db][r];
                red[((kb * 2 + 1) * D + db * 32 + crow(r, half)) * 32 + l32] = dv[db][r];
            }
    }
    __syncthreads();
    if (qh == 0) {
        bf16* dkp = a.dK + b * a.dk_sb + hkv * a.dk_sh + (int64_t)kv_lane * a.dk_ss;
        bf16* dvp = a.dV + b * a.dv_sb + hkv * a.dv_sh + (int64_t)kv_lane * a.dv_ss;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float k4[4], v4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * rg + e;
                    k4[e] = (dk[db][r] + red[((kb * 2 + 0) * D + db * 32 + crow(r, half)) * 32 + l32]) * a.scale;
                    v4[e] = dv[db][r] + red[((kb * 2 + 1) * D + db * 32 + crow(r, half)) * 32 + l32];
                }
                u32x2 ko, vo;
                ko[0] = pack_bf16(k4[0], k4[1]);
                ko[1] = pack_bf16(k4[2], k4[3]);
                vo[0] = pack_bf16(v4[0], v4[1]);
                vo[1] = pack_bf16(v4[2], v4[3]);
                *(u32x2*)(dkp + db * 32 + 8 * rg + 4 * half) = ko;
                *(u32x2*)(dvp + db * 32 + 8 * rg + 4 * half) = vo;
            }
    }
}

// ------------------------------------------------------------------------------------------
// dQ.  NW waves, each owning 32 query rows of the row of blocks; structure of the forward kernel.
template <int D, int NW, uint32_t MASK, uint32_t SCORE>
__global__ __launch_bounds__(NW * 64, 1) void bwd_dq_kernel(const BwdArgs a) {
    constexpr int NT = NW * 64;
    constexpr int Bq = NW * 32;
    constexpr int DC = D / 8;
    constexpr int NS = D + 8;
    constexpr int TS = 64 + 8;
    constexpr int NU = 16 * DC;
    constexpr int UPT = (NU + NT - 1) / NT;

    __shared__ __attribute__((aligned(16))) bf16 Kn[64 * NS];
    __shared__ __attribute__((aligned(16))) bf16 Vn[64 * NS];
    __shared__ __attribute__((aligned(16))) bf16 Kt[D * TS];

    const int units = a.B * a.Hkv;
    const int id = blockIdx.x, xcd = id & 7, kk = id >> 3;
    const int per_unit = a.G * a.NR;
    const int unit = (kk / per_unit) * 8 + xcd;
    if (unit >= units) return;
    const int rem = kk % per_unit;
    const int row = a.NR - 1 - rem / a.G;
    const int g = rem % a.G;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv, hq = hkv * a.G + g;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int q_row = row * Bq + w * 32 + l32;

    const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NR + row;
    const int n_full = a.full_kv_num[line], n_part = a.kv_num[line];
    const int32_t* full_idx = a.full_kv_idx + line * a.NC;
    const int32_t* part_idx = a.kv_idx + line * a.NC;
    const int sub = a.Bk / 64;
    const int T = (n_full + n_part) * sub;

    bf16* dq_ptr = a.dQ + b * a.dq_sb + hq * a.dq_sh + (int64_t)q_row * a.dq_ss;
    if (T == 0) {
        for (int d0 = half * 8; d0 < D; d0 += 16) *(u32x4*)(dq_ptr + d0) = u32x4{0, 0, 0, 0};
        return;
    }

    bf16x8 qf[D / 16], dof[D / 16];
    {
        const bf16* qp = a.Q + b * a.q_sb + hq * a.q_sh + (int64_t)q_row * a.q_ss + half * 8;
        const bf16* dp = a.dO + b * a.do_sb + hq * a.do_sh + (int64_t)q_row * a.do_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            qf[ks] = *(const bf16x8*)(qp + ks * 16);
            dof[ks] = *(const bf16x8*)(dp + ks * 16);
        }
    }
    const int64_t rowi = ((int64_t)b * a.Hq + hq) * a.q_len + q_row;
    const float lse2 = a.lse2[rowi], delta = a.delta[rowi];
    const bf16* k_base = a.K + b * a.k_sb + hkv * a.k_sh;
    const bf16* v_base = a.V + b * a.v_sb + hkv * a.v_sh;
    const ScoreMod<SCORE> smod(a.p, hq, a.scale);
    const MaskRow<MASK> mrow(a.p, b, hq, q_row);

    u32x4 kreg[UPT][4], vreg[UPT][4];
    auto tile_kv0 = [&](int t) {
        const int pos = t / sub, s = t - pos * sub;
        const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
        return blk * a.Bk + s * 64;
    };
    auto gload = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = tid + i * NT;
            if (NU % NT == 0 || u < NU) {
                const int gq = u / DC, cc = u % DC;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    kreg[i][r4] = *(const u32x4*)(k_base + (int64_t)(kv0 + 4 * gq + r4) * a.k_ss + cc * 8);
                    vreg[i][r4] = *(const u32x4*)(v_base + (int64_t)(kv0 + 4 * gq + r4) * a.v_ss + cc * 8);
                }
            }
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = tid + i * NT;
            if (NU % NT == 0 || u < NU) {
                const int gq = u / DC, cc = u % DC;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    *(u32x4*)(&Kn[(4 * gq + r4) * NS + cc * 8]) = kreg[i][r4];
                    *(u32x4*)(&Vn[(4 * gq + r4) * NS + cc * 8]) = vreg[i][r4];
                }
                const int pos = 16 * (gq >> 2) + tr_pos16(4 * (gq & 3));
                store_unit_transposed(Kt, TS, cc * 8, pos, kreg[i]);
            }
        }
    };

    f32x16 dq[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.0f;

    int kv0 = tile_kv0(0);
    gload(kv0);
    for (int t = 0; t < T; ++t) {
        __syncthreads();
        sstore();
        __syncthreads();
        const int kv0_cur = kv0;
        if (t + 1 < T) {
            kv0 = tile_kv0(t + 1);
            gload(kv0);
        }
        const bool partial = (t / sub) >= n_full;

        u32x4 dsk[2][2];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
            f32x16 sacc, dpacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sacc[r] = 0.0f;
                dpacc[r] = 0.0f;
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 ka = *(const bf16x8*)(&Kn[(kvb * 32 + l32) * NS + ks * 16 + half * 8]);
                sacc = mfma32(ka, qf[ks], sacc);
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 va = *(const bf16x8*)(&Vn[(kvb * 32 + l32) * NS + ks * 16 + half * 8]);
                dpacc = mfma32(va, dof[ks], dpacc);
            }
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    float dsv[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int r = 8 * c + 2 * jj + e;
                        const int kv = kv0_cur + kvb * 32 + crow(r, half);
                        const float x = smod.apply(sacc[r], q_row - kv);
                        float pe = fast_exp2(x - lse2);
                        if (partial) pe = mrow(kv) ? pe : 0.0f;
                        dsv[e] = pe * (dpacc[r] - delta) * smod.dscore(x);
                    }
                    dsk[kvb][c][jj] = pack_bf16(dsv[0], dsv[1]);
                }
        }
        // dQ^T += K^T dS^T
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 kt = *(const bf16x8*)(&Kt[(db * 32 + l32) * TS + (kvb * 2 + c) * 16 + half * 8]);
                    dq[db] = mfma32(kt, __builtin_bit_cast(bf16x8, dsk[kvb][c]), dq[db]);
                }
    }

#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            u32x2 pk;
            pk[0] = pack_bf16(dq[db][4 * rg] * a.scale, dq[db][4 * rg + 1] * a.scale);
            pk[1] = pack_bf16(dq[db][4 * rg + 2] * a.scale, dq[db][4 * rg + 3] * a.scale);
            *(u32x2*)(dq_ptr + db * 32 + 8 * rg + 4 * half) = pk;
        }
}

template <uint32_t MASK, uint32_t SCORE>
int launch_bwd_variant(const BwdArgs& a, int D, uint32_t stages, hipStream_t st) {
    const int units = a.B * a.Hkv;
    const unsigned grid_kv = (unsigned)(((units + 7) / 8) * 8 * (a.kv_len / 64));
    const unsigned grid_q = (unsigned)(((units + 7) / 8) * 8 * a.G * a.NR);
    const bool kv = stages & FLEXATTN_BWD_DKDV, q = stages & FLEXATTN_BWD_DQ;
    if (D == 128) {
        if (kv) hipLaunchKernelGGL((bwd_dkdv_kernel<128, MASK, SCORE>), dim3(grid_kv), dim3(256), 0, st, a);
        if (q && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<128, 4, MASK, SCORE>), dim3(grid_q), dim3(256), 0, st, a);
        if (q && a.Bq == 64) hipLaunchKernelGGL((bwd_dq_kernel<128, 2, MASK, SCORE>), dim3(grid_q), dim3(128), 0, st, a);
    } else {
        if (kv) hipLaunchKernelGGL((bwd_dkdv_kernel<64, MASK, SCORE>), dim3(grid_kv), dim3(256), 0, st, a);
        if (q && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<64, 4, MASK, SCORE>), dim3(grid_q), dim3(256), 0, st, a);
        if (q && a.Bq == 64) hipLaunchKernelGGL((bwd_dq_kernel<64, 2, MASK, SCORE>), dim3(grid_q), dim3(128), 0, st, a);
    }
    return FLEXATTN_OK;
}

}  // namespace flexattn
