// FlexAttention forward kernel for gfx950 (paper Eq. 1; forward template of section 4.1; block
// skipping, full/partial split and indirect KV-block access of section 4.2; the KV prefetch of
// the "Data Prefetching Pipeline" paragraph is the register-staged double buffer below).
//
// One workgroup owns one row of BlockMask blocks (Bq = NW * 32 query rows of one (b, hq)); each
// wave owns 32 of those rows.  The score tile is computed TRANSPOSED, S^T = K Q^T, so that in the
// MFMA result layout every lane holds scores of ONE query (column l % 32) and 16 keys per 32-key
// block in its registers: the row max / row sum of the online softmax are in-register reductions
// plus one exchange between the two halves of the wave, and P^T is already laid out as the B
// operand of O^T += V^T P^T.  K tiles sit in LDS row-major (A operand of K Q^T), V tiles are
// transposed on their way into LDS (A operand V^T), Q lives in registers for the whole kernel.
#pragma once

#include "flex_common.h"

namespace flexattn {

struct FwdArgs {
    const bf16* Q;
    const bf16* K;
    const bf16* V;
    bf16* O;
    float* LSE;
    int64_t q_sb, q_sh, q_ss, k_sb, k_sh, k_ss, v_sb, v_sh, v_ss, o_sb, o_sh, o_ss;
    int B, Hq, Hkv, G, q_len, kv_len;
    int NR, NC, Bk, sub;   // BlockMask geometry; sub = Bk / 64 kernel tiles per block
    int bm_Bm, bm_Hm;
    const int32_t* kv_num;
    const int32_t* kv_idx;
    const int32_t* full_num;
    const int32_t* full_idx;
    float scale;
    flexattn_mod_params p;
};

constexpr int kTileKV = 64;   // keys per kernel tile

// Position inside a 16-key chunk of V^T rows at which key t (0..15) is stored, chosen so that the
// eight keys a lane of half h needs for one MFMA (t = 4h + 8 * (j / 4) + j % 4, j = 0..7: the keys
// its P^T registers hold) are contiguous: pos = 8 h + j.
__device__ __forceinline__ constexpr int vt_pos16(int t) { return 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3); }

template <int D, int NW, uint32_t MASK, uint32_t SCORE>
__global__ __launch_bounds__(NW * 64, 2) void fwd_kernel(const FwdArgs a) {
    constexpr int NT = NW * 64;
    constexpr int Bq = NW * 32;
    constexpr int DC = D / 8;                      // 16-byte chunks per row
    constexpr int KS = D + 8;                      // K row stride in LDS (elements), padded
    constexpr int VS = kTileKV + 8;                // V^T row stride in LDS (elements), padded
    constexpr int NKC = kTileKV * DC / NT;         // K chunks per thread
    constexpr int NVU = (kTileKV / 4) * DC;        // V units (4 keys x 8 dims) per tile
    constexpr int NVT = (NVU + NT - 1) / NT;       // V units per thread
    static_assert(kTileKV * DC % NT == 0, "K tile must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) bf16 Ks[2][kTileKV * KS];
    __shared__ __attribute__((aligned(16))) bf16 Vt[2][D * VS];

    // ---- workgroup -> (b, hkv, g, row of blocks).  Consecutive workgroup ids go to the 8 XCDs in
    // turn; all rows and all G query heads of one (b, hkv) are sent to the same XCD so that its K/V
    // stay in that XCD's L2.  Rows are taken last-first (causal-like masks: longest first).
    const int units = a.B * a.Hkv;
    const int id = blockIdx.x;
    const int xcd = id & 7, k = id >> 3;
    const int per_unit = a.G * a.NR;
    const int unit = (k / per_unit) * 8 + xcd;
    if (unit >= units) return;
    const int rem = k % per_unit;
    const int row = a.NR - 1 - rem / a.G;
    const int g = rem % a.G;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv, hq = hkv * a.G + g;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int q_row = row * Bq + w * 32 + l32;

    const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NR + row;
    const int n_full = a.full_num[line], n_part = a.kv_num[line];
    const int32_t* full_idx = a.full_idx + line * a.NC;
    const int32_t* part_idx = a.kv_idx + line * a.NC;
    const int T = (n_full + n_part) * a.sub;

    bf16* o_ptr = a.O + b * a.o_sb + hq * a.o_sh + (int64_t)q_row * a.o_ss;
    float* lse_ptr = a.LSE + ((int64_t)b * a.Hq + hq) * a.q_len + q_row;
    if (T == 0) {   // every key of these rows is masked
        for (int d0 = half * 8; d0 < D; d0 += 16) *(u32x4*)(o_ptr + d0) = u32x4{0, 0, 0, 0};
        if (half == 0) *lse_ptr = -INFINITY;
        return;
    }

    // Q fragments: B operand of K Q^T, column q_row, k-slots d = 16 ks + 8 half + [0, 8)
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.Q + b * a.q_sb + hq * a.q_sh + (int64_t)q_row * a.q_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *(const bf16x8*)(qp + ks * 16);
    }
    const bf16* k_base = a.K + b * a.k_sb + hkv * a.k_sh;
    const bf16* v_base = a.V + b * a.v_sb + hkv * a.v_sh;

    const ScoreMod<SCORE> smod(a.p, hq, a.scale);
    const MaskRow<MASK> mrow(a.p, b, hq, q_row);

    bf16x8 kreg[NKC];
    u32x4 vreg[NVT][4];

    auto tile_kv0 = [&](int t) {
        const int pos = t / a.sub, s = t - pos * a.sub;
        const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
        return blk * a.Bk + s * kTileKV;
    };
    auto gload = [&](int kv0) {
        const bf16* kp = k_base + (int64_t)kv0 * a.k_ss;
        const bf16* vp = v_base + (int64_t)kv0 * a.v_ss;
#pragma unroll
        for (int i = 0; i < NKC; ++i) {
            const int c = tid + i * NT, r = c / DC, cc = c % DC;
            kreg[i] = *(const bf16x8*)(kp + (int64_t)r * a.k_ss + cc * 8);
        }
#pragma unroll
        for (int i = 0; i < NVT; ++i) {
            const int u = tid + i * NT;
            if (NVU % NT == 0 || u < NVU) {
                const int gq = u / DC, cc = u % DC;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4)
                    vreg[i][r4] = *(const u32x4*)(vp + (int64_t)(4 * gq + r4) * a.v_ss + cc * 8);
            }
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NKC; ++i) {
            const int c = tid + i * NT, r = c / DC, cc = c % DC;
            *(bf16x8*)(&Ks[buf][r * KS + cc * 8]) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < NVT; ++i) {
            const int u = tid + i * NT;
            if (NVU % NT == 0 || u < NVU) {
                const int gq = u / DC, cc = u % DC;
                const int pos = 16 * (gq >> 2) + vt_pos16(4 * (gq & 3));
                // 4 keys x 8 dims -> 8 dims x 4 keys
#pragma unroll
                for (int wd = 0; wd < 4; ++wd) {
                    const uint32_t r0 = vreg[i][0][wd], r1 = vreg[i][1][wd], r2 = vreg[i][2][wd], r3 = vreg[i][3][wd];
                    u32x2 lo, hi;
                    lo[0] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
                    lo[1] = __builtin_amdgcn_perm(r3, r2, 0x05040100u);
                    hi[0] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
                    hi[1] = __builtin_amdgcn_perm(r3, r2, 0x07060302u);
                    *(u32x2*)(&Vt[buf][(cc * 8 + 2 * wd) * VS + pos]) = lo;
                    *(u32x2*)(&Vt[buf][(cc * 8 + 2 * wd + 1) * VS + pos]) = hi;
                }
            }
        }
    };

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    int kv0 = tile_kv0(0);
    gload(kv0);
    sstore(0);
    __syncthreads();

    for (int t = 0; t < T; ++t) {
        const int buf = t & 1;
        int kv0_next = 0;
        if (t + 1 < T) {
            kv0_next = tile_kv0(t + 1);
            gload(kv0_next);
        }
        const bool partial = (t / a.sub) >= n_full;

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 sacc[2];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kvb][r] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 kf = *(const bf16x8*)(&Ks[buf][(kvb * 32 + l32) * KS + ks * 16 + half * 8]);
                sacc[kvb] = mfma32(kf, qf[ks], sacc[kvb]);
            }
        }

        // ---- score_mod, mask_mod (partial blocks only), online softmax in base 2
        const int dq_base = q_row - kv0;
        float mx = -INFINITY;
        if (partial) {
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvo = kvb * 32 + crow(r, half);
                    float x = smod.apply(sacc[kvb][r], dq_base - kvo);
                    x = mrow(kv0 + kvo) ? x : -INFINITY;
                    sacc[kvb][r] = x;
                    mx = fmaxf(mx, x);
                }
        } else {
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvo = kvb * 32 + crow(r, half);
                    const float x = smod.apply(sacc[kvb][r], dq_base - kvo);
                    sacc[kvb][r] = x;
                    mx = fmaxf(mx, x);
                }
        }
        mx = fmaxf(mx, swap_halves(mx));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
        const float alpha = fast_exp2(m_run - m_use);
        m_run = m_new;
        float psum = 0.0f;
        bf16x8 pf[2][2];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                u32x4 pk;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float p0 = fast_exp2(sacc[kvb][8 * c + 2 * jj] - m_use);
                    const float p1 = fast_exp2(sacc[kvb][8 * c + 2 * jj + 1] - m_use);
                    psum += p0 + p1;
                    pk[jj] = pack_bf16(p0, p1);
                }
                pf[kvb][c] = __builtin_bit_cast(bf16x8, pk);
            }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 vf =
                        *(const bf16x8*)(&Vt[buf][(db * 32 + l32) * VS + (kvb * 2 + c) * 16 + half * 8]);
                    oacc[db] = mfma32(vf, pf[kvb][c], oacc[db]);
                }

        if (t + 1 < T) sstore(buf ^ 1);
        __syncthreads();
        kv0 = kv0_next;
    }

    // ---- epilogue: O = O^T / l, LSE = ln 2 * (m + log2 l)
    const float l_tot = l_run + swap_halves(l_run);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            u32x2 pk;
            pk[0] = pack_bf16(oacc[db][4 * rg] * inv, oacc[db][4 * rg + 1] * inv);
            pk[1] = pack_bf16(oacc[db][4 * rg + 2] * inv, oacc[db][4 * rg + 3] * inv);
            *(u32x2*)(o_ptr + db * 32 + 8 * rg + 4 * half) = pk;
        }
    if (half == 0) *lse_ptr = l_tot > 0.0f ? (m_run + fast_log2(l_tot)) * kLn2 : -INFINITY;
}

template <uint32_t MASK, uint32_t SCORE>
int launch_fwd_variant(const FwdArgs& a, int D, int Bq, hipStream_t st) {
    const int units = a.B * a.Hkv;
    const unsigned grid = (unsigned)(((units + 7) / 8) * 8 * a.G * a.NR);
#define FLEXATTN_LAUNCH(DD, NW)                                                                         \
    hipLaunchKernelGGL((fwd_kernel<DD, NW, MASK, SCORE>), dim3(grid), dim3(NW * 64), 0, st, a);         \
    return FLEXATTN_OK;
    if (D == 128 && Bq == 128) { FLEXATTN_LAUNCH(128, 4) }
    if (D == 128 && Bq == 64) { FLEXATTN_LAUNCH(128, 2) }
    if (D == 64 && Bq == 128) { FLEXATTN_LAUNCH(64, 4) }
    if (D == 64 && Bq == 64) { FLEXATTN_LAUNCH(64, 2) }
#undef FLEXATTN_LAUNCH
    return FLEXATTN_ERR_UNSUPPORTED;
}

}  // namespace flexattn
