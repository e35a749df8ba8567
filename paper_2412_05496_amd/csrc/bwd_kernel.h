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
// Tiles (Q, dO in the first kernel; K, V in the second) go from global memory straight into
// XOR-swizzled LDS tiles, double buffered, one barrier per tile; the transposed operands
// (dO^T, Q^T, K^T) come out of the same row-major tiles through transposing LDS reads.
#pragma once

#include <type_traits>

#include "flex_common.h"
#include "lds_tiles.h"

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
// dK, dV.  256 threads = 4 waves; one workgroup per 64 keys.  The listed q-blocks are walked in
// steps of two 64-row half-tiles; wave w owns keys 32 * (w & 1) .. +32 and the half-tile w >> 1,
// which it processes as two 32 x 32 score blocks so that the MFMAs of one block sit next to the
// exp / dS arithmetic of the other.  The two waves that share keys add their accumulators
// through LDS at the end.
template <int D, uint32_t MASK, uint32_t SCORE>
__global__ __launch_bounds__(256, 1) void bwd_dkdv_kernel(const BwdArgs a) {
    constexpr int HQ = 64;                         // query rows per half-tile
    constexpr int TILE = HQ * D;                   // elements per LDS tile
    // per buffer: Q half a, Q half b, dO half a, dO half b; two buffers; reused for the final reduction
    __shared__ __attribute__((aligned(1024))) bf16 smem[8 * TILE];
    __shared__ __attribute__((aligned(16))) float s_row[2][2][2 * HQ];   // [buffer][lse2 | delta][row]
    static_assert(sizeof(bf16) * 8 * TILE >= sizeof(float) * 4 * D * 32, "reduction buffer must fit");

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

    const int sub = a.Bq / HQ;          // half-tiles per BlockMask row block
    const TileLoader<D, 4> q_loader(a.q_ss, w, lane), do_loader(a.do_ss, w, lane);
    // per-lane LDS addresses of this wave's half-tile (Q copy; the dO copy is 2 tiles further on)
    const uint32_t my_tile = lds_addr(smem) + qh * (TILE * 2);
    const RowReader<D> row_reader(l32, half, my_tile);
    const TrReader<D> tr_reader(lane, my_tile);

    for (int g = 0; g < a.G; ++g) {
        const int hq = hkv * a.G + g;
        const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NC + col;
        const int n_full = a.full_q_num[line], n_part = a.q_num[line];
        const int32_t* full_idx = a.full_q_idx + line * a.NR;
        const int32_t* part_idx = a.q_idx + line * a.NR;
        const int H = (n_full + n_part) * sub;      // half-tiles to visit
        if (H == 0) continue;
        const int U = (H + 1) / 2;                  // steps
        const bf16* q_base = a.Q + b * a.q_sb + hq * a.q_sh;
        const bf16* do_base = a.dO + b * a.do_sb + hq * a.do_sh;
        const float* lse_base = a.lse2 + ((int64_t)b * a.Hq + hq) * a.q_len;
        const float* delta_base = a.delta + ((int64_t)b * a.Hq + hq) * a.q_len;
        const ScoreMod<SCORE> smod(a.p, hq, a.scale);

        auto half_q0 = [&](int h) {                 // first query row of half-tile h (h < H)
            const int pos = h / sub, s = h - pos * sub;
            const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
            return blk * a.Bq + s * HQ;
        };
        // starts the loads of step u into buffer u & 1; returns this thread's row scalar
        auto load_step = [&](int u) {
            bf16* buf = smem + (u & 1) * 4 * TILE;
            const int qa = half_q0(2 * u);
            const bool has_b = 2 * u + 1 < H;
            const int qb = has_b ? half_q0(2 * u + 1) : qa;
            // row scalars first: waiting for them later must not wait for the tiles behind them
            const int rr = tid & (2 * HQ - 1);
            const int qrow = (rr < HQ ? qa : qb) + (rr & (HQ - 1));
            const float v = tid < 2 * HQ ? lse_base[qrow] : delta_base[qrow];
            q_loader.start(buf, q_base + (int64_t)qa * a.q_ss);
            do_loader.start(buf + 2 * TILE, do_base + (int64_t)qa * a.do_ss);
            if (has_b) {
                q_loader.start(buf + TILE, q_base + (int64_t)qb * a.q_ss);
                do_loader.start(buf + 3 * TILE, do_base + (int64_t)qb * a.do_ss);
            }
            return v;
        };
        // lse2 is stored as the row constant of ScoreMod::p_with_grad
        auto store_rows = [&](int u, float v) {
            s_row[u & 1][tid >> 7][tid & (2 * HQ - 1)] = tid < 2 * HQ ? smod.row_const(v) : v;
        };

        store_rows(0, load_step(0));
        wait_vmem();
        __syncthreads();

        // One step on buffer BUF (compile-time, so that every LDS read is "VGPR + immediate").
        auto step = [&](int u, auto buf_tag) {
            constexpr int BUF = decltype(buf_tag)::value;
            float row_next = 0.0f;
            if (u + 1 < U) row_next = load_step(u + 1);     // buffer BUF ^ 1 was last read in step u-1
            const int h_mine = 2 * u + qh;
            if (h_mine < H) {
                const int q0 = half_q0(h_mine);
                const bool partial = (h_mine / sub) >= n_full;
                constexpr uint32_t qt = BUF * 4 * (TILE * 2), dot = (BUF * 4 + 2) * (TILE * 2);
                const float* lrow = &s_row[BUF][0][HQ * qh];
                const float* drow = &s_row[BUF][1][HQ * qh];

                // S = Q K^T and dP = dO V^T for both 32-row blocks of this wave
                f32x16 sacc[2], dpacc[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        sacc[j][r] = 0.0f;
                        dpacc[j][r] = 0.0f;
                    }
#pragma unroll
                    for (int ks = 0; ks < D / 16; ++ks) sacc[j] = mfma32(row_reader.read(qt, 32 * j, ks), kf[ks], sacc[j]);
#pragma unroll
                    for (int ks = 0; ks < D / 16; ++ks) dpacc[j] = mfma32(row_reader.read(dot, 32 * j, ks), vf[ks], dpacc[j]);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // P = exp2(x - lse2), dS = P * (dP - delta) * g; row = 32 j + crow(r, half)
                    f32x4 rc4[4], del4[4];
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        rc4[rg] = *(const f32x4*)(lrow + 32 * j + 8 * rg + 4 * half);
                        del4[rg] = *(const f32x4*)(drow + 32 * j + 8 * rg + 4 * half);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int qi = q0 + 32 * j + crow(r, half);
                        float gr;
                        const float pe = smod.p_with_grad(sacc[j][r], qi - kv_lane, rc4[r >> 2][r & 3], gr);
                        sacc[j][r] = pe;
                        dpacc[j][r] = pe * (dpacc[j][r] - del4[r >> 2][r & 3]) * gr;
                    }
                    if (partial) {
                        asm volatile("" ::: "memory");   // keep this a branch
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const MaskRow<MASK> mrow(a.p, b, hq, q0 + 32 * j + crow(r, half));
                            const bool keep = mrow(kv_lane);
                            sacc[j][r] = keep ? sacc[j][r] : 0.0f;
                            dpacc[j][r] = keep ? dpacc[j][r] : 0.0f;
                        }
                    }
                    // dV^T += dO^T P, dK^T += Q^T dS  (contraction over these 32 query rows)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        u32x4 pk, dsk;
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            pk[jj] = pack_bf16(sacc[j][8 * c + 2 * jj], sacc[j][8 * c + 2 * jj + 1]);
                            dsk[jj] = pack_bf16(dpacc[j][8 * c + 2 * jj], dpacc[j][8 * c + 2 * jj + 1]);
                        }
#pragma unroll
                        for (int db = 0; db < D / 32; ++db) {
                            dv[db] = mfma32(tr_reader.read(dot, 32 * j + 16 * c, db), __builtin_bit_cast(bf16x8, pk), dv[db]);
                            dk[db] = mfma32(tr_reader.read(qt, 32 * j + 16 * c, db), __builtin_bit_cast(bf16x8, dsk), dk[db]);
                        }
                    }
                }
            }
            if (u + 1 < U) store_rows(u + 1, row_next);
            wait_vmem();
            __syncthreads();
        };
        int u = 0;
        for (; u + 1 < U; u += 2) {
            step(u, std::integral_constant<int, 0>{});
            step(u + 1, std::integral_constant<int, 1>{});
        }
        if (u < U) step(u, std::integral_constant<int, 0>{});
    }

    // ---- add the two query-halves through LDS and write dK, dV (bf16)
    float* red = (float*)smem;          // [key block][dK | dV][D][32 keys] floats
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
        const float kscale = a.scale * ScoreMod<SCORE>::grad_scale();
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
                    k4[e] = (dk[db][r] + red[((kb * 2 + 0) * D + db * 32 + crow(r, half)) * 32 + l32]) * kscale;
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
__global__ __launch_bounds__(NW * 64, 2) void bwd_dq_kernel(const BwdArgs a) {
    constexpr int Bq = NW * 32;
    constexpr int TILE = 64 * D;
    __shared__ __attribute__((aligned(1024))) bf16 smem[4 * TILE];   // K(even), K(odd), V(even), V(odd)

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

    auto tile_kv0 = [&](int t) {
        const int pos = t / sub, s = t - pos * sub;
        const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
        return blk * a.Bk + s * 64;
    };
    const TileLoader<D, NW> k_loader(a.k_ss, w, lane), v_loader(a.v_ss, w, lane);
    auto load_tiles = [&](int t, int kv0) {
        k_loader.start(smem + (t & 1) * TILE, k_base + (int64_t)kv0 * a.k_ss);
        v_loader.start(smem + (2 + (t & 1)) * TILE, v_base + (int64_t)kv0 * a.v_ss);
    };
    const RowReader<D> row_reader(l32, half, lds_addr(smem));
    const TrReader<D> tr_reader(lane, lds_addr(smem));
    const float rc = smod.row_const(lse2);

    f32x16 dq[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.0f;

    int kv0 = tile_kv0(0);
    load_tiles(0, kv0);
    wait_vmem();
    __syncthreads();

    // One tile on buffer BUF (compile-time, so that every LDS read is "VGPR + immediate").
    auto step = [&](int t, auto buf_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int kv0_cur = kv0;
        if (t + 1 < T) {
            kv0 = tile_kv0(t + 1);
            load_tiles(t + 1, kv0);          // buffer BUF ^ 1 was last read in step t-1
        }
        const bool partial = (t / sub) >= n_full;
        constexpr uint32_t kt = BUF * (TILE * 2), vt = (2 + BUF) * (TILE * 2);

#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
            // S^T = K Q^T and dP^T = V dO^T for 32 keys
            f32x16 sacc, dpacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sacc[r] = 0.0f;
                dpacc[r] = 0.0f;
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) sacc = mfma32(row_reader.read(kt, kvb * 32, ks), qf[ks], sacc);
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) dpacc = mfma32(row_reader.read(vt, kvb * 32, ks), dof[ks], dpacc);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = kv0_cur + kvb * 32 + crow(r, half);
                float gr;
                const float pe = smod.p_with_grad(sacc[r], q_row - kv, rc, gr);
                dpacc[r] = pe * (dpacc[r] - delta) * gr;
            }
            if (partial) {
                asm volatile("" ::: "memory");   // keep this a branch
#pragma unroll
                for (int r = 0; r < 16; ++r) dpacc[r] = mrow(kv0_cur + kvb * 32 + crow(r, half)) ? dpacc[r] : 0.0f;
            }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                u32x4 dsk;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) dsk[jj] = pack_bf16(dpacc[8 * c + 2 * jj], dpacc[8 * c + 2 * jj + 1]);
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
                    dq[db] = mfma32(tr_reader.read(kt, kvb * 32 + 16 * c, db), __builtin_bit_cast(bf16x8, dsk), dq[db]);
            }
        }
        wait_vmem();
        __syncthreads();
    };
    {
        int t = 0;
        for (; t + 1 < T; t += 2) {
            step(t, std::integral_constant<int, 0>{});
            step(t + 1, std::integral_constant<int, 1>{});
        }
        if (t < T) step(t, std::integral_constant<int, 0>{});
    }

    const float qscale = a.scale * ScoreMod<SCORE>::grad_scale();
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            u32x2 pk;
            pk[0] = pack_bf16(dq[db][4 * rg] * qscale, dq[db][4 * rg + 1] * qscale);
            pk[1] = pack_bf16(dq[db][4 * rg + 2] * qscale, dq[db][4 * rg + 3] * qscale);
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
