// FlexAttention backward kernels for gfx950 (backward template of paper section 4.1, walking the
// BlockMask in both orientations, section 4.2).  The paper gives no formulas; with P recomputed
// from the saved LSE this is the usual softmax-attention calculus:
//     dV = P^T dO,  dP = dO V^T,  dS' = P * (dP - delta),  delta = rowsum(dO * O),
//     dS = dS' * d score_mod / d s,  dQ = scale * dS K,  dK = scale * dS^T Q.
// Three kernels, no floating-point atomics (results are deterministic):
//   bwd_delta_kernel   -delta and the row constant of P = exp2(f(score) + rc) per query row.
//   bwd_dkdv_kernel    one workgroup per 64 keys of one (b, hkv); walks the q-blocks listed for
//                      that column of blocks (transposed BlockMask) for every query head of the
//                      group; score tile in S = Q K^T orientation so that P and dS are the B
//                      operands of dV^T += dO^T P and dK^T += Q^T dS; the two waves that share
//                      keys split the outputs (one dV, one dK) and exchange P / dS through LDS.
//   bwd_dq_kernel      one workgroup per row of blocks of one (b, hq); walks the kv-blocks listed
//                      for it; score tile transposed (S^T = K Q^T) so that dS^T is the B operand of
//                      dQ^T += K^T dS^T and LSE / delta are per-lane scalars.
// Tiles (Q, dO in the first kernel; K, V in the second) go from global memory straight into
// XOR-swizzled LDS tiles, double buffered; the transposed operands (dO^T, Q^T, K^T) come out of
// the same row-major tiles through transposing LDS reads.  dP accumulates on top of -delta.
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
    float* delta;   // [B, Hq, q_len]  MINUS rowsum(dO * O): the dP accumulators start from it
    float* lse2;    // [B, Hq, q_len]  row constant rc of ScoreMod::p_with_grad (from LSE); -inf for dead rows
    // gradients of captured tensors: per-workgroup partial sums, [B, Hq, NR] and [B, Hq, NR, rel_len]
    float* cap_alibi;
    float* cap_rel;
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
    const int32_t* kv_order;   // nullable work orders (rows / columns of blocks, longest first)
    const int32_t* q_order;
    // dS kept in memory (bwd_stored.h): the dK/dV kernel writes the dS of every block it visits, a lean
    // kernel contracts it with K.  Null ds_store: nothing is written.
    bf16* ds_store;            // [heads that share no dS, ds_blocks, Bk / 64, Bq / 64, 4096] (see ds_chunk)
    const int32_t* ds_colbase; // [planes * NC] first block slot of every column of blocks
    const int32_t* ds_grid;    // [planes, NR, NC] slot of block (row, column)
    int64_t ds_blocks;         // slots per head (capacity)
    float scale;
    flexattn_mod_params p;
};

// dS in memory.  The non-empty blocks of all BlockMask planes are numbered column by column of blocks,
// in the order of the merged (FULL, then PARTIAL) column lists: that number is the block's slot.
// Heads that share a plane share the numbering and differ in `rep`.  A block is cut into Bk / 64 tiles
// of 64 keys, a tile into Bq / 64 steps of 64 query rows, and a step is the 8 KiB the four waves of
// the dK/dV workgroup hold in registers after the step: wave (kb, x) two chunks of 1 KiB, lane
// (key 32 kb + l32, half h) 16 bytes of each -- chunk c holds rows 32 x + 16 c + 8 jj + 4 h + i at
// position 4 jj + i.  Slots are clamped to the capacity: a caller that passes too small a capacity
// gets wrong gradients, never an access outside the workspace.
__device__ __forceinline__ int64_t ds_rep(const BwdArgs& a, int b, int hq) {
    return (int64_t)(a.bm_Bm > 1 ? 0 : b) * (a.bm_Hm > 1 ? 1 : a.Hq) + (a.bm_Hm > 1 ? 0 : hq);
}
// index of the 8 KiB step (in units of 4096 bf16) of block `slot`, key tile `st`, row step `sidx`
__device__ __forceinline__ int64_t ds_chunk(const BwdArgs& a, int64_t rep, int slot, int st, int sidx) {
    const int64_t sl = min(max((int64_t)slot, (int64_t)0), a.ds_blocks - 1);
    return ((rep * a.ds_blocks + sl) * (a.Bk / 64) + st) * (a.Bq / 64) + sidx;
}

// ------------------------------------------------------------------------------------------
// -delta = -rowsum(dO * O) and the per-row constant rc of ScoreMod::p_with_grad (so that the main
// kernels get P = exp2(f(score) + rc) with no further per-row arithmetic); rc = -inf for rows
// without a visible key (LSE = -inf), which makes their P vanish.
template <int D, uint32_t SCORE>
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
        a.delta[row] = -s;
        const float l = a.LSE[row];
        const ScoreMod<SCORE> smod(a.p, h, a.scale);
        a.lse2[row] = smod.row_const((l == -INFINITY) ? INFINITY : l * kLog2e);
    }
}

// ------------------------------------------------------------------------------------------
// dK, dV.  256 threads = 4 waves, one workgroup per 64 keys of one (b, hkv), two workgroups per CU
// (two waves per SIMD, from different workgroups, so that one wave's exp / dS arithmetic runs
// beside the other's MFMAs).  The listed q-blocks are walked in steps of 64 query rows.  Wave
// w = (kb, x), kb = w & 1, x = w >> 1:
//   scores     S and dP - delta of the 32 x 32 block (rows 32 x .. +32 of the step, keys 32 kb .. +32),
//              turned into P and dS (bf16, B-operand layout);
//   exchange   the x = 0 wave hands its dS to the x = 1 wave of the same keys through LDS and gets
//              that wave's P;
//   outputs    the x = 0 wave accumulates dV^T += dO^T P over all 64 rows (its own P, then its
//              partner's), the x = 1 wave dK^T += Q^T dS.  Each output row belongs to one wave: no
//              reduction at the end, and 64 accumulator registers per lane instead of 128, which
//              is what lets two workgroups share a CU.
// Q / dO tiles and the per-row scalars are double buffered in LDS; the loads of step v+1 are
// issued at the top of step v.  Two barriers per step: after the exchange writes, and at the end
// (exchange buffer and ring slot free again, next tiles landed).
// M0 RULE: this kernel fills LDS through the LDS-DMA helpers of lds_tiles.h, which write M0 behind the
// compiler's back.  Keep every register array in it indexed by compile-time constants (no movrel /
// s_set_gpr_idx code, which would also use M0) and add no other LDS-DMA or M0-based construct.
template <int D, uint32_t MASK, uint32_t SCORE>
__global__ __launch_bounds__(256, (bwd_waves_per_simd<D, MASK>())) void bwd_dkdv_kernel(const BwdArgs a) {
    constexpr int TQ = 64;                         // query rows per step
    constexpr int TILE = TQ * D;                   // elements per LDS tile
    constexpr int NKS = D / 16, NDB = D / 32;
    using Loader = WaveTileLoader<D, 4>;
    __shared__ __attribute__((aligned(1024))) bf16 smem[2 * 2 * TILE];        // 2 x (Q tile, dO tile)
    __shared__ __attribute__((aligned(1024))) u32x4 s_xchg[4][2][64];         // [wave][16-row slice][lane]
    __shared__ __attribute__((aligned(256))) float s_row[2][2][TQ];           // [slot][rc | -delta][row]
    constexpr int kListMax = 512;
    __shared__ int s_steps[kListMax + 2];          // the walk of the current head, see below
    using Score = ScoreMod<SCORE, true>;
    __shared__ float s_rel[Score::kRel ? kRelTableMax : 1];   // relative-bias row of the current head

    // workgroup -> (b, hkv, 64-key tile); all tiles of one (b, hkv) on one XCD.  The columns of
    // blocks are taken in the BlockMask's work order (longest first; that of the group's first query
    // head where the mask has a plane per head), the 64-key tiles of a column side by side.
    const int units = a.B * a.Hkv;
    const int sub_k = a.Bk / 64;                   // tiles per column of blocks
    const int slots = a.NC * sub_k;                // >= tiles: the last column may be cut short
    const int id = blockIdx.x, xcd = id & 7, kk = id >> 3;
    const int unit = (kk / slots) * 8 + xcd;
    if (unit >= units) return;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv;
    const int slot = kk % slots;
    int col = slot / sub_k;
    if (a.q_order) {
        const int64_t plane0 = (int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hkv * a.G : 0);
        col = min(max(a.q_order[plane0 * a.NC + col], 0), a.NC - 1);   // clamped: a bad order array stays inside the lists
    }
    const int key_tile = slot % sub_k;             // which 64 keys of the column of blocks
    const int tile = col * sub_k + key_tile;
    const int kv0 = tile * 64;
    if (kv0 >= a.kv_len) return;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = w & 1, x = w >> 1;
    const int kv_lane = kv0 + 32 * kb + l32;

    // K, V fragments of this wave's 32 keys: B operands (column = key, k-slots = dims)
    bf16x8 kf[NKS], vf[NKS];
    {
        // keys past kv_len (last tile of a length that is no multiple of 64) take a copy of the last
        // real key; the mask hides them and they are never stored
        const int kv_ld = min(kv_lane, a.kv_len - 1);
        const bf16* kp = a.K + b * a.k_sb + hkv * a.k_sh + (int64_t)kv_ld * a.k_ss + half * 8;
        const bf16* vp = a.V + b * a.v_sb + hkv * a.v_sh + (int64_t)kv_ld * a.v_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            kf[ks] = *(const bf16x8*)(kp + ks * 16);
            vf[ks] = *(const bf16x8*)(vp + ks * 16);
        }
    }

    f32x16 acc[NDB];                    // x = 0: dV^T, x = 1: dK^T (row = dim, column = key)
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;

    const int sub = a.Bq / TQ;          // steps per BlockMask row block (1 or 2)
    const int sub_shift = sub >> 1;
    const Loader q_loader(a.q_ss, w, lane), do_loader(a.do_ss, w, lane);
    const uint32_t ring = lds_addr(smem);
    const uint32_t wave_row = lds_addr(&s_row[0][w & 1][0]);
    const uint32_t q_bytes = (uint32_t)((a.q_len - 1) * a.q_ss + D) * 2u;
    const uint32_t do_bytes = (uint32_t)((a.q_len - 1) * a.do_ss + D) * 2u;
    const int q_row_bytes = (int)a.q_ss * 2, do_row_bytes = (int)a.do_ss * 2;
    // scores: this wave's 32 rows of the Q tile (the dO tile is one tile further)
    const RowReader<D> row_reader(l32, half, ring + x * 32 * D * 2);
    // outputs: the tile this wave contracts with (x = 0: dO, x = 1: Q), its own rows first, then
    // its partner's
    const uint32_t out_tile = ring + (x ? 0 : TILE * 2);
    const TrReader<D> tr_own(lane, out_tile + x * 32 * D * 2), tr_other(lane, out_tile + (1 - x) * 32 * D * 2);
    const uint32_t row_lds = lds_addr(&s_row[0][0][0]) + (32 * x + 4 * half) * 4;
    const uint32_t xchg_mine = lds_addr(&s_xchg[w][0][lane]), xchg_theirs = lds_addr(&s_xchg[w ^ 2][0][lane]);
    const int q_off = q_offset_of(a.p, b);
    const int ds_lane = w * 1024 + lane * 8;     // this lane's place inside a step of dS in memory (bf16 elements)

    for (int g = 0; g < a.G; ++g) {
        const int hq = hkv * a.G + g;
        const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NC + col;
        const int n_full = a.full_q_num[line], n_part = a.q_num[line];
        const int32_t* full_idx = a.full_q_idx + line * a.NR;
        const int32_t* part_idx = a.q_idx + line * a.NR;
        const int H_all = (n_full + n_part) * sub;  // steps
        if (H_all == 0) continue;
        // dS to memory: where step u of this column's walk goes is ds_col + (pos * sub_k * sub + sidx) * 4096
        // for u = pos * sub + sidx (everything that does not change with u folded into ds_col, so that a
        // step pays a handful of scalar instructions); pos is clamped to the capacity
        bf16* ds_col = nullptr;
        int ds_pos_max = 0;
        if (a.ds_store) {
            const int slot0 = min(max(ldc(a.ds_colbase + line), 0), (int)a.ds_blocks - 1);
            ds_col = a.ds_store + ds_chunk(a, ds_rep(a, b, hq), slot0, key_tile, 0) * 4096 + ds_lane;
            ds_pos_max = (int)a.ds_blocks - 1 - slot0;
        }
        const i32x4 q_rsrc = make_rsrc(a.Q + b * a.q_sb + hq * a.q_sh, q_bytes);
        const i32x4 do_rsrc = make_rsrc(a.dO + b * a.do_sb + hq * a.do_sh, do_bytes);
        // waves 0, 2 fetch the rc row, waves 1, 3 the -delta row (the duplicates write the same values)
        const i32x4 row_rsrc =
            make_rsrc(((w & 1) ? a.delta : a.lse2) + ((int64_t)b * a.Hq + hq) * a.q_len, (uint32_t)a.q_len * 4u);
        const Score smod(a.p, hq, a.scale, lds_addr(s_rel));
        // (the previous head's last step ended with a barrier: nobody reads its row any more; the
        // barrier behind the first segment's walk makes this one visible)
        smod.fill_table(tid, 256);

        // The merged list (FULL blocks, then PARTIAL ones) is walked from its END: every workgroup of
        // a head then spends most of its time descending from the last row block, so the workgroups
        // that run side by side on an XCD ask its L2 for the same Q / dO tiles at about the same
        // time.  The walk is laid out in LDS first, kListMax steps at a time -- one entry per step:
        // first query row | 1 if the block is PARTIAL -- so that the main loop finds the next row
        // offset with one LDS read issued a step ahead.
        for (int seg0 = 0; seg0 < H_all; seg0 += kListMax) {
            const int H = min(kListMax, H_all - seg0);
            for (int i = tid; i < H; i += 256) {
                const int u = H_all - 1 - (seg0 + i), pos = u / sub, sidx = u - pos * sub;
                const int blk = pos < n_full ? full_idx[pos] : part_idx[pos - n_full];
                s_steps[i] = (blk * a.Bq + sidx * TQ) | (pos >= n_full ? 1 : 0);
                // loads are issued for one step past the end as well (into the free ring slot,
                // never read): it repeats the last step's rows
                if (i == H - 1) s_steps[H] = s_steps[i];
            }
            __syncthreads();
            int ld_v = 0;                           // step whose loads are issued next
            int u_step = H_all - 1 - seg0;          // position of the current step in the column's walk (counts down)
            int e_next = s_steps[0];
            int q0_of[2];                           // first query row of the step in each ring slot,
            bool part_of[2];                        // and whether its block is PARTIAL

            int ld_q0 = 0;                          // first row of the step being loaded
            constexpr int kLoads = 2 * Loader::NI + 1;      // load instructions per wave and step
            auto load_begin = [&](auto slot_tag) {
                constexpr int SLOT = decltype(slot_tag)::value;
                const int e = __builtin_amdgcn_readfirstlane(e_next);
                ld_q0 = e & ~1;
                q0_of[SLOT] = ld_q0;
                part_of[SLOT] = e & 1;
                e_next = s_steps[++ld_v];
            };
            // piece P of the loads of a step: NI for the Q tile, NI for the dO tile, one row of scalars
            auto load_piece = [&](auto slot_tag, auto piece_tag) {
                constexpr int SLOT = decltype(slot_tag)::value, P = decltype(piece_tag)::value;
                if constexpr (P < Loader::NI)
                    q_loader.template start_one<P>(q_rsrc, ring + SLOT * 2 * (TILE * 2), ld_q0 * q_row_bytes);
                else if constexpr (P < 2 * Loader::NI)
                    do_loader.template start_one<P - Loader::NI>(do_rsrc, ring + (SLOT * 2 + 1) * (TILE * 2),
                                                                 ld_q0 * do_row_bytes);
                else
                    dma_dword(row_rsrc, wave_row + SLOT * 2 * TQ * 4, lane * 4, ld_q0 * 4);
            };
            auto load_step = [&](auto slot_tag) {   // all at once (prologue)
                load_begin(slot_tag);
                static_for<0, kLoads>([&](auto piece_tag) { load_piece(slot_tag, piece_tag); });
            };
            // this lane's 16 row scalars of a step: rows 8 rg + 4 half + {0..3} of the wave's 32
            auto read_rows = [&](int slot, int which, f32x4 (&out)[4]) {
#pragma unroll
                for (int rg = 0; rg < 4; ++rg)
                    out[rg] = *(const __attribute__((address_space(3))) f32x4*)(uintptr_t)(
                        row_lds + (uint32_t)((slot * 2 + which) * TQ + 8 * rg) * 4);
            };

            load_step(std::integral_constant<int, 0>{});
            wait_vmem();
            __syncthreads();

            // ---- one step; SLOT = v & 1 is compile-time so that every LDS access is "VGPR + immediate"
            auto step = [&](auto slot_tag) {
                constexpr int SLOT = decltype(slot_tag)::value;
                constexpr uint32_t q_cur = SLOT * 2 * (TILE * 2), do_cur = q_cur + TILE * 2;
                // step v+1 (or the dummy past the end); its loads are issued between the MFMAs below: a
                // wave waits on every load instruction until the memory pipe has taken it
                constexpr std::integral_constant<int, SLOT ^ 1> ld_slot{};
                load_begin(ld_slot);
                const bool partial = part_of[SLOT];
                const int q_first = q0_of[SLOT] + 32 * x;

                // scores
                f32x4 nd[4], rcv4[4];
                read_rows(SLOT, 1, nd);
                f32x16 sacc, dpacc;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    sacc[r] = 0.0f;
                    dpacc[r] = nd[r >> 2][r & 3];    // dP - delta comes out of the accumulation
                }
                {   // operand fragments are read PF MFMAs ahead of their use
                    constexpr int NM = 2 * NKS, PF = 4;
                    auto frag = [&](int m) { return row_reader.read((m & 1) ? do_cur : q_cur, 0, m >> 1); };
                    bf16x8 fr[NM];
#pragma unroll
                    for (int m = 0; m < PF; ++m) fr[m] = frag(m);
                    static_for<0, NM>([&](auto m_tag) {
                        constexpr int m = decltype(m_tag)::value;
                        if constexpr (m + PF < NM) fr[m + PF] = frag(m + PF);
                        if (m & 1) dpacc = mfma32(fr[m], vf[m >> 1], dpacc);
                        else sacc = mfma32(fr[m], kf[m >> 1], sacc);
                        static_for<0, kLoads>([&](auto piece_tag) {
                            if constexpr (decltype(piece_tag)::value * NM / kLoads == m) load_piece(ld_slot, piece_tag);
                        });
                        __builtin_amdgcn_sched_barrier(0);
                    });
                }
                read_rows(SLOT, 0, rcv4);
                // relative bias: one value for the whole 32 x 32 block unless it lies near the diagonal
                float rel_uni;
                const bool rel_is_uni = smod.rel_uniform(q_off + q_first - (kv0 + 32 * kb + 31),
                                                         q_off + q_first + 31 - (kv0 + 32 * kb), rel_uni);
                u32x4 pk[2], dsk[2];
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) {
                    float sv[4], rcv[4], gr[4], pe[4], ds[4];
                    // alibi / rel-bias need q - kv = dq0 + 8 (r >> 2) + (r & 3); the soft-cap and the plain score do not
                    using RelPos = typename decltype(smod)::RelPos;
                    constexpr bool kNeedsPos = Score::kAlibi || Score::kRel;
                    const int dq0 = kNeedsPos ? q_off + q_first + 4 * half - kv_lane : 0;
                    const float abase = smod.alibi_base(dq0);
                    auto rel = [&](int r) __attribute__((always_inline)) {
                        return kNeedsPos ? RelPos(dq0, abase, 8 * (r >> 2) + (r & 3)) : RelPos(0);
                    };
                    const RelPos dqk[4] = {rel(4 * c4), rel(4 * c4 + 1), rel(4 * c4 + 2), rel(4 * c4 + 3)};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = 4 * c4 + i;
                        sv[i] = sacc[r];
                        rcv[i] = rcv4[r >> 2][r & 3];
                    }
                    if (rel_is_uni) smod.template p_with_grad4<true>(sv, dqk, rcv, gr, pe, rel_uni);
                    else smod.template p_with_grad4<false>(sv, dqk, rcv, gr, pe);
#pragma unroll
                    for (int i = 0; i < 4; ++i) ds[i] = pe[i] * gr[i] * dpacc[4 * c4 + i];
                    if (partial) {
                        asm volatile("" ::: "memory");   // keep this a (scalar, rarely taken) branch
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            // (rows past q_len hold zeros in Q and dO: whatever the mask says there adds nothing)
                            const MaskRow<MASK> mrow(a.p, b, hq, q_off + min(q_first + crow(4 * c4 + i, half), a.q_len - 1),
                                                     a.kv_len);
                            const bool keep = mrow(kv_lane);
                            pe[i] = keep ? pe[i] : 0.0f;
                            ds[i] = keep ? ds[i] : 0.0f;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int e = 2 * c4 + i;
                        pk[e >> 2][e & 3] = pack_bf16(pe[2 * i], pe[2 * i + 1]);
                        dsk[e >> 2][e & 3] = pack_bf16(ds[2 * i], ds[2 * i + 1]);
                    }
                }
                if (a.ds_store) {       // (wave-uniform) this wave's dS of the step, as it sits in the registers
                    const int u = u_step, pos = u >> sub_shift;
                    bf16* dst = ds_col + (int64_t)(min(pos, ds_pos_max) * (sub_k * sub) + (u - (pos << sub_shift))) * 4096;
                    // (written once, read once by another kernel much later: no reason to keep it in a cache)
                    __builtin_nontemporal_store(dsk[0], (u32x4*)dst);
                    __builtin_nontemporal_store(dsk[1], (u32x4*)(dst + 512));
                }
                --u_step;
                // exchange: keep what this wave's output needs, hand over the other
                u32x4 own[2];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    own[c] = x ? dsk[c] : pk[c];
                    *(__attribute__((address_space(3))) u32x4*)(uintptr_t)(xchg_mine + c * 1024) = x ? pk[c] : dsk[c];
                }
                // outputs: contraction over this wave's own 32 rows (while the exchange settles), then,
                // after the barrier, over its partner's
                constexpr uint32_t slot_off = SLOT * 2 * (TILE * 2);
                constexpr int NMH = 2 * NDB, PF = 4;          // MFMAs per half: [slice c][block db]
                u32x4 theirs[2];
                auto out_half = [&](const TrReader<D>& reader, const u32x4 (&bop)[2]) {
                    auto frag = [&](int m) { return reader.read(slot_off, 16 * (m / NDB), m % NDB); };
                    bf16x8 fr[NMH];
#pragma unroll
                    for (int m = 0; m < PF; ++m) fr[m] = frag(m);
#pragma unroll
                    for (int m = 0; m < NMH; ++m) {
                        if (m + PF < NMH) fr[m + PF] = frag(m + PF);
                        acc[m % NDB] = mfma32(fr[m], __builtin_bit_cast(bf16x8, bop[m / NDB]), acc[m % NDB]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };
                out_half(tr_own, own);
                __syncthreads();
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    theirs[c] = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(xchg_theirs + c * 1024);
                out_half(tr_other, theirs);
                // the next step's tiles must have landed; the two dS stores, the youngest vector-memory
                // operations of the step (the counter retires in issue order), may still be under way
                if (a.ds_store) wait_vmem_but<2>();
                else wait_vmem();
                __syncthreads();
            };

            int v = 0;
            for (; v + 1 < H; v += 2) {
                step(std::integral_constant<int, 0>{});
                step(std::integral_constant<int, 1>{});
            }
            if (v < H) step(std::integral_constant<int, 0>{});
        }
    }

    // ---- dV (x = 0) or dK (x = 1, with the scale and the score_mod's gradient factor), bf16
    {
        const float oscale = x ? a.scale * ScoreMod<SCORE>::grad_scale() : 1.0f;
        bf16* op = x ? a.dK + b * a.dk_sb + hkv * a.dk_sh + (int64_t)kv_lane * a.dk_ss
                     : a.dV + b * a.dv_sb + hkv * a.dv_sh + (int64_t)kv_lane * a.dv_ss;
        if (kv_lane >= a.kv_len) return;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                u32x2 o;
                o[0] = pack_bf16(acc[db][4 * rg] * oscale, acc[db][4 * rg + 1] * oscale);
                o[1] = pack_bf16(acc[db][4 * rg + 2] * oscale, acc[db][4 * rg + 3] * oscale);
                *(u32x2*)(op + db * 32 + 8 * rg + 4 * half) = o;
            }
    }
}

// ------------------------------------------------------------------------------------------
// dQ.  NW waves, each owning 32 query rows of the row of blocks; structure of the forward kernel.
// CAPTURED: the same walk and the same dS, but instead of dQ the kernel sums what the score_mod's
// captured tensors receive: dS * (q_idx - kv_idx) for the ALiBi bias of the head, dS per table entry
// for the relative bias (the factor ScoreMod::grad_scale() is applied by the reduction that follows).
// One partial result per workgroup; the blocks whose every pair falls on the table's last (or first)
// entry are summed in registers, the others entry by entry with LDS atomics.
// M0 RULE: this kernel fills LDS through the LDS-DMA helpers of lds_tiles.h, which write M0 behind the
// compiler's back.  Keep every register array in it indexed by compile-time constants (no movrel /
// s_set_gpr_idx code, which would also use M0) and add no other LDS-DMA or M0-based construct.
template <int D, int NW, uint32_t MASK, uint32_t SCORE, bool CAPTURED = false>
__global__ __launch_bounds__(NW * 64, (bwd_waves_per_simd<D, MASK>())) void bwd_dq_kernel(const BwdArgs a) {
    constexpr int Bq = NW * 32;
    constexpr int TILE = 64 * D;
    __shared__ __attribute__((aligned(1024))) bf16 smem[4 * TILE];   // K(even), K(odd), V(even), V(odd)
    constexpr int kTabAlibi = 1024;                                  // the table has at most 1024 entries
    __shared__ float s_tab[CAPTURED ? kTabAlibi + 1 : 1];            // relative-bias entries, then the ALiBi sum
    __shared__ float s_rel[ScoreMod<SCORE>::kRel ? kRelTableMax : 1]; // relative-bias row of the head (values)

    const int units = a.B * a.Hkv;
    const int id = blockIdx.x, xcd = id & 7, kk = id >> 3;
    const int per_unit = a.G * a.NR;
    const int unit = (kk / per_unit) * 8 + xcd;
    if (unit >= units) return;
    const int rem = kk % per_unit;
    const int g = rem % a.G;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv, hq = hkv * a.G + g;
    const int64_t plane = (int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0);
    const int row = a.kv_order ? min(max(ldc(a.kv_order + plane * a.NR + rem / a.G), 0), a.NR - 1) : a.NR - 1 - rem / a.G;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q_row = row * Bq + w * 32 + l32;

    const int64_t line = ((int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0)) * a.NR + row;
    const int n_full = ldc(a.full_kv_num + line), n_part = ldc(a.kv_num + line);
    const int sub = a.Bk / 64;
    const int T = (n_full + n_part) * sub;

    bf16* dq_ptr = a.dQ + b * a.dq_sb + hq * a.dq_sh + (int64_t)q_row * a.dq_ss;
    // rows past q_len are computed on a copy of the last real row and never stored
    const bool real_row = q_row < a.q_len;
    const int q_ld = min(q_row, a.q_len - 1);
    const int64_t cap_slot = ((int64_t)b * a.Hq + hq) * a.NR + row;
    if (T == 0) {
        if constexpr (CAPTURED) {
            if constexpr (ScoreMod<SCORE>::kRel)
                for (int i = tid; i < a.p.rel_len; i += NW * 64) a.cap_rel[cap_slot * a.p.rel_len + i] = 0.0f;
            if constexpr (ScoreMod<SCORE>::kAlibi)
                if (tid == 0) a.cap_alibi[cap_slot] = 0.0f;
        } else if (real_row) {
            for (int d0 = half * 8; d0 < D; d0 += 16) *(u32x4*)(dq_ptr + d0) = u32x4{0, 0, 0, 0};
        }
        return;
    }
    if constexpr (CAPTURED)
        for (int i = tid; i <= kTabAlibi; i += NW * 64) s_tab[i] = 0.0f;   // before the first barrier below

    bf16x8 qf[D / 16], dof[D / 16];
    {
        const bf16* qp = a.Q + b * a.q_sb + hq * a.q_sh + (int64_t)q_ld * a.q_ss + half * 8;
        const bf16* dp = a.dO + b * a.do_sb + hq * a.do_sh + (int64_t)q_ld * a.do_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            qf[ks] = *(const bf16x8*)(qp + ks * 16);
            dof[ks] = *(const bf16x8*)(dp + ks * 16);
        }
    }
    const int64_t rowi = ((int64_t)b * a.Hq + hq) * a.q_len + q_ld;
    const float lse2 = a.lse2[rowi], neg_delta = a.delta[rowi];
    const i32x4 k_rsrc = make_rsrc(a.K + b * a.k_sb + hkv * a.k_sh, (uint32_t)((a.kv_len - 1) * a.k_ss + D) * 2u);
    const i32x4 v_rsrc = make_rsrc(a.V + b * a.v_sb + hkv * a.v_sh, (uint32_t)((a.kv_len - 1) * a.v_ss + D) * 2u);
    const int k_row_bytes = (int)a.k_ss * 2, v_row_bytes = (int)a.v_ss * 2;
    const ScoreMod<SCORE, true> smod(a.p, hq, a.scale, lds_addr(s_rel));
    smod.fill_table(tid, NW * 64);                  // visible after the prologue's barrier
    const int q_pos = q_ld + q_offset_of(a.p, b);   // as the mods see it
    const MaskRow<MASK> mrow(a.p, b, hq, q_pos, a.kv_len);

    TileWalk<> walk(a.full_kv_idx + line * a.NC, a.kv_idx + line * a.NC, n_full, n_part, sub, a.Bk);
    const WaveTileLoader<D, NW> k_loader(a.k_ss, w, lane), v_loader(a.v_ss, w, lane);
    auto load_tiles = [&](int buf, int kv0) {
        k_loader.start(k_rsrc, lds_addr(smem) + buf * (TILE * 2), kv0 * k_row_bytes);
        v_loader.start(v_rsrc, lds_addr(smem) + (2 + buf) * (TILE * 2), kv0 * v_row_bytes);
    };
    const RowReader<D> row_reader(l32, half, lds_addr(smem));
    const TrReader<D> tr_reader(lane, lds_addr(smem));
    // the delta kernel stored the row constant; a row past q_len must add nothing to the sums
    const float rc = (CAPTURED && !real_row) ? -INFINITY : lse2;
    const int q_wave_min = row * Bq + w * 32 + q_offset_of(a.p, b);   // smallest q_idx of this wave's rows
    float g_alibi = 0.0f, g_hi = 0.0f, g_lo = 0.0f;

    f32x16 dq[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.0f;

    bool part_next = false;
    int kv0 = walk.next(part_next);
    load_tiles(0, kv0);
    wait_vmem();
    __syncthreads();

    // One tile on buffer BUF (compile-time, so that every LDS read is "VGPR + immediate").
    auto step = [&](int t, auto buf_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int kv0_cur = kv0;
        const bool partial = part_next;
        int tile_docs = 0;          // document ids of this tile's keys: one coalesced read, used after the MFMAs
        if constexpr (MaskRow<MASK>::kUsesDoc) {
            if (partial) tile_docs = MaskRow<MASK>::tile_docs(a.p, b, kv0_cur, a.kv_len - 1, lane);
        }
        // K(t+1), V(t+1) go to buffer BUF ^ 1, last read in step t-1.  Their loads are issued piece by
        // piece between the first MFMAs below: a wave waits on every load instruction until the
        // memory pipe has taken it.
        const bool ld = t + 1 < T;
        if (ld) kv0 = walk.next(part_next);
        constexpr uint32_t kt = BUF * (TILE * 2), vt = (2 + BUF) * (TILE * 2);
        using L = WaveTileLoader<D, NW>;
        constexpr int NKS = D / 16, NDB = D / 32, PF = 4;

        static_for<0, 2>([&](auto kvb_tag) {
            constexpr int kvb = decltype(kvb_tag)::value;
            // S^T = K Q^T and dP^T = V dO^T for 32 keys; operand fragments read PF MFMAs ahead
            f32x16 sacc, dpacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sacc[r] = 0.0f;
                dpacc[r] = neg_delta;        // dP - delta comes out of the accumulation
            }
            {
                constexpr int NM = 2 * NKS, NP = 2 * L::NI;
                auto frag = [&](int m) { return row_reader.read((m & 1) ? vt : kt, kvb * 32, m >> 1); };
                bf16x8 fr[NM];
#pragma unroll
                for (int m = 0; m < PF; ++m) fr[m] = frag(m);
                static_for<0, NM>([&](auto m_tag) {
                    constexpr int m = decltype(m_tag)::value;
                    if constexpr (m + PF < NM) fr[m + PF] = frag(m + PF);
                    if (m & 1) dpacc = mfma32(fr[m], dof[m >> 1], dpacc);
                    else sacc = mfma32(fr[m], qf[m >> 1], sacc);
                    if constexpr (kvb == 0) {
                        static_for<0, NP>([&](auto p_tag) {
                            constexpr int p = decltype(p_tag)::value;
                            if constexpr (p * NM / NP == m) {
                                if (ld) {
                                    if constexpr (p < L::NI)
                                        k_loader.template start_one<p>(k_rsrc, lds_addr(smem) + (BUF ^ 1) * (TILE * 2),
                                                                       kv0 * k_row_bytes);
                                    else
                                        v_loader.template start_one<p - L::NI>(
                                            v_rsrc, lds_addr(smem) + (2 + (BUF ^ 1)) * (TILE * 2), kv0 * v_row_bytes);
                                }
                            }
                        });
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            }
            // q_idx - kv_idx of element r is dq0 - 8 (r >> 2) - (r & 3)
            const int dq0 = q_pos - (kv0_cur + kvb * 32 + 4 * half);
            const float abase = smod.alibi_base(dq0);
            float rel_uni;
            const int kvs_blk = kv0_cur + kvb * 32;
            const bool rel_is_uni = smod.rel_uniform(q_wave_min - (kvs_blk + 31), q_wave_min + 31 - kvs_blk, rel_uni);
            auto rel = [&](int r) __attribute__((always_inline)) {
                return typename decltype(smod)::RelPos(dq0, abase, -(8 * (r >> 2) + (r & 3)));
            };
            if (rel_is_uni) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float gr;
                    const float pe = smod.template p_with_grad<true>(sacc[r], rel(r), rc, gr, rel_uni);
                    dpacc[r] = pe * gr * dpacc[r];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float gr;
                    const float pe = smod.template p_with_grad<false>(sacc[r], rel(r), rc, gr);
                    dpacc[r] = pe * gr * dpacc[r];
                }
            }
            if (partial) {
                asm volatile("" ::: "memory");   // keep this a branch
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int off = kvb * 32 + crow(r, half);
                    bool keep;
                    if constexpr (MaskRow<MASK>::kUsesDoc) keep = mrow.eval(kv0_cur + off, MaskRow<MASK>::doc_at(tile_docs, off));
                    else keep = mrow(kv0_cur + off);
                    dpacc[r] = keep ? dpacc[r] : 0.0f;
                }
            }
            if constexpr (CAPTURED) {
                const int kvs = kv0_cur + kvb * 32;
                if constexpr (ScoreMod<SCORE>::kAlibi) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        g_alibi = __builtin_fmaf(dpacc[r], (float)(q_pos - (kvs + crow(r, half))), g_alibi);
                }
                if constexpr (ScoreMod<SCORE>::kRel) {
                    if (q_wave_min - (kvs + 31) >= smod.rel_max) {          // every pair on the last entry
#pragma unroll
                        for (int r = 0; r < 16; ++r) g_hi += dpacc[r];
                    } else if (q_wave_min + 31 <= kvs) {                     // every pair on the first entry
#pragma unroll
                        for (int r = 0; r < 16; ++r) g_lo += dpacc[r];
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dqk = q_pos - (kvs + crow(r, half));
                            atomicAdd(&s_tab[dqk < 0 ? 0 : (dqk > smod.rel_max ? smod.rel_max : dqk)], dpacc[r]);
                        }
                    }
                }
                return;
            }
            // dQ^T += K^T dS^T
            u32x4 dsk[2];
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) dsk[c][jj] = pack_bf16(dpacc[8 * c + 2 * jj], dpacc[8 * c + 2 * jj + 1]);
            {
                constexpr int NM = 2 * NDB;              // [slice c][block db]
                auto frag = [&](int m) { return tr_reader.read(kt, kvb * 32 + 16 * (m / NDB), m % NDB); };
                bf16x8 fr[NM];
#pragma unroll
                for (int m = 0; m < PF; ++m) fr[m] = frag(m);
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    if (m + PF < NM) fr[m + PF] = frag(m + PF);
                    dq[m % NDB] = mfma32(fr[m], __builtin_bit_cast(bf16x8, dsk[m / NDB]), dq[m % NDB]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        });
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

    if constexpr (CAPTURED) {
        auto wave_sum = [](float v) {
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            return v;
        };
        if constexpr (ScoreMod<SCORE>::kAlibi) {
            const float g = wave_sum(g_alibi);
            if (lane == 0) atomicAdd(&s_tab[kTabAlibi], g);
        }
        if constexpr (ScoreMod<SCORE>::kRel) {
            const float hi = wave_sum(g_hi), lo = wave_sum(g_lo);
            if (lane == 0) {
                atomicAdd(&s_tab[smod.rel_max], hi);
                atomicAdd(&s_tab[0], lo);
            }
        }
        __syncthreads();
        if constexpr (ScoreMod<SCORE>::kRel)
            for (int i = tid; i < a.p.rel_len; i += NW * 64) a.cap_rel[cap_slot * a.p.rel_len + i] = s_tab[i];
        if constexpr (ScoreMod<SCORE>::kAlibi)
            if (tid == 0) a.cap_alibi[cap_slot] = s_tab[kTabAlibi];
        return;
    }
    const float qscale = a.scale * ScoreMod<SCORE>::grad_scale();
    if (!real_row) return;
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

constexpr uint32_t kBwdStageCaptured = 8u;   // internal: the captured-tensor sums instead of dQ

template <uint32_t MASK, uint32_t SCORE>
int launch_bwd_variant(const BwdArgs& a, int D, uint32_t stages, hipStream_t st) {
    const int units = a.B * a.Hkv;
    const unsigned grid_kv = (unsigned)(((units + 7) / 8) * 8 * (a.NC * (a.Bk / 64)));
    const unsigned grid_q = (unsigned)(((units + 7) / 8) * 8 * a.G * a.NR);
    const bool kv = stages & FLEXATTN_BWD_DKDV, q = stages & FLEXATTN_BWD_DQ;
    if (stages & FLEXATTN_BWD_DELTA) {
        const size_t rows = (size_t)a.B * a.Hq * a.q_len;
        if (D == 128) hipLaunchKernelGGL((bwd_delta_kernel<128, SCORE>), dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, a);
        else hipLaunchKernelGGL((bwd_delta_kernel<64, SCORE>), dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, st, a);
    }
    if (D == 128) {
        if (kv) hipLaunchKernelGGL((bwd_dkdv_kernel<128, MASK, SCORE>), dim3(grid_kv), dim3(256), 0, st, a);
        if (q && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<128, 4, MASK, SCORE>), dim3(grid_q), dim3(256), 0, st, a);
        if (q && a.Bq == 64) hipLaunchKernelGGL((bwd_dq_kernel<128, 2, MASK, SCORE>), dim3(grid_q), dim3(128), 0, st, a);
    } else {
        if (kv) hipLaunchKernelGGL((bwd_dkdv_kernel<64, MASK, SCORE>), dim3(grid_kv), dim3(256), 0, st, a);
        if (q && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<64, 4, MASK, SCORE>), dim3(grid_q), dim3(256), 0, st, a);
        if (q && a.Bq == 64) hipLaunchKernelGGL((bwd_dq_kernel<64, 2, MASK, SCORE>), dim3(grid_q), dim3(128), 0, st, a);
    }
    if (stages & kBwdStageCaptured) {
        if constexpr ((SCORE & (FLEXATTN_SCORE_ALIBI | FLEXATTN_SCORE_REL_BIAS)) != 0) {
            if (D == 128 && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<128, 4, MASK, SCORE, true>), dim3(grid_q), dim3(256), 0, st, a);
            else if (D == 128) hipLaunchKernelGGL((bwd_dq_kernel<128, 2, MASK, SCORE, true>), dim3(grid_q), dim3(128), 0, st, a);
            else if (a.Bq == 128) hipLaunchKernelGGL((bwd_dq_kernel<64, 4, MASK, SCORE, true>), dim3(grid_q), dim3(256), 0, st, a);
            else hipLaunchKernelGGL((bwd_dq_kernel<64, 2, MASK, SCORE, true>), dim3(grid_q), dim3(128), 0, st, a);
        } else {
            return FLEXATTN_ERR_UNSUPPORTED;     // this score_mod captures no tensor
        }
    }
    return FLEXATTN_OK;
}

}  // namespace flexattn
