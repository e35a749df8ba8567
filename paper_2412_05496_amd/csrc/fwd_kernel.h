// FlexAttention forward kernel for gfx950 (paper Eq. 1; forward template of section 4.1; block
// skipping, full/partial split and indirect KV-block access of section 4.2; the KV prefetch of
// the "Data Prefetching Pipeline" paragraph is the two-deep asynchronous LDS pipeline below).
//
// One workgroup owns one row of BlockMask blocks (Bq = NW * 32 query rows of one (b, hq)); each
// wave owns 32 of those rows.  The score tile is computed TRANSPOSED, S^T = K Q^T, so that in the
// MFMA result layout every lane holds scores of ONE query (column l % 32) and 16 keys per 32-key
// block in its registers: the row max / row sum of the online softmax are in-register reductions
// plus one exchange between the two halves of the wave, and P^T is already laid out as the B
// operand of O^T += V^T P^T.  K and V tiles go from global memory straight into LDS (LDS-DMA buffer
// loads, issued one at a time between the MFMAs of the next score tile); K rows are
// the A operand of K Q^T as they are, V^T fragments come out of the row-major V tile through the
// transposing LDS read.  Q lives in registers for the whole kernel.
//
// Software pipeline, one barrier per tile: while the VALU works on the softmax of tile t, the
// MFMA unit computes S^T of tile t+1; K(t+2) and V(t+1) are in flight from HBM/L2 meanwhile.
#pragma once

#include <type_traits>

#include "flex_common.h"
#include "lds_tiles.h"

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
    const int32_t* kv_order;   // nullable: rows of blocks, longest first
    float scale;
    flexattn_mod_params p;
    // paged K/V (section 5.1): K, V point at the pools, k_sb = v_sb = 0, k_sh = v_sh = page_size * D,
    // k_ss = v_ss = D; page p starts page_stride elements after page p - 1; the physical block of
    // every BlockMask entry stands at the same place in phys_kv_idx / phys_full_idx
    const int32_t* phys_kv_idx;
    const int32_t* phys_full_idx;
    int64_t page_stride;
    int n_pool_pages;
};

constexpr int kTileKV = 64;   // keys per kernel tile

// BOUNDED: the score_mod ends in a soft-cap small enough that the cap itself serves as the fixed
// softmax maximum (see ScoreMod::bounded); chosen by the host from the cap value.
// PAGED: the tiles of K and V are fetched from a paged pool through the converted block lists;
// the mods keep seeing the logical key index.
// M0 RULE: this kernel fills LDS through the LDS-DMA helpers of lds_tiles.h, which write M0 behind the
// compiler's back.  Keep every register array in it indexed by compile-time constants (no movrel /
// s_set_gpr_idx code, which would also use M0) and add no other LDS-DMA or M0-based construct.
template <int D, int NW, uint32_t MASK, uint32_t SCORE, bool BOUNDED, bool PAGED = false>
__global__ __launch_bounds__(NW * 64, (waves_per_simd<D, MASK, SCORE>())) void fwd_kernel(const FwdArgs a) {
    constexpr int Bq = NW * 32;
    constexpr int TILE = kTileKV * D;              // elements per LDS tile

    __shared__ __attribute__((aligned(1024))) bf16 smem[4 * TILE];   // K(even), K(odd), V(even), V(odd)
    using Score = ScoreMod<SCORE, true>;
    __shared__ float s_rel[Score::kRel ? kRelTableMax : 1];           // relative-bias row of the head

    // ---- workgroup -> (b, hkv, g, row of blocks).  Consecutive workgroup ids go to the 8 XCDs in
    // turn; all rows and all G query heads of one (b, hkv) are sent to the same XCD so that its K/V
    // stay in that XCD's L2.  Rows are taken longest first (the BlockMask's work order), or
    // last-first without one (causal-like masks: longest first).
    const int units = a.B * a.Hkv;
    const int id = blockIdx.x;
    const int xcd = id & 7, k = id >> 3;
    const int per_unit = a.G * a.NR;
    const int unit = (k / per_unit) * 8 + xcd;
    if (unit >= units) return;
    const int rem = k % per_unit;
    const int g = rem % a.G;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv, hq = hkv * a.G + g;
    const int64_t plane = (int64_t)(a.bm_Bm > 1 ? b : 0) * a.bm_Hm + (a.bm_Hm > 1 ? hq : 0);
    // (an order array that is no permutation gives wrong rows; clamped so that it cannot leave the arrays)
    const int row = a.kv_order ? min(max(ldc(a.kv_order + plane * a.NR + rem / a.G), 0), a.NR - 1) : a.NR - 1 - rem / a.G;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q_row = row * Bq + w * 32 + l32;

    const int64_t line = plane * a.NR + row;
    const int n_full = ldc(a.full_num + line), n_part = ldc(a.kv_num + line);
    const int T = (n_full + n_part) * a.sub;

    bf16* o_ptr = a.O + b * a.o_sb + hq * a.o_sh + (int64_t)q_row * a.o_ss;
    float* lse_ptr = a.LSE + ((int64_t)b * a.Hq + hq) * a.q_len + q_row;
    // rows past q_len (last block of a length that is no multiple of Bq) are computed on a copy of
    // the last real row and never stored
    const bool real_row = q_row < a.q_len;
    const int q_ld = min(q_row, a.q_len - 1);
    if (T == 0) {   // every key of these rows is masked
        if (real_row) {
            for (int d0 = half * 8; d0 < D; d0 += 16) *(u32x4*)(o_ptr + d0) = u32x4{0, 0, 0, 0};
            if (half == 0) *lse_ptr = -INFINITY;
        }
        return;
    }

    // Q fragments: B operand of K Q^T, column q_row, k-slots d = 16 ks + 8 half + [0, 8)
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.Q + b * a.q_sb + hq * a.q_sh + (int64_t)q_ld * a.q_ss + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *(const bf16x8*)(qp + ks * 16);
    }
    const bf16* k_head = a.K + b * a.k_sb + hkv * a.k_sh;
    const bf16* v_head = a.V + b * a.v_sb + hkv * a.v_sh;
    const i32x4 k_rsrc = make_rsrc(k_head, (uint32_t)((a.kv_len - 1) * a.k_ss + D) * 2u);
    const i32x4 v_rsrc = make_rsrc(v_head, (uint32_t)((a.kv_len - 1) * a.v_ss + D) * 2u);
    const int k_row_bytes = (int)a.k_ss * 2, v_row_bytes = (int)a.v_ss * 2;
    // Where the 64 rows of a tile come from: a buffer descriptor and the byte offset of the first
    // row in it.  Contiguous K/V: one descriptor per head, the tile chosen by the offset.  PAGED: a
    // descriptor of exactly the tile, based at row `row` of pool page `page` (clamped to the pool,
    // so that a wrong page table reads wrong rows and never faults).
    auto tile_src = [&](const bf16* head, i32x4 whole, int row_bytes, int kv0, int page, int row, i32x4& rsrc,
                        int& soff) __attribute__((always_inline)) {
        if constexpr (PAGED) {
            const int pg = min(max(page, 0), a.n_pool_pages - 1);
            rsrc = make_rsrc(head + (int64_t)pg * a.page_stride + row * D, (uint32_t)(kTileKV * D * 2));
            soff = 0;
        } else {
            rsrc = whole;
            soff = kv0 * row_bytes;
        }
    };

    const Score smod(a.p, hq, a.scale, lds_addr(s_rel));
    smod.fill_table(tid, NW * 64);                  // visible after the prologue's barrier
    const int q_pos = q_ld + q_offset_of(a.p, b);   // as the mods see it
    const int q_wave_min = row * Bq + w * 32 + q_offset_of(a.p, b);   // the wave's rows: q_wave_min .. +31
    const MaskRow<MASK> mrow(a.p, b, hq, q_pos, a.kv_len);
    const float inv_neg2c = smod.capl2 > 0.0f ? -0.5f / smod.capl2 : 0.0f;   // 1 / (-2 cap log2 e)

    // first key and PARTIAL flag of tiles t, t+1, t+2 (the walk is always two tiles ahead)
    TileWalk<PAGED> walk(a.full_idx + line * a.NC, a.kv_idx + line * a.NC, n_full, n_part, a.sub, a.Bk,
                         PAGED ? a.phys_full_idx + line * a.NC : nullptr, PAGED ? a.phys_kv_idx + line * a.NC : nullptr);
    int kv_t = 0, kv_t1 = 0, kv_t2 = 0;
    bool part_t = false, part_t1 = false, part_t2 = false;
    int pg_t = 0, pg_t1 = 0, pg_t2 = 0, pr_t = 0, pr_t1 = 0, pr_t2 = 0;   // PAGED: page, row in page
    const uint32_t smem_bytes = lds_addr(smem);
    const WaveTileLoader<D, NW> k_loader(a.k_ss, w, lane), v_loader(a.v_ss, w, lane);
    // buf = tile index & 1
    auto load_k = [&](int buf, int kv0, int page, int row) {
        i32x4 rsrc;
        int soff;
        tile_src(k_head, k_rsrc, k_row_bytes, kv0, page, row, rsrc, soff);
        k_loader.start(rsrc, smem_bytes + buf * (TILE * 2), soff);
    };
    auto load_v = [&](int buf, int kv0, int page, int row) {
        i32x4 rsrc;
        int soff;
        tile_src(v_head, v_rsrc, v_row_bytes, kv0, page, row, rsrc, soff);
        v_loader.start(rsrc, smem_bytes + (2 + buf) * (TILE * 2), soff);
    };
    const RowReader<D> k_reader(l32, half);
    const TrReader<D> v_reader(lane);

    // S^T = K Q^T for the two 32-key blocks of the K tile in buffer BUF (compile-time);
    // between(m) runs after the m-th of the 2 D / 16 MFMAs (used to spread out tile loads)
    auto qk = [&](auto buf_tag, f32x16 (&s)[2], auto&& between) {
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr int NKS = D / 16;
        static_for<0, 2 * NKS>([&](auto m_tag) {
            constexpr int m = decltype(m_tag)::value, kvb = m / NKS, ks = m % NKS;
            if constexpr (ks == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kvb][r] = 0.0f;
            }
            s[kvb] = mfma32(k_reader.read(smem_bytes + BUF * (TILE * 2), kvb * 32, ks), qf[ks], s[kvb]);
            between(m_tag);
        });
    };

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.0f;
    // base-2 running max and this lane's part of the running sum; with a bounded soft-cap the
    // maximum is fixed at the cap from the start
    float m_run = BOUNDED ? smod.capl2 : -INFINITY, l_run = 0.0f;
    float m_use = 0.0f;     // the maximum the exponentials subtract: m_run, or 0 while the row has seen no key
    float m_thr = -INFINITY; // what a block's largest shifted score must exceed for the maximum to move

    // score_mod, mask_mod (partial blocks only) and softmax of one 32-key block whose first key is
    // kvs: s -> P^T as two bf16 fragments.  The mask is a separate, rarely taken pass (kept a real
    // branch) so that the common path is one straight run of VALU work next to the MFMAs around it.
    int tile_docs = 0, tile_first = 0;   // document ids of the current tile's keys (partial tiles of document masks)
    auto keep = [&](int kv) __attribute__((always_inline)) {
        if constexpr (MaskRow<MASK>::kUsesDoc) return mrow.eval(kv, MaskRow<MASK>::doc_at(tile_docs, kv - tile_first));
        else return mrow(kv);
    };
    auto softmax = [&](f32x16& s, int kvs, bool partial, bf16x8 (&pf)[2]) {
        // q_idx - kv_idx of element r is dq0 - 8 (r >> 2) - (r & 3)
        const int dq0 = q_pos - kvs - 4 * half;
        const float abase = smod.alibi_base(dq0);
        auto rel = [&](int r) __attribute__((always_inline)) {
            return typename Score::RelPos(dq0, abase, -(8 * (r >> 2) + (r & 3)));
        };
        // relative bias: one value for the whole block unless it lies near the diagonal
        float rel_uni;
        const bool rel_is_uni = smod.rel_uniform(q_wave_min - (kvs + 31), q_wave_min + 31 - kvs, rel_uni);
        if constexpr (BOUNDED) {
            // p = 2^(x - cap log2 e) = 2^(-2 cap log2 e * r), r = 1 / (1 + e): no maximum to track
            auto prob = [&](float e) __attribute__((always_inline)) {
                // -2 cap log2e / (1 + e) as ONE reciprocal: rcp((1 + e) / (-2 cap log2e))
                return fast_exp2(fast_rcp(__builtin_fmaf(e, inv_neg2c, inv_neg2c)));
            };
            if (rel_is_uni) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = prob(fast_exp2(smod.template pre<true>(s[r], rel(r), rel_uni)));
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = prob(fast_exp2(smod.template pre<false>(s[r], rel(r))));
            }
            if (partial) {
                asm volatile("" ::: "memory");   // keep this a branch, not 16 selects on every tile
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = keep(kvs + crow(r, half)) ? s[r] : 0.0f;
            }
        } else {
            // Online softmax.  The running maximum only has to keep exp2(s - m) in range, so it follows
            // the scores lazily: a row keeps its maximum until a block exceeds it by more than kLazyMax
            // (P then reaches 2^kLazyMax at most, the row sum as much more; O / l and LSE = m + log2 l
            // come out the same).  The score_mod therefore subtracts the CURRENT maximum on its way (folded
            // into its multiply-adds), and only when some row of the wave moves its maximum -- rare after a
            // row's first blocks -- are the scores shifted again and O^T and l rescaled.
            constexpr float kLazyMax = 8.0f;
            const float shift = -m_use;
            if (rel_is_uni) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = smod.template apply_shifted<true>(s[r], rel(r), rel_uni, shift);
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = smod.template apply_shifted<false>(s[r], rel(r), 0.0f, shift);
            }
            if (partial) {
                asm volatile("" ::: "memory");
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = keep(kvs + crow(r, half)) ? s[r] : -INFINITY;
            }
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            mx = fmaxf(mx, swap_halves(mx));
            if (__any(mx > m_thr)) {                 // some row of the wave moves its maximum (by mx)
                const float up = mx > m_thr ? mx : 0.0f;
                // (a row's first keys: nothing to rescale yet, and 2^-mx could overflow)
                const float alpha = m_thr == -INFINITY ? 0.0f : fast_exp2(-up);
                m_use += up;                         // (0 before the row's first key)
                m_run = mx > m_thr ? m_use : m_run;
                m_thr = mx > m_thr ? kLazyMax : m_thr;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] -= up;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = fast_exp2(s[r]);
        }
        // The row sum adds up the bf16-rounded probabilities, the values P V is computed from, two at
        // a time (dot product of a packed pair with (1, 1), fp32 accumulation).
        float psum[2] = {0.0f, 0.0f};
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            u32x4 pk;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                pk[jj] = pack_bf16(s[8 * c + 2 * jj], s[8 * c + 2 * jj + 1]);
                psum[jj & 1] = pair_sum_bf16(pk[jj], psum[jj & 1]);
            }
            pf[c] = __builtin_bit_cast(bf16x8, pk);
        }
        l_run += psum[0] + psum[1];
    };

    // O^T += V^T P^T for the 32-key block kvb (compile-time) of the V tile in buffer BUF
    auto pv = [&](auto buf_tag, int kvb, const bf16x8 (&pf)[2]) {
        constexpr int BUF = decltype(buf_tag)::value;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                oacc[db] = mfma32(v_reader.read(smem_bytes + (2 + BUF) * (TILE * 2), kvb * 32 + 16 * c, db), pf[c], oacc[db]);
    };

    // ---- prologue: K(0), V(0), K(1) in flight; S^T(0)
    kv_t = walk.next(part_t, pg_t, pr_t);
    load_k(0, kv_t, pg_t, pr_t);
    load_v(0, kv_t, pg_t, pr_t);
    if (T > 1) {
        kv_t1 = walk.next(part_t1, pg_t1, pr_t1);
        load_k(1, kv_t1, pg_t1, pr_t1);
    }
    wait_vmem();
    __syncthreads();
    f32x16 s_cur[2], s_next[2];
    qk(std::integral_constant<int, 0>{}, s_cur, [](auto) {});

    // One tile (t & 1 == BUF).  S^T of tile t+1 (MFMA) is issued next to the softmax of tile t (VALU),
    // P V of the first 32 keys next to the softmax of the second 32.
    auto tile_step = [&](int t, auto buf_tag, auto has_next_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
        // Everything this wave asked for has landed; after the barrier so has everyone else's, and
        // nobody still reads K(t) [buffer BUF] or V(t-1) [buffer BUF ^ 1], which are refilled next.
        wait_vmem();
        __syncthreads();
        // K(t+2) and V(t+1) are loaded piece by piece between the MFMAs of S^T(t+1): a wave waits on
        // every load instruction until the memory pipe has taken it, and a burst of them from all
        // waves at once keeps everybody waiting
        const bool ld_k = t + 2 < T;
        if (ld_k) kv_t2 = walk.next(part_t2, pg_t2, pr_t2);
        i32x4 k_src, v_src;
        int k_soff, v_soff;
        tile_src(k_head, k_rsrc, k_row_bytes, kv_t2, pg_t2, pr_t2, k_src, k_soff);
        tile_src(v_head, v_rsrc, v_row_bytes, kv_t1, pg_t1, pr_t1, v_src, v_soff);
        const int kv0 = kv_t;
        const bool partial = part_t;
        if constexpr (MaskRow<MASK>::kUsesDoc) {
            if (partial) {      // one coalesced read, behind the MFMAs that follow
                tile_first = kv0;
                tile_docs = MaskRow<MASK>::tile_docs(a.p, b, kv0, a.kv_len - 1, lane);
            }
        }
        bf16x8 pf[2];
        if constexpr (HAS_NEXT) {
            using L = WaveTileLoader<D, NW>;
            constexpr int NP = 2 * L::NI, NMQ = 2 * (D / 16);
            qk(std::integral_constant<int, BUF ^ 1>{}, s_next, [&](auto m_tag) {
                static_for<0, NP>([&](auto p_tag) {
                    constexpr int p = decltype(p_tag)::value;
                    if constexpr (p * NMQ / NP == decltype(m_tag)::value) {
                        if constexpr (p < L::NI) {
                            if (ld_k) k_loader.template start_one<p>(k_src, smem_bytes + BUF * (TILE * 2), k_soff);
                        } else {
                            v_loader.template start_one<p - L::NI>(v_src, smem_bytes + (2 + (BUF ^ 1)) * (TILE * 2), v_soff);
                        }
                    }
                });
            });
        }
        softmax(s_cur[0], kv0, partial, pf);
        pv(buf_tag, 0, pf);
        softmax(s_cur[1], kv0 + 32, partial, pf);
        pv(buf_tag, 1, pf);
        if constexpr (HAS_NEXT) {
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb) s_cur[kvb] = s_next[kvb];
        }
        kv_t = kv_t1, part_t = part_t1;
        kv_t1 = kv_t2, part_t1 = part_t2;
        if constexpr (PAGED) pg_t1 = pg_t2, pr_t1 = pr_t2;
    };
    {
        const std::integral_constant<int, 0> b0;
        const std::integral_constant<int, 1> b1;
        int t = 0;
        for (; t + 2 < T; t += 2) {
            tile_step(t, b0, std::true_type{});
            tile_step(t + 1, b1, std::true_type{});
        }
        if (T - t == 2) {
            tile_step(t, b0, std::true_type{});
            tile_step(t + 1, b1, std::false_type{});
        } else {
            tile_step(t, b0, std::false_type{});
        }
    }

    // ---- epilogue: O = O^T / l, LSE = ln 2 * (m + log2 l)
    const float l_tot = l_run + swap_halves(l_run);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    if (!real_row) return;
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

template <uint32_t MASK, uint32_t SCORE, bool BOUNDED, bool PAGED>
int launch_fwd_shape(const FwdArgs& a, int D, int Bq, hipStream_t st) {
    const int units = a.B * a.Hkv;
    const unsigned grid = (unsigned)(((units + 7) / 8) * 8 * a.G * a.NR);
#define FLEXATTN_LAUNCH(DD, NW)                                                                            \
    hipLaunchKernelGGL((fwd_kernel<DD, NW, MASK, SCORE, BOUNDED, PAGED>), dim3(grid), dim3(NW * 64), 0, st, a); \
    return FLEXATTN_OK;
    if (D == 128 && Bq == 128) { FLEXATTN_LAUNCH(128, 4) }
    if (D == 128 && Bq == 64) { FLEXATTN_LAUNCH(128, 2) }
    if (D == 64 && Bq == 128) { FLEXATTN_LAUNCH(64, 4) }
    if (D == 64 && Bq == 64) { FLEXATTN_LAUNCH(64, 2) }
#undef FLEXATTN_LAUNCH
    return FLEXATTN_ERR_UNSUPPORTED;
}

template <uint32_t MASK, uint32_t SCORE, bool PAGED = false>
int launch_fwd_variant(const FwdArgs& a, int D, int Bq, hipStream_t st) {
    if constexpr (SCORE & FLEXATTN_SCORE_SOFTCAP) {
        if (2.0f * a.p.softcap * kLog2e <= 100.0f) return launch_fwd_shape<MASK, SCORE, true, PAGED>(a, D, Bq, st);
    }
    return launch_fwd_shape<MASK, SCORE, false, PAGED>(a, D, Bq, st);
}

}  // namespace flexattn
