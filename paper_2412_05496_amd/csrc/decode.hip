// Paged split-KV decode (decoding template of paper section 4.1; page-table indirection fused
// into the KV-block walk as in section 5.1) and the partial-softmax combine.
//
// The path is bound by reading K and V once from HBM.  One WAVE owns one (sequence, KV head,
// KV split): it walks its logical pages, looks each up in the page table and reads K rows straight
// from the pool into the A-operand layout of S^T = K Q^T (each lane: 16-byte pieces of one key
// row), with the G query heads of the group as (zero-padded) columns, so K and V are read once
// per KV head, never once per query head.  V rows are read 16 bytes per lane, four keys at a
// time, transposed through a wave-private LDS tile and used as V^T in O^T += V^T P^T.  No
// workgroup barrier is needed.  Each wave leaves (m, l, O) of its split in the workspace; the
// combine kernel merges the splits of a (sequence, head) with the usual log-sum-exp weights.
#include "flex_common.h"

namespace flexattn {

constexpr int kDecWaves = 4;       // waves (= splits) per workgroup
constexpr int kDecTile = 64;       // keys per inner tile
constexpr int kDecSplit = 512;     // keys per split

struct DecodeArgs {
    const bf16* Q;
    int64_t q_stride_seq;
    const bf16* K_pool;
    const bf16* V_pool;
    const int32_t* page_table;
    int64_t pt_stride;
    const int32_t* ctx_lens;
    int nseq, Hq, Hkv, G, page_size, page_shift, max_splits;
    float scale;
    flexattn_mod_params p;
    float* part_O;    // [nseq, Hq, max_splits, D]
    float* part_ml;   // [nseq, Hq, max_splits, 2]  (running max in base 2, sum)
    bf16* O;
    float* LSE;
};

__device__ __forceinline__ constexpr int dec_vt_pos16(int t) { return 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3); }

template <int D, uint32_t SCORE>
__global__ __launch_bounds__(kDecWaves * 64, 2) void decode_split_kernel(const DecodeArgs a) {
    constexpr int DC = D / 8;
    constexpr int VS = kDecTile + 8;
    constexpr int NVU = (kDecTile / 4) * DC;   // 4-key x 8-dim units per tile
    constexpr int NVT = NVU / 64;              // per lane
    __shared__ __attribute__((aligned(16))) bf16 Vt_all[kDecWaves][D * VS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int b = blockIdx.x / a.Hkv, hkv = blockIdx.x % a.Hkv;
    const int split = blockIdx.y * kDecWaves + wave;
    const int ctx = a.ctx_lens[b];
    const int tok_begin = split * kDecSplit;
    if (tok_begin >= ctx) return;                       // wave-uniform; the kernel has no barriers
    const int tok_end = min(ctx, tok_begin + kDecSplit);
    bf16* Vt = Vt_all[wave];

    const int g_lane = l32;                             // query head of the group held by this lane
    const bool g_ok = g_lane < a.G;
    const int hq = hkv * a.G + (g_ok ? g_lane : 0);
    bf16x8 qf[D / 16];
    {
        const bf16* qp = a.Q + (int64_t)b * a.q_stride_seq + (int64_t)hq * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            u32x4 v = *(const u32x4*)(qp + ks * 16);
            if (!g_ok) v = u32x4{0, 0, 0, 0};
            qf[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }
    const ScoreMod<SCORE> smod(a.p, hq, a.scale);
    const int q_idx = ctx - 1;
    const int32_t* pt = a.page_table + (int64_t)b * a.pt_stride;
    const int page_mask = a.page_size - 1;
    const int64_t slab = (int64_t)a.page_size * D;      // elements per (page, head)

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    for (int tok0 = tok_begin; tok0 < tok_end; tok0 += kDecTile) {
        // ---- gather K rows (A operand of K Q^T) through the page table
        bf16x8 kf[2][D / 16];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
            const int tok = min(tok0 + kvb * 32 + l32, ctx - 1);     // rows past the context re-read the last key
            const int pg = pt[tok >> a.page_shift];
            const bf16* kp = a.K_pool + ((int64_t)pg * a.Hkv + hkv) * slab + (int64_t)(tok & page_mask) * D + half * 8;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) kf[kvb][ks] = *(const bf16x8*)(kp + ks * 16);
        }
        // ---- gather V: each lane takes units of 4 consecutive keys x 8 dims
        u32x4 vreg[NVT][4];
#pragma unroll
        for (int i = 0; i < NVT; ++i) {
            const int u = lane + i * 64, gq = u / DC, cc = u % DC;
            const int tok = min(tok0 + 4 * gq, ((ctx - 1) >> 2) << 2);  // 4-key groups never straddle a page
            const int pg = pt[tok >> a.page_shift];
            const bf16* vp = a.V_pool + ((int64_t)pg * a.Hkv + hkv) * slab + (int64_t)(tok & page_mask) * D + cc * 8;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) vreg[i][r4] = *(const u32x4*)(vp + r4 * D);
        }

        // ---- S^T = K Q^T
        f32x16 sacc[2];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kvb][r] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) sacc[kvb] = mfma32(kf[kvb][ks], qf[ks], sacc[kvb]);
        }

        // ---- V^T into the wave's LDS tile
#pragma unroll
        for (int i = 0; i < NVT; ++i) {
            const int u = lane + i * 64, gq = u / DC, cc = u % DC;
            const int pos = 16 * (gq >> 2) + dec_vt_pos16(4 * (gq & 3));
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                const uint32_t r0 = vreg[i][0][wd], r1 = vreg[i][1][wd], r2 = vreg[i][2][wd], r3 = vreg[i][3][wd];
                u32x2 lo, hi;
                lo[0] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
                lo[1] = __builtin_amdgcn_perm(r3, r2, 0x05040100u);
                hi[0] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
                hi[1] = __builtin_amdgcn_perm(r3, r2, 0x07060302u);
                *(u32x2*)(&Vt[(cc * 8 + 2 * wd) * VS + pos]) = lo;
                *(u32x2*)(&Vt[(cc * 8 + 2 * wd + 1) * VS + pos]) = hi;
            }
        }

        // ---- score_mod, mask kv < ctx_len (only the last tile can hold masked keys), softmax
        const bool ragged = tok0 + kDecTile > tok_end;
        float mx = -INFINITY;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = tok0 + kvb * 32 + crow(r, half);
                float x = smod.apply(sacc[kvb][r], q_idx - kv);
                if (ragged && kv >= tok_end) x = -INFINITY;
                sacc[kvb][r] = x;
                mx = fmaxf(mx, x);
            }
        mx = fmaxf(mx, swap_halves(mx));
        const float m_new = fmaxf(m_run, mx);          // finite: every split holds at least one key
        const float alpha = fast_exp2(m_run - m_new);
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
                    const float p0 = fast_exp2(sacc[kvb][8 * c + 2 * jj] - m_new);
                    const float p1 = fast_exp2(sacc[kvb][8 * c + 2 * jj + 1] - m_new);
                    psum += p0 + p1;
                    pk[jj] = pack_bf16(p0, p1);
                }
                pf[kvb][c] = __builtin_bit_cast(bf16x8, pk);
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;

        // ---- O^T += V^T P^T  (LDS writes above are ordered before these reads within the wave)
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 vf = *(const bf16x8*)(&Vt[(db * 32 + l32) * VS + (kvb * 2 + c) * 16 + half * 8]);
                    oacc[db] = mfma32(vf, pf[kvb][c], oacc[db]);
                }
    }

    const float l_tot = l_run + swap_halves(l_run);
    if (g_ok) {
        const int64_t item = ((int64_t)b * a.Hq + hq) * a.max_splits + split;
        float* po = a.part_O + item * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                f32x4 v = {oacc[db][4 * rg], oacc[db][4 * rg + 1], oacc[db][4 * rg + 2], oacc[db][4 * rg + 3]};
                *(f32x4*)(po + db * 32 + 8 * rg + 4 * half) = v;
            }
        if (half == 0) {
            a.part_ml[item * 2] = m_run;
            a.part_ml[item * 2 + 1] = l_tot;
        }
    }
}

// One wave per (sequence, query head): O = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max m).
template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const DecodeArgs a) {
    const int lane = threadIdx.x;
    const int b = blockIdx.x / a.Hq, hq = blockIdx.x % a.Hq;
    const int ctx = a.ctx_lens[b];
    const int ns = (ctx + kDecSplit - 1) / kDecSplit;
    const int64_t base = ((int64_t)b * a.Hq + hq) * a.max_splits;
    bf16* o = a.O + ((int64_t)b * a.Hq + hq) * D;
    constexpr int PER = D / 64;
    if (ns == 0) {
#pragma unroll
        for (int i = 0; i < PER; ++i) o[lane * PER + i] = (bf16)0.0f;
        if (lane == 0 && a.LSE) a.LSE[(int64_t)b * a.Hq + hq] = -INFINITY;
        return;
    }
    float m = -INFINITY;
    for (int s = 0; s < ns; ++s) m = fmaxf(m, a.part_ml[(base + s) * 2]);
    float L = 0.0f, acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.0f;
    for (int s = 0; s < ns; ++s) {
        const float wgt = fast_exp2(a.part_ml[(base + s) * 2] - m);
        L += wgt * a.part_ml[(base + s) * 2 + 1];
        const float* po = a.part_O + (base + s) * D + lane * PER;
#pragma unroll
        for (int i = 0; i < PER; ++i) acc[i] += wgt * po[i];
    }
    const float inv = 1.0f / L;
#pragma unroll
    for (int i = 0; i < PER; ++i) o[lane * PER + i] = (bf16)(acc[i] * inv);
    if (lane == 0 && a.LSE) a.LSE[(int64_t)b * a.Hq + hq] = (m + fast_log2(L)) * kLn2;
}

static int max_splits_of(const flexattn_decode_dims* d) {
    const long long max_tokens = (long long)d->max_pages * d->page_size;
    return (int)((max_tokens + kDecSplit - 1) / kDecSplit);
}

template <int D>
static int launch_decode(const DecodeArgs& a, uint32_t score_id, hipStream_t st) {
    const dim3 grid((unsigned)(a.nseq * a.Hkv), (unsigned)((a.max_splits + kDecWaves - 1) / kDecWaves));
    switch (score_id) {
#define CASE(S)                                                                                           \
    case S:                                                                                               \
        hipLaunchKernelGGL((decode_split_kernel<D, S>), grid, dim3(kDecWaves * 64), 0, st, a);            \
        break;
        CASE(FLEXATTN_SCORE_IDENTITY)
        CASE(FLEXATTN_SCORE_ALIBI)
        CASE(FLEXATTN_SCORE_SOFTCAP)
        CASE(FLEXATTN_SCORE_REL_BIAS)
#undef CASE
        default: return FLEXATTN_ERR_UNSUPPORTED;
    }
    hipLaunchKernelGGL((decode_combine_kernel<D>), dim3((unsigned)(a.nseq * a.Hq)), dim3(64), 0, st, a);
    return FLEXATTN_OK;
}

}  // namespace flexattn

using namespace flexattn;

static int check_decode_dims(const flexattn_decode_dims* d) {
    if (!d) return FLEXATTN_ERR_INVALID_ARG;
    if (d->nseq <= 0 || d->Hq <= 0 || d->Hkv <= 0 || d->max_pages <= 0 || d->n_pool_pages <= 0)
        return FLEXATTN_ERR_INVALID_ARG;
    if (d->Hq % d->Hkv != 0) return FLEXATTN_ERR_INVALID_ARG;
    if (d->D != 64 && d->D != 128) return FLEXATTN_ERR_UNSUPPORTED;
    if (d->Hq / d->Hkv > 16) return FLEXATTN_ERR_UNSUPPORTED;
    if (d->page_size != 16 && d->page_size != 32 && d->page_size != 64 && d->page_size != 128)
        return FLEXATTN_ERR_UNSUPPORTED;
    return FLEXATTN_OK;
}

extern "C" size_t flexattn_paged_decode_workspace_bytes(const flexattn_decode_dims* d) {
    if (check_decode_dims(d) != FLEXATTN_OK) return 0;
    const size_t items = (size_t)d->nseq * d->Hq * max_splits_of(d);
    return items * ((size_t)d->D + 2) * sizeof(float);
}

extern "C" int flexattn_paged_decode(const flexattn_decode_dims* d, const void* Q, int64_t stride_q_seq,
                                     const void* K_pool, const void* V_pool, const int32_t* page_table,
                                     int64_t pt_stride, const int32_t* ctx_lens, uint32_t score_id, uint32_t mask_id,
                                     const flexattn_mod_params* params, float scale, void* O, float* LSE, void* ws,
                                     size_t ws_bytes, void* stream) {
    int rc = check_decode_dims(d);
    if (rc != FLEXATTN_OK) return rc;
    if (!Q || !K_pool || !V_pool || !page_table || !ctx_lens || !O || !ws) return FLEXATTN_ERR_INVALID_ARG;
    if (pt_stride < d->max_pages || stride_q_seq < (int64_t)d->Hq * d->D || (stride_q_seq % 8) != 0)
        return FLEXATTN_ERR_INVALID_ARG;
    if (((uintptr_t)Q & 15) || ((uintptr_t)K_pool & 15) || ((uintptr_t)V_pool & 15) || ((uintptr_t)ws & 15))
        return FLEXATTN_ERR_INVALID_ARG;
    if (!(scale > 0.0f)) return FLEXATTN_ERR_INVALID_ARG;
    if (mask_id != FLEXATTN_MASK_CTX_LEN) return FLEXATTN_ERR_UNSUPPORTED;
    flexattn_mod_params p = {};
    if (params) p = *params;
    p.ctx_lens = ctx_lens;
    if ((rc = check_mod_params(mask_id, score_id, &p)) != FLEXATTN_OK) return rc;
    if (ws_bytes < flexattn_paged_decode_workspace_bytes(d)) return FLEXATTN_ERR_WORKSPACE;

    DecodeArgs a = {};
    a.Q = (const bf16*)Q; a.q_stride_seq = stride_q_seq;
    a.K_pool = (const bf16*)K_pool; a.V_pool = (const bf16*)V_pool;
    a.page_table = page_table; a.pt_stride = pt_stride; a.ctx_lens = ctx_lens;
    a.nseq = d->nseq; a.Hq = d->Hq; a.Hkv = d->Hkv; a.G = d->Hq / d->Hkv;
    a.page_size = d->page_size;
    a.page_shift = __builtin_ctz((unsigned)d->page_size);
    a.max_splits = max_splits_of(d);
    a.scale = scale; a.p = p;
    const size_t items = (size_t)d->nseq * d->Hq * a.max_splits;
    a.part_O = (float*)ws;
    a.part_ml = (float*)ws + items * d->D;
    a.O = (bf16*)O; a.LSE = LSE;
    rc = d->D == 128 ? launch_decode<128>(a, score_id, (hipStream_t)stream)
                     : launch_decode<64>(a, score_id, (hipStream_t)stream);
    if (rc != FLEXATTN_OK) return rc;
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}
