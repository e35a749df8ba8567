// Paged split-KV decode (decoding template of paper section 4.1; page-table indirection fused
// into the KV-block walk as in section 5.1) and the partial-softmax combine.
//
// The path is bound by reading K and V once from HBM.  One WAVE owns one (sequence, KV head,
// KV split) and never synchronises with another: it walks its logical pages 32 keys at a time,
// looks each key's page up in the page table and pulls the K and V rows straight from the pool into
// its private, XOR-swizzled LDS tiles (global_load_lds_dwordx4: every wave instruction moves 1 KiB
// of whole 256-byte rows, so the page gather is fully coalesced; non-temporal, since a decode step
// reads every K / V row exactly once); the gather of the next tile is
// started as soon as the current tile's operand fragments sit in registers.  S^T = K Q^T takes K rows from
// LDS as the A operand with the G query heads of the group as (zero-padded) columns of the B
// operand, so K and V are read once per KV head, never once per query head; V^T comes out of the
// row-major V tile through the transposing LDS read.  Each wave leaves (m, l, O) of its split in
// the workspace; the combine kernel merges the splits of a (sequence, head) with log-sum-exp weights.
#include <mutex>

#include "flex_common.h"
#include "lds_tiles.h"

// Workspace of flexattn_paged_decode_static(): lives in the library's device image, one copy per
// GPU, for callers that cannot allocate.  In host code this name is only a handle for
// hipGetSymbolAddress(); kernels receive the device address it returns, like any other workspace.
constexpr size_t kStaticScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace flexattn {

constexpr int kDecWaves = 4;       // waves per workgroup (the mapping below assumes 4)
constexpr int kDecTile = 32;       // keys per inner tile
constexpr int kDecSplitMax = 1024; // keys per split: a power of two in [kDecSplitMin, kDecSplitMax],
constexpr int kDecSplitMin = 128;  // chosen by the host so that the launch fills the chip (split_len_of)
constexpr int kDecTargetWaves = 256 * 4;   // one wave per SIMD: finer cuts cost more per-wave start-up than they gain

struct DecodeArgs {
    const bf16* Q;
    int64_t q_stride_seq;
    const bf16* K_pool;
    const bf16* V_pool;
    const int32_t* page_table;
    int64_t pt_stride;
    const int32_t* ctx_lens;
    int nseq, Hq, Hkv, G, page_size, page_shift, max_splits;
    int split_len;       // keys per split
    int max_ctx;         // max_pages * page_size: context lengths are clamped to what the page table can address
    int n_pool_pages;    // page ids are clamped to [0, n_pool_pages)
    int window;          // sliding window (q_idx - kv <= window), -1 if none
    float scale;
    flexattn_mod_params p;
    float* part_O;    // [nseq, Hq, max_splits, D]
    float* part_ml;   // [nseq, Hq, max_splits, 2]  (running max in base 2, sum)
    bf16* O;
    float* LSE;
};

// M0 RULE: this kernel fills LDS through the LDS-DMA helpers of lds_tiles.h, which write M0 behind the
// compiler's back.  Keep every register array in it indexed by compile-time constants (no movrel /
// s_set_gpr_idx code, which would also use M0) and add no other LDS-DMA or M0-based construct.
template <int D, uint32_t SCORE>
__global__ __launch_bounds__(kDecWaves * 64, 2) void decode_split_kernel(const DecodeArgs a) {
    constexpr int DC = D / 8;                  // 16-byte chunks per row
    constexpr int RPI = 64 / DC;               // rows per wave instruction
    constexpr int NI = kDecTile / RPI;         // instructions per tile and tensor
    constexpr int TILE = kDecTile * D;         // elements
    __shared__ __attribute__((aligned(1024))) bf16 smem[kDecWaves * 2 * TILE];   // per wave: K tile, V tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    // workgroup -> consecutive splits of one (sequence, KV head): blockIdx.x walks the (sequence, KV
    // head) units, blockIdx.y the groups of splits, so the splits of a long sequence are spread over the
    // launch.  When a sequence has fewer splits than a workgroup has waves, the spare waves take the
    // following units instead of idling.
    const int spw = a.max_splits >= 4 ? 4 : (a.max_splits >= 2 ? 2 : 1);   // splits per workgroup
    const int upw = kDecWaves / spw;                     // units per workgroup
    const int split = blockIdx.y * spw + wave % spw;
    const int unit = blockIdx.x * upw + wave / spw;
    if (unit >= a.nseq * a.Hkv || split >= a.max_splits) return;
    const int b = unit / a.Hkv, hkv = unit % a.Hkv;
    // A context length beyond what the page table addresses (or a negative one) is clamped, and so is
    // every page id below: wrong device-side tables give wrong rows, never an access outside the
    // table, the pools or the workspace.
    const int ctx = min(max(a.ctx_lens[b], 0), a.max_ctx);
    // The query sits at q_idx = ctx - 1 (the offset of the decode step), so "causal" is kv < ctx and a
    // sliding window adds the lower bound kv >= q_idx - window.
    const int kv_lo = a.window >= 0 ? max(ctx - 1 - a.window, 0) : 0;
    const int tok_begin = split * a.split_len;
    if (tok_begin >= ctx || tok_begin + a.split_len <= kv_lo) return;   // wave-uniform; the kernel has no barriers
    const int tok_end = min(ctx, tok_begin + a.split_len);
    const int tok_first = max(tok_begin, kv_lo & ~(kDecTile - 1));    // first tile that holds a visible key
    bf16* k_tile = smem + wave * 2 * TILE;
    bf16* v_tile = k_tile + TILE;

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
    const RowReader<D> k_reader(l32, half, lds_addr(k_tile));
    const TrReader<D> v_reader(lane, lds_addr(v_tile));

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    // Page ids of the rows this lane fetches for one tile (NI wave instructions, RPI rows each; rows
    // past the context re-read the last key).
    auto lookup = [&](int tok0, int (&pg)[NI]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int tok = min(tok0 + i * RPI + lane / DC, ctx - 1);
            pg[i] = min(max(pt[tok >> a.page_shift], 0), a.n_pool_pages - 1);
        }
    };
    // Gather of the 32 K rows and 32 V rows of a tile through the page table, straight into LDS.  The
    // LDS-DMA loads are inline assembly so that the compiler does not make later LDS reads wait for
    // them (see lds_tiles.h); completion is awaited with wait_vmem() at the top of the next iteration.
    auto gather = [&](int tok0, const int (&pg)[NI]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = i * RPI + lane / DC;
            const int tok = min(tok0 + row, ctx - 1);
            const int64_t off = ((int64_t)pg[i] * a.Hkv + hkv) * slab + (int64_t)(tok & page_mask) * D +
                                (((lane % DC) ^ swz<D>(row)) * 8);
            dma_global_nt(lds_addr(k_tile + i * 512), a.K_pool + off);
            dma_global_nt(lds_addr(v_tile + i * 512), a.V_pool + off);
        }
    };

    int pg_next[NI];
    lookup(tok_first, pg_next);
    gather(tok_first, pg_next);
    if (tok_first + kDecTile < tok_end) lookup(tok_first + kDecTile, pg_next);

    for (int tok0 = tok_first; tok0 < tok_end; tok0 += kDecTile) {
        // ---- tile tok0 has landed; take every operand fragment out of LDS, then start the gather of
        // the next tile into the same (wave-private) buffers so that it runs beside this tile's compute
        wait_vmem();
        bf16x8 kfr[D / 16], vfr[D / 32][2];
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) kfr[ks] = k_reader.read(0, 0, ks);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int c = 0; c < 2; ++c) vfr[db][c] = v_reader.read(0, 16 * c, db);
        if (tok0 + kDecTile < tok_end) {
            __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): the fragments are in registers
            gather(tok0 + kDecTile, pg_next);
            if (tok0 + 2 * kDecTile < tok_end) lookup(tok0 + 2 * kDecTile, pg_next);
        }

        // ---- S^T = K Q^T
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) sacc = mfma32(kfr[ks], qf[ks], sacc);

        // ---- score_mod, mask kv_lo <= kv < ctx_len (only the first and the last tile can hold masked
        // keys), softmax
        const bool ragged = tok0 + kDecTile > tok_end || tok0 < kv_lo;
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kv = tok0 + crow(r, half);
            float x = smod.apply(sacc[r], q_idx - kv);
            if (ragged && (kv >= tok_end || kv < kv_lo)) x = -INFINITY;
            sacc[r] = x;
            mx = fmaxf(mx, x);
        }
        mx = fmaxf(mx, swap_halves(mx));
        const float m_new = fmaxf(m_run, mx);          // finite: every tile holds at least one key
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float psum = 0.0f;
        bf16x8 pf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            u32x4 pk;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float p0 = fast_exp2(sacc[8 * c + 2 * jj] - m_new);
                const float p1 = fast_exp2(sacc[8 * c + 2 * jj + 1] - m_new);
                psum += p0 + p1;
                pk[jj] = pack_bf16(p0, p1);
            }
            pf[c] = __builtin_bit_cast(bf16x8, pk);
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
            for (int c = 0; c < 2; ++c) oacc[db] = mfma32(vfr[db][c], pf[c], oacc[db]);
    }

    const float l_tot = l_run + swap_halves(l_run);
    if (g_ok) {
        const int64_t out_item = ((int64_t)b * a.Hq + hq) * a.max_splits + split;
        float* po = a.part_O + out_item * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                f32x4 v = {oacc[db][4 * rg], oacc[db][4 * rg + 1], oacc[db][4 * rg + 2], oacc[db][4 * rg + 3]};
                *(f32x4*)(po + db * 32 + 8 * rg + 4 * half) = v;
            }
        if (half == 0) {
            a.part_ml[out_item * 2] = m_run;
            a.part_ml[out_item * 2 + 1] = l_tot;
        }
    }
}

// One wave per (sequence, query head): O = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max m).
template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const DecodeArgs a) {
    const int lane = threadIdx.x;
    const int b = blockIdx.x / a.Hq, hq = blockIdx.x % a.Hq;
    const int ctx = min(max(a.ctx_lens[b], 0), a.max_ctx);                          // as in the split kernel
    const int ns = (ctx + a.split_len - 1) / a.split_len;                           // <= max_splits
    const int s0 = a.window >= 0 ? max(ctx - 1 - a.window, 0) / a.split_len : 0;    // splits below the window are empty
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
    for (int s = s0; s < ns; ++s) m = fmaxf(m, a.part_ml[(base + s) * 2]);
    float L = 0.0f, acc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) acc[i] = 0.0f;
    for (int s = s0; s < ns; ++s) {
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

// Keys per split.  One wave works on one (sequence, KV head, split), so a launch offers
// nseq * Hkv * ceil(ctx / split_len) waves; the host cannot see the context lengths and sizes the
// split for the longest context the page table addresses: the largest power of two in
// [kDecSplitMin, kDecSplitMax] that still gives every SIMD of the chip a wave, so that a small batch
// of long sequences is cut finer than a large one (measured: aiming at two waves per SIMD instead
// makes one sequence of 32k tokens 1.5x slower -- each wave's start-up outweighs its 128 keys).
static int split_len_of(const flexattn_decode_dims* d) {
    const long long max_tokens = (long long)d->max_pages * d->page_size;
    const long long per_wave = max_tokens * d->nseq * d->Hkv / kDecTargetWaves;
    int len = kDecSplitMin;
    while (len < kDecSplitMax && 2 * len <= per_wave) len *= 2;
    return len;
}

static int max_splits_of(const flexattn_decode_dims* d) {
    const long long max_tokens = (long long)d->max_pages * d->page_size;
    const int len = split_len_of(d);
    return (int)((max_tokens + len - 1) / len);
}

template <int D>
static int launch_decode(const DecodeArgs& a, uint32_t score_id, hipStream_t st) {
    const int spw = a.max_splits >= 4 ? 4 : (a.max_splits >= 2 ? 2 : 1), upw = kDecWaves / spw;
    const dim3 grid((unsigned)((a.nseq * a.Hkv + upw - 1) / upw), (unsigned)((a.max_splits + spw - 1) / spw));
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
    if (d->page_size < 16 || d->page_size > 1024 || (d->page_size & (d->page_size - 1)))
        return FLEXATTN_ERR_UNSUPPORTED;
    if ((long long)d->max_pages * d->page_size > (1ll << 30)) return FLEXATTN_ERR_UNSUPPORTED;
    return FLEXATTN_OK;
}

extern "C" size_t flexattn_paged_decode_workspace_bytes(const flexattn_decode_dims* d) {
    if (check_decode_dims(d) != FLEXATTN_OK) return 0;
    const size_t items = (size_t)d->nseq * d->Hq * max_splits_of(d);
    return items * ((size_t)d->D + 2) * sizeof(float);
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* addr[kMaxDevices] = {};
    int dev = -1;
    FLEXATTN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return FLEXATTN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        FLEXATTN_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return FLEXATTN_ERR_HIP;
        addr[dev] = p;
    }
    *out = addr[dev];
    return FLEXATTN_OK;
}

extern "C" size_t flexattn_paged_decode_static_capacity(void) { return kStaticScratchBytes; }

extern "C" int flexattn_paged_decode_static(const flexattn_decode_dims* d, const void* Q, int64_t stride_q_seq,
                                            const void* K_pool, const void* V_pool, const int32_t* page_table,
                                            int64_t pt_stride, const int32_t* ctx_lens, uint32_t score_id,
                                            uint32_t mask_id, const flexattn_mod_params* params, float scale, void* O,
                                            float* LSE, void* stream) {
    int rc = check_decode_dims(d);
    if (rc != FLEXATTN_OK) return rc;
    // Every partial the combine kernel reads was written by the split kernel of the same call, so
    // nothing in the array has to start at zero.
    if (flexattn_paged_decode_workspace_bytes(d) > kStaticScratchBytes) return FLEXATTN_ERR_WORKSPACE;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != FLEXATTN_OK) return rc;
    return flexattn_paged_decode(d, Q, stride_q_seq, K_pool, V_pool, page_table, pt_stride, ctx_lens, score_id,
                                 mask_id, params, scale, O, LSE, ws, kStaticScratchBytes, stream);
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
    const uint32_t kCtxWindow = FLEXATTN_M_CTX_LEN | FLEXATTN_M_SLIDING_WINDOW;   // one AND-term
    if (mask_id != FLEXATTN_MASK_CTX_LEN && mask_id != kCtxWindow) return FLEXATTN_ERR_UNSUPPORTED;
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
    a.split_len = split_len_of(d);
    a.max_ctx = d->max_pages * d->page_size;
    a.n_pool_pages = d->n_pool_pages;
    a.window = mask_id == kCtxWindow ? p.window : -1;
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
