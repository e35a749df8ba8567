// flexattn_backward: argument validation, the delta pre-pass and dispatch to the compiled variant.
#include "bwd_stored.h"
#include "variants.h"

namespace flexattn {

#define DECL(i) int bwd_launch_##i(const BwdArgs&, int, uint32_t, hipStream_t);
FLEXATTN_VARIANT_INDICES(DECL)
#undef DECL
typedef int (*BwdLauncher)(const BwdArgs&, int, uint32_t, hipStream_t);
#define ENTRY(i) bwd_launch_##i,
static const BwdLauncher kBwdLaunchers[kNumVariants] = {FLEXATTN_VARIANT_INDICES(ENTRY)};
#undef ENTRY
int check_tensor(const flexattn_tensor* t);
int check_extent(const flexattn_tensor* t, int len, int D);
int check_problem(const flexattn_dims* d, const flexattn_blockmask* bm);

}  // namespace flexattn

using namespace flexattn;

extern "C" size_t flexattn_backward_workspace_bytes(const flexattn_dims* d) {
    if (!d || d->B <= 0 || d->Hq <= 0 || d->q_len <= 0) return 0;
    return (size_t)2 * d->B * d->Hq * d->q_len * sizeof(float);
}

namespace {
// Workspace of the backward that keeps dS in memory: the row scalars of the recomputing backward,
// then the slot numbering (column bases, grid), then the dS blocks.
struct StoredLayout {
    size_t colbase_off, grid_off, store_off, total;
    int64_t cap;        // slots per head
    int lines, planes;
};
size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
bool stored_layout(const flexattn_dims* d, const flexattn_blockmask* bm, int64_t n_blocks, StoredLayout* out) {
    if (!d || !bm || d->B <= 0 || d->Hq <= 0 || d->q_len <= 0 || d->kv_len <= 0 || n_blocks < 0) return false;
    if (bm->Bq <= 0 || bm->Bk <= 0 || bm->Bm <= 0 || bm->Hm <= 0) return false;
    const int64_t NR = (d->q_len + bm->Bq - 1) / bm->Bq, NC = (d->kv_len + bm->Bk - 1) / bm->Bk;
    const int64_t planes = (int64_t)bm->Bm * bm->Hm, lines = planes * NC;
    const int64_t cap = n_blocks > 0 ? n_blocks : 1;    // (times Bk / 64 tiles and Bq / 64 steps it must fit an int)
    if (lines >= (1ll << 30) || planes * NR * NC >= (1ll << 40) || cap * 4 >= (1ll << 31)) return false;
    const int64_t reps = (int64_t)(bm->Bm > 1 ? 1 : d->B) * (bm->Hm > 1 ? 1 : d->Hq);
    out->cap = cap;
    out->lines = (int)lines;
    out->planes = (int)planes;
    out->colbase_off = align256(flexattn_backward_workspace_bytes(d));
    out->grid_off = out->colbase_off + align256((size_t)(lines + 1) * sizeof(int32_t));
    out->store_off = out->grid_off + align256((size_t)(planes * NR * NC) * sizeof(int32_t));
    out->total = out->store_off + (size_t)reps * (size_t)cap * (size_t)bm->Bq * (size_t)bm->Bk * sizeof(bf16);
    return true;
}

// ds_blocks < 0: dQ recomputes S and dP; otherwise dS goes through memory (every stage runs).
int backward_impl(const flexattn_dims* dims, const flexattn_tensor* Q,
                                        const flexattn_tensor* K, const flexattn_tensor* V, const flexattn_tensor* O,
                                        const flexattn_tensor* dO, const float* LSE, uint32_t score_id,
                                        uint32_t mask_id, const flexattn_mod_params* params,
                                        const flexattn_blockmask* bm, float scale, const flexattn_tensor* dQ,
                                        const flexattn_tensor* dK, const flexattn_tensor* dV, void* ws,
                                        size_t ws_bytes, void* stream, uint32_t stages, int64_t ds_blocks) {
    int rc = check_problem(dims, bm);
    if (rc != FLEXATTN_OK) return rc;
    if (stages == 0 || (stages & ~FLEXATTN_BWD_ALL)) return FLEXATTN_ERR_INVALID_ARG;
    const flexattn_tensor* ts[] = {Q, K, V, O, dO};
    for (const flexattn_tensor* t : ts)
        if ((rc = check_tensor(t)) != FLEXATTN_OK) return rc;
    if ((stages & FLEXATTN_BWD_DQ) && (rc = check_tensor(dQ)) != FLEXATTN_OK) return rc;
    if ((stages & FLEXATTN_BWD_DKDV) && ((rc = check_tensor(dK)) != FLEXATTN_OK || (rc = check_tensor(dV)) != FLEXATTN_OK))
        return rc;
    if ((rc = check_extent(Q, dims->q_len, dims->D)) != FLEXATTN_OK) return rc;
    if ((rc = check_extent(dO, dims->q_len, dims->D)) != FLEXATTN_OK) return rc;
    if ((rc = check_extent(K, dims->kv_len, dims->D)) != FLEXATTN_OK) return rc;
    if ((rc = check_extent(V, dims->kv_len, dims->D)) != FLEXATTN_OK) return rc;
    static const flexattn_tensor kNoTensor = {nullptr, 0, 0, 0};
    if (!(stages & FLEXATTN_BWD_DQ)) dQ = &kNoTensor;
    if (!(stages & FLEXATTN_BWD_DKDV)) dK = dV = &kNoTensor;
    if (!LSE || !ws || !(scale > 0.0f) || ((uintptr_t)ws & 15)) return FLEXATTN_ERR_INVALID_ARG;
    if (!bm->q_num_blocks || !bm->q_indices || !bm->full_q_num_blocks || !bm->full_q_indices)
        return FLEXATTN_ERR_INVALID_ARG;
    if ((rc = check_mod_params(mask_id, score_id, params)) != FLEXATTN_OK) return rc;
    if ((rc = check_canvas(mask_id, params, dims->q_len, dims->kv_len)) != FLEXATTN_OK) return rc;
    const int vi = find_variant(mask_id, score_id);
    if (vi < 0) return FLEXATTN_ERR_UNSUPPORTED;
    const bool stored = ds_blocks >= 0;
    StoredLayout lay = {};
    if (stored) {
        if (!stored_layout(dims, bm, ds_blocks, &lay)) return FLEXATTN_ERR_INVALID_ARG;
        if (((uintptr_t)ws & 255)) return FLEXATTN_ERR_INVALID_ARG;
        if (ws_bytes < lay.total) return FLEXATTN_ERR_WORKSPACE;
    } else if (ws_bytes < flexattn_backward_workspace_bytes(dims)) {
        return FLEXATTN_ERR_WORKSPACE;
    }

    BwdArgs a = {};
    a.Q = (const bf16*)Q->ptr; a.K = (const bf16*)K->ptr; a.V = (const bf16*)V->ptr;
    a.O = (const bf16*)O->ptr; a.dO = (const bf16*)dO->ptr; a.LSE = LSE;
    a.dQ = (bf16*)dQ->ptr; a.dK = (bf16*)dK->ptr; a.dV = (bf16*)dV->ptr;
    const size_t rows = (size_t)dims->B * dims->Hq * dims->q_len;
    a.delta = (float*)ws; a.lse2 = (float*)ws + rows;
    int32_t* colbase = nullptr;
    int32_t* grid = nullptr;
    if (stored) {
        colbase = (int32_t*)((char*)ws + lay.colbase_off);
        grid = (int32_t*)((char*)ws + lay.grid_off);
        a.ds_colbase = colbase;
        a.ds_grid = grid;
        a.ds_store = (bf16*)((char*)ws + lay.store_off);
        a.ds_blocks = lay.cap;
    }
    a.q_sb = Q->stride_b; a.q_sh = Q->stride_h; a.q_ss = Q->stride_s;
    a.k_sb = K->stride_b; a.k_sh = K->stride_h; a.k_ss = K->stride_s;
    a.v_sb = V->stride_b; a.v_sh = V->stride_h; a.v_ss = V->stride_s;
    a.o_sb = O->stride_b; a.o_sh = O->stride_h; a.o_ss = O->stride_s;
    a.do_sb = dO->stride_b; a.do_sh = dO->stride_h; a.do_ss = dO->stride_s;
    a.dq_sb = dQ->stride_b; a.dq_sh = dQ->stride_h; a.dq_ss = dQ->stride_s;
    a.dk_sb = dK->stride_b; a.dk_sh = dK->stride_h; a.dk_ss = dK->stride_s;
    a.dv_sb = dV->stride_b; a.dv_sh = dV->stride_h; a.dv_ss = dV->stride_s;
    a.B = dims->B; a.Hq = dims->Hq; a.Hkv = dims->Hkv; a.G = dims->Hq / dims->Hkv;
    a.q_len = dims->q_len; a.kv_len = dims->kv_len;
    a.NR = (dims->q_len + bm->Bq - 1) / bm->Bq; a.NC = (dims->kv_len + bm->Bk - 1) / bm->Bk;
    a.Bq = bm->Bq; a.Bk = bm->Bk;
    a.bm_Bm = bm->Bm; a.bm_Hm = bm->Hm;
    a.kv_num = bm->kv_num_blocks; a.kv_idx = bm->kv_indices;
    a.full_kv_num = bm->full_kv_num_blocks; a.full_kv_idx = bm->full_kv_indices;
    a.q_num = bm->q_num_blocks; a.q_idx = bm->q_indices;
    a.full_q_num = bm->full_q_num_blocks; a.full_q_idx = bm->full_q_indices;
    a.kv_order = bm->kv_order; a.q_order = bm->q_order;
    a.scale = scale;
    if (params) a.p = *params;

    hipStream_t st = (hipStream_t)stream;
    if (stored) {
        if (stages & FLEXATTN_BWD_DELTA) {      // the block numbering belongs to the pre-pass
            hipLaunchKernelGGL(bwd_slots_scan_kernel, dim3(1), dim3(1024), 0, st, a.q_num, a.full_q_num, lay.lines,
                               a.NR, colbase);
            hipLaunchKernelGGL(bwd_slots_fill_kernel, dim3((unsigned)lay.lines), dim3(256), 0, st, a.q_num, a.q_idx,
                               a.full_q_num, a.full_q_idx, a.NR, a.NC, colbase, grid);
        }
        // delta and dK/dV (which writes dS) from the compiled variant; dQ from what it wrote
        if (stages & (FLEXATTN_BWD_DELTA | FLEXATTN_BWD_DKDV)) {
            rc = kBwdLaunchers[vi](a, dims->D, stages & (FLEXATTN_BWD_DELTA | FLEXATTN_BWD_DKDV), st);
            if (rc != FLEXATTN_OK) return rc;
        }
        if (stages & FLEXATTN_BWD_DQ) {
            const float qscale = scale * ((score_id & FLEXATTN_SCORE_SOFTCAP) ? 4.0f : 1.0f);   // ScoreMod::grad_scale()
            launch_bwd_stored_dq(a, dims->D, qscale, st);
        }
    } else {
        rc = kBwdLaunchers[vi](a, dims->D, stages, st);     // the delta pre-pass depends on the score_mod too
        if (rc != FLEXATTN_OK) return rc;
    }
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}
}  // namespace

extern "C" int flexattn_backward_stages(const flexattn_dims* dims, const flexattn_tensor* Q,
                                        const flexattn_tensor* K, const flexattn_tensor* V, const flexattn_tensor* O,
                                        const flexattn_tensor* dO, const float* LSE, uint32_t score_id,
                                        uint32_t mask_id, const flexattn_mod_params* params,
                                        const flexattn_blockmask* bm, float scale, const flexattn_tensor* dQ,
                                        const flexattn_tensor* dK, const flexattn_tensor* dV, void* ws,
                                        size_t ws_bytes, void* stream, uint32_t stages) {
    return backward_impl(dims, Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, scale, dQ, dK, dV, ws, ws_bytes,
                         stream, stages, -1);
}

extern "C" int flexattn_backward(const flexattn_dims* dims, const flexattn_tensor* Q, const flexattn_tensor* K,
                                 const flexattn_tensor* V, const flexattn_tensor* O, const flexattn_tensor* dO,
                                 const float* LSE, uint32_t score_id, uint32_t mask_id,
                                 const flexattn_mod_params* params, const flexattn_blockmask* bm, float scale,
                                 const flexattn_tensor* dQ, const flexattn_tensor* dK, const flexattn_tensor* dV,
                                 void* ws, size_t ws_bytes, void* stream) {
    return flexattn_backward_stages(dims, Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, scale, dQ, dK, dV, ws,
                                    ws_bytes, stream, FLEXATTN_BWD_ALL);
}

extern "C" size_t flexattn_backward_stored_workspace_bytes(const flexattn_dims* dims, const flexattn_blockmask* bm,
                                                           int64_t n_blocks) {
    StoredLayout lay;
    return stored_layout(dims, bm, n_blocks, &lay) ? lay.total : 0;
}

extern "C" int flexattn_backward_stored(const flexattn_dims* dims, const flexattn_tensor* Q, const flexattn_tensor* K,
                                        const flexattn_tensor* V, const flexattn_tensor* O, const flexattn_tensor* dO,
                                        const float* LSE, uint32_t score_id, uint32_t mask_id,
                                        const flexattn_mod_params* params, const flexattn_blockmask* bm, float scale,
                                        const flexattn_tensor* dQ, const flexattn_tensor* dK, const flexattn_tensor* dV,
                                        int64_t n_blocks, void* ws, size_t ws_bytes, void* stream, uint32_t stages) {
    if (n_blocks < 0) return FLEXATTN_ERR_INVALID_ARG;
    return backward_impl(dims, Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, scale, dQ, dK, dV, ws, ws_bytes,
                         stream, stages, n_blocks);
}

// ---- gradients of captured tensors -----------------------------------------------------------
namespace {
// Sum of the per-workgroup partials over batch and rows of blocks, in a fixed order, times `factor`:
// out[hq, i] = factor * sum_{b, row} part[((b * Hq + hq) * NR + row) * width + i].
__global__ __launch_bounds__(256) void captured_reduce_kernel(const float* __restrict__ part, int B, int Hq, int NR,
                                                              int width, float factor, float* __restrict__ out) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Hq * width) return;
    const int hq = idx / width, i = idx - hq * width;
    double sum = 0.0;
    for (int b = 0; b < B; ++b)
        for (int row = 0; row < NR; ++row) sum += (double)part[(((int64_t)b * Hq + hq) * NR + row) * width + i];
    out[idx] = (float)(sum * (double)factor);
}

size_t captured_rows(const flexattn_dims* d) { return (size_t)d->B * d->Hq * d->q_len; }
size_t captured_slots(const flexattn_dims* d, const flexattn_blockmask* bm) {
    return (size_t)d->B * d->Hq * ((d->q_len + bm->Bq - 1) / bm->Bq);
}
}  // namespace

extern "C" size_t flexattn_backward_captured_workspace_bytes(const flexattn_dims* d, const flexattn_blockmask* bm,
                                                             uint32_t score_id, const flexattn_mod_params* params) {
    if (!d || !bm || d->B <= 0 || d->Hq <= 0 || d->q_len <= 0 || bm->Bq <= 0) return 0;
    size_t n = 2 * captured_rows(d);                                   // -delta and the row constants
    if (score_id & FLEXATTN_SCORE_ALIBI) n += captured_slots(d, bm);
    if ((score_id & FLEXATTN_SCORE_REL_BIAS) && params && params->rel_len > 0)
        n += captured_slots(d, bm) * (size_t)params->rel_len;
    return n * sizeof(float);
}

extern "C" int flexattn_backward_captured(const flexattn_dims* dims, const flexattn_tensor* Q,
                                          const flexattn_tensor* K, const flexattn_tensor* V, const flexattn_tensor* O,
                                          const flexattn_tensor* dO, const float* LSE, uint32_t score_id,
                                          uint32_t mask_id, const flexattn_mod_params* params,
                                          const flexattn_blockmask* bm, float scale, float* d_alibi_bias,
                                          float* d_rel_bias, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_problem(dims, bm);
    if (rc != FLEXATTN_OK) return rc;
    const flexattn_tensor* ts[] = {Q, K, V, O, dO};
    for (const flexattn_tensor* t : ts)
        if ((rc = check_tensor(t)) != FLEXATTN_OK) return rc;
    if ((rc = check_extent(K, dims->kv_len, dims->D)) != FLEXATTN_OK) return rc;
    if ((rc = check_extent(V, dims->kv_len, dims->D)) != FLEXATTN_OK) return rc;
    if (!LSE || !ws || !(scale > 0.0f) || ((uintptr_t)ws & 15)) return FLEXATTN_ERR_INVALID_ARG;
    if ((rc = check_mod_params(mask_id, score_id, params)) != FLEXATTN_OK) return rc;
    if ((rc = check_canvas(mask_id, params, dims->q_len, dims->kv_len)) != FLEXATTN_OK) return rc;
    const bool alibi = score_id & FLEXATTN_SCORE_ALIBI, rel = score_id & FLEXATTN_SCORE_REL_BIAS;
    if (!alibi && !rel) return FLEXATTN_ERR_UNSUPPORTED;               // nothing is captured
    if ((alibi && !d_alibi_bias) || (rel && !d_rel_bias)) return FLEXATTN_ERR_INVALID_ARG;
    const int vi = find_variant(mask_id, score_id);
    if (vi < 0) return FLEXATTN_ERR_UNSUPPORTED;
    if (ws_bytes < flexattn_backward_captured_workspace_bytes(dims, bm, score_id, params)) return FLEXATTN_ERR_WORKSPACE;

    BwdArgs a = {};
    a.Q = (const bf16*)Q->ptr; a.K = (const bf16*)K->ptr; a.V = (const bf16*)V->ptr;
    a.O = (const bf16*)O->ptr; a.dO = (const bf16*)dO->ptr; a.LSE = LSE;
    const size_t rows = captured_rows(dims), slots = captured_slots(dims, bm);
    a.delta = (float*)ws; a.lse2 = (float*)ws + rows;
    a.cap_alibi = (float*)ws + 2 * rows;
    a.cap_rel = a.cap_alibi + (alibi ? slots : 0);
    a.q_sb = Q->stride_b; a.q_sh = Q->stride_h; a.q_ss = Q->stride_s;
    a.k_sb = K->stride_b; a.k_sh = K->stride_h; a.k_ss = K->stride_s;
    a.v_sb = V->stride_b; a.v_sh = V->stride_h; a.v_ss = V->stride_s;
    a.o_sb = O->stride_b; a.o_sh = O->stride_h; a.o_ss = O->stride_s;
    a.do_sb = dO->stride_b; a.do_sh = dO->stride_h; a.do_ss = dO->stride_s;
    a.B = dims->B; a.Hq = dims->Hq; a.Hkv = dims->Hkv; a.G = dims->Hq / dims->Hkv;
    a.q_len = dims->q_len; a.kv_len = dims->kv_len;
    a.NR = (dims->q_len + bm->Bq - 1) / bm->Bq; a.NC = (dims->kv_len + bm->Bk - 1) / bm->Bk;
    a.Bq = bm->Bq; a.Bk = bm->Bk;
    a.bm_Bm = bm->Bm; a.bm_Hm = bm->Hm;
    a.kv_num = bm->kv_num_blocks; a.kv_idx = bm->kv_indices;
    a.full_kv_num = bm->full_kv_num_blocks; a.full_kv_idx = bm->full_kv_indices;
    a.scale = scale;
    a.p = *params;

    hipStream_t st = (hipStream_t)stream;
    rc = kBwdLaunchers[vi](a, dims->D, FLEXATTN_BWD_DELTA | kBwdStageCaptured, st);
    if (rc != FLEXATTN_OK) return rc;
    // the kernels' dS lacks the constant factor of the score_mod's derivative
    const float factor = (score_id & FLEXATTN_SCORE_SOFTCAP) ? 4.0f : 1.0f;
    if (alibi)
        hipLaunchKernelGGL(captured_reduce_kernel, dim3((unsigned)((a.Hq + 255) / 256)), dim3(256), 0, st, a.cap_alibi,
                           a.B, a.Hq, a.NR, 1, factor, d_alibi_bias);
    if (rel)
        hipLaunchKernelGGL(captured_reduce_kernel, dim3((unsigned)((a.Hq * a.p.rel_len + 255) / 256)), dim3(256), 0, st,
                           a.cap_rel, a.B, a.Hq, a.NR, a.p.rel_len, factor, d_rel_bias);
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}
