// flexattn_forward: argument validation and dispatch to the compiled (mask, score) variant.
#include "fwd_kernel.h"
#include "variants.h"

namespace flexattn {

#define DECL(i) int fwd_launch_##i(const FwdArgs&, int, int, hipStream_t);
FLEXATTN_VARIANT_INDICES(DECL)
#undef DECL
typedef int (*FwdLauncher)(const FwdArgs&, int, int, hipStream_t);
#define ENTRY(i) fwd_launch_##i,
static const FwdLauncher kFwdLaunchers[kNumVariants] = {FLEXATTN_VARIANT_INDICES(ENTRY)};
#undef ENTRY
#define DECL(i) int fwd_paged_launch_##i(const FwdArgs&, int, int, hipStream_t);
FLEXATTN_VARIANT_INDICES(DECL)
#undef DECL
#define ENTRY(i) fwd_paged_launch_##i,
static const FwdLauncher kFwdPagedLaunchers[kNumVariants] = {FLEXATTN_VARIANT_INDICES(ENTRY)};
#undef ENTRY

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

int check_tensor(const flexattn_tensor* t) {
    if (!t || !t->ptr) return FLEXATTN_ERR_INVALID_ARG;
    if (t->stride_s <= 0 || t->stride_h < 0 || t->stride_b < 0) return FLEXATTN_ERR_INVALID_ARG;
    if (((uintptr_t)t->ptr & 15) || (t->stride_s % 8) || (t->stride_h % 8) || (t->stride_b % 8))
        return FLEXATTN_ERR_INVALID_ARG;   // rows are moved 16 bytes at a time
    return FLEXATTN_OK;
}

// The kernels address the rows of one (b, h) slice with 32-bit byte offsets.
int check_extent(const flexattn_tensor* t, int len, int D) {
    if (t->stride_s < D) return FLEXATTN_ERR_INVALID_ARG;
    const int64_t bytes = ((int64_t)(len - 1) * t->stride_s + D) * 2;
    return bytes < ((int64_t)1 << 31) ? FLEXATTN_OK : FLEXATTN_ERR_UNSUPPORTED;
}

int check_problem(const flexattn_dims* d, const flexattn_blockmask* bm) {
    if (!d || !bm) return FLEXATTN_ERR_INVALID_ARG;
    if (d->B <= 0 || d->Hq <= 0 || d->Hkv <= 0 || d->q_len <= 0 || d->kv_len <= 0) return FLEXATTN_ERR_INVALID_ARG;
    if (d->Hq % d->Hkv != 0) return FLEXATTN_ERR_INVALID_ARG;
    if (d->D != 64 && d->D != 128) return FLEXATTN_ERR_UNSUPPORTED;
    if (bm->q_len != d->q_len || bm->kv_len != d->kv_len) return FLEXATTN_ERR_INVALID_ARG;
    if (!(bm->Bm == 1 || bm->Bm == d->B) || !(bm->Hm == 1 || bm->Hm == d->Hq)) return FLEXATTN_ERR_INVALID_ARG;
    if (!(bm->Bq == 64 || bm->Bq == 128) || !(bm->Bk == 64 || bm->Bk == 128)) return FLEXATTN_ERR_UNSUPPORTED;
    if (!bm->kv_num_blocks || !bm->kv_indices || !bm->full_kv_num_blocks || !bm->full_kv_indices)
        return FLEXATTN_ERR_INVALID_ARG;
    return FLEXATTN_OK;
}

}  // namespace flexattn

using namespace flexattn;

extern "C" const char* flexattn_strerror(int status) {
    switch (status) {
        case FLEXATTN_OK: return "ok";
        case FLEXATTN_ERR_INVALID_ARG: return "invalid argument";
        case FLEXATTN_ERR_UNSUPPORTED: return "unsupported head dimension, block size or (mask, score) variant";
        case FLEXATTN_ERR_WORKSPACE: return "workspace too small";
        case FLEXATTN_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}
extern "C" int flexattn_last_hip_error(void) { return g_last_hip_error; }
extern "C" int flexattn_version(void) { return 120; }   // 120: flexattn_backward_stored (110: work-order arrays, probes, static decode)
extern "C" int flexattn_is_supported(uint32_t mask_id, uint32_t score_id, int32_t D) {
    return (D == 64 || D == 128) && find_variant(mask_id, score_id) >= 0;
}

extern "C" int flexattn_forward(const flexattn_dims* dims, const flexattn_tensor* Q, const flexattn_tensor* K,
                                const flexattn_tensor* V, uint32_t score_id, uint32_t mask_id,
                                const flexattn_mod_params* params, const flexattn_blockmask* bm, float scale,
                                const flexattn_tensor* O, float* LSE, void* stream) {
    int rc = check_problem(dims, bm);
    if (rc != FLEXATTN_OK) return rc;
    if ((rc = check_tensor(Q)) || (rc = check_tensor(K)) || (rc = check_tensor(V)) || (rc = check_tensor(O))) return rc;
    if ((rc = check_extent(K, dims->kv_len, dims->D)) || (rc = check_extent(V, dims->kv_len, dims->D))) return rc;
    if (!LSE || !(scale > 0.0f)) return FLEXATTN_ERR_INVALID_ARG;
    if ((rc = check_mod_params(mask_id, score_id, params)) != FLEXATTN_OK) return rc;
    if ((rc = check_canvas(mask_id, params, dims->q_len, dims->kv_len)) != FLEXATTN_OK) return rc;
    const int vi = find_variant(mask_id, score_id);
    if (vi < 0) return FLEXATTN_ERR_UNSUPPORTED;

    FwdArgs a = {};
    a.Q = (const bf16*)Q->ptr; a.K = (const bf16*)K->ptr; a.V = (const bf16*)V->ptr;
    a.O = (bf16*)O->ptr; a.LSE = LSE;
    a.q_sb = Q->stride_b; a.q_sh = Q->stride_h; a.q_ss = Q->stride_s;
    a.k_sb = K->stride_b; a.k_sh = K->stride_h; a.k_ss = K->stride_s;
    a.v_sb = V->stride_b; a.v_sh = V->stride_h; a.v_ss = V->stride_s;
    a.o_sb = O->stride_b; a.o_sh = O->stride_h; a.o_ss = O->stride_s;
    a.B = dims->B; a.Hq = dims->Hq; a.Hkv = dims->Hkv; a.G = dims->Hq / dims->Hkv;
    a.q_len = dims->q_len; a.kv_len = dims->kv_len;
    a.NR = (dims->q_len + bm->Bq - 1) / bm->Bq; a.NC = (dims->kv_len + bm->Bk - 1) / bm->Bk;
    a.Bk = bm->Bk; a.sub = bm->Bk / kTileKV;
    a.bm_Bm = bm->Bm; a.bm_Hm = bm->Hm;
    a.kv_num = bm->kv_num_blocks; a.kv_idx = bm->kv_indices;
    a.full_num = bm->full_kv_num_blocks; a.full_idx = bm->full_kv_indices;
    a.kv_order = bm->kv_order;
    a.scale = scale;
    if (params) a.p = *params;
    rc = kFwdLaunchers[vi](a, dims->D, bm->Bq, (hipStream_t)stream);
    if (rc != FLEXATTN_OK) return rc;
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}

extern "C" int flexattn_paged_forward(const flexattn_dims* dims, const flexattn_tensor* Q, const void* K_pool,
                                      const void* V_pool, int32_t page_size, int32_t n_pool_pages, uint32_t score_id,
                                      uint32_t mask_id, const flexattn_mod_params* params,
                                      const flexattn_blockmask* bm, const int32_t* phys_kv_indices,
                                      const int32_t* phys_full_kv_indices, float scale, const flexattn_tensor* O,
                                      float* LSE, void* stream) {
    int rc = check_problem(dims, bm);
    if (rc != FLEXATTN_OK) return rc;
    if ((rc = check_tensor(Q)) || (rc = check_tensor(O))) return rc;
    if (!K_pool || !V_pool || ((uintptr_t)K_pool & 15) || ((uintptr_t)V_pool & 15)) return FLEXATTN_ERR_INVALID_ARG;
    if (!phys_kv_indices || !phys_full_kv_indices || n_pool_pages <= 0) return FLEXATTN_ERR_INVALID_ARG;
    if (!LSE || !(scale > 0.0f)) return FLEXATTN_ERR_INVALID_ARG;
    if (page_size != bm->Bk) return FLEXATTN_ERR_UNSUPPORTED;     // a block of the BlockMask is a page
    if (bm->Bm != dims->B) return FLEXATTN_ERR_INVALID_ARG;        // every sequence has its own pages
    if ((rc = check_mod_params(mask_id, score_id, params)) != FLEXATTN_OK) return rc;
    if ((rc = check_canvas(mask_id, params, dims->q_len, dims->kv_len)) != FLEXATTN_OK) return rc;
    const int vi = find_variant(mask_id, score_id);
    if (vi < 0) return FLEXATTN_ERR_UNSUPPORTED;

    FwdArgs a = {};
    a.Q = (const bf16*)Q->ptr; a.K = (const bf16*)K_pool; a.V = (const bf16*)V_pool;
    a.O = (bf16*)O->ptr; a.LSE = LSE;
    a.q_sb = Q->stride_b; a.q_sh = Q->stride_h; a.q_ss = Q->stride_s;
    a.k_sb = 0; a.k_sh = (int64_t)page_size * dims->D; a.k_ss = dims->D;
    a.v_sb = 0; a.v_sh = a.k_sh; a.v_ss = dims->D;
    a.o_sb = O->stride_b; a.o_sh = O->stride_h; a.o_ss = O->stride_s;
    a.B = dims->B; a.Hq = dims->Hq; a.Hkv = dims->Hkv; a.G = dims->Hq / dims->Hkv;
    a.q_len = dims->q_len; a.kv_len = dims->kv_len;
    a.NR = (dims->q_len + bm->Bq - 1) / bm->Bq; a.NC = (dims->kv_len + bm->Bk - 1) / bm->Bk;
    a.Bk = bm->Bk; a.sub = bm->Bk / kTileKV;
    a.bm_Bm = bm->Bm; a.bm_Hm = bm->Hm;
    a.kv_num = bm->kv_num_blocks; a.kv_idx = bm->kv_indices;
    a.full_num = bm->full_kv_num_blocks; a.full_idx = bm->full_kv_indices;
    a.kv_order = bm->kv_order;
    a.phys_kv_idx = phys_kv_indices; a.phys_full_idx = phys_full_kv_indices;
    a.page_stride = (int64_t)dims->Hkv * page_size * dims->D;
    a.n_pool_pages = n_pool_pages;
    a.scale = scale;
    if (params) a.p = *params;
    rc = kFwdPagedLaunchers[vi](a, dims->D, bm->Bq, (hipStream_t)stream);
    if (rc != FLEXATTN_OK) return rc;
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}
