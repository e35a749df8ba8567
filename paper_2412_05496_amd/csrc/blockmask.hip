// BlockMask construction (paper section 4.2) and the paged BlockMask conversion (section 5.1).
//
// classify: one wave per block evaluates mask_mod on all Bq x Bk scalars and counts the unmasked
// ones (0 -> skipped, Bq*Bk -> full, else partial).  compact: one wave per row (or column) of
// blocks turns the per-block kinds into ascending index lists with a zero tail.
#include "flex_common.h"

namespace flexattn {

constexpr int kClassifyWaves = 4;

template <uint32_t MASK>
__global__ __launch_bounds__(kClassifyWaves * 64) void classify_blocks_kernel(
    flexattn_mod_params p, int Bm, int Hm, int NR, int NC, int Bq, int Bk, int q_len, int kv_len,
    uint8_t* __restrict__ kinds, unsigned long long* __restrict__ stats) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long nblocks = (long long)Bm * Hm * NR * NC;
    const long long blk = (long long)blockIdx.x * kClassifyWaves + wave;
    __shared__ unsigned long long s_acc[3];
    if (threadIdx.x < 3) s_acc[threadIdx.x] = 0;
    __syncthreads();
    if (blk < nblocks) {
        const int j = (int)(blk % NC);
        const int i = (int)((blk / NC) % NR);
        const int h = (int)((blk / ((long long)NC * NR)) % Hm);
        const int b = (int)(blk / ((long long)NC * NR * Hm));
        const int n = Bq * Bk;
        const int q_off = q_offset_of(p, b);
        int cnt = 0;
        // Blocks that lie wholly inside the score matrix and that the index comparisons of the mask
        // settle as a whole are not enumerated; everything else is evaluated scalar by scalar.
        bool settled = false;
        if ((i + 1) * Bq <= q_len && (j + 1) * Bk <= kv_len) {
            const MaskRow<MASK> corner(p, b, h, q_off + i * Bq, kv_len);
            const int q_lo = q_off + i * Bq, q_hi = q_lo + Bq - 1, kv_lo = j * Bk, kv_hi = kv_lo + Bk - 1;
            if (corner.block_empty(q_lo, q_hi, kv_lo, kv_hi)) {
                settled = true;
            } else if (corner.block_full(q_lo, q_hi, kv_lo, kv_hi)) {
                settled = true;
                cnt = lane == 0 ? n : 0;
            }
        }
        for (int e = lane; e < (settled ? 0 : n); e += 64) {
            // rows and keys past the end of the score matrix count as masked
            const int q = i * Bq + e / Bk, kv = j * Bk + e % Bk;
            MaskRow<MASK> row(p, b, h, q_off + min(q, q_len - 1), kv_len);
            cnt += (q < q_len && row(kv)) ? 1 : 0;
        }
        for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
        if (lane == 0) {
            const uint8_t kind = cnt == 0 ? 0 : (cnt == n ? 2 : 1);
            kinds[blk] = kind;
            if (stats) {
                if (kind == 1) atomicAdd(&s_acc[0], 1ull);
                if (kind == 2) atomicAdd(&s_acc[1], 1ull);
                atomicAdd(&s_acc[2], (unsigned long long)cnt);
            }
        }
    }
    __syncthreads();
    if (stats && threadIdx.x == 0) {
        if (s_acc[0]) atomicAdd(&stats[0], s_acc[0]);
        if (s_acc[1]) atomicAdd(&stats[1], s_acc[1]);
        if (s_acc[2]) atomicAdd(&stats[3], s_acc[2]);
        if (blockIdx.x == 0) atomicAdd(&stats[2], (unsigned long long)nblocks);
    }
}

// One wave per line.  Line `ln` of the plane `pl` reads kinds[pl * plane + ln * line_stride + k * elem_stride],
// k = 0 .. len-1, and writes the partial (kind 1) and full (kind 2) lists of that line.
__global__ __launch_bounds__(64) void compact_lines_kernel(
    const uint8_t* __restrict__ kinds, int nlines, int len, long long plane, long long line_stride,
    long long elem_stride, int32_t* __restrict__ num_partial, int32_t* __restrict__ idx_partial,
    int32_t* __restrict__ num_full, int32_t* __restrict__ idx_full) {
    const int lane = threadIdx.x;
    const long long line = blockIdx.x;                  // global line = pl * nlines + ln
    const long long pl = line / nlines, ln = line % nlines;
    const uint8_t* src = kinds + pl * plane + ln * line_stride;
    int32_t* out_p = idx_partial + line * len;
    int32_t* out_f = idx_full + line * len;
    int np = 0, nf = 0;
    for (int k0 = 0; k0 < len; k0 += 64) {
        const int k = k0 + lane;
        const int kind = k < len ? src[(long long)k * elem_stride] : 0;
        const unsigned long long mp = __ballot(kind == 1), mf = __ballot(kind == 2);
        const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
        if (kind == 1) out_p[np + __popcll(mp & below)] = k;
        if (kind == 2) out_f[nf + __popcll(mf & below)] = k;
        np += __popcll(mp);
        nf += __popcll(mf);
    }
    for (int k = lane; k < len; k += 64) {
        if (k >= np) out_p[k] = 0;
        if (k >= nf) out_f[k] = 0;
    }
    if (lane == 0) {
        num_partial[line] = np;
        num_full[line] = nf;
    }
}

// Work order of one orientation: per plane, the lines sorted by descending num_a + num_b (ties by
// ascending index) with a bitonic sort of (kOrderCountMax - count, index) keys in LDS; more than
// kOrderMax lines are left in the fixed order (descending index if `reversed`, else ascending).
constexpr int kOrderMax = 8192, kOrderIdxBits = 13, kOrderCountMax = (1 << 18) - 1;
__global__ __launch_bounds__(256) void order_lines_kernel(const int32_t* __restrict__ num_a,
                                                          const int32_t* __restrict__ num_b, int n, int reversed,
                                                          int32_t* __restrict__ order) {
    __shared__ uint32_t keys[kOrderMax];
    const int64_t base = (int64_t)blockIdx.x * n;
    if (n > kOrderMax) {
        for (int i = threadIdx.x; i < n; i += 256) order[base + i] = reversed ? n - 1 - i : i;
        return;
    }
    int n_pad = 1;
    while (n_pad < n) n_pad <<= 1;
    for (int i = threadIdx.x; i < n_pad; i += 256) {
        uint32_t key = 0xffffffffu;
        if (i < n) {
            const int cnt = min(num_a[base + i] + num_b[base + i], kOrderCountMax);
            key = ((uint32_t)(kOrderCountMax - cnt) << kOrderIdxBits) | (uint32_t)i;
        }
        keys[i] = key;
    }
    __syncthreads();
    for (int k = 2; k <= n_pad; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < n_pad; i += 256) {
                const int partner = i ^ j;
                if (partner > i) {
                    const uint32_t x = keys[i], y = keys[partner];
                    const bool ascending = (i & k) == 0;
                    if ((x > y) == ascending) {
                        keys[i] = y;
                        keys[partner] = x;
                    }
                }
            }
            __syncthreads();
        }
    }
    for (int i = threadIdx.x; i < n; i += 256) order[base + i] = (int32_t)(keys[i] & ((1u << kOrderIdxBits) - 1));
}

__global__ void zero_stats_kernel(unsigned long long* stats) {
    if (threadIdx.x < 4) stats[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void paged_convert_kernel(
    const int32_t* __restrict__ num_blocks, const int32_t* __restrict__ indices, int Hm, int NR, int NC,
    const int32_t* __restrict__ page_table, long long pt_stride, int32_t* __restrict__ phys_indices,
    int32_t* __restrict__ phys2log, int n_pool_pages, long long total) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const long long line = e / NC;
    const int k = (int)(e % NC);
    const long long b = line / ((long long)Hm * NR);
    int32_t out = 0;
    if (k < num_blocks[line]) {
        const int32_t logical = indices[e];
        out = page_table[b * pt_stride + logical];
        if (phys2log && out >= 0 && out < n_pool_pages) phys2log[out] = logical;
    }
    phys_indices[e] = out;
}

template <uint32_t MASK>
static int launch_classify(const flexattn_mod_params& p, const flexattn_blockmask* bm, uint8_t* kinds,
                           unsigned long long* stats, hipStream_t st) {
    const int NR = (bm->q_len + bm->Bq - 1) / bm->Bq, NC = (bm->kv_len + bm->Bk - 1) / bm->Bk;
    const long long nblocks = (long long)bm->Bm * bm->Hm * NR * NC;
    const long long grid = (nblocks + kClassifyWaves - 1) / kClassifyWaves;
    hipLaunchKernelGGL(classify_blocks_kernel<MASK>, dim3((unsigned)grid), dim3(kClassifyWaves * 64), 0, st, p,
                       bm->Bm, bm->Hm, NR, NC, bm->Bq, bm->Bk, bm->q_len, bm->kv_len, kinds, stats);
    return FLEXATTN_OK;
}

}  // namespace flexattn

using namespace flexattn;

extern "C" int flexattn_blockmask_sizes(int32_t Bm, int32_t Hm, int32_t q_len, int32_t kv_len, int32_t Bq,
                                           int32_t Bk, flexattn_blockmask_counts* sizes) {
    if (!sizes || Bm <= 0 || Hm <= 0 || q_len <= 0 || kv_len <= 0 || Bq <= 0 || Bk <= 0)
        return FLEXATTN_ERR_INVALID_ARG;
    const int64_t NR = ((int64_t)q_len + Bq - 1) / Bq, NC = ((int64_t)kv_len + Bk - 1) / Bk;
    const int64_t planes = (int64_t)Bm * Hm;
    if (planes * NR * NC > (1ll << 31)) return FLEXATTN_ERR_UNSUPPORTED;
    sizes->NR = (int32_t)NR;
    sizes->NC = (int32_t)NC;
    sizes->kv_num_blocks = sizes->full_kv_num_blocks = planes * NR;
    sizes->kv_indices = sizes->full_kv_indices = planes * NR * NC;
    sizes->q_num_blocks = sizes->full_q_num_blocks = planes * NC;
    sizes->q_indices = sizes->full_q_indices = planes * NC * NR;
    sizes->kv_order = planes * NR;
    sizes->q_order = planes * NC;
    return FLEXATTN_OK;
}

extern "C" size_t flexattn_blockmask_workspace_bytes(int32_t Bm, int32_t Hm, int32_t q_len, int32_t kv_len,
                                                     int32_t Bq, int32_t Bk) {
    if (Bm <= 0 || Hm <= 0 || q_len <= 0 || kv_len <= 0 || Bq <= 0 || Bk <= 0) return 0;
    const size_t NR = ((size_t)q_len + Bq - 1) / Bq, NC = ((size_t)kv_len + Bk - 1) / Bk;
    return ((size_t)Bm * Hm * NR * NC + 255) & ~(size_t)255;
}

extern "C" int flexattn_blockmask_build(uint32_t mask_id, const flexattn_mod_params* params,
                                        const flexattn_blockmask* bm, int64_t* stats, void* ws, size_t ws_bytes,
                                        void* stream) {
    if (!bm || !ws) return FLEXATTN_ERR_INVALID_ARG;
    if (bm->Bm <= 0 || bm->Hm <= 0 || bm->q_len <= 0 || bm->kv_len <= 0 || bm->Bq <= 0 || bm->Bk <= 0)
        return FLEXATTN_ERR_INVALID_ARG;
    if (!bm->kv_num_blocks || !bm->kv_indices || !bm->full_kv_num_blocks || !bm->full_kv_indices ||
        !bm->q_num_blocks || !bm->q_indices || !bm->full_q_num_blocks || !bm->full_q_indices)
        return FLEXATTN_ERR_INVALID_ARG;
    int rc = check_mod_params(mask_id, 0, params);
    if (rc != FLEXATTN_OK) return rc;
    if ((rc = check_canvas(mask_id, params, bm->q_len, bm->kv_len)) != FLEXATTN_OK) return rc;
    const int NR = (bm->q_len + bm->Bq - 1) / bm->Bq, NC = (bm->kv_len + bm->Bk - 1) / bm->Bk;
    const long long nblocks = (long long)bm->Bm * bm->Hm * NR * NC;
    if (nblocks > (1ll << 31) || (long long)bm->Bq * bm->Bk > (1ll << 24)) return FLEXATTN_ERR_UNSUPPORTED;
    if (ws_bytes < flexattn_blockmask_workspace_bytes(bm->Bm, bm->Hm, bm->q_len, bm->kv_len, bm->Bq, bm->Bk))
        return FLEXATTN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    flexattn_mod_params p = {};
    if (params) p = *params;
    uint8_t* kinds = (uint8_t*)ws;
    unsigned long long* st_dev = (unsigned long long*)stats;
    if (st_dev) hipLaunchKernelGGL(zero_stats_kernel, dim3(1), dim3(64), 0, st, st_dev);

    // The block classifier is instantiated for every mask the two-term encoding can express with
    // the primitives below; unknown combinations are rejected rather than approximated.
    switch (mask_id) {
#define CASE(M) case M: launch_classify<M>(p, bm, kinds, st_dev, st); break;
        CASE(FLEXATTN_MASK_NONE)
        CASE(FLEXATTN_MASK_CAUSAL)
        CASE(FLEXATTN_MASK_SLIDING_WINDOW)
        CASE(FLEXATTN_MASK_SWA_CAUSAL)
        CASE(FLEXATTN_MASK_DOCUMENT)
        CASE(FLEXATTN_MASK_DOCUMENT_CAUSAL)
        CASE(FLEXATTN_MASK_PREFIX_LM)
        CASE(FLEXATTN_MASK_SWA_CAUSAL_OR_PREFIX)
        CASE(FLEXATTN_MASK_CTX_LEN)
        CASE(FLEXATTN_MASK_NEIGHBORHOOD)
        CASE((FLEXATTN_M_CTX_LEN | FLEXATTN_M_CAUSAL))
        CASE((FLEXATTN_MASK_SWA_CAUSAL | FLEXATTN_M_DOCUMENT))
#undef CASE
        default: return FLEXATTN_ERR_UNSUPPORTED;
    }
    FLEXATTN_HIP_TRY(hipGetLastError());

    const long long planes = (long long)bm->Bm * bm->Hm;
    // rows of blocks: line = row i, elements = columns j
    hipLaunchKernelGGL(compact_lines_kernel, dim3((unsigned)(planes * NR)), dim3(64), 0, st, kinds, NR, NC,
                       (long long)NR * NC, (long long)NC, 1ll, bm->kv_num_blocks, bm->kv_indices,
                       bm->full_kv_num_blocks, bm->full_kv_indices);
    // columns of blocks: line = column j, elements = rows i
    hipLaunchKernelGGL(compact_lines_kernel, dim3((unsigned)(planes * NC)), dim3(64), 0, st, kinds, NC, NR,
                       (long long)NR * NC, 1ll, (long long)NC, bm->q_num_blocks, bm->q_indices,
                       bm->full_q_num_blocks, bm->full_q_indices);
    if (bm->kv_order)
        hipLaunchKernelGGL(order_lines_kernel, dim3((unsigned)planes), dim3(256), 0, st, bm->kv_num_blocks,
                           bm->full_kv_num_blocks, NR, 1, bm->kv_order);
    if (bm->q_order)
        hipLaunchKernelGGL(order_lines_kernel, dim3((unsigned)planes), dim3(256), 0, st, bm->q_num_blocks,
                           bm->full_q_num_blocks, NC, 0, bm->q_order);
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}

extern "C" int flexattn_paged_convert_blockmask(const int32_t* num_blocks, const int32_t* indices, int32_t Bm,
                                                int32_t Hm, int32_t NR, int32_t NC, const int32_t* page_table,
                                                int64_t pt_stride, int32_t* phys_indices, int32_t* phys2log,
                                                int32_t n_pool_pages, void* stream) {
    if (!num_blocks || !indices || !page_table || !phys_indices) return FLEXATTN_ERR_INVALID_ARG;
    if (Bm <= 0 || Hm <= 0 || NR <= 0 || NC <= 0 || pt_stride < NC || n_pool_pages <= 0)
        return FLEXATTN_ERR_INVALID_ARG;
    const long long total = (long long)Bm * Hm * NR * NC;
    hipLaunchKernelGGL(paged_convert_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, num_blocks, indices, Hm, NR, NC, page_table, (long long)pt_stride,
                       phys_indices, phys2log, n_pool_pages, total);
    FLEXATTN_HIP_TRY(hipGetLastError());
    return FLEXATTN_OK;
}
