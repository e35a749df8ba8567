/*
 * flexattn.h -- C ABI of libflexattn: the FlexAttention hot path on AMD MI355X (gfx950).
 *
 * Paper: "Flex Attention: a Programming Model for Generating Optimized Attention Kernels"
 * (arXiv 2412.05496).  The library computes
 *
 *     FlexAttention(Q, K, V) = softmax( mod( Q K^T * scale ) ) V            (Eq. 1)
 *
 * where mod applies a score_mod to every scaled score and then sets the scores whose
 * mask_mod is false to -inf (section 3.1), with work skipped per block through a BlockMask
 * (section 4.2) and a paged KV cache addressed through a page table (section 5.1).
 *
 * General conventions
 *   - Every entry point returns an int status (FLEXATTN_OK or a negative FLEXATTN_ERR_*),
 *     never throws and never aborts.  flexattn_strerror() names a status;
 *     flexattn_last_hip_error() returns the hipError_t behind the last FLEXATTN_ERR_HIP on
 *     the calling thread.
 *   - All tensor, BlockMask and workspace pointers are DEVICE pointers owned by the caller.
 *     The library allocates and frees nothing.  Pointers inside flexattn_mod_params are
 *     device pointers as well.  Descriptor structs themselves are host memory, read during
 *     the call only.
 *   - Every launch is asynchronous on the caller's stream (`stream` is a hipStream_t passed
 *     as void*; NULL is the default stream).  No call synchronises, copies or clears memory
 *     through the runtime: a call only launches kernels, so it may be made on a stream that
 *     is being captured into a HIP graph (for flexattn_paged_decode_static after one call
 *     outside a capture, which looks up the static array's address).
 *   - Float tensors are bf16 (Q, K, V, O, dO, dQ, dK, dV) unless stated; LSE is fp32.
 *     Head dimension D is 64 or 128 and has unit stride; other strides are in ELEMENTS.
 *   - Grouped-query attention: query head hq reads KV head hq / (Hq / Hkv); mods see hq.
 *   - A query row whose keys are all masked yields O = 0, LSE = -inf and zero gradients.
 *   - Results are deterministic run to run (no floating-point atomics), with the one exception
 *     stated at flexattn_backward_captured.
 */
#ifndef FLEXATTN_H
#define FLEXATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---------------------------------------------------------------- */
#define FLEXATTN_OK               0
#define FLEXATTN_ERR_INVALID_ARG  (-1)   /* null pointer, non-positive size, bad stride, ...      */
#define FLEXATTN_ERR_UNSUPPORTED  (-2)   /* D, block size or (mask, score) pair not compiled in   */
#define FLEXATTN_ERR_WORKSPACE    (-3)   /* workspace smaller than *_workspace_bytes() asks for   */
#define FLEXATTN_ERR_HIP          (-4)   /* a HIP call failed; see flexattn_last_hip_error()      */

/* ---- mask_mod (sections 3.1, 3.2) --------------------------------------------------
 * A mask_mod is a boolean function of (b, h, q_idx, kv_idx).  The library offers the
 * paper's primitives and their and_mask / or_mask compositions as a two-term disjunction
 * of conjunctions:   mask = AND(term0 primitives)  OR  AND(term1 primitives)
 * encoded as  term0 | (term1 << 8).  term0 == 0 means "no mask" (always true); term1 == 0
 * means "no second term".
 */
#define FLEXATTN_M_CAUSAL          1u   /* q_idx >= kv_idx                                        */
#define FLEXATTN_M_SLIDING_WINDOW  2u   /* q_idx - kv_idx <= window   (one-sided, as the paper)   */
#define FLEXATTN_M_DOCUMENT        4u   /* doc_ids[b, q_idx] == doc_ids[b, kv_idx]                */
#define FLEXATTN_M_PREFIX          8u   /* kv_idx < prefix_len                                    */
#define FLEXATTN_M_CTX_LEN        16u   /* kv_idx < ctx_lens[b]                                   */
#define FLEXATTN_M_NEIGHBORHOOD   32u   /* neighborhood attention on a 2-D canvas (appendix "NA"):
                                           the tokens are the pixels of an na_width x na_height
                                           canvas; a query pixel sees the na_kernel x na_kernel
                                           pixels nearest to it (the window centred on it, moved
                                           inside the canvas where it would stick out)           */
#define FLEXATTN_MASK_OR(term0, term1) ((uint32_t)(term0) | ((uint32_t)(term1) << 8))

#define FLEXATTN_MASK_NONE                  0u
#define FLEXATTN_MASK_CAUSAL                FLEXATTN_M_CAUSAL
#define FLEXATTN_MASK_SLIDING_WINDOW        FLEXATTN_M_SLIDING_WINDOW
#define FLEXATTN_MASK_SWA_CAUSAL            (FLEXATTN_M_CAUSAL | FLEXATTN_M_SLIDING_WINDOW)
#define FLEXATTN_MASK_DOCUMENT              FLEXATTN_M_DOCUMENT
#define FLEXATTN_MASK_DOCUMENT_CAUSAL       (FLEXATTN_M_DOCUMENT | FLEXATTN_M_CAUSAL)
#define FLEXATTN_MASK_PREFIX_LM             FLEXATTN_MASK_OR(FLEXATTN_M_CAUSAL, FLEXATTN_M_PREFIX)
#define FLEXATTN_MASK_SWA_CAUSAL_OR_PREFIX  FLEXATTN_MASK_OR(FLEXATTN_MASK_SWA_CAUSAL, FLEXATTN_M_PREFIX)
#define FLEXATTN_MASK_CTX_LEN               FLEXATTN_M_CTX_LEN
#define FLEXATTN_MASK_CTX_LEN_WINDOW        (FLEXATTN_M_CTX_LEN | FLEXATTN_M_SLIDING_WINDOW)
#define FLEXATTN_MASK_NEIGHBORHOOD          FLEXATTN_M_NEIGHBORHOOD

/* Token order of the canvas for NEIGHBORHOOD (pixel (x, y) -> token index):
 *   ROW_MAJOR  y * W + x
 *   TILED      T x T squares, the squares row after row, the pixels of a square row after row:
 *              ((y / T) * (W / T) + x / T) * T * T + (y % T) * T + x % T
 *   MORTON     the bits of x and y interleaved, x in the even positions (Z-order curve) */
#define FLEXATTN_NA_ROW_MAJOR 0
#define FLEXATTN_NA_TILED     1
#define FLEXATTN_NA_MORTON    2

/* ---- score_mod (section 3.1; nested score_mods, section 1.1) -------------------------
 * A bit set; the selected modifications are applied to the scaled score in this order:
 *   ALIBI     score + alibi_bias[h] * (q_idx - kv_idx)
 *   REL_BIAS  score + rel_bias[h, clamp(q_idx - kv_idx, 0, rel_len - 1)]
 *   SOFTCAP   softcap * tanh(score / softcap)
 */
#define FLEXATTN_SCORE_IDENTITY  0u
#define FLEXATTN_SCORE_ALIBI     1u
#define FLEXATTN_SCORE_REL_BIAS  2u
#define FLEXATTN_SCORE_SOFTCAP   4u

/* Values the mods capture.  Only the fields a selected mod uses are read. */
typedef struct flexattn_mod_params {
    int32_t        window;        /* SLIDING_WINDOW                                            */
    int32_t        prefix_len;    /* PREFIX                                                    */
    float          softcap;       /* SOFTCAP, > 0                                              */
    int32_t        rel_len;       /* REL_BIAS: row length of rel_bias (<= 1024)                */
    const int32_t* doc_ids;       /* DOCUMENT: [B, seq] token -> document index; read at the
                                     positions the mods see (q_idx + q_offsets[b], kv_idx)       */
    int64_t        doc_stride_b;  /*           elements between batches (0 = shared row)       */
    const float*   alibi_bias;    /* ALIBI: [Hq] fp32                                          */
    const float*   rel_bias;      /* REL_BIAS: [Hq, rel_len] fp32, row-major                   */
    const int32_t* ctx_lens;      /* CTX_LEN: [B] int32                                        */
    const int32_t* q_offsets;     /* nullable [B] int32: every mod sees q_idx + q_offsets[b], the
                                     offset conversion for inference of section 5.2 (number of
                                     tokens of sequence b processed before this call's first
                                     query); BlockMask build, forward and backward honour it    */
    int32_t        na_width;      /* NEIGHBORHOOD: canvas W x H; q_len == kv_len == W * H <= 2^20 */
    int32_t        na_height;
    int32_t        na_kernel;     /*   odd K, 1 <= K <= min(W, H): K x K keys per query          */
    int32_t        na_layout;     /*   FLEXATTN_NA_*                                              */
    int32_t        na_tile;       /*   TILED: T, a power of two that divides W and H;
                                       MORTON needs W == H == a power of two                     */
} flexattn_mod_params;

/* A 4-D tensor [batch, head, seq, D] with unit stride in D.  ptr is 16-byte aligned, the
 * strides are multiples of 8 elements, stride_s >= D, and one (batch, head) slice spans less
 * than 2 GiB ((seq_len - 1) * stride_s + D elements): rows are addressed with 32-bit offsets.
 * A larger slice is refused with FLEXATTN_ERR_UNSUPPORTED. */
typedef struct flexattn_tensor {
    void*   ptr;
    int64_t stride_b, stride_h, stride_s;   /* in elements */
} flexattn_tensor;

/* ---- BlockMask (section 4.2) -------------------------------------------------------
 * The score matrix is cut into Bq x Bk blocks: NR = ceil(q_len / Bq) rows and
 * NC = ceil(kv_len / Bk) columns of blocks.  A block with every scalar masked is skipped; one
 * with none masked is FULL (mask_mod is not evaluated in it); any other is PARTIAL.  Where a
 * length is no multiple of the block size, the part of the last block that lies outside the
 * score matrix counts as masked: such a block is PARTIAL or skipped, never FULL.
 *
 *   kv_num_blocks      [Bm, Hm, NR]      number of PARTIAL blocks in each row of blocks
 *   kv_indices         [Bm, Hm, NR, NC]  their column indices, ascending; entries past the
 *                                        count are 0
 *   full_kv_num_blocks / full_kv_indices the same for FULL blocks
 *   q_num_blocks       [Bm, Hm, NC]      PARTIAL blocks of each column of blocks
 *   q_indices          [Bm, Hm, NC, NR]  their row indices (the transpose the backward walks)
 *   full_q_num_blocks / full_q_indices   the same for FULL blocks
 *
 * Bm is 1 (the mask ignores b) or the batch size; Hm is 1 or the number of QUERY heads.
 * All arrays are int32, dense, row-major.
 *
 * Work order (nullable, optional; not in the paper): the workgroups of a launch start in index
 * order and a launch ends with its slowest workgroup, so for masks whose rows differ in length
 * (documents, sliding windows with a prefix, ...) the kernels take the rows of blocks longest first:
 *   kv_order [Bm, Hm, NR]  the rows of blocks sorted by descending number of listed blocks
 *                          (kv_num_blocks + full_kv_num_blocks), ties by ascending index
 *   q_order  [Bm, Hm, NC]  the same for the columns of blocks (q_num_blocks + full_q_num_blocks)
 * A line count above 8192 is not sorted: kv_order is then NR-1, ..., 0 and q_order 0, ..., NC-1
 * (the best fixed orders for causal-like masks).  flexattn_blockmask_build fills the arrays that
 * are non-NULL; forward / backward use them when present and those fixed orders otherwise.  The
 * order changes which workgroup computes which block of rows, never a result.
 */
typedef struct flexattn_blockmask {
    int32_t  Bm, Hm, q_len, kv_len, Bq, Bk;
    int32_t* kv_num_blocks;
    int32_t* kv_indices;
    int32_t* full_kv_num_blocks;
    int32_t* full_kv_indices;
    int32_t* q_num_blocks;
    int32_t* q_indices;
    int32_t* full_q_num_blocks;
    int32_t* full_q_indices;
    int32_t* kv_order;      /* nullable */
    int32_t* q_order;       /* nullable */
} flexattn_blockmask;

/* Geometry and element counts of the eight arrays of a BlockMask (section 4.2), so that a caller
 * can allocate them without repeating the library's rounding: NR = ceil(q_len / Bq),
 * NC = ceil(kv_len / Bk); counts are in int32 elements, in the order of flexattn_blockmask
 * (the eight lists, then the two optional order arrays).
 * Host-only arithmetic.  FLEXATTN_ERR_INVALID_ARG for a non-positive argument or a NULL `sizes`,
 * FLEXATTN_ERR_UNSUPPORTED if Bm * Hm * NR * NC exceeds 2^31 (the limit of flexattn_blockmask_build). */
typedef struct flexattn_blockmask_counts {
    int32_t NR, NC;
    int64_t kv_num_blocks, kv_indices, full_kv_num_blocks, full_kv_indices;
    int64_t q_num_blocks, q_indices, full_q_num_blocks, full_q_indices;
    int64_t kv_order, q_order;
} flexattn_blockmask_counts;
int flexattn_blockmask_sizes(int32_t Bm, int32_t Hm, int32_t q_len, int32_t kv_len, int32_t Bq, int32_t Bk,
                                flexattn_blockmask_counts* sizes);

/* Problem shape of flex_attention (section 2.1). */
typedef struct flexattn_dims {
    int32_t B, Hq, Hkv, q_len, kv_len, D;
} flexattn_dims;

const char* flexattn_strerror(int status);
int         flexattn_last_hip_error(void);
int         flexattn_version(void);

/* 1 if forward/backward kernels for this (mask, score, D) were compiled into the library.
 * The BlockMask builder accepts every mask listed above; forward and backward are template
 * instantiations over a table of (mask_id, score_id) pairs (csrc/flex_common.h,
 * FLEXATTN_FOR_EACH_VARIANT): the pairs of the paper's examples and benchmarks.  The mask and score
 * functors compose freely, so another pair is one more line in that table and a rebuild; a pair
 * that is not in it is refused with FLEXATTN_ERR_UNSUPPORTED, never approximated. */
int flexattn_is_supported(uint32_t mask_id, uint32_t score_id, int32_t D);

/* ---- BlockMask construction (section 4.2; create_block_mask, section 1.1) ----------
 * Evaluates mask_mod on every (q_idx, kv_idx) of every block -- brute force, so the result
 * is exact for any mask; a block that the mask's index comparisons alone settle (every pair
 * hidden, or none) is classified without the enumeration -- and fills the eight arrays of
 * `bm` (both orientations).
 * Any q_len, kv_len >= 1.
 *   stats  nullable device int64[4]: {#partial blocks, #full blocks, #blocks, #unmasked
 *          scalars}, summed over Bm * Hm.
 *   ws     device workspace of at least flexattn_blockmask_workspace_bytes() bytes.
 */
size_t flexattn_blockmask_workspace_bytes(int32_t Bm, int32_t Hm, int32_t q_len, int32_t kv_len,
                                          int32_t Bq, int32_t Bk);
int flexattn_blockmask_build(uint32_t mask_id, const flexattn_mod_params* params,
                             const flexattn_blockmask* bm, int64_t* stats,
                             void* ws, size_t ws_bytes, void* stream);

/* ---- forward (Eq. 1; forward template of section 4.1; block skipping, full-block
 * optimisation and indirect block access of section 4.2) -----------------------------
 * O [B, Hq, q_len, D] bf16 and LSE [B, Hq, q_len] fp32 (natural log of the sum of exp of the
 * modified, masked, scaled scores; dense, row-major).  `bm` must have been built for the
 * same mask_id/params, with Bq in {64, 128} and Bk in {64, 128}.  Full blocks are processed
 * without evaluating mask_mod, partial blocks with it, all other blocks not at all.
 */
int flexattn_forward(const flexattn_dims* dims,
                     const flexattn_tensor* Q, const flexattn_tensor* K, const flexattn_tensor* V,
                     uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                     const flexattn_blockmask* bm, float scale,
                     const flexattn_tensor* O, float* LSE, void* stream);

/* ---- backward (backward template of section 4.1) -----------------------------------
 * With P = softmax of the modified masked scores recomputed from LSE:
 *   dV = P^T dO;  dP = dO V^T;  dS' = P * (dP - rowsum(dO * O));  dS = dS' * d score_mod/d s;
 *   dQ = scale * dS K;  dK = scale * dS^T Q;  dK and dV are summed over the Hq / Hkv query
 * heads that share a KV head.  Gradients with respect to captured buffers (alibi_bias,
 * rel_bias) come from flexattn_backward_captured.  dQ [B,Hq,q_len,D], dK, dV [B,Hkv,kv_len,D] bf16.
 *   ws     device workspace of at least flexattn_backward_workspace_bytes(dims) bytes.
 */
size_t flexattn_backward_workspace_bytes(const flexattn_dims* dims);
int flexattn_backward(const flexattn_dims* dims,
                      const flexattn_tensor* Q, const flexattn_tensor* K, const flexattn_tensor* V,
                      const flexattn_tensor* O, const flexattn_tensor* dO, const float* LSE,
                      uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                      const flexattn_blockmask* bm, float scale,
                      const flexattn_tensor* dQ, const flexattn_tensor* dK, const flexattn_tensor* dV,
                      void* ws, size_t ws_bytes, void* stream);

/* The same computation by stage, for callers that need only part of the gradients (frozen K/V:
 * DQ only; frozen Q: DKDV only) or that time the stages separately.  DELTA fills the workspace
 * from (O, dO, LSE) and must have run on the same workspace before DKDV or DQ; DKDV writes dK
 * and dV; DQ writes dQ.  Output tensors of stages that are not selected may be NULL.
 * flexattn_backward() is flexattn_backward_stages(..., FLEXATTN_BWD_ALL).
 */
#define FLEXATTN_BWD_DELTA 1u
#define FLEXATTN_BWD_DKDV  2u
#define FLEXATTN_BWD_DQ    4u
#define FLEXATTN_BWD_ALL   7u
int flexattn_backward_stages(const flexattn_dims* dims,
                             const flexattn_tensor* Q, const flexattn_tensor* K, const flexattn_tensor* V,
                             const flexattn_tensor* O, const flexattn_tensor* dO, const float* LSE,
                             uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                             const flexattn_blockmask* bm, float scale,
                             const flexattn_tensor* dQ, const flexattn_tensor* dK, const flexattn_tensor* dV,
                             void* ws, size_t ws_bytes, void* stream, uint32_t stages);

/* The same gradients with dS kept in device memory instead of being recomputed (a trade of HBM
 * capacity and bandwidth for arithmetic; the result is as deterministic as flexattn_backward's, and
 * equal to it up to the rounding of dS to bf16, which both take before the dQ and dK products).
 * The dK/dV kernel writes the gradient of the scores of every non-empty block it visits (section
 * 4.2's transposed walk) and dQ = scale * dS K is then one block-sparse product over the written
 * blocks: the backward executes the five matrix products of its definition instead of seven.
 * Whether it pays depends on what the recomputation costs against 4 bytes of HBM traffic per
 * unmasked score: measured on MI355X it is 9-12 % faster at D = 128 (soft-cap or relative bias),
 * 23-25 % faster for masks whose blocks are mostly PARTIAL (neighborhood attention, D = 64), even
 * at D = 64 with a soft-cap, and 15-25 % slower at D = 64 with a plain score_mod.
 *   n_blocks  capacity, in blocks of Bq x Bk scores: at least the number of non-empty (PARTIAL +
 *             FULL) blocks of the BlockMask, all planes together -- stats[0] + stats[1] of
 *             flexattn_blockmask_build.  A smaller value gives wrong gradients for the blocks that
 *             do not fit (slots are clamped; nothing is accessed outside the workspace).
 *   ws        device workspace, 256-byte aligned, of flexattn_backward_stored_workspace_bytes()
 *             bytes: the row scalars, one int32 per block position of the BlockMask grid, and
 *             2 * Bq * Bk bytes per block and per head that does not share the BlockMask plane with
 *             an equal (b, hq) -- B * Hq * n_blocks blocks for a broadcast BlockMask (config 2:
 *             64 heads x 4160 blocks x 16 KiB = 4.4 GB).  Returns 0 for invalid arguments.
 *   stages    as in flexattn_backward_stages (FLEXATTN_BWD_ALL for the whole backward): DELTA also
 *             numbers the blocks and must have run on the workspace first; DKDV writes dK, dV and
 *             the dS blocks; DQ reads them, so it must follow DKDV on the same workspace.
 * All other arguments and errors as flexattn_backward.
 */
size_t flexattn_backward_stored_workspace_bytes(const flexattn_dims* dims, const flexattn_blockmask* bm,
                                                int64_t n_blocks);
int flexattn_backward_stored(const flexattn_dims* dims,
                             const flexattn_tensor* Q, const flexattn_tensor* K, const flexattn_tensor* V,
                             const flexattn_tensor* O, const flexattn_tensor* dO, const float* LSE,
                             uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                             const flexattn_blockmask* bm, float scale,
                             const flexattn_tensor* dQ, const flexattn_tensor* dK, const flexattn_tensor* dV,
                             int64_t n_blocks, void* ws, size_t ws_bytes, void* stream, uint32_t stages);

/* Gradients of the tensors the score_mod captures (the bias of the ALiBi example, the table of the
 * relative-bias example, section 3.1), which flexattn_backward does not produce:
 *   d_alibi_bias [Hq] fp32          sum over b, q, kv of dS * (q_idx - kv_idx)
 *   d_rel_bias   [Hq, rel_len] fp32 sum of dS over the pairs that read each table entry
 * with dS the gradient of the loss with respect to the biased score (before a soft-cap that
 * follows it).  Each is written (not accumulated) if the score_id selects its mod and must then
 * be non-NULL; FLEXATTN_ERR_UNSUPPORTED if the score_mod captures nothing.  Arguments as in
 * flexattn_backward (O and LSE from the forward); ws of at least
 * flexattn_backward_captured_workspace_bytes() bytes.  The sums over one workgroup's pairs use
 * LDS atomics, so the last bits can differ between runs; the sum over workgroups has a fixed order.
 */
size_t flexattn_backward_captured_workspace_bytes(const flexattn_dims* dims, const flexattn_blockmask* bm,
                                                  uint32_t score_id, const flexattn_mod_params* params);
int flexattn_backward_captured(const flexattn_dims* dims,
                               const flexattn_tensor* Q, const flexattn_tensor* K, const flexattn_tensor* V,
                               const flexattn_tensor* O, const flexattn_tensor* dO, const float* LSE,
                               uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                               const flexattn_blockmask* bm, float scale,
                               float* d_alibi_bias, float* d_rel_bias,
                               void* ws, size_t ws_bytes, void* stream);

/* ---- paged attention (section 5.1) --------------------------------------------------
 * BlockMask conversion: each of the first num_blocks[b,h,i] entries j of indices[b,h,i,:]
 * (logical KV block numbers; Bk == page size) becomes page_table[b, j]; the tail stays 0 and
 * the counts are unchanged.  phys2log (nullable, int32[n_pool_pages], pre-filled by the
 * caller, e.g. with -1) receives phys2log[page_table[b, j]] = j for every converted entry:
 * the vector that turns a physical KV index back into the logical one the user's mods expect.
 *   num_blocks [Bm,Hm,NR], indices/phys_indices [Bm,Hm,NR,NC], page_table [Bm, pt_stride].
 */
int flexattn_paged_convert_blockmask(const int32_t* num_blocks, const int32_t* indices,
                                     int32_t Bm, int32_t Hm, int32_t NR, int32_t NC,
                                     const int32_t* page_table, int64_t pt_stride,
                                     int32_t* phys_indices, int32_t* phys2log, int32_t n_pool_pages,
                                     void* stream);

/* Paged forward: a chunk of q_len query tokens per sequence against a paged KV cache (chunked
 * prefill: fused indirect access of section 5.1 with the offset conversion of section 5.2).
 * The computation is that of flexattn_forward over the LOGICAL BlockMask `bm`, which must have
 * Bm == B (every sequence has its own pages) and Bk == page_size, and is normally built with
 * params->q_offsets[b] = number of tokens of sequence b that precede the chunk.  K and V rows
 * come from the pools: the page of the j-th entry of a list of `bm` is the j-th entry of the
 * converted list (phys_kv_indices beside bm->kv_indices, phys_full_kv_indices beside
 * bm->full_kv_indices; same shapes, made by flexattn_paged_convert_blockmask), so the kernel
 * never looks the page table up and the mods keep seeing the logical kv_idx.  Pages are whole
 * blocks: keys past the end of a sequence inside its last page must be hidden by the mask (a
 * causal mask with q_offsets does so).
 *   dims->kv_len    logical KV length `bm` was built for (a multiple of page_size)
 *   K_pool, V_pool  [n_pool_pages, Hkv, page_size, D] bf16, dense; page_size is 64 or 128
 *   converted entries are clamped to [0, n_pool_pages): a wrong entry reads the wrong page, never
 *   outside the pools.
 * O, LSE as in flexattn_forward.
 */
int flexattn_paged_forward(const flexattn_dims* dims, const flexattn_tensor* Q,
                           const void* K_pool, const void* V_pool, int32_t page_size, int32_t n_pool_pages,
                           uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                           const flexattn_blockmask* bm, const int32_t* phys_kv_indices,
                           const int32_t* phys_full_kv_indices, float scale,
                           const flexattn_tensor* O, float* LSE, void* stream);

/* Paged decode: one query token per sequence against a paged KV cache (decoding template of
 * section 4.1 + fused indirect access of section 5.1), split over KV and combined.
 *   Q       [nseq, Hq, D] bf16 (stride_q_seq elements between sequences, heads contiguous)
 *   K_pool, V_pool  [n_pool_pages, Hkv, page_size, D] bf16, dense
 *   page_table [nseq, pt_stride] int32: logical page j of sequence b lives in pool page
 *              page_table[b, j]; only the first ceil(ctx_lens[b] / page_size) entries are read
 *   ctx_lens   [nseq] int32: visible keys are kv_idx < ctx_lens[b] (0 is legal: O = 0,
 *              LSE = -inf).  score_mods see q_idx = ctx_lens[b] - 1 and the LOGICAL kv_idx.
 *   O [nseq, Hq, D] bf16 dense; LSE nullable [nseq, Hq] fp32.
 * page_size must be a power of two from 16 to 1024; Hq / Hkv <= 16; max_pages * page_size <= 2^30.
 * Device-side values are not trusted: a context length outside [0, max_pages * page_size] is clamped to
 * that range and a page id outside [0, n_pool_pages) to the nearest valid page, so that wrong tables
 * give wrong rows and never an access outside the table, the pools or the workspace.
 * The KV range is cut into splits of 128 ... 1024 keys, one wave each; the split length is chosen
 * from nseq * Hkv * max_pages * page_size so that the launch still fills the chip when the batch is
 * small (flexattn_paged_decode_workspace_bytes accounts for it).  mask_id: FLEXATTN_MASK_CTX_LEN (which, with the query at
 * q_idx = ctx_len - 1, is also the causal mask of a decode step: the offset conversion of section 5.2) or
 * FLEXATTN_MASK_CTX_LEN_WINDOW (additionally q_idx - kv_idx <= params->window; splits wholly below the
 * window are skipped).
 */
typedef struct flexattn_decode_dims {
    int32_t nseq, Hq, Hkv, D, page_size, max_pages, n_pool_pages;
} flexattn_decode_dims;

size_t flexattn_paged_decode_workspace_bytes(const flexattn_decode_dims* dims);
int flexattn_paged_decode(const flexattn_decode_dims* dims,
                          const void* Q, int64_t stride_q_seq,
                          const void* K_pool, const void* V_pool,
                          const int32_t* page_table, int64_t pt_stride, const int32_t* ctx_lens,
                          uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                          float scale, void* O, float* LSE,
                          void* ws, size_t ws_bytes, void* stream);

/* ---- measurement aids ------------------------------------------------------------------
 * What the chip sustains for the two resources the hot path is bound by, from the simplest kernels
 * that can reach them (bench.py times them with events and reports the library's kernels against
 * these rates beside the datasheet peaks).  Asynchronous on `stream`, like every other call.
 *   flexattn_probe_mfma         512 workgroups of 4 waves (two waves per SIMD) issue 16 * iters
 *                               32x32x16 bf16 MFMAs each on register operands;
 *                               flexattn_probe_mfma_flops(iters) is the FLOP count of one launch.
 *                               valu_mix = 1 puts behind every MFMA, independent of it, the vector
 *                               instructions the soft-capped forward spends per MFMA (4 multiply-adds,
 *                               3 transcendentals): the hot loop's instruction mix with nothing to
 *                               wait for; valu_mix = 2 does the same for the soft-capped backward
 *                               (3 multiply-adds, 2 transcendentals per MFMA of its two kernels).  random_operands != 0 feeds the MFMAs bf16 values of random
 *                               sign, exponent and mantissa instead of small integers and ones: the
 *                               chip's clock under load depends on how much the operands toggle.
 *                               clocks: nullable device int64[2 * flexattn_probe_mfma_waves()]; wave w
 *                               stores the core cycles and the 100 MHz ticks it spent in its loop
 *                               (their ratio is the sustained core clock in units of 100 MHz).
 *   flexattn_probe_stream_read  reads `bytes` bytes (device pointer, 16-byte aligned) once with
 *                               16-byte loads.
 * `sink` is a device float the kernels never really write (it keeps their work alive). */
double  flexattn_probe_mfma_flops(int64_t iters);
int32_t flexattn_probe_mfma_waves(void);
int     flexattn_probe_mfma(int64_t iters, int32_t valu_mix, int32_t random_operands, float* sink,
                            int64_t* clocks, void* stream);
int     flexattn_probe_stream_read(const void* src, size_t bytes, float* sink, void* stream);

/* flexattn_paged_decode without a workspace argument, for callers that cannot allocate device
 * memory: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * partial results live in an array inside the library's device image (one copy per GPU, held until
 * the process ends) of flexattn_paged_decode_static_capacity() bytes = 40 MiB -- enough for 64
 * sequences x 32 query heads x 32 splits at D = 128.  The call allocates and frees nothing; it
 * returns FLEXATTN_ERR_WORKSPACE, launching nothing, when
 * flexattn_paged_decode_workspace_bytes(dims) exceeds the capacity.  Arguments, results and every
 * other error as flexattn_paged_decode (same kernels, bit-identical output).
 * The FIRST call on each device looks the array's address up (hipGetSymbolAddress): make it before
 * a capture begins.  All calls on one GPU share the array: calls that may overlap there (different
 * streams, different threads) race -- serialise them or use flexattn_paged_decode with separate
 * workspaces.  Nothing in the array needs clearing between calls. */
size_t flexattn_paged_decode_static_capacity(void);
int flexattn_paged_decode_static(const flexattn_decode_dims* dims,
                                 const void* Q, int64_t stride_q_seq,
                                 const void* K_pool, const void* V_pool,
                                 const int32_t* page_table, int64_t pt_stride, const int32_t* ctx_lens,
                                 uint32_t score_id, uint32_t mask_id, const flexattn_mod_params* params,
                                 float scale, void* O, float* LSE, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXATTN_H */
