// Shared device/host pieces of libflexattn (gfx950 only): vector types, MFMA wrappers,
// the mask_mod / score_mod functors (paper sections 3.1 and 3.2) and host-side status helpers.
#pragma once

#include <type_traits>

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flexattn.h"

namespace flexattn {

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// D[32x32] += A[32x16] * B[16x32], bf16 inputs, fp32 accumulate.
// Operand layout (wave64): lane l supplies A[row = l % 32][k-slots of half l / 32] and
// B[k-slots of half l / 32][col = l % 32], eight bf16 each; the k-slot <-> k mapping is the same
// for A and B, so any consistent choice contracts correctly.
// Result layout: register r of lane l holds D[row = 8 * (r / 4) + 4 * (l / 32) + r % 4][col = l % 32].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of the 32x32 result tile held in register r by a lane of half `half` (= lane / 32).
__device__ __forceinline__ constexpr int crow(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>)
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// acc + lo(pair) + hi(pair) for a packed pair of bf16 values (v_dot2c_f32_bf16).
__device__ __forceinline__ float pair_sum_bf16(uint32_t pair, float acc) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, 0x3f803f80u),
                                           acc, false);
}

// Load of read-only data at a wave-uniform address: constant address space, so the compiler may
// use the scalar cache and keep the load off the vector memory counter.
__device__ __forceinline__ int32_t ldc(const int32_t* p) {
    return *(const __attribute__((address_space(4))) int32_t*)(uintptr_t)p;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Exchange a value with the lane 32 away (the other half of the wave).
__device__ __forceinline__ float swap_halves(float v) { return __shfl_xor(v, 32, 64); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 v;
    v[0] = (bf16)lo;
    v[1] = (bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// ---------------------------------------------------------------------------------------
// mask_mod: OR of up to two AND-terms over the primitive predicates.
// A MaskRow caches what depends only on (b, h, q_idx); operator() takes kv_idx.
// ---------------------------------------------------------------------------------------
// Token index -> pixel of the canvas, for the neighborhood mask (appendix, Neighborhood Attention).
struct CanvasOrder {
    int width, layout, tile_log2, tiles_x;
    float inv_width, inv_tiles_x;
    __device__ __forceinline__ explicit CanvasOrder(const flexattn_mod_params& p) {
        width = p.na_width;
        layout = p.na_layout;
        tile_log2 = p.na_tile > 0 ? 31 - __builtin_clz((unsigned)p.na_tile) : 0;
        tiles_x = width >> tile_log2;
        inv_width = fast_rcp((float)width);
        inv_tiles_x = fast_rcp((float)tiles_x);
    }
    // n = quot * d + rem for 0 <= n < 2^24: a float estimate of the quotient (off by one at most),
    // then one exact correction step
    __device__ __forceinline__ static void divmod(int n, int d, float inv_d, int& quot, int& rem) {
        int qq = (int)(((float)n + 0.5f) * inv_d);
        int rr = n - qq * d;
        const bool lo = rr < 0, hi = rr >= d;
        quot = qq + (hi ? 1 : 0) - (lo ? 1 : 0);
        rem = rr + (lo ? d : 0) - (hi ? d : 0);
    }
    // every second bit of v, packed (the inverse of interleaving with zeros)
    __device__ __forceinline__ static int even_bits(uint32_t v) {
        v &= 0x55555555u;
        v = (v | (v >> 1)) & 0x33333333u;
        v = (v | (v >> 2)) & 0x0f0f0f0fu;
        v = (v | (v >> 4)) & 0x00ff00ffu;
        v = (v | (v >> 8)) & 0x0000ffffu;
        return (int)v;
    }
    __device__ __forceinline__ void pixel(int n, int& x, int& y) const {
        if (layout == FLEXATTN_NA_MORTON) {
            x = even_bits((uint32_t)n);
            y = even_bits((uint32_t)n >> 1);
        } else if (layout == FLEXATTN_NA_TILED) {
            const int in_tile = n & ((1 << (2 * tile_log2)) - 1);
            int ty, tx;
            divmod(n >> (2 * tile_log2), tiles_x, inv_tiles_x, ty, tx);
            y = (ty << tile_log2) + (in_tile >> tile_log2);
            x = (tx << tile_log2) + (in_tile & ((1 << tile_log2) - 1));
        } else {
            divmod(n, width, inv_width, y, x);
        }
    }
};

struct NoCanvas {
    __device__ __forceinline__ explicit NoCanvas(const flexattn_mod_params&) {}
    __device__ __forceinline__ void pixel(int, int&, int&) const {}
};

template <uint32_t TERM>
struct MaskTermRow {
    int q, window, prefix_len, doc_q, ctx;
    const int32_t* doc_row;
    // NEIGHBORHOOD: the window of the query pixel, [x0, x0 + span] x [y0, y0 + span]
    std::conditional_t<(TERM & FLEXATTN_M_NEIGHBORHOOD) != 0, CanvasOrder, NoCanvas> canvas;
    int x0, y0, span;
    // doc_q_known >= 0: the caller already holds doc_ids[b, q_idx] (no table read here)
    __device__ __forceinline__ MaskTermRow(const flexattn_mod_params& p, int b, int /*h*/, int q_idx, int doc_q_known = -1)
        : canvas(p) {
        q = q_idx;
        window = p.window;
        prefix_len = p.prefix_len;
        doc_row = nullptr;
        doc_q = 0;
        ctx = 0;
        x0 = y0 = span = 0;
        if constexpr (TERM & FLEXATTN_M_NEIGHBORHOOD) {
            const int r = p.na_kernel >> 1;
            int qx, qy;
            canvas.pixel(q_idx, qx, qy);
            x0 = min(max(qx, r), p.na_width - 1 - r) - r;
            y0 = min(max(qy, r), p.na_height - 1 - r) - r;
            span = 2 * r;
        }
        if constexpr (TERM & FLEXATTN_M_DOCUMENT) {
            doc_row = p.doc_ids + (int64_t)b * p.doc_stride_b;
            doc_q = doc_q_known >= 0 ? doc_q_known : doc_row[q_idx];
        }
        if constexpr (TERM & FLEXATTN_M_CTX_LEN) ctx = p.ctx_lens[b];
    }
    __device__ __forceinline__ bool operator()(int kv) const {
        int doc_kv = 0;
        if constexpr (TERM & FLEXATTN_M_DOCUMENT) doc_kv = doc_row[kv];
        return eval(kv, doc_kv);
    }
    // Rectangle tests on q_lo <= q <= q_hi, kv_lo <= kv <= kv_hi, decided from the primitives that are
    // plain index comparisons: block_empty is true only if NO pair can pass this term, block_full only
    // if EVERY pair does (a term with a table lookup or the canvas decode is never declared full).
    __device__ __forceinline__ bool block_empty(int q_lo, int q_hi, int kv_lo, int kv_hi) const {
        bool e = false;
        if constexpr (TERM & FLEXATTN_M_CAUSAL) e = e || (q_hi < kv_lo);
        if constexpr (TERM & FLEXATTN_M_SLIDING_WINDOW) e = e || (q_lo - kv_hi > window);
        if constexpr (TERM & FLEXATTN_M_PREFIX) e = e || (kv_lo >= prefix_len);
        if constexpr (TERM & FLEXATTN_M_CTX_LEN) e = e || (kv_lo >= ctx);
        return e;
    }
    __device__ __forceinline__ bool block_full(int q_lo, int q_hi, int kv_lo, int kv_hi) const {
        if constexpr ((TERM & (FLEXATTN_M_DOCUMENT | FLEXATTN_M_NEIGHBORHOOD)) != 0) return false;
        bool f = true;
        if constexpr (TERM & FLEXATTN_M_CAUSAL) f = f && (q_lo >= kv_hi);
        if constexpr (TERM & FLEXATTN_M_SLIDING_WINDOW) f = f && (q_hi - kv_lo <= window);
        if constexpr (TERM & FLEXATTN_M_PREFIX) f = f && (kv_hi < prefix_len);
        if constexpr (TERM & FLEXATTN_M_CTX_LEN) f = f && (kv_hi < ctx);
        return f;
    }
    // the same with doc_ids[b, kv] supplied by the caller
    __device__ __forceinline__ bool eval(int kv, int doc_kv) const {
        bool r = true;
        if constexpr (TERM & FLEXATTN_M_CAUSAL) r = r && (q >= kv);
        if constexpr (TERM & FLEXATTN_M_SLIDING_WINDOW) r = r && (q - kv <= window);
        if constexpr (TERM & FLEXATTN_M_DOCUMENT) r = r && (doc_kv == doc_q);
        if constexpr (TERM & FLEXATTN_M_PREFIX) r = r && (kv < prefix_len);
        if constexpr (TERM & FLEXATTN_M_CTX_LEN) r = r && (kv < ctx);
        if constexpr (TERM & FLEXATTN_M_NEIGHBORHOOD) {
            int kx, ky;
            canvas.pixel(kv, kx, ky);
            r = r && ((unsigned)(kx - x0) <= (unsigned)span) && ((unsigned)(ky - y0) <= (unsigned)span);
        }
        return r;
    }
};

// Offset conversion for inference (section 5.2): the position the mods see for query row 0 of
// batch entry b.
__device__ __forceinline__ int q_offset_of(const flexattn_mod_params& p, int b) {
    return p.q_offsets ? ldc(p.q_offsets + b) : 0;
}

template <uint32_t MASK>
struct MaskRow {
    static constexpr uint32_t T0 = MASK & 0xffu, T1 = (MASK >> 8) & 0xffu;
    MaskTermRow<T0> t0;
    MaskTermRow<T1> t1;
    int kv_last;
    // Masks that read the document table can take the ids from the caller instead, who fetches
    // them for a whole tile with one coalesced load (lane j: entry first + j) and hands them from
    // lane to lane (tile_docs / doc_at), rather than with one table read per score element.
    static constexpr bool kUsesDoc = (((MASK | (MASK >> 8)) & 0xffu) & FLEXATTN_M_DOCUMENT) != 0;
    __device__ __forceinline__ static int tile_docs(const flexattn_mod_params& p, int b, int first, int last, int lane) {
        return (p.doc_ids + (int64_t)b * p.doc_stride_b)[min(first + lane, last)];
    }
    __device__ __forceinline__ static int doc_at(int docs, int offset_in_tile) { return __shfl(docs, offset_in_tile, 64); }
    // kv_len: keys at or past it do not exist (last block of a length that is no multiple of the
    // block size): they are masked, and the primitives are evaluated at the last real key instead
    // so that no table is read out of range.  q_idx must be a real row.
    __device__ __forceinline__ MaskRow(const flexattn_mod_params& p, int b, int h, int q_idx, int kv_len,
                                       int doc_q_known = -1)
        : t0(p, b, h, q_idx, doc_q_known), t1(p, b, h, q_idx, doc_q_known), kv_last(kv_len - 1) {}
    // Whole-rectangle shortcuts (exact implications of the index comparisons, never a guess): the
    // mask hides every pair / no pair of the rectangle.  The rectangle must lie inside the score matrix.
    __device__ __forceinline__ bool block_empty(int q_lo, int q_hi, int kv_lo, int kv_hi) const {
        bool e = T0 != 0 && t0.block_empty(q_lo, q_hi, kv_lo, kv_hi);
        if constexpr (T1 != 0) e = e && t1.block_empty(q_lo, q_hi, kv_lo, kv_hi);
        return e;
    }
    __device__ __forceinline__ bool block_full(int q_lo, int q_hi, int kv_lo, int kv_hi) const {
        bool f = T0 == 0 || t0.block_full(q_lo, q_hi, kv_lo, kv_hi);
        if constexpr (T1 != 0) f = f || t1.block_full(q_lo, q_hi, kv_lo, kv_hi);
        return f;
    }
    // with the document id of key kv supplied (any value for keys past the end)
    __device__ __forceinline__ bool eval(int kv, int doc_kv) const {
        bool r = t0.eval(kv, doc_kv);
        if constexpr (T1 != 0) r = r || t1.eval(kv, doc_kv);
        return r && kv <= kv_last;
    }
    __device__ __forceinline__ bool operator()(int kv) const {
        const int kc = min(kv, kv_last);
        bool r = t0(kc);
        if constexpr (T1 != 0) r = r || t1(kc);
        return r && kv <= kv_last;
    }
};

// ---------------------------------------------------------------------------------------
// score_mod in the base-2 domain.  apply(acc, q - kv) returns log2(e) * score_mod(acc * scale),
// so that exp(score') = exp2(apply(...)).  Order: ALiBi, relative bias, soft-cap.
// dscore(x) is d score_mod / d s given x = apply(...), used by the backward pass.
// ---------------------------------------------------------------------------------------
// Compiler-only fence on four values: everything that produces them is ordered before everything
// that uses them afterwards (no instruction is emitted).
__device__ __forceinline__ void pin4(float (&v)[4]) {
    asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
}

// LDSTAB: the relative-bias row of the head has been copied to LDS (fill_table), pre-multiplied, and
// is looked up there: one 32-bit address per score instead of a 64-bit global address, which is
// what keeps the table variant of the MFMA kernels inside their register budget.
constexpr int kRelTableMax = 1024;         // flexattn_mod_params::rel_len is at most this

template <uint32_t SCORE, bool LDSTAB = false>
struct ScoreMod {
    static constexpr bool kAlibi = SCORE & FLEXATTN_SCORE_ALIBI;
    static constexpr bool kRel = SCORE & FLEXATTN_SCORE_REL_BIAS;
    static constexpr bool kCap = SCORE & FLEXATTN_SCORE_SOFTCAP;
    float k_acc;      // multiplies the raw dot product
    float k_bias;     // alibi_bias[h], pre-multiplied like k_acc
    float k_tab;      // factor applied to table entries
    float capl2;      // softcap * log2(e)
    const float* tab; // rel_bias row of head h
    int rel_max;
    float rel_first, rel_last;   // first and last table entry, times k_tab
    uint32_t tab_lds; // LDSTAB: LDS byte address of the pre-multiplied row

    __device__ __forceinline__ ScoreMod(const flexattn_mod_params& p, int h, float scale, uint32_t tab_lds_ = 0)
        : tab_lds(tab_lds_) {
        float mul = kCap ? (2.0f * kLog2e / p.softcap) : kLog2e;   // soft-cap needs exp(2 s / cap)
        k_acc = scale * mul;
        k_bias = kAlibi ? p.alibi_bias[h] * mul : 0.0f;
        k_tab = mul;
        tab = kRel ? p.rel_bias + (int64_t)h * p.rel_len : nullptr;
        rel_max = kRel ? p.rel_len - 1 : 0;
        capl2 = kCap ? p.softcap * kLog2e : 0.0f;
        rel_first = kRel ? __builtin_bit_cast(float, ldc((const int32_t*)tab)) * k_tab : 0.0f;
        rel_last = kRel ? __builtin_bit_cast(float, ldc((const int32_t*)tab + rel_max)) * k_tab : 0.0f;
    }

    // LDSTAB: every thread of the workgroup copies its share of the head's row (a barrier must follow
    // before the first lookup, and precede the next fill)
    __device__ __forceinline__ void fill_table(int tid, int nthreads) const {
        if constexpr (kRel && LDSTAB) {
            for (int i = tid; i <= rel_max; i += nthreads)
                *(__attribute__((address_space(3))) float*)(uintptr_t)(tab_lds + 4u * (uint32_t)i) = tab[i] * k_tab;
        }
    }

    // Relative bias of a whole block of scores whose q_idx - kv_idx spans [dq_min, dq_max]
    // (wave-uniform bounds): the index is clamped to the table, so a block that lies at or beyond the
    // last entry, or at or before the first, adds ONE value to all its scores -- almost every block
    // of a long sequence -- and only the blocks near the diagonal look the table up per element.
    // The functions below take UNI = true and that value (pre-multiplied like k_tab) for such blocks.
    __device__ __forceinline__ bool rel_uniform(int dq_min, int dq_max, float& value) const {
        value = 0.0f;
        if constexpr (!kRel) return true;
        if (dq_min >= rel_max) {
            value = rel_last;
            return true;
        }
        if (dq_max <= 0) {
            value = rel_first;
            return true;
        }
        return false;
    }

    // q_idx - kv_idx of one score element.  The kernels know it as dq0 + c with dq0 shared by the 16
    // elements a lane holds of a 32 x 32 block and c a compile-time constant, so the ALiBi term
    // bias * (dq0 + c) costs one addition of abase = alibi_base(dq0), computed once per block, and
    // one fma with a literal instead of a subtraction, a conversion and an fma per element.
    struct RelPos {
        int dq;
        float abase, c;
        __device__ __forceinline__ RelPos(int dq_) : dq(dq_), abase(0.0f), c((float)dq_) {}
        __device__ __forceinline__ RelPos(int dq0, float abase_, int c_) : dq(dq0 + c_), abase(abase_), c((float)c_) {}
    };
    __device__ __forceinline__ float alibi_base(int dq0) const { return kAlibi ? k_bias * (float)dq0 : 0.0f; }

    // Scaled score plus the additive biases, times the factor the following exp2 needs.
    template <bool UNI = false>
    __device__ __forceinline__ float pre(float acc, RelPos rp, float uni = 0.0f) const {
        float y;
        if constexpr (kRel && UNI) y = __builtin_fmaf(acc, k_acc, uni);
        else y = acc * k_acc;
        if constexpr (kAlibi) y = __builtin_fmaf(k_bias, rp.c, y + rp.abase);
        if constexpr (kRel && !UNI) {
            int r = rp.dq < 0 ? 0 : (rp.dq > rel_max ? rel_max : rp.dq);
            if constexpr (LDSTAB) y += *(const __attribute__((address_space(3))) float*)(uintptr_t)(tab_lds + 4u * (uint32_t)r);
            else y = __builtin_fmaf(tab[r], k_tab, y);
        }
        return y;
    }

    // Soft-cap only: r = 1 / (1 + exp(2 s / cap)), so that cap * tanh(s / cap) = cap * (1 - 2 r).
    template <bool UNI = false>
    __device__ __forceinline__ float cap_r(float acc, RelPos dq, float uni = 0.0f) const {
        return fast_rcp(1.0f + fast_exp2(pre<UNI>(acc, dq, uni)));
    }

    template <bool UNI = false>
    __device__ __forceinline__ float apply(float acc, RelPos dq, float uni = 0.0f) const {
        if constexpr (kCap) {
            return __builtin_fmaf(-2.0f * capl2, cap_r<UNI>(acc, dq, uni), capl2);
        } else {
            return pre<UNI>(acc, dq, uni);
        }
    }

    // apply() + shift with the addition folded into the multiply-adds that are there anyway (the
    // online softmax passes minus its running maximum: the score arrives ready for exp2).
    template <bool UNI = false>
    __device__ __forceinline__ float apply_shifted(float acc, RelPos rp, float uni, float shift) const {
        if constexpr (kCap) {
            return __builtin_fmaf(-2.0f * capl2, cap_r<UNI>(acc, rp, uni), capl2 + shift);
        } else if constexpr (kAlibi) {
            float y = __builtin_fmaf(acc, k_acc, __builtin_fmaf(k_bias, rp.c, rp.abase + ((kRel && UNI) ? uni + shift : shift)));
            if constexpr (kRel && !UNI) y += rel_entry(rp.dq);
            return y;
        } else {
            float y = __builtin_fmaf(acc, k_acc, (kRel && UNI) ? uni + shift : shift);
            if constexpr (kRel && !UNI) y += rel_entry(rp.dq);
            return y;
        }
    }
    // the relative-bias entry of q_idx - kv_idx = dq, times k_tab
    __device__ __forceinline__ float rel_entry(int dq) const {
        const int r = dq < 0 ? 0 : (dq > rel_max ? rel_max : dq);
        if constexpr (LDSTAB) return *(const __attribute__((address_space(3))) float*)(uintptr_t)(tab_lds + 4u * (uint32_t)r);
        else return tab[r] * k_tab;
    }

    // A soft-capped score never exceeds the cap, so softmax can use the cap itself as its
    // (fixed) maximum when 2^(-2 cap log2 e) is still far from fp32 underflow: no running max,
    // no rescaling, and p = exp2(-2 capl2 r) directly.
    __device__ __forceinline__ bool bounded() const { return kCap && 2.0f * capl2 <= 100.0f; }

    // The backward needs d score_mod / d s up to the constant factor grad_scale(): for the soft-cap,
    // 1 - tanh^2 = 4 r (1 - r) with r from cap_r(), so g = r - r^2 and the 4 is folded into the
    // final scaling of dQ / dK (see p_with_grad).
    static constexpr float grad_scale() { return kCap ? 4.0f : 1.0f; }

    // Backward: P = exp(score' - LSE) from the raw dot product, with the row's constant folded in.
    // row_const() maps LSE * log2(e) (+inf for a row without visible keys) to that constant.
    __device__ __forceinline__ float row_const(float lse2) const { return kCap ? capl2 - lse2 : -lse2; }
    // The same for four independent elements, written stage by stage (pin4 keeps the stages apart):
    // a wave that is alone on its SIMD loses several cycles on every vector instruction that
    // consumes the result of the one before it.
    template <bool UNI = false>
    __device__ __forceinline__ void p_with_grad4(const float (&acc)[4], const RelPos (&dq)[4], const float (&rc)[4],
                                                 float (&g)[4], float (&p)[4], float uni = 0.0f) const {
        float x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)   // (without a soft-cap the row constant rides on the score_mod's multiply-adds)
            x[i] = kCap ? pre<UNI>(acc[i], dq[i], uni) : apply_shifted<UNI>(acc[i], dq[i], uni, rc[i]);
        pin4(x);
        if constexpr (kCap) {
            float r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = fast_exp2(x[i]);
            pin4(x);
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = 1.0f + x[i];
            pin4(x);
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = fast_rcp(x[i]);
            pin4(r);
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = __builtin_fmaf(-2.0f * capl2, r[i], rc[i]);
            pin4(x);
#pragma unroll
            for (int i = 0; i < 4; ++i) g[i] = __builtin_fmaf(-r[i], r[i], r[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) g[i] = 1.0f;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = fast_exp2(x[i]);
        pin4(p);
    }
    template <bool UNI = false>
    __device__ __forceinline__ float p_with_grad(float acc, RelPos dq, float rc, float& g, float uni = 0.0f) const {
        if constexpr (kCap) {
            const float r = cap_r<UNI>(acc, dq, uni);
            g = __builtin_fmaf(-r, r, r);
            return fast_exp2(__builtin_fmaf(-2.0f * capl2, r, rc));
        } else {
            g = 1.0f;
            return fast_exp2(apply_shifted<UNI>(acc, dq, uni, rc));
        }
    }
};

// Waves per SIMD the MFMA kernels are compiled for.  At D = 64 the lean variants fit 168 registers,
// so three workgroups share a CU (more latency hiding, more chances for one wave's MFMAs to run
// beside another's VALU work); the variants that carry a relative-bias table or the canvas decode
// would spill there and stay at two, as does everything at D = 128.
template <int D, uint32_t MASK, uint32_t SCORE>
constexpr int waves_per_simd() {
    constexpr uint32_t prims = (MASK | (MASK >> 8)) & 0xffu;
    constexpr bool lean = !(prims & FLEXATTN_M_NEIGHBORHOOD) && !(SCORE & FLEXATTN_SCORE_REL_BIAS);
    return (D == 64 && lean) ? 3 : 2;
}

// The backward kernels need fewer registers: at D = 64 only the canvas decode does not fit three waves.
template <int D, uint32_t MASK>
constexpr int bwd_waves_per_simd() {
    return (D == 64 && !(((MASK | (MASK >> 8)) & 0xffu) & FLEXATTN_M_NEIGHBORHOOD)) ? 3 : 2;
}

// ---------------------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------------------
void set_last_hip_error(int e);

#define FLEXATTN_HIP_TRY(expr)                          \
    do {                                                \
        hipError_t _e = (expr);                         \
        if (_e != hipSuccess) {                         \
            ::flexattn::set_last_hip_error((int)_e);    \
            return FLEXATTN_ERR_HIP;                    \
        }                                               \
    } while (0)

inline bool mask_id_valid(uint32_t m) {
    return (m & ~0x3f3fu) == 0 && !((m & 0xffu) == 0 && (m >> 8) != 0);
}
inline bool score_id_valid(uint32_t s) { return (s & ~7u) == 0; }
inline bool mask_uses(uint32_t m, uint32_t prim) { return ((m | (m >> 8)) & prim) != 0; }

// Pointers the selected mods will dereference must be present.
inline int check_mod_params(uint32_t mask_id, uint32_t score_id, const flexattn_mod_params* p) {
    if (!mask_id_valid(mask_id) || !score_id_valid(score_id)) return FLEXATTN_ERR_INVALID_ARG;
    bool need = mask_id != 0 || score_id != 0;
    if (need && !p) return FLEXATTN_ERR_INVALID_ARG;
    if (!p) return FLEXATTN_OK;
    if (mask_uses(mask_id, FLEXATTN_M_DOCUMENT) && !p->doc_ids) return FLEXATTN_ERR_INVALID_ARG;
    if (mask_uses(mask_id, FLEXATTN_M_CTX_LEN) && !p->ctx_lens) return FLEXATTN_ERR_INVALID_ARG;
    if ((score_id & FLEXATTN_SCORE_ALIBI) && !p->alibi_bias) return FLEXATTN_ERR_INVALID_ARG;
    if ((score_id & FLEXATTN_SCORE_REL_BIAS) && (!p->rel_bias || p->rel_len <= 0 || p->rel_len > 1024))
        return FLEXATTN_ERR_INVALID_ARG;
    if ((score_id & FLEXATTN_SCORE_SOFTCAP) && !(p->softcap > 0.0f)) return FLEXATTN_ERR_INVALID_ARG;
    if (mask_uses(mask_id, FLEXATTN_M_NEIGHBORHOOD)) {
        const int w = p->na_width, h = p->na_height, k = p->na_kernel, t = p->na_tile;
        if (w <= 0 || h <= 0 || (int64_t)w * h > (1 << 20)) return FLEXATTN_ERR_INVALID_ARG;
        if (k < 1 || !(k & 1) || k > w || k > h) return FLEXATTN_ERR_INVALID_ARG;
        if (p->na_layout == FLEXATTN_NA_TILED) {
            if (t <= 0 || (t & (t - 1)) || w % t || h % t) return FLEXATTN_ERR_INVALID_ARG;
        } else if (p->na_layout == FLEXATTN_NA_MORTON) {
            if (w != h || (w & (w - 1))) return FLEXATTN_ERR_INVALID_ARG;
        } else if (p->na_layout != FLEXATTN_NA_ROW_MAJOR) {
            return FLEXATTN_ERR_INVALID_ARG;
        }
    }
    return FLEXATTN_OK;
}

// The neighborhood mask is defined on a canvas of exactly q_len == kv_len tokens.
inline int check_canvas(uint32_t mask_id, const flexattn_mod_params* p, int q_len, int kv_len) {
    if (!mask_uses(mask_id, FLEXATTN_M_NEIGHBORHOOD)) return FLEXATTN_OK;
    const int64_t n = (int64_t)p->na_width * p->na_height;
    return (q_len == n && kv_len == n) ? FLEXATTN_OK : FLEXATTN_ERR_INVALID_ARG;
}

// The (mask, score) pairs that forward/backward kernels are instantiated for: the paper's examples
// and benchmark variants, and three compositions of them (sliding window with a soft-cap; nested
// score_mods: ALiBi then soft-cap, relative bias then soft-cap under a document mask).  The functors
// compose freely -- another pair is one more line here (and in the launcher lists that
// FLEXATTN_VARIANT_INDICES drives), nothing else.
// X(mask_id, score_id)
#define FLEXATTN_FOR_EACH_VARIANT(X)                                                    \
    X(FLEXATTN_MASK_NONE, FLEXATTN_SCORE_IDENTITY)                                      \
    X(FLEXATTN_MASK_CAUSAL, FLEXATTN_SCORE_IDENTITY)                                    \
    X(FLEXATTN_MASK_CAUSAL, FLEXATTN_SCORE_ALIBI)                                       \
    X(FLEXATTN_MASK_CAUSAL, FLEXATTN_SCORE_SOFTCAP)                                     \
    X(FLEXATTN_MASK_SWA_CAUSAL, FLEXATTN_SCORE_IDENTITY)                                \
    X(FLEXATTN_MASK_PREFIX_LM, FLEXATTN_SCORE_IDENTITY)                                 \
    X(FLEXATTN_MASK_DOCUMENT_CAUSAL, FLEXATTN_SCORE_IDENTITY)                           \
    X(FLEXATTN_MASK_DOCUMENT_CAUSAL, FLEXATTN_SCORE_ALIBI)                              \
    X(FLEXATTN_MASK_SWA_CAUSAL_OR_PREFIX, FLEXATTN_SCORE_REL_BIAS)                      \
    X(FLEXATTN_MASK_NEIGHBORHOOD, FLEXATTN_SCORE_IDENTITY)                              \
    X(FLEXATTN_MASK_SWA_CAUSAL, FLEXATTN_SCORE_SOFTCAP)                                 \
    X(FLEXATTN_MASK_CAUSAL, (FLEXATTN_SCORE_ALIBI | FLEXATTN_SCORE_SOFTCAP))            \
    X(FLEXATTN_MASK_DOCUMENT_CAUSAL, (FLEXATTN_SCORE_REL_BIAS | FLEXATTN_SCORE_SOFTCAP))

// One entry per line of FLEXATTN_FOR_EACH_VARIANT: X(index)
#define FLEXATTN_VARIANT_INDICES(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12)

}  // namespace flexattn
