// The backward with dS kept in memory (an alternative to recomputing S and dP in a dQ kernel).
//
// The dK/dV kernel computes dS for every block it visits anyway; with ds_store set it also writes it
// out, and dQ = scale * dS K (section 4.1's backward, written out at the top of bwd_kernel.h) becomes
// one block-sparse GEMM over what was written: 1 GEMM and no softmax arithmetic instead of 3 GEMMs
// and all of it -- the backward executes 5 GEMMs, its algorithmic count, instead of 7.  The price is
// HBM: 2 bytes per unmasked score written once and read once, and a workspace of that size -- which
// this GPU has (288 GB; 4.4 GB for 64 heads of dense-causal S = 8192).  Still no floating-point
// atomics: every dQ row is summed by one wave in the order of its BlockMask row.
//
//   bwd_slots_scan_kernel / bwd_slots_fill_kernel   number the non-empty blocks (see ds_chunk in
//                      bwd_kernel.h) and lay the numbers out as a [planes, NR, NC] grid, so that the
//                      row-walking kernel finds the block the column-walking kernel wrote;
//   bwd_dq_stored_kernel   one workgroup per row of blocks of one (b, hq): K and dS tiles stream
//                      through LDS, dQ^T += K^T dS^T with both operands from transposing LDS
//                      reads.  Bound by the HBM read of dS.
#pragma once

#include "bwd_kernel.h"

namespace flexattn {

// Exclusive prefix sum of the merged column-list lengths over all `lines` = planes * NC columns of
// blocks; colbase[lines] = total.  One workgroup.
__global__ __launch_bounds__(1024) void bwd_slots_scan_kernel(const int32_t* __restrict__ q_num,
                                                              const int32_t* __restrict__ full_q_num, int lines, int NR,
                                                              int32_t* __restrict__ colbase) {
    __shared__ int s_sum[1024];
    const int tid = threadIdx.x;
    const int per = (lines + 1023) / 1024;
    const int lo = min(tid * per, lines), hi = min(lo + per, lines);
    auto count = [&](int l) { return min(max(full_q_num[l], 0), NR) + min(max(q_num[l], 0), NR); };
    int sum = 0;
    for (int l = lo; l < hi; ++l) sum += count(l);
    s_sum[tid] = sum;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {      // inclusive scan of the per-thread sums
        const int v = tid >= off ? s_sum[tid - off] : 0;
        __syncthreads();
        s_sum[tid] += v;
        __syncthreads();
    }
    int base = s_sum[tid] - sum;
    for (int l = lo; l < hi; ++l) {
        colbase[l] = base;
        base += count(l);
    }
    if (tid == 1023) colbase[lines] = s_sum[1023];
}

// grid[plane, r, c] = colbase[plane * NC + c] + j for the j-th entry r of the merged list of column c.
// One workgroup per column of blocks.
__global__ __launch_bounds__(256) void bwd_slots_fill_kernel(const int32_t* __restrict__ q_num,
                                                             const int32_t* __restrict__ q_idx,
                                                             const int32_t* __restrict__ full_q_num,
                                                             const int32_t* __restrict__ full_q_idx, int NR, int NC,
                                                             const int32_t* __restrict__ colbase,
                                                             int32_t* __restrict__ grid) {
    const int l = blockIdx.x, plane = l / NC, c = l - plane * NC;
    const int n_full = min(max(full_q_num[l], 0), NR), n_part = min(max(q_num[l], 0), NR);
    const int base = colbase[l];
    for (int j = threadIdx.x; j < n_full + n_part; j += 256) {
        const int r = j < n_full ? full_q_idx[(int64_t)l * NR + j] : q_idx[(int64_t)l * NR + j - n_full];
        if (r >= 0 && r < NR) grid[((int64_t)plane * NR + r) * NC + c] = base + j;
    }
}

// Transposing reads of a wave's own slice of a dS tile: 64 keys x 32 query columns, row-major and
// unpadded in LDS (a transposing read of 64 lanes covers 8 rows x 64 bytes = 512 contiguous bytes:
// no bank conflicts without any swizzle).  Fragment: column lane % 32, k-slots = rows
// r0 + 4 h + {0..3} and r0 + 8 + 4 h + {0..3}, like TrReader.
struct SliceTrReader {
    uint32_t off;
    __device__ __forceinline__ SliceTrReader(int lane, uint32_t base) {
        const int j = lane & 15, grp = lane >> 4;
        const int row = 4 * (grp >> 1) + (j >> 2), col = 16 * (grp & 1) + 4 * (j & 3);
        off = base + 2u * (uint32_t)(row * 32 + col);
    }
    __device__ __forceinline__ bf16x8 read(uint32_t slot_bytes, int r0) const {
        const u32x2 lo = lds_read_tr4(slot_bytes + off + 2u * r0 * 32);
        const u32x2 hi = lds_read_tr4(slot_bytes + off + 2u * (r0 + 8) * 32);
        u32x4 f = {lo[0], lo[1], hi[0], hi[1]};
        return __builtin_bit_cast(bf16x8, f);
    }
};

// M0 RULE: this kernel fills LDS through the LDS-DMA helpers of lds_tiles.h, which write M0 behind the
// compiler's back.  Keep every register array in it indexed by compile-time constants (no movrel /
// s_set_gpr_idx code, which would also use M0) and add no other LDS-DMA or M0-based construct.
//
// Pipeline.  K tiles are shared by the workgroup: double buffered, one barrier per tile.  A wave
// needs only ITS 32 query columns of a dS tile -- 4 KiB that the dK/dV kernel wrote contiguously --
// so every wave keeps a private ring of two slices and no barrier guards it.  Per tile t a wave
// issues K(t+1) and then dS(t+2); the vector-memory counter retires in issue order, so
// "all but the last four" at the top of a tile means K(t) and dS(t) have landed while dS(t+1) is
// still under way: the HBM read of dS runs two tiles ahead of its use, the L2 read of K one.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 2) void bwd_dq_stored_kernel(const BwdArgs a, const float qscale) {
    constexpr int Bq = NW * 32;
    constexpr int TILE_K = 64 * D, TILE_S = 64 * Bq, SLICE = 64 * 32;   // bf16 elements
    constexpr int kList = 512;
    __shared__ __attribute__((aligned(1024))) bf16 smem[2 * TILE_K + NW * 2 * SLICE];   // K(even), K(odd); per wave dS(even), dS(odd)
    __shared__ int s_kv0[kList + 2];                                 // first key of a tile, -1: nothing to add
    __shared__ int s_chunk[kList + 2];                               // where its dS starts (ds_chunk without the rep)

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
    // the dS tile's columns are the block's query rows with bits 2 and 3 of the index exchanged (the
    // order in which the dK/dV kernel's registers hold them): lane l32 of wave w owns this row
    const int q_in_block = 32 * w + (l32 & 19) + ((l32 & 4) << 1) + ((l32 & 8) >> 1);
    const int q_row = row * Bq + q_in_block;
    const bool real_row = q_row < a.q_len;
    bf16* dq_ptr = a.dQ + b * a.dq_sb + hq * a.dq_sh + (int64_t)q_row * a.dq_ss;

    const int64_t line = plane * a.NR + row;
    const int n_full = ldc(a.full_kv_num + line), n_part = ldc(a.kv_num + line);
    const int sub_k = a.Bk / 64;
    const int T_all = (n_full + n_part) * sub_k;
    if (T_all == 0) {
        if (real_row)
            for (int d0 = half * 8; d0 < D; d0 += 16) *(u32x4*)(dq_ptr + d0) = u32x4{0, 0, 0, 0};
        return;
    }
    const int32_t* full_idx = a.full_kv_idx + line * a.NC;
    const int32_t* part_idx = a.kv_idx + line * a.NC;
    const int32_t* grid_row = a.ds_grid + line * a.NC;
    // this wave's slice of the head's tiles: columns 32 w .. of a tile are the 4 KiB at w * 4096
    const bf16* ds_head = a.ds_store + ds_rep(a, b, hq) * a.ds_blocks * ((int64_t)a.Bk * Bq) + w * SLICE;

    const i32x4 k_rsrc = make_rsrc(a.K + b * a.k_sb + hkv * a.k_sh, (uint32_t)((a.kv_len - 1) * a.k_ss + D) * 2u);
    const int k_row_bytes = (int)a.k_ss * 2;
    const WaveTileLoader<D, NW> k_loader(a.k_ss, w, lane);
    // slice position (key, 8 columns) <- where the dK/dV kernel put those 8 values: chunk c = columns
    // 16 c .., lane 32 h + key % 32 of the wave that had keys 32 kb ..
    int32_t s_voff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int pos = i * 64 + lane, key = pos >> 2, pc = pos & 3;
        s_voff[i] = (key >> 5) * 2048 + (pc >> 1) * 1024 + (32 * (pc & 1) + (key & 31)) * 16;
    }
    const uint32_t k_lds = lds_addr(smem), s_lds = k_lds + 2 * TILE_K * 2 + w * (2 * SLICE * 2);
    const TrReader<D> tr_k(lane, k_lds);
    const SliceTrReader tr_s(lane, s_lds);

    f32x16 dq[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[db][r] = 0.0f;

    for (int seg0 = 0; seg0 < T_all; seg0 += kList) {
        const int T = min(kList, T_all - seg0);
        for (int i = tid; i < T; i += NW * 64) {
            const int t = seg0 + i, pos = t / sub_k, st = t - pos * sub_k;
            const int c = min(max(pos < n_full ? full_idx[pos] : part_idx[pos - n_full], 0), a.NC - 1);
            const int kv0 = c * a.Bk + st * 64;
            const int slot = (int)min(max((int64_t)grid_row[c], (int64_t)0), a.ds_blocks - 1);
            s_kv0[i] = kv0 < a.kv_len ? kv0 : -1;      // the dK/dV kernel has no workgroup for keys past kv_len
            s_chunk[i] = slot * sub_k + st;
        }
        __syncthreads();

        auto load_k = [&](int i, auto buf_tag) {
            constexpr int BUF = decltype(buf_tag)::value;
            const int kv0 = max(__builtin_amdgcn_readfirstlane(s_kv0[i]), 0);
            k_loader.start(k_rsrc, k_lds + BUF * (TILE_K * 2), kv0 * k_row_bytes);
        };
        // a tile with nothing to add is loaded through an empty descriptor, which fills the slice with zeros
        auto load_s = [&](int i, auto buf_tag) {
            constexpr int BUF = decltype(buf_tag)::value;
            const int kv0 = __builtin_amdgcn_readfirstlane(s_kv0[i]);
            const int chunk = __builtin_amdgcn_readfirstlane(s_chunk[i]);
            const i32x4 rsrc = make_rsrc(ds_head + (int64_t)chunk * TILE_S, kv0 >= 0 ? (uint32_t)SLICE * 2u : 0u);
#pragma unroll
            for (int i = 0; i < 4; ++i) dma_x1_nt(rsrc, s_lds + BUF * (SLICE * 2) + i * 1024, s_voff[i], 0);
        };
        const std::integral_constant<int, 0> b0;
        const std::integral_constant<int, 1> b1;
        load_k(0, b0);
        load_s(0, b0);
        if (T > 1) load_s(1, b1);

        auto step = [&](int t, auto buf_tag) {
            constexpr int BUF = decltype(buf_tag)::value;
            constexpr std::integral_constant<int, BUF ^ 1> nxt{};
            // K(t) and dS(t) have landed; dS(t+1), if there is one, may still be under way
            if (t + 1 < T) wait_vmem_but<4>();
            else wait_vmem();
            __syncthreads();
            constexpr uint32_t kt = BUF * (TILE_K * 2), stl = BUF * (SLICE * 2);
            bf16x8 bfr[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bfr[ks] = tr_s.read(stl, 16 * ks);
            // (the slot is refilled below: the reads above must have left LDS first)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bfr[0]), "+v"(bfr[1]), "+v"(bfr[2]), "+v"(bfr[3]) :: "memory");
            if (t + 1 < T) load_k(t + 1, nxt);
            if (t + 2 < T) load_s(t + 2, buf_tag);
            constexpr int NDB = D / 32, NM = 4 * NDB, PF = 4;       // [16-key slice][block db]
            auto frag = [&](int m) { return tr_k.read(kt, 16 * (m / NDB), m % NDB); };
            bf16x8 fr[NM];
#pragma unroll
            for (int m = 0; m < PF; ++m) fr[m] = frag(m);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                if (m + PF < NM) fr[m + PF] = frag(m + PF);
                dq[m % NDB] = mfma32(fr[m], bfr[m / NDB], dq[m % NDB]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int t = 0;
        for (; t + 1 < T; t += 2) {
            step(t, b0);
            step(t + 1, b1);
        }
        if (t < T) step(t, b0);
        __syncthreads();        // everybody has read the last K tile and the lists
    }

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

inline int launch_bwd_stored_dq(const BwdArgs& a, int D, float qscale, hipStream_t st) {
    const int units = a.B * a.Hkv;
    const unsigned grid_q = (unsigned)(((units + 7) / 8) * 8 * a.G * a.NR);
    if (D == 128 && a.Bq == 128) hipLaunchKernelGGL((bwd_dq_stored_kernel<128, 4>), dim3(grid_q), dim3(256), 0, st, a, qscale);
    else if (D == 128) hipLaunchKernelGGL((bwd_dq_stored_kernel<128, 2>), dim3(grid_q), dim3(128), 0, st, a, qscale);
    else if (a.Bq == 128) hipLaunchKernelGGL((bwd_dq_stored_kernel<64, 4>), dim3(grid_q), dim3(256), 0, st, a, qscale);
    else hipLaunchKernelGGL((bwd_dq_stored_kernel<64, 2>), dim3(grid_q), dim3(128), 0, st, a, qscale);
    return FLEXATTN_OK;
}

}  // namespace flexattn
