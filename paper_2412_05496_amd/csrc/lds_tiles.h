// LDS tile helpers shared by the forward and backward kernels (gfx950).
//
// A tile is 64 rows x D bf16, row-major and UNPADDED in LDS, with the 16-byte chunks of every row
// permuted by an XOR that depends on the row.  The permutation keeps both access patterns the
// kernels use free of bank conflicts (64 banks x 4 bytes):
//   row read         32 consecutive lanes read the same logical chunk of 32 consecutive rows
//                    (A/B operand of an MFMA whose contraction runs along D);
//   transposing read ds_read_b64_tr_b16: 16 lanes cover a 4-row x 16-column block and lane i gets
//                    column i of the 4 rows (operand of an MFMA whose contraction runs along rows).
// Tiles are filled straight from global memory (buffer_load_dwordx4 ... lds): each wave instruction
// deposits 64 x 16 bytes contiguously in LDS, so the permutation is applied on the global side --
// lane L fetches the chunk that belongs at LDS position L.
//
// Per-lane byte offsets for the reads are computed once (RowReader / TrReader) so that every
// read in the main loops is "precomputed VGPR + immediate".
#pragma once

#include "flex_common.h"

namespace flexattn {

// XOR applied to the chunk index (0 .. D/8-1) of row `row`.
template <int D>
__device__ __forceinline__ constexpr int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

// Element offset of logical chunk `chunk` of row `row`.
template <int D>
__device__ __forceinline__ constexpr int tile_off(int row, int chunk) {
    return row * D + 8 * (chunk ^ swz<D>(row));
}

// vmcnt(0): every global load (including loads into LDS) this wave issued has completed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// vmcnt(N): all but the N most recently issued vector-memory operations of this wave have completed
// (loads, LDS-DMA loads and stores retire from the counter in the order they were issued).
template <int N>
__device__ __forceinline__ void wait_vmem_but() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Raw buffer resource (four scalar dwords) over `bytes` bytes at `p`: no stride, loads beyond
// the end return zero instead of faulting.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 make_rsrc(const void* p, uint32_t bytes) {
    const uint64_t addr = (uint64_t)p;
    // (readfirstlane: the descriptor must sit in scalar registers whatever the compiler believes
    // about the uniformity of p)
    return i32x4{__builtin_amdgcn_readfirstlane((int)(uint32_t)addr),
                 __builtin_amdgcn_readfirstlane((int)((uint32_t)(addr >> 32) & 0xffffu)),
                 __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}

// The descriptor as four values the compiler knows to be scalar (an "s" operand that it believes
// to live in vector registers is not moved for us).
__device__ __forceinline__ i32x4 scalar_rsrc(i32x4 r) {
    return i32x4{__builtin_amdgcn_readfirstlane(r[0]), __builtin_amdgcn_readfirstlane(r[1]),
                 __builtin_amdgcn_readfirstlane(r[2]), __builtin_amdgcn_readfirstlane(r[3])};
}

// LDS-DMA loads are issued from inline assembly on purpose.  When the compiler sees such a load it
// makes every later LDS read that it cannot prove disjoint wait for vmcnt(0), which serialises the
// prefetch with the compute it is meant to overlap; completion is tracked by hand instead
// (s_waitcnt vmcnt + barrier before a buffer is read).  s_nop 4 covers the wait states between a
// write of M0 (or of a scalar operand by a vector instruction) and the loads that use it.  M0 is
// written without telling the compiler (it does not accept M0 as a clobber): the kernels that
// use these helpers contain nothing else that needs M0.
//
// dma_dword: 64 lanes x 4 bytes to `lds` .. +256.
__device__ __forceinline__ void dma_dword(i32x4 rsrc, uint32_t lds, int voff, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(voff), "s"(scalar_rsrc(rsrc)), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

// dma_x4 / dma_x2: four (two) 1 KiB loads to `lds` + 0, 1024, 2048, 3072.  The immediate offset
// moves the LDS destination and, because it is added to the memory address as well, has been
// taken out of the per-lane offsets v0..v3 by the caller.
__device__ __forceinline__ void dma_x4(i32x4 rsrc, uint32_t lds, int v0, int v1, int v2, int v3, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\t"
                 "buffer_load_dwordx4 %1, %5, %6 offen lds\n\t"
                 "buffer_load_dwordx4 %2, %5, %6 offen offset:1024 lds\n\t"
                 "buffer_load_dwordx4 %3, %5, %6 offen offset:2048 lds\n\t"
                 "buffer_load_dwordx4 %4, %5, %6 offen offset:3072 lds"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(scalar_rsrc(rsrc)), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}
__device__ __forceinline__ void dma_x2(i32x4 rsrc, uint32_t lds, int v0, int v1, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\t"
                 "buffer_load_dwordx4 %1, %3, %4 offen lds\n\t"
                 "buffer_load_dwordx4 %2, %3, %4 offen offset:1024 lds"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(v0), "v"(v1), "s"(scalar_rsrc(rsrc)), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

// 64 lanes x 16 bytes from per-lane global addresses to `lds` .. +1024, with the non-temporal hint:
// for data that is read exactly once (the K / V pages of a decode step), which then stream past the
// caches instead of displacing each other there.
__device__ __forceinline__ void dma_global_nt(uint32_t lds, const void* gptr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(gptr) : "memory");
}

__device__ __forceinline__ void dma_x1(i32x4 rsrc, uint32_t lds, int v0, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(v0), "s"(scalar_rsrc(rsrc)), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

// The same with the non-temporal hint, for data that is read exactly once.
__device__ __forceinline__ void dma_x1_nt(i32x4 rsrc, uint32_t lds, int v0, int soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds)), "v"(v0), "s"(scalar_rsrc(rsrc)), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

// The tile copy with buffer loads, for a workgroup of NW waves: the row of the tile is selected by
// a scalar byte offset, so starting a tile costs an M0 write per four loads and no vector
// arithmetic.  Wave w fills the contiguous LDS bytes [w * 1024 * NI, (w + 1) * 1024 * NI) of the
// tile.  The per-lane offsets stay non-negative as long as the row stride is >= D.
// Completion: s_waitcnt vmcnt by every wave, then a barrier.
template <int D, int NW>
struct WaveTileLoader {
    static constexpr int DC = D / 8, RPI = 64 / DC, NI = DC / NW;   // NI loads per wave
    static_assert(NI == 2 || NI == 4 || NI == 8, "D is 64 or 128, 2 or 4 waves");
    int32_t voff[NI];                           // per-lane byte offsets
    uint32_t wave_off;                          // of this wave's part inside a tile
    __device__ __forceinline__ WaveTileLoader(int64_t gs, int wave, int lane) : wave_off(wave * NI * 1024) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = (wave * NI + i) * RPI + lane / DC;
            voff[i] = (int32_t)(row * gs * 2) + (((lane % DC) ^ swz<D>(row)) * 16) - (i & 3) * 1024;
        }
    }
    // `tile`: LDS byte address of the tile (wave-uniform);
    // `soff`: byte offset of the tile's first row inside the resource (wave-uniform)
    __device__ __forceinline__ void start(i32x4 rsrc, uint32_t tile, int soff) const {
        if constexpr (NI == 2) {
            dma_x2(rsrc, tile + wave_off, voff[0], voff[1], soff);
        } else {
            dma_x4(rsrc, tile + wave_off, voff[0], voff[1], voff[2], voff[3], soff);
            if constexpr (NI == 8) dma_x4(rsrc, tile + wave_off + 4096, voff[4], voff[5], voff[6], voff[7], soff);
        }
    }
    // One of the NI loads on its own (I compile-time), for callers that spread the loads of a tile
    // over their compute instead of issuing them back to back: the vector memory path takes a
    // 1 KiB load every ~16 cycles per CU and a wave that finds its queue full stalls.
    template <int I>
    __device__ __forceinline__ void start_one(i32x4 rsrc, uint32_t tile, int soff) const {
        dma_x1(rsrc, tile + wave_off + I * 1024, voff[I] + (I & 3) * 1024, soff);
    }
};

// Row reads: fragment (row0 + lane % 32, dims 16 ks + 8 half ..) for row0 a multiple of 32.
template <int D>
struct RowReader {
    uint32_t off[D / 16];                       // byte offsets inside a tile, row0 = 0
    // `base`: a per-lane byte offset added to every read (e.g. the LDS address of the buffer set
    // plus a wave-specific tile), so that reads are "this VGPR + immediate"
    __device__ __forceinline__ RowReader(int l32, int half, uint32_t base = 0) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) off[ks] = base + 2u * (uint32_t)tile_off<D>(l32, 2 * ks + half);
    }
    // `tile_bytes`: LDS byte address of the tile (wave-uniform); row0 and ks are compile-time
    __device__ __forceinline__ bf16x8 read(uint32_t tile_bytes, int row0, int ks) const {
        return *(const __attribute__((address_space(3))) bf16x8*)(uintptr_t)(tile_bytes + off[ks] + 2u * row0 * D);
    }
};

__device__ __forceinline__ u32x2 lds_read_tr4(uint32_t addr) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
    return __builtin_bit_cast(u32x2, v);
}

// Transposing reads: operand fragment of tile^T for one MFMA contracting over tile ROWS.  The
// fragment's row (or column) index is tile column c0 + lane % 32; the eight k-slots of half
// h = lane / 32 are tile rows r0 + 4 h + {0,1,2,3} and r0 + 8 + 4 h + {0,1,2,3} -- exactly the rows
// that registers 0..7 of a 32x32 MFMA result starting at row r0 hold in a lane of that half.
// r0 is a multiple of 16, c0 a multiple of 32.
template <int D>
struct TrReader {
    uint32_t off[D / 32][2];                    // [column block][low / high four rows], r0 = 0
    __device__ __forceinline__ TrReader(int lane, uint32_t base = 0) {
        const int j = lane & 15, grp = lane >> 4;
        const int row = 4 * (grp >> 1) + (j >> 2);
#pragma unroll
        for (int cb = 0; cb < D / 32; ++cb) {
            const int col = cb * 32 + 16 * (grp & 1) + 4 * (j & 3);
            off[cb][0] = base + 2u * (uint32_t)(tile_off<D>(row, col >> 3) + (col & 7));
            off[cb][1] = base + 2u * (uint32_t)(tile_off<D>(row + 8, col >> 3) + (col & 7));
        }
    }
    // r0 (multiple of 16) and cb are compile-time: swz depends on r0 only through (r0 >> 2) & 3 == 0
    __device__ __forceinline__ bf16x8 read(uint32_t tile_bytes, int r0, int cb) const {
        const u32x2 lo = lds_read_tr4(tile_bytes + off[cb][0] + 2u * r0 * D);
        const u32x2 hi = lds_read_tr4(tile_bytes + off[cb][1] + 2u * r0 * D);
        u32x4 f = {lo[0], lo[1], hi[0], hi[1]};
        return __builtin_bit_cast(bf16x8, f);
    }
};

// Walk over the 64-wide tiles of the blocks a BlockMask lists for one row (or column) of blocks:
// FULL blocks first, then PARTIAL ones, each block cut into `sub` tiles.  Written without
// branches, and the index of the following block is fetched (scalar cache) on every call and only
// consumed by the call after it, so that the fetch has a tile's worth of work to hide behind.
template <bool PAGED = false>
struct TileWalk {
    const int32_t* full_idx;
    const int32_t* part_idx;
    const int32_t* full_phys;                   // PAGED: the converted lists (section 5.1), read entry
    const int32_t* part_phys;                   // by entry beside the logical ones
    int n_full, n_blocks, sub, block_len;
    int pos, s, blk, fetched, pblk, pfetched;
    bool entered;                               // the previous call moved on to the next block
    __device__ __forceinline__ int block_at(int p) const {
        return ldc(p < n_full ? full_idx + p : part_idx + (p - n_full));
    }
    __device__ __forceinline__ int phys_at(int p) const {
        return ldc(p < n_full ? full_phys + p : part_phys + (p - n_full));
    }
    __device__ __forceinline__ TileWalk(const int32_t* full_idx_, const int32_t* part_idx_, int n_full_, int n_part,
                                        int sub_, int block_len_, const int32_t* full_phys_ = nullptr,
                                        const int32_t* part_phys_ = nullptr)
        : full_idx(full_idx_), part_idx(part_idx_), full_phys(full_phys_), part_phys(part_phys_), n_full(n_full_),
          n_blocks(n_full_ + n_part), sub(sub_), block_len(block_len_), pos(0), s(0), fetched(0), pblk(0),
          pfetched(0), entered(false) {
        blk = n_blocks > 0 ? block_at(0) : 0;
        if constexpr (PAGED) pblk = n_blocks > 0 ? phys_at(0) : 0;
    }
    // first row (column) of the next tile, and whether its block is PARTIAL; must not be called
    // more than n_blocks * sub times.  PAGED: `page` and `row_in_page` receive where the tile starts
    // in the pool (the page is the physical block); otherwise they are not touched.
    __device__ __forceinline__ int next(bool& partial, int& page, int& row_in_page) {
        blk = entered ? fetched : blk;
        const int x0 = blk * block_len + s * 64;
        if constexpr (PAGED) {
            pblk = entered ? pfetched : pblk;
            page = pblk;
            row_in_page = s * 64;
            pfetched = phys_at(min(pos + 1, n_blocks - 1));
        }
        partial = pos >= n_full;
        fetched = block_at(min(pos + 1, n_blocks - 1));
        entered = s + 1 == sub;
        s = entered ? 0 : s + 1;
        pos += entered ? 1 : 0;
        return x0;
    }
    __device__ __forceinline__ int next(bool& partial) {
        static_assert(!PAGED, "the paged walk also yields the physical position");
        int page, row;
        return next(partial, page, row);
    }
};

// LDS byte address of a __shared__ object.
template <typename T>
__device__ __forceinline__ uint32_t lds_addr(const T* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) T*)p;
}

}  // namespace flexattn
