// Tile transport of the query-tiled kernels (gfx950): 32-row tiles of a [tokens, H, D] bf16
// tensor travel from global memory straight into LDS (buffer_load ... lds, no staging
// registers) into a ring of stages, so that several tiles are in flight while one is consumed.
//
// The loads are written in assembly: once the compiler sees a load that writes LDS it waits
// for ALL outstanding vector-memory operations before every LDS read, which would serialise
// the ring.  The kernels count their own loads instead (wait_vmcnt); loads of one wave
// complete in order.
//
// A load instruction writes 64 consecutive 16-byte LDS slots, so tiles are unpadded
// (D*2 bytes per row) and bank conflicts are avoided by an XOR swizzle of the 16-byte chunk
// index that is applied on the GLOBAL side: slot (row, pos) receives chunk pos ^ x(row) of the
// row; readers use TileLayout::k_offset / v_offset / u_offset with the same x.
#pragma once
#include "mfma_tile.h"

namespace kunlun {

// 128-bit buffer descriptor: base address, byte count, raw 32-bit addressing.
__device__ __forceinline__ u32x4 make_rsrc_words(const void* base, uint32_t bytes) {
    const uint64_t a = (uint64_t)base;
    const u32x4 r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
    return r;
}

// One wave-wide load from a buffer straight into LDS: lane l's 16 (4) bytes land at
// lds_addr + 16*l (4*l).  voff: per-lane byte offset, soff: uniform byte offset.  Counted by vmcnt.
// The statements overwrite M0 (the LDS base of such a load) and say so in their clobber lists, so that the
// compiler never assumes a value of its own survives in M0 across them.  M0 is a reserved register on this
// target; the compiler's remark that it cannot save and restore a reserved register is what is meant here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds_b128(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds_b32(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

#pragma clang diagnostic pop

// s_waitcnt that waits only for the vector-memory counter to drop to N (other counters untouched).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// LDS byte address (the value M0 takes) of a pointer into a __shared__ array.
__device__ __forceinline__ uint32_t lds_address(const char* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

enum { SWZ_K = 0, SWZ_V = 1, SWZ_U = 2 };

// The chunk XOR of a tile row for each swizzle kind (see TileLayout).
template <int D, int SWZ>
__device__ __forceinline__ int swizzle_of_row(int row) {
    if (SWZ == SWZ_K) return (D == 128) ? (row & 15) : (D == 64) ? ((row >> 1) & 7) : ((row >> 2) & 3);
    if (SWZ == SWZ_V) return ((D == 128) ? (row & 3) : (D == 64) ? ((row >> 1) & 1) : 0) << 2;
    return TileLayout<D>::u_swizzle(row);
}

// A wave's share of the loads of one 32-row tile, cooperatively with the NW waves of the
// workgroup: load instruction j = wave*IPW + i fills the LDS bytes [1024 j, 1024 (j+1)) of the
// tile, i.e. rows RPI*j ..  A tile of fewer than NW instructions (D = 32 with four waves) is
// loaded by the first ACTIVE_WAVES waves alone; the others issue nothing.  Every load stays
// inside the valid rows of the tile: rows past the end fetch the last valid row again (finite
// data; the kernels give them zero weight).
template <int D, int NW, int SWZ>
struct TileDma {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = KT * ROW;
    static constexpr int CHUNKS = D / 8;
    static constexpr int RPI = 1024 / ROW;        // rows written by one load instruction
    static constexpr int INSTR = TILE / 1024;     // load instructions per tile
    static constexpr int IPW = INSTR >= NW ? INSTR / NW : 1;  // load instructions per (active) wave per tile
    static constexpr int ACTIVE_WAVES = INSTR / IPW;
    static_assert(ACTIVE_WAVES >= 1 && ACTIVE_WAVES <= NW && ACTIVE_WAVES * IPW * 1024 == TILE,
                  "tile does not split evenly over the waves");
    uint32_t voff[IPW], row_bytes;
    int lane_, wave_;

    __device__ __forceinline__ static int row_of(int lane, int wave, int i) { return (wave * IPW + i) * RPI + lane / CHUNKS; }
    __device__ __forceinline__ static int chunk16_of(int lane, int row) {
        return ((lane % CHUNKS) ^ swizzle_of_row<D, SWZ>(row)) * 16;
    }
    __device__ __forceinline__ void init(int lane, int wave, uint32_t row_stride_bytes) {
        row_bytes = row_stride_bytes;
        lane_ = lane;
        wave_ = wave;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int row = row_of(lane, wave, i);
            voff[i] = (uint32_t)row * row_bytes + chunk16_of(lane, row);
        }
    }
    // tile_base: first row of the tile (this head's columns); rows_left: valid rows from there
    // on (>= 1); lds_tile: LDS address of the tile.  Issues IPW loads (none in an idle wave).
    __device__ __forceinline__ bool active() const { return ACTIVE_WAVES == NW || wave_ < ACTIVE_WAVES; }
    __device__ __forceinline__ void issue(const char* tile_base, int rows_left, uint32_t lds_tile) const {
        if (!active()) return;
        const int rows = rows_left < KT ? rows_left : KT;
        // the descriptor and the LDS address are wave-uniform by construction; say so where the compiler
        // cannot prove it (they are scalar operands of the load)
        u32x4 rsrc = make_rsrc_words(tile_base, (uint32_t)(rows - 1) * row_bytes + ROW);
#pragma unroll
        for (int i = 0; i < 4; ++i) rsrc[i] = __builtin_amdgcn_readfirstlane(rsrc[i]);
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_tile + wave_ * IPW * 1024);
        if (rows == KT) {
#pragma unroll
            for (int i = 0; i < IPW; ++i) load_to_lds_b128(rsrc, voff[i], 0, dst + i * 1024);
        } else {  // the last tile of a sequence: offsets recomputed with the row clamped
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                const int row = row_of(lane_, wave_, i);
                const uint32_t rb = (uint32_t)(row < rows ? row : rows - 1) * row_bytes;
                load_to_lds_b128(rsrc, rb + chunk16_of(lane_, row), 0, dst + i * 1024);
            }
        }
    }
};

// Prologue staging of up to 32*NW rows (global rows from `base`, row stride row_bytes, n_rows
// valid, the rest read as zero) through registers into LDS as NW consecutive 32-row tiles in the
// K-tile swizzle, whole rows coalesced.  Caller synchronises.
template <int D, int NW>
__device__ __forceinline__ void stage_rows_swizzled(char* lds, const char* base, uint32_t row_bytes, int n_rows, int tid) {
    using L = TileLayout<D>;
    constexpr int CHUNKS = D / 8;
    constexpr int ROWS_PER_LOAD = 64 * NW / CHUNKS;
    constexpr int N_LOADS = 32 * NW / ROWS_PER_LOAD;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (n_rows - 1) * (int)row_bytes + D * 2, 0x00020000);
    const int row0 = tid / CHUNKS, ch = tid % CHUNKS;
    u32x4 st[N_LOADS];
#pragma unroll
    for (int i = 0; i < N_LOADS; ++i)
        st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (uint32_t)row0 * row_bytes + ch * 16, i * ROWS_PER_LOAD * row_bytes, 0);
#pragma unroll
    for (int i = 0; i < N_LOADS; ++i) {
        const int row = i * ROWS_PER_LOAD + row0;
        *(u32x4*)(lds + (row / KT) * L::TILE_BYTES + L::k_offset(row % KT, ch)) = st[i];
    }
}

}  // namespace kunlun
