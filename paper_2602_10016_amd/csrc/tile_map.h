// Work mapping of the tiled launches (query tiles of the forward kernel and of the backward
// dQ pass, key tiles of the backward dK/dV pass): grid = H * (tiles of all examples), cut into
// 8 contiguous ranges, one per XCD (workgroup i runs on XCD i % 8), so that the tiles of one
// (example, head) - which share their operands - meet in the same L2.  Items are ordered by
// example, then tile, then head.  tile_start[b] = number of tiles before example b and
// tile_example[t] = example of tile t (both written by the prefix kernel), so a workgroup finds
// its item with two dependent loads.
// An XCD's range is further cut into `runs` contiguous runs that are issued round-robin:
// workgroups that follow each other in a run start `runs` slots apart, so that the next tile of
// an (example, head) starts when its predecessor is about one tile width into its window and
// both read the rows they share at about the same time.
#pragma once
#include "common.h"

namespace kunlun {

constexpr int TILE_ROWS = 128;  // rows (queries or keys) per tile of every tiled launch: 4 waves x 32

inline size_t tile_table_bytes(int B, int64_t total_rows) {
    return align_up((size_t)(B + 1) * sizeof(int32_t), 256) +
           align_up((size_t)(total_rows / TILE_ROWS + B) * sizeof(int32_t), 256);
}
inline int32_t* tile_example_of(int32_t* tile_start, int B) {
    return (int32_t*)((char*)tile_start + align_up((size_t)(B + 1) * sizeof(int32_t), 256));
}
// grid size (an upper bound of the tile count sizes it; surplus workgroups exit at once)
inline unsigned tile_grid(int B, int H, int64_t total_rows, int runs) {
    const int64_t per_xcd = ((total_rows / TILE_ROWS + B) * H + 7) / 8;
    return (unsigned)((per_xcd + runs) * 8);
}
// Stagger for a window of finite reach: a tile shares rows with (reach / tile) neighbours on
// each side; with about 96 workgroups resident per XCD, the next tile of an (example, head) -
// H items further in item order - should start 96 / (neighbours + 1) slots later.
inline int tile_runs(bool windowed, int left, int right, int H) {
    if (!windowed || left < 0 || right < 0) return 1;
    const int64_t span_tiles = ((int64_t)left + right + TILE_ROWS - 1) / TILE_ROWS + 1;
    const int64_t want = 96 / span_tiles / H;
    return (int)(want < 1 ? 1 : (want > 32 ? 32 : want));
}

#ifdef __HIPCC__
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ tile_start,
                                            const int32_t* __restrict__ tile_example, int B, int H, int runs, int& b,
                                            int& h, int& t) {
    const int64_t n_items = (int64_t)tile_start[B] * H;
    const int64_t per_xcd = (n_items + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t run_len = (per_xcd + runs - 1) / runs;
    const int64_t in_xcd = (slot % runs) * run_len + slot / runs;
    if (slot >= run_len * runs || in_xcd >= per_xcd) return false;
    const int64_t item = xcd * per_xcd + in_xcd;
    if (item >= n_items) return false;
    const int tile = (int)(item / H);
    h = (int)(item % H);
    b = tile_example[tile];
    t = tile - tile_start[b];
    return true;
}

// Exclusive prefix sum of ceil(len_b / tile_rows) over the examples, and the example of every
// tile; single workgroup of 1024 threads.  off == null: every example has `dense_len` rows.
// tile_rows is TILE_ROWS or a multiple of it (a workgroup that walks several tiles).
// (A template only so that every translation unit that launches it carries its own copy.)
template <int UNUSED>
__global__ __launch_bounds__(1024) void tile_prefix_kernel(const int32_t* __restrict__ off, int dense_len, int B,
                                                           int32_t* __restrict__ tile_start,
                                                           int32_t* __restrict__ tile_example, int tile_rows) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (B + 1023) / 1024;
    const int b0 = tid * per, b1 = (b0 + per < B) ? b0 + per : B;
    auto tiles_of = [&](int b) { return ((off ? off[b + 1] - off[b] : dense_len) + tile_rows - 1) / tile_rows; };
    int sum = 0;
    for (int b = b0; b < b1; ++b) sum += tiles_of(b);
    part[tid] = sum;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int v = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int run = part[tid] - sum;
    for (int b = b0; b < b1; ++b) {
        tile_start[b] = run;
        const int n = tiles_of(b);
        for (int t = 0; t < n; ++t) tile_example[run + t] = b;
        run += n;
    }
    if (tid == 1023) tile_start[B] = part[1023];
}
#endif  // __HIPCC__

}  // namespace kunlun
