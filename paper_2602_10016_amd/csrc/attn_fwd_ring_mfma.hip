// bf16 matrix-core forward kernel for the query-tiled launches (gfx950): sliding-window
// self-attention (Eq. (sliding window)) and GDPA with long query sequences (Eq. (GDPA), the
// PFFN direction: sequence tokens are the queries, a few context tokens per example are keys).
//
// A workgroup of NW wavefronts owns one (example, head, tile of 32*NW queries); each wave owns
// 32 of those queries and the waves walk the 32-key K/V tiles of the item together.  The
// arithmetic per tile is that of the streaming forward kernel (S^T = K Q^T, score function in
// registers, O^T += V^T P^T); what differs is how tiles travel.  A step of this kernel costs
// one full memory round trip if only one tile is in flight, and the window makes steps many
// and short, so the tiles are moved by the buffer-load-to-LDS path (no staging registers)
// into a ring of three LDS stages: while tile t is consumed, tiles t+1 and t+2 are in flight.
// The loads are written in assembly because the compiler would otherwise wait for ALL
// outstanding loads before every LDS read; the kernel counts its own loads (vmcnt) instead.
//
// LDS tiles are unpadded (a load instruction writes 64 consecutive 16-byte slots) and bank
// conflicts are avoided by an XOR swizzle that is applied on the global side: slot (row, pos)
// of a K tile receives the 16-byte chunk pos ^ xk(row) of the row, of a V tile the chunk
// pos ^ 4*xv(row) (TileLayout::k_offset / v_offset give the matching read addresses).
#include "attn_fwd_score.h"

namespace kunlun {

template <int D, int NW>
struct RingSmem {
    static constexpr int ROW = D * 2;
    static constexpr int TILE = KT * ROW;          // one K or V tile
    static constexpr int STAGE = 2 * TILE;         // K tile, then V tile
    static constexpr int STAGES = 3;
    static constexpr int TOTAL = STAGES * STAGE;
    static constexpr int QT = 32 * NW;             // queries per workgroup
    static constexpr int Q_BYTES = QT * ROW;       // query tile, K-tile layout, at the END of the ring
    static constexpr int O_STRIDE = ROW + 16;      // output staging rows (padded)
    static_assert(Q_BYTES <= 2 * STAGE, "the query tile may cover at most the last two stages");
    static_assert(QT * O_STRIDE <= TOTAL, "output staging must fit");
    // true: the query tile also covers the stage of the second key tile
    static constexpr bool Q_COVERS_STAGE1 = Q_BYTES > STAGE;
};

// 128-bit buffer descriptor: base address, byte count, raw 32-bit addressing.
__device__ __forceinline__ u32x4 make_rsrc_words(const void* base, uint32_t bytes) {
    const uint64_t a = (uint64_t)base;
    const u32x4 r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
    return r;
}

// One wave-wide 16-byte-per-lane load from a buffer straight into LDS: lane l's 16 bytes land
// at lds_addr + 16*l.  voff: per-lane byte offset, soff: uniform byte offset.  Counted by vmcnt.
__device__ __forceinline__ void load_to_lds_b128(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory");
}

// s_waitcnt that waits only for the vector-memory counter to drop to n (other counters untouched).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void attn_fwd_ring_item(const AttnParams& p, char* lds, int h, int64_t q_row0, int nq_wg,
                                                   int64_t t0_wg, int64_t k0, int n_kv) {
    using SM = RingSmem<D, NW>;
    using L = TileLayout<D>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16;
    constexpr int DB = D / 32;
    constexpr int CHUNKS = D / 8;
    constexpr int RPI = 1024 / SM::ROW;            // rows written by one load instruction
    constexpr int IPW = SM::TILE / 1024 / NW;      // load instructions per wave per tile and tensor
    static_assert(IPW >= 1 && SM::TILE % (1024 * NW) == 0, "tile does not split evenly over the waves");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* K = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* V = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

    // this wave's queries
    const int q_lo_w = wave * 32;
    int nq = nq_wg - q_lo_w;
    nq = nq < 0 ? 0 : (nq > 32 ? 32 : nq);
    const bool wave_active = nq > 0;
    const int64_t t0 = t0_wg + q_lo_w;

    // key tiles of the workgroup, and of this wave
    int kt_begin = 0, kt_end = (n_kv + KT - 1) / KT;
    int w_begin = 0, w_end = kt_end;
    if (WINDOWED && n_kv > 0) {
        int64_t lo = 0, hi = n_kv - 1;
        if (p.left >= 0 && t0_wg - p.left > lo) lo = t0_wg - p.left;
        if (p.right >= 0 && t0_wg + nq_wg - 1 + p.right < hi) hi = t0_wg + nq_wg - 1 + p.right;
        kt_begin = (int)(lo / KT);
        kt_end = (int)(hi / KT) + 1;
        lo = 0; hi = n_kv - 1;
        if (p.left >= 0 && t0 - p.left > lo) lo = t0 - p.left;
        if (p.right >= 0 && t0 + nq - 1 + p.right < hi) hi = t0 + nq - 1 + p.right;
        w_begin = (int)(lo / KT);
        w_end = (int)(hi / KT) + 1;
    }

    // ---- tile transport.  Load instruction j = wave*IPW + i of a tile fills the LDS bytes
    // [1024 j, 1024 (j+1)): rows RPI*j .. ; lane -> (row, slot) -> swizzled source chunk.
    uint32_t k_voff[IPW], v_voff[IPW];
    int src_row[IPW], k_chunk[IPW], v_chunk[IPW];
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int row = (wave * IPW + i) * RPI + lane / CHUNKS, pos = lane % CHUNKS;
        const int xk = (D == 128) ? (row & 15) : ((row >> 1) & 7);
        const int xv = (D == 128) ? (row & 3) : ((row >> 1) & 1);
        src_row[i] = row;
        k_chunk[i] = (pos ^ xk) * 16;
        v_chunk[i] = (pos ^ (xv << 2)) * 16;
        k_voff[i] = (uint32_t)row * row_bytes + k_chunk[i];
        v_voff[i] = (uint32_t)row * row_bytes + v_chunk[i];
    }
    // Every load stays inside the valid rows of its tile: rows past the end of the history
    // fetch the last valid row again (finite data; their weights are zero).
    auto issue = [&](int kt, int stage) {
        const int rows_left = n_kv - kt * KT;
        const int rows = rows_left < KT ? rows_left : KT;
        const uint32_t bytes = (uint32_t)(rows - 1) * row_bytes + SM::ROW;
        const u32x4 kr = make_rsrc_words(K + kt * tile_bytes, bytes);
        const u32x4 vr = make_rsrc_words(V + kt * tile_bytes, bytes);
        const uint32_t dst = lds0 + stage * SM::STAGE + wave * IPW * 1024;
        if (rows == KT) {
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                load_to_lds_b128(kr, k_voff[i], 0, dst + i * 1024);
                load_to_lds_b128(vr, v_voff[i], 0, dst + SM::TILE + i * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                const uint32_t rb = (uint32_t)(src_row[i] < rows ? src_row[i] : rows - 1) * row_bytes;
                load_to_lds_b128(kr, rb + k_chunk[i], 0, dst + i * 1024);
                load_to_lds_b128(vr, rb + v_chunk[i], 0, dst + SM::TILE + i * 1024);
            }
        }
    };

    // ---- prologue.  The first key tile starts its journey at once (stage 0); the query tile
    // goes through registers into the end of the ring (whole rows, K-tile swizzle) and every
    // wave picks its B-operand fragments: column = query r, contraction = channels 16*kc + 8g ..
    const int n_steps = kt_end - kt_begin;
    if (n_steps > 0) issue(kt_begin, 0);
    if (!SM::Q_COVERS_STAGE1 && n_steps > 1) issue(kt_begin + 1, 1);
    constexpr int Q_LOADS = SM::QT * CHUNKS / (64 * NW);
    bf16x8 qf[KC];
    {
        char* qstage = lds + SM::TOTAL - SM::Q_BYTES;
        const char* qbase = (const char*)((const bf16_t*)p.q + q_row0 * hd + (int64_t)h * D);
        const __amdgpu_buffer_rsrc_t qrsrc =
            __builtin_amdgcn_make_buffer_rsrc((void*)qbase, 0, (nq_wg - 1) * (int)row_bytes + D * 2, 0x00020000);
        u32x4 qst[Q_LOADS];
        constexpr int ROWS_PER_LOAD = 64 * NW / CHUNKS;
        const int qrow = tid / CHUNKS, qch = tid % CHUNKS;
#pragma unroll
        for (int i = 0; i < Q_LOADS; ++i)  // rows past the tile read as zero
            qst[i] = __builtin_amdgcn_raw_buffer_load_b128(qrsrc, (uint32_t)qrow * row_bytes + qch * 16,
                                                           i * ROWS_PER_LOAD * row_bytes, 0);
#pragma unroll
        for (int i = 0; i < Q_LOADS; ++i) {
            const int row = i * ROWS_PER_LOAD + qrow;  // the swizzle has period 16 (or 32) rows
            *(u32x4*)(qstage + (row / KT) * SM::TILE + L::k_offset(row % KT, qch)) = qst[i];
        }
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
            qf[kc] = *(const bf16x8*)(qstage + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
        __syncthreads();  // the query tile's stages may now receive key tiles
    }
    if (SM::Q_COVERS_STAGE1 && n_steps > 1) issue(kt_begin + 1, 1);

    // visible keys of this lane's query: key_lo .. key_lo + key_span (an empty range for padding
    // lanes whose query lies past the end)
    int key_lo;
    unsigned key_span;
    {
        const int tq = (int)t0 + r;
        int lo = 0, hi = n_kv - 1;
        if (WINDOWED) {
            if (p.left >= 0 && tq - p.left > lo) lo = tq - p.left;
            if (p.right >= 0 && tq + p.right < hi) hi = tq + p.right;
        }
        const bool empty = hi < lo;
        key_lo = empty ? 0x3fffffff : lo;
        key_span = empty ? 0u : (unsigned)(hi - lo);
    }

    f32x16 oacc[DB][1];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][0][v] = 0.f;
    float m_ref = -INFINITY, l_run = 0.f;
    const float sc = SOFTMAX ? p.scale * LOG2E : p.scale;

    // LDS read offsets of this lane inside a stage.  K fragment of contraction step kc (A
    // operand: row r, channels 16*kc + 8g ..): k_rd ^ (kc << 5).  V^T fragment of channel block db
    // for the keys in registers 8c..8c+7 of the score layout (keys 16c + 4g + 0..3 and 16c + 8 +
    // 4g + 0..3): two transposing reads at (v_rd ^ (db << 6)) + 16c rows (+ 8 rows); in each,
    // the 16 lanes of a group address a 4 (keys) x 16 (channels) block - lane s points at key
    // s/4, channels 4*(s%4) .. - and lane i receives channel i of the four keys.
    const int k_rd = L::k_offset(r, g);
    const int v_rd = SM::TILE + L::v_offset(4 * g + ((lane & 15) >> 2), (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);

    auto compute = [&](const char* st, int kt) {
        if (!wave_active || kt < w_begin || kt >= w_end) return;
        // ---- S^T = K Q^T
        f32x16 sacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 a = *(const bf16x8*)(st + (k_rd ^ (kc << 5)));
            sacc = mfma32(a, qf[kc], sacc);
        }
        // ---- score function, masking, packing
        const int key_base = kt * KT;
        bool need_mask = key_base + KT > n_kv;
        if (WINDOWED) {
            // interior tile: every (query, key) pair of the tile is inside the window
            const int tq_lo = (int)t0, tq_hi = (int)t0 + nq - 1;
            if (p.left >= 0 && key_base < tq_hi - p.left) need_mask = true;
            if (p.right >= 0 && key_base + KT - 1 > tq_lo + p.right) need_mask = true;
        }
        bf16x8 pf[2];
        score_to_weights<ACT, DB, 1>(sacc, need_mask, (unsigned)(key_base + 4 * g - key_lo), key_span, sc, m_ref, l_run,
                                     oacc, 0, pf);
        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const char* src = st + (v_rd ^ (db << 6)) + c * 16 * SM::ROW;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src + 8 * SM::ROW));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const bf16x8 a = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[db][0] = mfma32(a, pf[c], oacc[db][0]);
            }
        }
    };

    // ---- main loop: tile kt_begin + i lives in stage i % 3.  Per step: wait for the wave's own
    // loads of the tile (the loads of the next tile may still be in flight), barrier (the tile
    // is complete, and every wave is done with the stage of the tile before it), send the loads
    // of the tile two steps ahead into that freed stage, compute.
    int stage = 0;
    for (int i = 0; i < n_steps; ++i) {
        if (i + 1 < n_steps) wait_vmcnt<2 * IPW>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (i + 2 < n_steps) issue(kt_begin + i + 2, stage == 0 ? 2 : stage - 1);
        compute(lds + stage * SM::STAGE, kt_begin + i);
        stage = stage == 2 ? 0 : stage + 1;
    }

    // ---- epilogue: lane holds query r, channels 32*db + 8*(v/4) + 4g + (v%4).  The wave
    // transposes its O tile through LDS (its own region of the now idle ring) and writes whole
    // rows, 16 bytes per lane.
    __syncthreads();  // every wave is done with the K/V tiles
    if (!wave_active) return;
    char* ostage = lds + wave * (32 * SM::O_STRIDE);
    {
        float inv = 1.f;
        if (SOFTMAX) {
            const float l_tot = halves_sum(l_run);
            inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            if (p.lse && g == 0 && r < nq)
                p.lse[(int64_t)h * p.total_q + q_row0 + q_lo_w + r] =
                    l_tot > 0.f ? (m_ref + __builtin_amdgcn_logf(l_tot)) * (1.f / LOG2E) : -INFINITY;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                bf16x4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (bf16_t)(oacc[db][0][4 * vg + e] * inv);
                *(bf16x4*)(ostage + r * SM::O_STRIDE + (32 * db + 8 * vg + 4 * g) * 2) = out;
            }
    }
    {
        bf16_t* obase = (bf16_t*)p.o + (q_row0 + q_lo_w) * hd + (int64_t)h * D;
        constexpr int O_STORES = 32 * CHUNKS / 64;
        const int chunk = lane % CHUNKS, rsub = lane / CHUNKS;
#pragma unroll
        for (int i = 0; i < O_STORES; ++i) {
            const int row = i * (64 / CHUNKS) + rsub;
            const u32x4 val = *(const u32x4*)(ostage + row * SM::O_STRIDE + chunk * 16);
            if (row < nq) *(u32x4*)(obase + row * hd + chunk * 8) = val;
        }
    }
}

// Query-tiled launch: grid = H * (query tiles of all examples), cut into 8 contiguous ranges,
// one per XCD (workgroup i runs on XCD i % 8), so that the query tiles of one (example, head)
// - which share their keys - meet in the same L2.  Items are ordered by example, then query
// tile, then head.  tile_start[b] = number of query tiles before example b and tile_example[t]
// = example of query tile t (both written by the prefix kernel), so a workgroup finds its
// item with two dependent loads.
// An XCD's range is further cut into `runs` contiguous runs that are issued round-robin:
// workgroups that follow each other in a run start `runs` slots apart, so that the next query
// tile of an (example, head) starts when its predecessor is about one tile width into its
// window and both read the keys they share at about the same time.
template <int D, int NW, int OCC, bool WINDOWED>
__global__ __launch_bounds__(64 * NW, OCC) void qtile_fwd_mfma_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                                      const int32_t* __restrict__ tile_example, int runs) {
    __shared__ __attribute__((aligned(1024))) char lds[RingSmem<D, NW>::TOTAL];
    constexpr int QT = 32 * NW;
    const int64_t n_items = (int64_t)tile_start[p.B] * p.H;
    const int64_t per_xcd = (n_items + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t run_len = (per_xcd + runs - 1) / runs;
    const int64_t in_xcd = (slot % runs) * run_len + slot / runs;
    if (slot >= run_len * runs || in_xcd >= per_xcd) return;
    const int64_t item = xcd * per_xcd + in_xcd;
    if (item >= n_items) return;
    const int tile = (int)(item / p.H);
    const int h = (int)(item % p.H);
    const int b = tile_example[tile];
    const int qt = tile - tile_start[b];
    const int64_t k0 = p.kv_off[b];
    const int n_kv = p.kv_off[b + 1] - (int)k0;
    const int64_t q0 = q_begin(p, b);
    const int64_t nq_all = q_end(p, b) - q0;
    const int64_t q_first = (int64_t)qt * QT;
    const int nq = (int)((nq_all - q_first) < QT ? (nq_all - q_first) : QT);
    if (WINDOWED) {
        attn_fwd_ring_item<D, NW, KUNLUN_ACT_SOFTMAX, true>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv);
    } else {
        switch (p.head_act[h]) {
        case KUNLUN_ACT_SOFTMAX: attn_fwd_ring_item<D, NW, KUNLUN_ACT_SOFTMAX, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        case KUNLUN_ACT_IDENTITY: attn_fwd_ring_item<D, NW, KUNLUN_ACT_IDENTITY, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        case KUNLUN_ACT_RELU: attn_fwd_ring_item<D, NW, KUNLUN_ACT_RELU, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        case KUNLUN_ACT_GELU: attn_fwd_ring_item<D, NW, KUNLUN_ACT_GELU, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        case KUNLUN_ACT_GELU_TANH: attn_fwd_ring_item<D, NW, KUNLUN_ACT_GELU_TANH, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        default: attn_fwd_ring_item<D, NW, KUNLUN_ACT_SILU, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        }
    }
}

// Exclusive prefix sum of ceil(len_b / tile) over the examples, and the example of every tile;
// single workgroup.  off == null: every example has `dense_len` rows.
__global__ __launch_bounds__(1024) void tile_prefix_kernel(const int32_t* __restrict__ off, int dense_len, int B,
                                                           int tile, int32_t* __restrict__ tile_start,
                                                           int32_t* __restrict__ tile_example) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (B + 1023) / 1024;
    const int b0 = tid * per, b1 = (b0 + per < B) ? b0 + per : B;
    auto tiles_of = [&](int b) { return ((off ? off[b + 1] - off[b] : dense_len) + tile - 1) / tile; };
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

size_t mfma_fwd_qtiled_workspace(int B, int64_t total_q) {
    return align_up((size_t)(total_q / 128 + B) * sizeof(int32_t), 256);  // tile_example
}

template <int D, int NW, int OCC, bool WINDOWED>
static hipError_t launch_qtiled(const AttnParams& p, void* workspace_tail, hipStream_t stream) {
    // an upper bound of the query-tile count sizes the grid
    constexpr int QT = 32 * NW;
    static_assert(QT == 128, "mfma_fwd_qtiled_workspace assumes 128-query tiles");
    const int64_t max_tiles = p.total_q / QT + p.B;
    const int64_t per_xcd = (max_tiles * p.H + 7) / 8;
    // Window of finite reach: a tile shares keys with (reach / QT) neighbours on each side.  With
    // about 96 workgroups resident per XCD, the next tile of an (example, head) - H items
    // further in item order - should start 96 / (neighbours + 1) slots later.
    int runs = 1;
    if (WINDOWED && p.left >= 0 && p.right >= 0) {
        const int64_t span_tiles = ((int64_t)p.left + p.right + QT - 1) / QT + 1;
        const int64_t want = 96 / span_tiles / p.H;
        runs = (int)(want < 1 ? 1 : (want > 32 ? 32 : want));
    }
    const unsigned grid = (unsigned)((per_xcd + runs) * 8);
    int32_t* tile_start = const_cast<int32_t*>(p.order);
    int32_t* tile_example = (int32_t*)workspace_tail;
    hipLaunchKernelGGL(tile_prefix_kernel, dim3(1), dim3(1024), 0, stream, p.q_off, p.max_q, p.B, QT, tile_start,
                       tile_example);
    hipLaunchKernelGGL((qtile_fwd_mfma_kernel<D, NW, OCC, WINDOWED>), dim3(grid), dim3(64 * NW), 0, stream, p, tile_start,
                       tile_example, runs);
    return hipGetLastError();
}

hipError_t launch_mfma_fwd_qtiled(const AttnParams& p, void* workspace_tail, hipStream_t stream) {
    // 128-query tiles (4 waves of 32 queries)
    if (p.windowed)
        return p.d == 128 ? launch_qtiled<128, 4, 2, true>(p, workspace_tail, stream)
                          : launch_qtiled<64, 4, 2, true>(p, workspace_tail, stream);
    return p.d == 128 ? launch_qtiled<128, 4, 2, false>(p, workspace_tail, stream)
                      : launch_qtiled<64, 4, 2, false>(p, workspace_tail, stream);
}

}  // namespace kunlun
