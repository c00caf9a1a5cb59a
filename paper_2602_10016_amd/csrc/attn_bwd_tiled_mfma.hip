// bf16 matrix-core backward in two passes, for the shapes the fused backward kernel does not
// take: sliding-window self-attention (Eq. (sliding window)) and GDPA / softmax attention with
// more than 64 queries per example (the PFFN direction of Eq. (GDPA): sequence tokens are the
// queries).  Scores are recomputed tile by tile in both passes; nothing of score size is stored.
//
//   pass A (dQ):     one workgroup per (example, 128-query tile, head), the mirror image of the
//                    forward kernel: each wave owns 32 queries (Q^T and dO^T fragments in
//                    registers) and the waves stream the K/V tiles of the tile's key range;
//                        S^T = K Q^T,  dP^T = V dO^T,  dS^T in registers,  dQ^T += K^T dS^T.
//   pass B (dK, dV): one workgroup per (example, 128-key tile, head): each wave owns 32 keys
//                    (K^T and V^T fragments in registers) and the waves stream the Q/dO tiles of
//                    the queries that see those keys;
//                        S = Q K^T,  dP = dO V^T,  P and dS in registers (one key per lane),
//                        dV^T += dO^T P,  dK^T += Q^T dS.
// In both passes the score tile comes out of the first contraction with the owned dimension
// on the lanes, so the packed registers are directly the B operand of the second contraction
// and the streamed operand is read transposed from LDS (ds_read_b64_tr_b16).  Streamed tiles
// travel by buffer-load-to-LDS into a ring of three stages (lds_ring.h); a tile that is read
// both as row fragments and transposed sits in LDS once, in the two-way swizzle.
// Softmax heads use the forward LSE and delta = rowsum(dO * O); pass A computes delta of its query
// tile from the O rows and leaves it in the workspace, pass B streams LSE and delta per query tile next
// to Q and dO.
// Long query sequences over at most 32 keys per example (the PFFN direction proper) take a third
// kernel at the end of this file that does everything in one pass over Q and dO.
#include "lds_ring.h"
#include "tile_map.h"

namespace kunlun {

constexpr float LOG2E_T = 1.4426950408889634f;

// Padded LDS tiles (32 rows): +16 bytes per row for row-fragment (A/B operand) reads, +64
// bytes per row for transposing reads; both conflict-free with affine offsets.
template <int D>
struct PadTiles {
    static constexpr int ROW_STRIDE = D * 2 + 16;
    static constexpr int TR_STRIDE = D * 2 + 64;
    static constexpr int ROW_TILE = KT * ROW_STRIDE;
    static constexpr int TR_TILE = KT * TR_STRIDE;
};

// A wave's 32 x D fp32 result tile in the C layout (lane: column r = row of the output tensor,
// registers: channels 32*db + 8*(v/4) + 4g + v%4) -> bf16 rows of a [tokens, H, D] tensor,
// transposed through the wave's own LDS region and written 16 bytes per lane.
template <int D>
__device__ __forceinline__ void store_block_staged(char* stage, const f32x16& acc, int db, int lane) {
    using PT = PadTiles<D>;
    const int r = lane & 31, g = lane >> 5;
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
        bf16x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (bf16_t)acc[4 * vg + e];
        *(bf16x4*)(stage + r * PT::ROW_STRIDE + (32 * db + 8 * vg + 4 * g) * 2) = out;
    }
}
template <int D>
__device__ __forceinline__ void store_staged_rows(const char* stage, bf16_t* out_rows, int64_t hd, int n_rows, int lane) {
    using PT = PadTiles<D>;
    constexpr int CHUNKS = D / 8;
    const int chunk = lane % CHUNKS, rsub = lane / CHUNKS;
#pragma unroll
    for (int i = 0; i < 32 * CHUNKS / 64; ++i) {
        const int row = i * (64 / CHUNKS) + rsub;
        const u32x4 val = *(const u32x4*)(stage + row * PT::ROW_STRIDE + chunk * 16);
        if (row < n_rows) __builtin_nontemporal_store(val, (u32x4*)(out_rows + row * hd + chunk * 8));
    }
}
template <int D>
__device__ __forceinline__ void store_tile_rows(char* stage, const f32x16 (&acc)[D / 32], bf16_t* out_rows, int64_t hd,
                                                int n_rows, int lane) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db) store_block_staged<D>(stage, acc[db], db, lane);
    store_staged_rows<D>(stage, out_rows, hd, n_rows, lane);
}

// One 8-element fragment from two transposing reads (rows .. +3 at a, rows .. +3 at b).
__device__ __forceinline__ bf16x8 tr_pair(const char* a, const char* b) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, b));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// LDS of both passes: a ring of three stages; the prologue stages the workgroup's own 128 rows
// (4 tiles, K-tile swizzle) in the end of the ring, and the epilogue transposes the results
// through padded rows.
template <int D, int STAGE_EXTRA>
struct TiledSmem {
    using PT = PadTiles<D>;
    static constexpr int TILE = KT * D * 2;
    static constexpr int STAGE = 2 * TILE + STAGE_EXTRA;
    static constexpr int TOTAL = 3 * STAGE;
    static constexpr int OWN_BYTES = 4 * TILE;
    static_assert(TOTAL - OWN_BYTES >= STAGE, "the staged rows must leave the first stage free");
    static_assert(4 * PT::ROW_TILE <= TOTAL, "output staging must fit");
};

// Per-lane LDS read offsets inside a tile in the two-way swizzle.
template <int D>
struct UFrag {
    int row0, trA, trB;
    __device__ __forceinline__ void init(int lane) {
        using L = TileLayout<D>;
        const int r = lane & 31, g = lane >> 5, s16 = lane & 15, hi16 = (lane >> 4) & 1;
        const int colb = (16 * hi16 + 4 * (s16 & 3)) * 2;
        row0 = L::u_offset(r, g * 16);                      // row fragment: row r, channels 16*kc + 8g ..: row0 ^ (kc << 5)
        trA = L::u_offset(4 * g + (s16 >> 2), colb);         // transposed: rows 16c + 4g + 0..3, channel block db: trA ^ (db << 6)
        trB = L::u_offset(8 + 4 * g + (s16 >> 2), colb);     //             rows 16c + 8 + 4g + 0..3
    }
    __device__ __forceinline__ bf16x8 row(const char* tile, int kc) const { return *(const bf16x8*)(tile + (row0 ^ (kc << 5))); }
    // A operand (row = channel 32*db + lane%32) for the 16 tile rows that the C layout puts in registers 8c .. 8c+7
    __device__ __forceinline__ bf16x8 transposed(const char* tile, int db, int c) const {
        const char* base = tile + c * 16 * D * 2;
        return tr_pair(base + (trA ^ (db << 6)), base + (trB ^ (db << 6)));
    }
};

#define KUNLUN_ACT_SWITCH(ACTV, CALL)                                   \
    switch (ACTV) {                                                     \
    case KUNLUN_ACT_SOFTMAX: { constexpr int A = KUNLUN_ACT_SOFTMAX; CALL; } break;     \
    case KUNLUN_ACT_IDENTITY: { constexpr int A = KUNLUN_ACT_IDENTITY; CALL; } break;   \
    case KUNLUN_ACT_RELU: { constexpr int A = KUNLUN_ACT_RELU; CALL; } break;           \
    case KUNLUN_ACT_GELU: { constexpr int A = KUNLUN_ACT_GELU; CALL; } break;           \
    case KUNLUN_ACT_GELU_TANH: { constexpr int A = KUNLUN_ACT_GELU_TANH; CALL; } break; \
    case KUNLUN_ACT_SILU: { constexpr int A = KUNLUN_ACT_SILU; CALL; } break;                        \
    default: { constexpr int A = KUNLUN_ACT_GELU_POLY; CALL; } break;                        \
    }

// ------------------------------------------------------------------ pass A: dQ

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void bwd_dq_item(const AttnParams& p, float* __restrict__ delta_ws, char* lds, int h,
                                            int64_t q_row0, int nq_wg, int64_t t0_wg, int64_t k0, int n_kv) {
    using PT = PadTiles<D>;
    using L = TileLayout<D>;
    using SM = TiledSmem<D, 0>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16, DB = D / 32;
    static_assert(NW == 4, "four waves of 32 queries");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* K = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* V = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);
    const uint32_t lds0 = lds_address(lds);

    const int q_lo_w = wave * 32;
    int nq = nq_wg - q_lo_w;
    nq = nq < 0 ? 0 : (nq > 32 ? 32 : nq);
    const bool wave_active = nq > 0;
    const int t0 = (int)t0_wg + q_lo_w;

    int kt_begin = 0, kt_end = (n_kv + KT - 1) / KT;
    int w_begin = 0, w_end = kt_end;
    if (WINDOWED && n_kv > 0) {
        int lo = 0, hi = n_kv - 1;
        if (p.left >= 0 && (int)t0_wg - p.left > lo) lo = (int)t0_wg - p.left;
        if (p.right >= 0 && (int)t0_wg + nq_wg - 1 + p.right < hi) hi = (int)t0_wg + nq_wg - 1 + p.right;
        kt_begin = lo / KT;
        kt_end = hi / KT + 1;
        lo = 0; hi = n_kv - 1;
        if (p.left >= 0 && t0 - p.left > lo) lo = t0 - p.left;
        if (p.right >= 0 && t0 + nq - 1 + p.right < hi) hi = t0 + nq - 1 + p.right;
        w_begin = lo / KT;
        w_end = hi / KT + 1;
    }

    // stage = K tile (two-way swizzle: row fragments and transposed reads) | V tile (row fragments)
    TileDma<D, NW, SWZ_U> kdma;
    TileDma<D, NW, SWZ_K> vdma;
    kdma.init(lane, wave, row_bytes);
    vdma.init(lane, wave, row_bytes);
    constexpr int LOADS_PER_TILE = 2 * TileDma<D, NW, SWZ_U>::IPW;
    auto issue = [&](int kt, int stage) {
        const uint32_t dst = lds0 + stage * SM::STAGE;
        kdma.issue(K + kt * tile_bytes, n_kv - kt * KT, dst);
        vdma.issue(V + kt * tile_bytes, n_kv - kt * KT, dst + SM::TILE);
    };
    const int n_steps = kt_end - kt_begin;
    if (n_steps > 0) issue(kt_begin, 0);

    // Q^T and dO^T fragments of this wave's queries (B operands), via the end of the ring
    bf16x8 qf[KC], dof[KC];
    {
        char* own = lds + SM::TOTAL - SM::OWN_BYTES;
        const int64_t goff = q_row0 * hd + (int64_t)h * D;
        stage_rows_swizzled<D, NW>(own, (const char*)((const bf16_t*)p.q + q_src_row(p, q_row0) * hd + (int64_t)h * D), row_bytes, nq_wg, tid);
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = *(const bf16x8*)(own + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
        __syncthreads();
        stage_rows_swizzled<D, NW>(own, (const char*)((const bf16_t*)p.d_o + goff), row_bytes, nq_wg, tid);
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) dof[kc] = *(const bf16x8*)(own + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
        __syncthreads();
    }
    // this lane's query: softmax statistics.  delta = rowsum(dO * O) is computed here from the O rows of the
    // tile (the dO fragments are at hand; each lane half covers half of the channels) and stored for pass B.
    float lse2 = INFINITY, delta = 0.f;
    if (SOFTMAX) {
        char* own = lds + SM::TOTAL - SM::OWN_BYTES;
        stage_rows_swizzled<D, NW>(own, (const char*)((const bf16_t*)p.o + q_row0 * hd + (int64_t)h * D), row_bytes, nq_wg, tid);
        __syncthreads();
        float part = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 of = *(const bf16x8*)(own + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
#pragma unroll
            for (int e = 0; e < 8; ++e) part = fmaf((float)of[e], (float)dof[kc][e], part);
        }
        delta = halves_sum(part);
        if (r < nq) {
            const int64_t idx = (int64_t)h * p.total_q + q_row0 + q_lo_w + r;
            lse2 = p.lse[idx] * LOG2E_T;
            if (g == 0) delta_ws[idx] = delta;
        }
        __syncthreads();
    }
    if (n_steps > 1) issue(kt_begin + 1, 1);
    int key_lo;
    unsigned key_span;
    {
        const int tq = t0 + r;
        int lo = 0, hi = n_kv - 1;
        if (WINDOWED) {
            if (p.left >= 0 && tq - p.left > lo) lo = tq - p.left;
            if (p.right >= 0 && tq + p.right < hi) hi = tq + p.right;
        }
        const bool empty = hi < lo || r >= nq;
        key_lo = empty ? 0x3fffffff : lo;
        key_span = empty ? 0u : (unsigned)(hi - lo);
    }

    f32x16 dqacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) dqacc[db][v] = 0.f;
    const float sc = SOFTMAX ? p.scale * LOG2E_T : p.scale;
    UFrag<D> uf;
    uf.init(lane);
    const int v_rd = L::k_offset(r, g);  // V row fragment: v_rd ^ (kc << 5)

    int stage = 0;
    for (int i = 0; i < n_steps; ++i) {
        // the loads above were issued before the lse / delta loads that the compiler tracks, so
        // its own waits can only be stricter than needed
        if (i + 1 < n_steps) wait_vmcnt<LOADS_PER_TILE>();
        else wait_vmcnt<0>();
        __syncthreads();  // tile i complete; every wave is done with the stage of tile i-1
        if (i + 2 < n_steps) issue(kt_begin + i + 2, stage == 0 ? 2 : stage - 1);
        const char* ldsK = lds + stage * SM::STAGE;
        const char* ldsV = ldsK + SM::TILE;
        stage = stage == 2 ? 0 : stage + 1;
        const int kt = kt_begin + i;
        if (!wave_active || kt < w_begin || kt >= w_end) continue;
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 ka = uf.row(ldsK, kc);
            const bf16x8 va = *(const bf16x8*)(ldsV + (v_rd ^ (kc << 5)));
            sacc = mfma32(ka, qf[kc], sacc);
            dpacc = mfma32(va, dof[kc], dpacc);
        }
        // dS^T in registers (lane: query, registers: keys of the tile).  Interior tiles - every
        // (query, key) pair inside the history and the window - skip the visibility test.
        const int key_base = kt * KT;
        bool need_mask = key_base + KT > n_kv;
        if (WINDOWED) {
            const int tq_lo = t0, tq_hi = t0 + nq - 1;
            if (p.left >= 0 && key_base < tq_hi - p.left) need_mask = true;
            if (p.right >= 0 && key_base + KT - 1 > tq_lo + p.right) need_mask = true;
        }
        float dsv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float s = sacc[v] * sc;
            if (SOFTMAX) {
                dsv[v] = fast_exp2(s - lse2) * (dpacc[v] - delta) * p.scale;
            } else {
                float val, der;
                act_fast_vd<ACT>(s, val, der);
                dsv[v] = dpacc[v] * der * p.scale;
            }
        }
        if (need_mask) {
            const unsigned rel0 = (unsigned)(key_base + 4 * g - key_lo);
#pragma unroll
            for (int v = 0; v < 16; ++v) dsv[v] = rel0 + (unsigned)(8 * (v >> 2) + (v & 3)) <= key_span ? dsv[v] : 0.f;
        }
        bf16x8 dsf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) dsf[c][e] = (bf16_t)dsv[8 * c + e];
        // dQ^T += K^T dS^T
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int c = 0; c < 2; ++c) dqacc[db] = mfma32(uf.transposed(ldsK, db, c), dsf[c], dqacc[db]);
    }
    __syncthreads();  // every wave is done with the ring
    if (!wave_active) return;
    store_tile_rows<D>(lds + wave * PT::ROW_TILE, dqacc, (bf16_t*)p.dq + (q_row0 + q_lo_w) * hd + (int64_t)h * D, hd, nq,
                       lane);
}

// ------------------------------------------------------------------ pass B: dK, dV

constexpr int STATS_BYTES = 512;  // per stage: lse of 64 queries (32 used), then delta of 64 queries

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void bwd_dkdv_item(const AttnParams& p, const float* __restrict__ delta_ws, char* lds, int h,
                                              int64_t k_row0, int nk_wg, int kpos0_wg, int64_t q0, int nq_all) {
    using PT = PadTiles<D>;
    using L = TileLayout<D>;
    using SM = TiledSmem<D, STATS_BYTES>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16, DB = D / 32;
    // At d = 128 the accumulators (128 registers) and the K^T, V^T fragments (64) leave too little
    // room for the rest; values parked in scratch memory would be reloaded with vector-memory
    // loads inside the loop, and the compiler waits for those together with the tile loads in flight.  The last K_LDS
    // K^T fragments of every wave are parked in LDS instead, lane by lane, behind the ring.
    constexpr int K_LDS = D == 128 ? 3 : 0, K_REG = KC - K_LDS;
    static_assert(NW == 4, "four waves of 32 keys");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* Q = (const char*)((const bf16_t*)p.q + (q_src_row(p, q0) * p.H + h) * D);
    const char* DO = (const char*)((const bf16_t*)p.d_o + (q0 * p.H + h) * D);
    const uint32_t lds0 = lds_address(lds);

    const int k_lo_w = wave * 32;
    int nk = nk_wg - k_lo_w;
    nk = nk < 0 ? 0 : (nk > 32 ? 32 : nk);
    const bool wave_active = nk > 0;
    const int kpos_w = kpos0_wg + k_lo_w;  // position of this wave's first key in its sequence

    // query tiles that see the workgroup's keys, and this wave's keys
    int qt_begin = 0, qt_end = (nq_all + KT - 1) / KT;
    int w_begin = 0, w_end = qt_end;
    if (WINDOWED && nq_all > 0) {
        int lo = 0, hi = nq_all - 1;
        if (p.right >= 0 && kpos0_wg - p.right > lo) lo = kpos0_wg - p.right;
        if (p.left >= 0 && kpos0_wg + nk_wg - 1 + p.left < hi) hi = kpos0_wg + nk_wg - 1 + p.left;
        qt_begin = lo / KT;
        qt_end = hi / KT + 1;
        lo = 0; hi = nq_all - 1;
        if (p.right >= 0 && kpos_w - p.right > lo) lo = kpos_w - p.right;
        if (p.left >= 0 && kpos_w + nk - 1 + p.left < hi) hi = kpos_w + nk - 1 + p.left;
        w_begin = lo / KT;
        w_end = hi / KT + 1;
    }

    // stage = Q tile | dO tile (both in the two-way swizzle) | lse and delta of the tile's queries
    TileDma<D, NW, SWZ_U> dma;
    dma.init(lane, wave, row_bytes);
    constexpr int LOADS_PER_TILE = 2 * TileDma<D, NW, SWZ_U>::IPW + (SOFTMAX ? 2 : 0);
    u32x4 lse_rsrc = {0, 0, 0, 0}, delta_rsrc = {0, 0, 0, 0};
    if (SOFTMAX && nq_all > 0) {
        const int64_t first = (int64_t)h * p.total_q + q0;
        lse_rsrc = make_rsrc_words(p.lse + first, (uint32_t)nq_all * 4);
        delta_rsrc = make_rsrc_words(delta_ws + first, (uint32_t)nq_all * 4);
    }
    auto issue = [&](int qt, int stage) {
        const uint32_t dst = lds0 + stage * SM::STAGE;
        dma.issue(Q + qt * tile_bytes, nq_all - qt * KT, dst);
        dma.issue(DO + qt * tile_bytes, nq_all - qt * KT, dst + SM::TILE);
        if (SOFTMAX && dma.active()) {  // every loading wave sends the same two loads (equal load counts); indices clamped
            const int qi = qt * KT + lane;
            const uint32_t voff = (uint32_t)(qi < nq_all ? qi : nq_all - 1) * 4;
            load_to_lds_b32(lse_rsrc, voff, 0, dst + 2 * SM::TILE);
            load_to_lds_b32(delta_rsrc, voff, 0, dst + 2 * SM::TILE + 256);
        }
    };
    const int n_steps = qt_end - qt_begin;
    if (n_steps > 0) issue(qt_begin, 0);

    // K^T and V^T fragments of this wave's keys (B operands: column = key r), via the end of the ring
    bf16x8 kf[K_REG], vf[KC];
    char* kpark = lds + SM::TOTAL + (wave * K_LDS * 64 + lane) * 16;  // + 1024 per fragment
    {
        char* own = lds + SM::TOTAL - SM::OWN_BYTES;
        const int64_t goff = k_row0 * hd + (int64_t)h * D;
        stage_rows_swizzled<D, NW>(own, (const char*)((const bf16_t*)p.k + goff), row_bytes, nk_wg, tid);
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 f = *(const bf16x8*)(own + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
            if (kc < K_REG) kf[kc < K_REG ? kc : 0] = f;
            else *(bf16x8*)(kpark + (kc - K_REG) * 1024) = f;
        }
        __syncthreads();
        stage_rows_swizzled<D, NW>(own, (const char*)((const bf16_t*)p.v + goff), row_bytes, nk_wg, tid);
        __syncthreads();
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) vf[kc] = *(const bf16x8*)(own + wave * SM::TILE + L::k_offset(r, 2 * kc + g));
        __syncthreads();
    }
    if (n_steps > 1) issue(qt_begin + 1, 1);

    // queries that see this lane's key: q_lo .. q_lo + q_span (empty for padding lanes)
    int q_lo;
    unsigned q_span;
    {
        const int kp = kpos_w + r;
        int lo = 0, hi = nq_all - 1;
        if (WINDOWED) {
            if (p.right >= 0 && kp - p.right > lo) lo = kp - p.right;
            if (p.left >= 0 && kp + p.left < hi) hi = kp + p.left;
        }
        const bool empty = hi < lo || r >= nk;
        q_lo = empty ? 0x3fffffff : lo;
        q_span = empty ? 0u : (unsigned)(hi - lo);
    }

    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dkacc[db][v] = 0.f; dvacc[db][v] = 0.f; }
    const float sc = SOFTMAX ? p.scale * LOG2E_T : p.scale;
    UFrag<D> uf;
    uf.init(lane);

    int stage = 0;
    for (int i = 0; i < n_steps; ++i) {
        if (i + 1 < n_steps) wait_vmcnt<LOADS_PER_TILE>();
        else wait_vmcnt<0>();
        __syncthreads();  // tile i complete; every wave is done with the stage of tile i-1
        const char* ldsQ = lds + stage * SM::STAGE;
        const char* ldsDO = ldsQ + SM::TILE;
        const float* stats = (const float*)(ldsDO + SM::TILE);
        const int free_stage = stage == 0 ? 2 : stage - 1;
        stage = stage == 2 ? 0 : stage + 1;
        const int qt = qt_begin + i;
        if (i + 2 < n_steps) issue(qt_begin + i + 2, free_stage);
        if (!wave_active || qt < w_begin || qt >= w_end) continue;
        // S = Q K^T and dP = dO V^T: lane = key column, registers = queries of the tile
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 qa = uf.row(ldsQ, kc);
            const bf16x8 da = uf.row(ldsDO, kc);
            const bf16x8 kb = kc < K_REG ? kf[kc < K_REG ? kc : 0] : *(const bf16x8*)(kpark + (kc - K_REG) * 1024);
            sacc = mfma32(qa, kb, sacc);
            dpacc = mfma32(da, vf[kc], dpacc);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads of the next phase behind this one (register pressure)
        // Interior tiles - every (query, key) pair inside the sequence and the window - skip the
        // visibility test.  (Padding key lanes hold zero K/V rows and are never stored.)
        const int q_base = qt * KT;
        bool need_mask = q_base + KT > nq_all;
        if (WINDOWED) {
            const int kp_lo = kpos_w, kp_hi = kpos_w + nk - 1;
            if (p.right >= 0 && q_base < kp_hi - p.right) need_mask = true;
            if (p.left >= 0 && q_base + KT - 1 > kp_lo + p.left) need_mask = true;
        }
        float pv[16], dsv[16];
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            f32x4 lse4 = {0.f, 0.f, 0.f, 0.f}, del4 = {0.f, 0.f, 0.f, 0.f};
            if (SOFTMAX) {  // natural-log LSE of queries 8*vg + 4g + 0..3 of the tile, and their delta
                lse4 = *(const f32x4*)(stats + 8 * vg + 4 * g);
                del4 = *(const f32x4*)(stats + 64 + 8 * vg + 4 * g);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = 4 * vg + e;
                if (SOFTMAX) {
                    pv[v] = fast_exp2(fmaf(sacc[v], sc, lse4[e] * -LOG2E_T));
                    dsv[v] = pv[v] * (dpacc[v] - del4[e]) * p.scale;
                } else {
                    float der;
                    act_fast_vd<ACT>(sacc[v] * sc, pv[v], der);
                    dsv[v] = dpacc[v] * der * p.scale;
                }
            }
        }
        if (need_mask) {
            const unsigned rel0 = (unsigned)(q_base + 4 * g - q_lo);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const bool ok = rel0 + (unsigned)(8 * (v >> 2) + (v & 3)) <= q_span;
                pv[v] = ok ? pv[v] : 0.f;
                dsv[v] = ok ? dsv[v] : 0.f;
            }
        }
        bf16x8 pf[2], dsf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) { pf[c][e] = (bf16_t)pv[8 * c + e]; dsf[c][e] = (bf16_t)dsv[8 * c + e]; }
        __builtin_amdgcn_sched_barrier(0);
        // dV^T += dO^T P and dK^T += Q^T dS (contraction over the queries of the tile)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                dvacc[db] = mfma32(uf.transposed(ldsDO, db, c), pf[c], dvacc[db]);
                dkacc[db] = mfma32(uf.transposed(ldsQ, db, c), dsf[c], dkacc[db]);
            }
    }
    __syncthreads();  // every wave is done with the ring
    if (!wave_active) return;
    char* out_stage = lds + wave * PT::ROW_TILE;
    store_tile_rows<D>(out_stage, dvacc, (bf16_t*)p.dv + (k_row0 + k_lo_w) * hd + (int64_t)h * D, hd, nk, lane);
    store_tile_rows<D>(out_stage, dkacc, (bf16_t*)p.dk + (k_row0 + k_lo_w) * hd + (int64_t)h * D, hd, nk, lane);
}

// ------------------------------------------------------------------ kernels


// work mapping of tile_map.h in both passes
template <int D, int NW, bool WINDOWED>
__global__ __launch_bounds__(64 * NW, D == 128 ? 2 : 3) void bwd_dq_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                            const int32_t* __restrict__ tile_example, int runs,
                                                            float* __restrict__ delta_ws) {
    __shared__ __attribute__((aligned(1024))) char lds[TiledSmem<D, 0>::TOTAL];
    static_assert(32 * NW == TILE_ROWS, "tile size of the work mapping");
    int b, h, qt;
    if (!locate_tile(tile_start, tile_example, p.B, p.H, runs, b, h, qt)) return;
    const int64_t k0 = p.kv_off[b];
    const int n_kv = p.kv_off[b + 1] - (int)k0;
    const int64_t q0 = q_begin(p, b);
    const int nq_all = (int)(q_end(p, b) - q0);
    const int q_first = qt * 32 * NW;
    const int nq = (nq_all - q_first) < 32 * NW ? (nq_all - q_first) : 32 * NW;
    if (WINDOWED) {
        bwd_dq_item<D, NW, KUNLUN_ACT_SOFTMAX, true>(p, delta_ws, lds, h, q0 + q_first, nq, q_first, k0, n_kv);
    } else {
        KUNLUN_ACT_SWITCH(p.head_act[h], (bwd_dq_item<D, NW, A, false>(p, delta_ws, lds, h, q0 + q_first, nq, q_first, k0, n_kv)));
    }
}

template <int D, int NW, bool WINDOWED>
__global__ __launch_bounds__(64 * NW, D == 128 ? 2 : 3) void bwd_dkdv_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                              const int32_t* __restrict__ tile_example, int runs,
                                                              const float* __restrict__ delta_ws) {
    __shared__ __attribute__((aligned(1024))) char lds[TiledSmem<D, STATS_BYTES>::TOTAL + (D == 128 ? 3 : 0) * NW * 1024];
    int b, h, kt;
    if (!locate_tile(tile_start, tile_example, p.B, p.H, runs, b, h, kt)) return;
    const int64_t k0 = p.kv_off[b];
    const int n_kv = p.kv_off[b + 1] - (int)k0;
    const int64_t q0 = q_begin(p, b);
    const int nq_all = (int)(q_end(p, b) - q0);
    const int k_first = kt * 32 * NW;
    const int nk = (n_kv - k_first) < 32 * NW ? (n_kv - k_first) : 32 * NW;
    if (WINDOWED) {
        bwd_dkdv_item<D, NW, KUNLUN_ACT_SOFTMAX, true>(p, delta_ws, lds, h, k0 + k_first, nk, k_first, q0, nq_all);
    } else {
        KUNLUN_ACT_SWITCH(p.head_act[h], (bwd_dkdv_item<D, NW, A, false>(p, delta_ws, lds, h, k0 + k_first, nk, k_first, q0, nq_all)));
    }
}

// delta[h, row] = sum_c dO[row, h, c] * O[row, h, c]: D/8 lanes per (row, head), 16 bytes each.
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o,
                                                    float* __restrict__ delta, int64_t total_q, int H) {
    constexpr int LANES = D / 8;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t item = gid / LANES;  // row * H + h
    const int part = (int)(gid % LANES);
    float acc = 0.f;
    if (item < total_q * H) {
        const bf16x8 a = *(const bf16x8*)(o + item * D + part * 8);
        const bf16x8 b = *(const bf16x8*)(d_o + item * D + part * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)b[e], acc);
    }
#pragma unroll
    for (int off = LANES / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (part == 0 && item < total_q * H) {
        const int64_t row = item / H;
        const int h = (int)(item % H);
        delta[(int64_t)h * total_q + row] = acc;
    }
}

// ------------------------------------------------------------------ few keys: one pass
//
// The PFFN direction proper: long query sequences, at most 32 keys per example (the context
// tokens).  With a single key tile there is no key loop and nothing to accumulate across tiles,
// so one workgroup per (example, 128-query tile, head) does all five contractions in one pass over
// Q and dO: per wave (32 queries)
//     S^T = K Q^T,  dP^T = V dO^T,  P^T / dS^T in registers  ->  dQ^T = K^T dS^T  (stored at once)
//     P, dS through a 2 KB LDS tile each (query-per-lane -> key-per-lane)
//     dV^T = dO^T P,  dK^T = Q^T dS  over the wave's 32 queries
// The dK / dV contributions of the four waves are added in LDS (fixed order) and written as one fp32
// partial tile per workgroup; a second kernel adds the partial tiles of an example in tile order
// (bit-reproducible, no atomics) and rounds once.  Against the two-pass kernels this reads Q and dO
// once instead of twice and keeps all four waves busy.

template <int D>
struct FewKeysSmem {
    using PT = PadTiles<D>;
    static constexpr int TILE = KT * D * 2;       // 32 rows of D bf16, two-way swizzle
    static constexpr int P_BYTES = KT * 64;       // [query][key] bf16, 64 bytes per row
    static constexpr int WAVE = 2 * TILE;         // a wave's Q and dO tiles; later its dQ staging rows, last its partial sums
    // K tile, then the V tile; once every wave has finished its reads of V, the P (then dS) tiles of the four
    // waves take its place (d < 128: the V tile is smaller than that, the region is sized for the larger use)
    static constexpr int V_REGION = TILE > 4 * P_BYTES ? TILE : 4 * P_BYTES;
    static constexpr int HEAD = TILE + V_REGION;
    static constexpr int TOTAL = HEAD + 4 * WAVE;
    static constexpr int PART = KT * D * 4;       // a wave's fp32 [key][channel] partial sums
    static_assert(PART <= WAVE, "a wave's partial sums go into its dead Q and dO tiles");
    static_assert(PT::ROW_TILE <= WAVE, "and so do its dQ staging rows");
};

// Query tiles that one workgroup walks (accumulating dK / dV in registers): more tiles mean fewer
// partial sums to write and read back, fewer workgroups mean an emptier machine.
inline int fewkeys_chunk_tiles(int B, int H, int64_t total_q) {
    const int64_t wgs = (total_q / TILE_ROWS + B) * H;
    return wgs >= 16384 ? 8 : (wgs >= 4096 ? 4 : (wgs >= 2048 ? 2 : 1));
}
inline size_t fewkeys_partial_bytes(int B, int H, int d, int64_t total_q) {
    const int chunk_rows = TILE_ROWS * fewkeys_chunk_tiles(B, H, total_q);
    return align_up((size_t)(total_q / chunk_rows + B) * H * 2 * KT * d * sizeof(float), 256);
}
inline bool fewkeys_applies(int d, int max_q, int max_kv, bool windowed) {
    return !windowed && max_q > 64 && max_kv <= KT && (d == 32 || d == 64 || d == 128);
}

// P / dS tile: row = query, 4 chunks of 16 bytes (8 keys) per row, chunk index swizzled by the row.
__device__ __forceinline__ int pq_offset(int row, int byte_in_row) {
    return row * 64 + ((((byte_in_row >> 4) ^ (row >> 2)) & 3) << 4) + (byte_in_row & 15);
}
// fp32 [key][channel] partial sums: 16-byte chunks swizzled by the row.
template <int D>
__device__ __forceinline__ int part_offset(int row, int chunk) {
    return row * D * 4 + ((chunk ^ (row & (D / 4 - 1))) << 4);
}

template <int D, int ACT>
__device__ __forceinline__ void bwd_fewkeys_item(const AttnParams& p, const float* __restrict__ delta_ws, char* lds, int h,
                                                 int64_t q_row0, int nq_chunk, int64_t k0, int n_kv,
                                                 float* __restrict__ part_out) {
    using L = TileLayout<D>;
    using SM = FewKeysSmem<D>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16, DB = D / 32;
    constexpr int CHUNKS = D / 8;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    char* ldsK = lds;
    char* ldsV = lds + SM::TILE;
    char* wbase = lds + SM::HEAD + wave * SM::WAVE;
    char* ldsQ = wbase;
    char* ldsDO = wbase + SM::TILE;
    char* ldsP = ldsV + wave * SM::P_BYTES;  // over the V tile, once that is dead: P first, then dS
    const int q_lo_w = wave * 32;

    UFrag<D> uf;
    uf.init(lane);
    const float sc = SOFTMAX ? p.scale * LOG2E_T : p.scale;
    const int s16 = lane & 15, hi16 = (lane >> 4) & 1;
    const int ptA = pq_offset(8 * g + (s16 >> 2), (16 * hi16 + 4 * (s16 & 3)) * 2);
    const int ptB = pq_offset(8 * g + 4 + (s16 >> 2), (16 * hi16 + 4 * (s16 & 3)) * 2);
    // A operands of the last two contractions (row = channel, contraction = queries 16j + 8g + 0..7):
    // transposing reads of the dO / Q tiles
    int qtA[DB], qtB[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        const int colb = (32 * db + 16 * hi16 + 4 * (s16 & 3)) * 2;
        qtA[db] = L::u_offset(8 * g + (s16 >> 2), colb);
        qtB[db] = L::u_offset(8 * g + 4 + (s16 >> 2), colb);
    }
    const unsigned keys_left = (unsigned)(n_kv - 4 * g);  // key 8*(v/4) + (v%4) + 4g < n_kv

    f32x16 dvacc[DB], dkacc[DB];  // lane = key r, registers = channels; summed over all tiles of the chunk
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dvacc[db][v] = 0.f; dkacc[db][v] = 0.f; }

    TileDma<D, 1, SWZ_U> dma;  // a wave loads its own tiles
    dma.init(lane, 0, (uint32_t)(hd * 2));
    const int n_tiles = (nq_chunk + TILE_ROWS - 1) / TILE_ROWS;
    for (int it = 0; it < n_tiles; ++it) {
        const int64_t rows0 = q_row0 + (int64_t)it * TILE_ROWS + q_lo_w;  // first query row of this wave
        int nq = nq_chunk - it * TILE_ROWS - q_lo_w;
        nq = nq < 0 ? 0 : (nq > 32 ? 32 : nq);
        if (it > 0) __syncthreads();  // every wave is done with the P / dS tiles of the previous tile (they lie over V)
        // ---- staging: whole rows, 16 bytes per lane, rows past the end are zero.  K (once) and V (for every
        // tile: it was overwritten) by the whole workgroup, Q and dO of a wave's 32 queries by that wave.
        {
            const u32x4 zero = {0, 0, 0, 0};
            for (int idx = tid; idx < KT * CHUNKS; idx += 256) {
                const int row = idx / CHUNKS, ch = idx % CHUNKS;
                u32x4 kv = zero, vv = zero;
                if (row < n_kv) {
                    if (it == 0) kv = *(const u32x4*)((const bf16_t*)p.k + (k0 + row) * hd + (int64_t)h * D + ch * 8);
                    vv = *(const u32x4*)((const bf16_t*)p.v + (k0 + row) * hd + (int64_t)h * D + ch * 8);
                }
                if (it == 0) *(u32x4*)(ldsK + L::u_offset(row, ch * 16)) = kv;
                *(u32x4*)(ldsV + L::u_offset(row, ch * 16)) = vv;
            }
            // Q and dO straight into LDS (no staging registers); rows past the wave's queries repeat the last
            // one and get zero weight below; a wave without queries loads nothing and computes nothing
            if (nq > 0) {
                dma.issue((const char*)((const bf16_t*)p.q + q_src_row(p, rows0) * hd + (int64_t)h * D), nq, lds_address(ldsQ));
                dma.issue((const char*)((const bf16_t*)p.d_o + rows0 * hd + (int64_t)h * D), nq, lds_address(ldsDO));
            }
        }
        // softmax statistics of this lane's query
        float lse2 = INFINITY, delta = 0.f;
        if (SOFTMAX && r < nq) {
            const int64_t idx = (int64_t)h * p.total_q + rows0 + r;
            lse2 = p.lse[idx] * LOG2E_T;
            delta = delta_ws[idx];
        }
        wait_vmcnt<0>();  // the loads into LDS are not tracked by the compiler
        __syncthreads();
        const bool wave_active = nq > 0;

        // packed P^T and dS^T in the register order of the C layout: element e of block c = key 16c + 8(e/4) + 4g + e%4
        bf16x8 pf[2], dsf[2];
        if (wave_active) {
            // ---- S^T = K Q^T and dP^T = V dO^T: lane = query r of the wave, registers = keys
            f32x16 sacc, dpacc;
#pragma unroll
            for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                sacc = mfma32(uf.row(ldsK, kc), uf.row(ldsQ, kc), sacc);
                dpacc = mfma32(uf.row(ldsV, kc), uf.row(ldsDO, kc), dpacc);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the phases apart (register pressure)
            // ---- score function; keys past the end of the example's keys and queries past the end of the
            // wave's queries (their rows repeat the last valid one) get zero weight
            const bool q_ok = r < nq;
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int v = 8 * c + e;
                    const float s = sacc[v] * sc;
                    float pval, dsval;
                    if (SOFTMAX) {
                        pval = fast_exp2(s - lse2);
                        dsval = pval * (dpacc[v] - delta) * p.scale;
                    } else {
                        float der;
                        act_fast_vd<ACT>(s, pval, der);
                        dsval = dpacc[v] * der * p.scale;
                    }
                    const bool ok = q_ok && n_kv > 4 * g && (unsigned)(8 * (v >> 2) + (v & 3)) < keys_left;
                    pf[c][e] = (bf16_t)(ok ? pval : 0.f);
                    dsf[c][e] = (bf16_t)(ok ? dsval : 0.f);
                }
        }
        __syncthreads();  // every wave is done with the V tile: the P / dS tiles take its place
        if (wave_active) {
            // ---- dV^T += dO^T P, then dK^T += Q^T dS, over the wave's 32 queries.  P (then dS, in the same 2 KB)
            // goes through LDS to come back as B operand (column = key, contraction over 16 queries per step);
            // registers 4*vg .. 4*vg+3 of the C layout hold keys 8*vg + 4g + 0..3 of query r.
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const bf16x8 src = which == 0 ? pf[vg >> 1] : dsf[vg >> 1];
                    const bf16x4 four = (vg & 1) ? __builtin_shufflevector(src, src, 4, 5, 6, 7) : __builtin_shufflevector(src, src, 0, 1, 2, 3);
                    *(bf16x4*)(ldsP + pq_offset(r, (8 * vg + 4 * g) * 2)) = four;
                }
                bf16x8 back[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) back[j] = tr_pair(ldsP + j * 16 * 64 + ptA, ldsP + j * 16 * 64 + ptB);
                const char* src_tile = which == 0 ? ldsDO : ldsQ;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int ro = j * 16 * L::ROW_BYTES;
                        const bf16x8 a = tr_pair(src_tile + ro + qtA[db], src_tile + ro + qtB[db]);
                        if (which == 0) dvacc[db] = mfma32(a, back[j], dvacc[db]);
                        else dkacc[db] = mfma32(a, back[j], dkacc[db]);
                    }
            }
            // ---- dQ^T = K^T dS^T, rows out through the wave's own Q / dO tiles: only this wave reads them,
            // and the LDS operations of a wave complete in order
            // (one 32-channel block at a time: 16 accumulator registers instead of 64)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                f32x16 dqacc;
#pragma unroll
                for (int v = 0; v < 16; ++v) dqacc[v] = 0.f;
#pragma unroll
                for (int c = 0; c < 2; ++c) dqacc = mfma32(uf.transposed(ldsK, db, c), dsf[c], dqacc);
                store_block_staged<D>(ldsQ, dqacc, db, lane);
            }
            store_staged_rows<D>(ldsQ, (bf16_t*)p.dq + rows0 * hd + (int64_t)h * D, hd, nq, lane);
        }
    }
    // ---- the four waves' contributions are added in LDS, dV first, then dK.  A wave's partial sums go
    // into its own Q / dO tiles.
    char* mine = ldsQ;
    const int n_chunks = KT * D / 4;  // 16-byte chunks of a [32][D] fp32 tile
#pragma unroll
    for (int which = 0; which < 2; ++which) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                f32x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = which == 0 ? dvacc[db][4 * vg + e] : dkacc[db][4 * vg + e];
                *(f32x4*)(mine + part_offset<D>(r, (32 * db + 8 * vg + 4 * g) / 4)) = x;
            }
        __syncthreads();
        float* dst = part_out + (size_t)which * KT * D;
        for (int idx = tid; idx < n_chunks; idx += 256) {
            const int row = idx / (D / 4), ch = idx % (D / 4);
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w) sum += *(const f32x4*)(lds + SM::HEAD + w * SM::WAVE + part_offset<D>(row, ch));
            *(f32x4*)(dst + row * D + ch * 4) = sum;
        }
        if (which == 0) __syncthreads();  // the partial tiles are rewritten for dK
    }
}

template <int D>
__global__ __launch_bounds__(256, 2) void bwd_fewkeys_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                          const int32_t* __restrict__ tile_example,
                                                          const float* __restrict__ delta_ws, float* __restrict__ partial,
                                                          int chunk_rows) {
    extern __shared__ __attribute__((aligned(1024))) char fk_lds[];
    int b, h, qt;
    if (!locate_tile(tile_start, tile_example, p.B, p.H, 1, b, h, qt)) return;
    const int64_t k0 = p.kv_off[b];
    int n_kv = p.kv_off[b + 1] - (int)k0;
    n_kv = n_kv > KT ? KT : n_kv;  // the launch condition (max_kv <= 32) promises this; never read past the tile
    const int64_t q0 = q_begin(p, b);
    const int nq_all = (int)(q_end(p, b) - q0);
    const int q_first = qt * chunk_rows;  // the tile table counts chunks of chunk_rows queries here
    const int nq = (nq_all - q_first) < chunk_rows ? (nq_all - q_first) : chunk_rows;
    float* part_out = partial + ((size_t)(tile_start[b] + qt) * p.H + h) * (2 * KT * D);
    KUNLUN_ACT_SWITCH(p.head_act[h], (bwd_fewkeys_item<D, A>(p, delta_ws, fk_lds, h, q0 + q_first, nq, k0, n_kv, part_out)));
}

// dK, dV rows of every example = sum of the partial tiles of its query tiles, in tile order; 4 channels per thread.
template <int D>
__global__ __launch_bounds__(256) void fewkeys_reduce_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                             const float* __restrict__ partial) {
    constexpr int PER_ROW = D / 4;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (((b*H + h)*2 + which)*32 + key)*PER_ROW + c4
    if (gid >= (int64_t)p.B * p.H * 2 * KT * PER_ROW) return;
    const int c4 = (int)(gid % PER_ROW);
    const int key = (int)((gid / PER_ROW) % KT);
    const int which = (int)((gid / (PER_ROW * KT)) % 2);
    const int h = (int)((gid / (PER_ROW * KT * 2)) % p.H);
    const int b = (int)(gid / ((int64_t)PER_ROW * KT * 2 * p.H));
    const int64_t k0 = p.kv_off[b];
    if (key >= p.kv_off[b + 1] - (int)k0) return;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int t = tile_start[b]; t < tile_start[b + 1]; ++t)
        sum += *(const f32x4*)(partial + (((size_t)t * p.H + h) * 2 + which) * (KT * D) + key * D + c4 * 4);
    bf16x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = (bf16_t)sum[e];
    bf16_t* dst = (bf16_t*)(which == 0 ? p.dv : p.dk) + (k0 + key) * (int64_t)p.H * D + (int64_t)h * D + c4 * 4;
    *(bf16x4*)dst = out;
}

bool mfma_bwd_tiled_supported(const AttnParams& p, int dtype) {
    return dtype == KUNLUN_BF16 && (p.d == 32 || p.d == 64 || p.d == 128);
}

size_t mfma_bwd_tiled_workspace(int B, int H, int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, bool windowed) {
    return tile_table_bytes(B, total_q) + tile_table_bytes(B, total_kv) + align_up((size_t)H * total_q * sizeof(float), 256) +
           (fewkeys_applies(d, max_q, max_kv, windowed) ? fewkeys_partial_bytes(B, H, d, total_q) : 0);
}

template <int D, bool WINDOWED>
static hipError_t launch_tiled(const AttnParams& p, char* ws, bool any_softmax, hipStream_t stream) {
    constexpr int NW = 4;
    int32_t* q_tiles = (int32_t*)ws;
    int32_t* k_tiles = (int32_t*)(ws + tile_table_bytes(p.B, p.total_q));
    float* delta = (float*)(ws + tile_table_bytes(p.B, p.total_q) + tile_table_bytes(p.B, p.total_kv));
    const int runs = tile_runs(WINDOWED, p.left, p.right, p.H);
    (void)any_softmax;  // pass A computes delta of its softmax heads itself and leaves it in the workspace for pass B
    if (p.total_q > 0) {
        hipLaunchKernelGGL(tile_prefix_kernel<1>, dim3(1), dim3(1024), 0, stream, p.q_off, p.max_q, p.B, q_tiles,
                           tile_example_of(q_tiles, p.B), TILE_ROWS);
        hipLaunchKernelGGL((bwd_dq_kernel<D, NW, WINDOWED>), dim3(tile_grid(p.B, p.H, p.total_q, runs)), dim3(64 * NW), 0,
                           stream, p, q_tiles, tile_example_of(q_tiles, p.B), runs, delta);
    }
    if (p.total_kv > 0) {
        hipLaunchKernelGGL(tile_prefix_kernel<1>, dim3(1), dim3(1024), 0, stream, p.kv_off, 0, p.B, k_tiles,
                           tile_example_of(k_tiles, p.B), TILE_ROWS);
        hipLaunchKernelGGL((bwd_dkdv_kernel<D, NW, WINDOWED>), dim3(tile_grid(p.B, p.H, p.total_kv, runs)), dim3(64 * NW), 0,
                           stream, p, k_tiles, tile_example_of(k_tiles, p.B), runs, delta);
    }
    return hipGetLastError();
}

template <int D>
static hipError_t launch_fewkeys(const AttnParams& p, char* ws, bool any_softmax, hipStream_t stream) {
    int32_t* q_tiles = (int32_t*)ws;
    float* delta = (float*)(ws + tile_table_bytes(p.B, p.total_q) + tile_table_bytes(p.B, p.total_kv));
    float* partial = (float*)((char*)delta + align_up((size_t)p.H * p.total_q * sizeof(float), 256));
    constexpr int bytes = FewKeysSmem<D>::TOTAL;
    if (bytes > 64 * 1024) {
        // once per process (thread-safe initialisation of a function-local static); not a stream operation
        static const hipError_t raised =
            hipFuncSetAttribute((const void*)bwd_fewkeys_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (raised != hipSuccess) return raised;
    }
    if (any_softmax && p.total_q > 0) {
        const int64_t threads = p.total_q * p.H * (D / 8);
        hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                           (const bf16_t*)p.o, (const bf16_t*)p.d_o, delta, p.total_q, p.H);
    }
    const int chunk_rows = TILE_ROWS * fewkeys_chunk_tiles(p.B, p.H, p.total_q);
    hipLaunchKernelGGL(tile_prefix_kernel<1>, dim3(1), dim3(1024), 0, stream, p.q_off, p.max_q, p.B, q_tiles,
                       tile_example_of(q_tiles, p.B), chunk_rows);
    if (p.total_q > 0) {
        const int64_t per_xcd = ((p.total_q / chunk_rows + p.B) * p.H + 7) / 8;  // an upper bound of the chunk count sizes the grid
        hipLaunchKernelGGL((bwd_fewkeys_kernel<D>), dim3((unsigned)((per_xcd + 1) * 8)), dim3(256), bytes, stream, p, q_tiles,
                           tile_example_of(q_tiles, p.B), delta, partial, chunk_rows);
    }
    if (p.total_kv > 0) {
        const int64_t threads = (int64_t)p.B * p.H * 2 * KT * (D / 4);
        hipLaunchKernelGGL((fewkeys_reduce_kernel<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, p, q_tiles,
                           partial);
    }
    return hipGetLastError();
}

hipError_t launch_mfma_bwd_tiled(const AttnParams& p, void* workspace_tail, bool any_softmax, hipStream_t stream) {
    char* ws = (char*)workspace_tail;
    if (fewkeys_applies(p.d, p.max_q, p.max_kv, p.windowed != 0))
        return p.d == 128 ? launch_fewkeys<128>(p, ws, any_softmax, stream)
               : p.d == 64 ? launch_fewkeys<64>(p, ws, any_softmax, stream) : launch_fewkeys<32>(p, ws, any_softmax, stream);
    if (p.windowed)
        return p.d == 128 ? launch_tiled<128, true>(p, ws, true, stream)
               : p.d == 64 ? launch_tiled<64, true>(p, ws, true, stream) : launch_tiled<32, true>(p, ws, true, stream);
    return p.d == 128 ? launch_tiled<128, false>(p, ws, any_softmax, stream)
           : p.d == 64 ? launch_tiled<64, false>(p, ws, any_softmax, stream) : launch_tiled<32, false>(p, ws, any_softmax, stream);
}

}  // namespace kunlun
