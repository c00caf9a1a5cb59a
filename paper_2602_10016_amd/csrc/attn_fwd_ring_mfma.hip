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
// into a ring of three LDS stages: while tile t is consumed, tiles t+1 and t+2 are in flight
// (lds_ring.h).  K tiles use the K swizzle, V tiles the V swizzle of TileLayout.
#include "attn_fwd_score.h"
#include "lds_ring.h"
#include "tile_map.h"

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

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void attn_fwd_ring_item(const AttnParams& p, char* lds, int h, int64_t q_row0, int nq_wg,
                                                   int64_t t0_wg, int64_t k0, int n_kv) {
    using SM = RingSmem<D, NW>;
    using L = TileLayout<D>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16;
    constexpr int DB = D / 32;
    constexpr int CHUNKS = D / 8;
    constexpr int IPW = TileDma<D, NW, SWZ_K>::IPW;  // load instructions per wave per tile and tensor
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* K = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* V = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);
    const uint32_t lds0 = lds_address(lds);

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

    // ---- tile transport
    TileDma<D, NW, SWZ_K> kdma;
    TileDma<D, NW, SWZ_V> vdma;
    kdma.init(lane, wave, row_bytes);
    vdma.init(lane, wave, row_bytes);
    auto issue = [&](int kt, int stage) {
        const uint32_t dst = lds0 + stage * SM::STAGE;
        kdma.issue(K + kt * tile_bytes, n_kv - kt * KT, dst);
        vdma.issue(V + kt * tile_bytes, n_kv - kt * KT, dst + SM::TILE);
    };

    // ---- prologue.  The first key tile starts its journey at once (stage 0); the query tile
    // goes through registers into the end of the ring (whole rows, K-tile swizzle) and every
    // wave picks its B-operand fragments: column = query r, contraction = channels 16*kc + 8g ..
    const int n_steps = kt_end - kt_begin;
    if (n_steps > 0) issue(kt_begin, 0);
    if (!SM::Q_COVERS_STAGE1 && n_steps > 1) issue(kt_begin + 1, 1);
    bf16x8 qf[KC];
    {
        char* qstage = lds + SM::TOTAL - SM::Q_BYTES;
        stage_rows_swizzled<D, NW>(qstage, (const char*)((const bf16_t*)p.q + q_src_row(p, q_row0) * hd + (int64_t)h * D), row_bytes, nq_wg, tid);
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
            if (row < nq) __builtin_nontemporal_store(val, (u32x4*)(obase + row * hd + chunk * 8));  // written once, not read back
        }
    }
}

// One workgroup per (example, query tile, head); work mapping of tile_map.h.
template <int D, int NW, int OCC, bool WINDOWED>
__global__ __launch_bounds__(64 * NW, OCC) void qtile_fwd_mfma_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                                      const int32_t* __restrict__ tile_example, int runs) {
    __shared__ __attribute__((aligned(1024))) char lds[RingSmem<D, NW>::TOTAL];
    constexpr int QT = 32 * NW;
    static_assert(QT == TILE_ROWS, "tile size of the work mapping");
    int b, h, qt;
    if (!locate_tile(tile_start, tile_example, p.B, p.H, runs, b, h, qt)) return;
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
        case KUNLUN_ACT_SILU: attn_fwd_ring_item<D, NW, KUNLUN_ACT_SILU, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        default: attn_fwd_ring_item<D, NW, KUNLUN_ACT_GELU_POLY, false>(p, lds, h, q0 + q_first, nq, q_first, k0, n_kv); break;
        }
    }
}

template <int D, int NW, int OCC, bool WINDOWED>
static hipError_t launch_qtiled(const AttnParams& p, hipStream_t stream) {
    const int runs = tile_runs(WINDOWED, p.left, p.right, p.H);
    int32_t* tile_start = const_cast<int32_t*>(p.order);
    int32_t* tile_example = tile_example_of(tile_start, p.B);
    hipLaunchKernelGGL(tile_prefix_kernel<0>, dim3(1), dim3(1024), 0, stream, p.q_off, p.max_q, p.B, tile_start,
                       tile_example, TILE_ROWS);
    hipLaunchKernelGGL((qtile_fwd_mfma_kernel<D, NW, OCC, WINDOWED>), dim3(tile_grid(p.B, p.H, p.total_q, runs)),
                       dim3(64 * NW), 0, stream, p, tile_start, tile_example, runs);
    return hipGetLastError();
}

// p.order points at tile_table_bytes(B, total_q) bytes of workspace.
hipError_t launch_mfma_fwd_qtiled(const AttnParams& p, hipStream_t stream) {
    // 128-query tiles (4 waves of 32 queries)
    if (p.windowed)
        return p.d == 128 ? launch_qtiled<128, 4, 2, true>(p, stream)
               : p.d == 64 ? launch_qtiled<64, 4, 2, true>(p, stream) : launch_qtiled<32, 4, 2, true>(p, stream);
    return p.d == 128 ? launch_qtiled<128, 4, 2, false>(p, stream)
           : p.d == 64 ? launch_qtiled<64, 4, 2, false>(p, stream) : launch_qtiled<32, 4, 2, false>(p, stream);
}

}  // namespace kunlun
