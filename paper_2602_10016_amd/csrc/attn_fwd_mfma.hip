// bf16 matrix-core forward kernel for gfx950, streaming launches: GDPA (Eq. (GDPA)) and softmax
// attention of a few seed / context queries (up to 64 per example) over a jagged history
// (Eq. (PMA), Eq. (seed-level attention)).  Longer query sequences and the sliding window are
// served by the query-tiled kernel (attn_fwd_ring_mfma.hip).
//
// A workgroup of NW wavefronts owns one work item = (example, head); each wave owns 32*NQB of
// its queries for the whole item.  The waves stream the 32-key K/V tiles of the item together:
// every thread fetches its share of tile t+1 (and t+2) into registers (whole rows, coalesced,
// non-temporal) while tile t, already in LDS, is being consumed; tiles are double-buffered in
// LDS, so there is one barrier per tile.  These operators do only Nq flops per byte of K/V (a
// key/value byte is used by the queries of its own example and head and by nobody else), far
// below the matrix-core ridge, so the design goal is bytes in flight and enough resident waves
// to hide latency, not MFMA occupancy.
//
// Per 32-key tile and wave:
//     S^T = K Q^T              (MFMA; Q^T fragments resident in registers)
//     P^T = score function of S^T * scale, in registers, zero past the end of the history,
//           packed to bf16
//     O^T += V^T P^T           (MFMA; V^T via transposing LDS reads)
// Softmax keeps a running maximum and sum per query (one query per lane column) and rescales
// O^T when the maximum grows; the activation path has no such stage.
#include "attn_fwd_score.h"

namespace kunlun {

// LDS tiles of the forward kernels: 32 rows, row-major, each row padded so that every access
// pattern is free of bank conflicts and every offset is affine in (row, column):
//   K rows + 16 bytes: the 16 lanes that read the same 16-byte chunk of 16 consecutive rows
//                      (A-operand reads) fall into 16 different 16-byte bank slots;
//   V rows + 64 bytes: the 4 consecutive rows of a transposing read fall into 4 different
//                      64-byte bank groups.
template <int D>
struct FwdSmem {
    static constexpr int K_STRIDE = D * 2 + 16;
    static constexpr int V_STRIDE = D == 32 ? 64 : D * 2 + 64;  // (D = 32: four rows of 64 bytes already cover all banks)
    static constexpr int K_TILE = KT * K_STRIDE;
    static constexpr int V_TILE = KT * V_STRIDE;
    static constexpr int BUF_BYTES = K_TILE + V_TILE;  // K tile, then V tile
    static constexpr int TOTAL = 2 * BUF_BYTES;        // double buffer (workgroups of several waves)
    // A wave that streams alone needs no second buffer (it writes a tile, reads it, and writes the next one in
    // program order); the key-split launches use that to fit four waves' buffers, the others keep two buffers
    // (the store of the next tile can then be scheduled before the reads of the current one end).
    static constexpr int bytes(int ks) { return ks > 1 ? BUF_BYTES : TOTAL; }
};

// Cooperative global -> register -> LDS staging of one 32-row tile by a workgroup of 64*NW
// threads: slot = i*64*NW + tid covers (row, 16-byte chunk) pairs row-major, so whole rows
// coalesce.  A thread's chunks sit ROWS_PER_LOAD rows apart, so every address is "uniform
// base + one per-thread offset + constant" and the key loop spends no vector arithmetic on it.
template <int D, int NW>
struct CoopTile {
    using SM = FwdSmem<D>;
    static constexpr int CHUNKS = D / 8;  // 16-byte chunks per row
    static constexpr int SLOTS = KT * CHUNKS;
    static constexpr int LOADS = SLOTS / (64 * NW);
    static constexpr int ROWS_PER_LOAD = 64 * NW / CHUNKS;
    static_assert(LOADS >= 1 && SLOTS % (64 * NW) == 0, "tile does not split evenly over the workgroup");

    uint32_t goff;   // byte offset of this thread's first chunk inside a tile of the [tokens,H,D] tensor
    int kw, vw;      // LDS byte offsets of the same chunk in the K / V tiles
    int row0, chunk;
    uint32_t row_bytes;

    __device__ __forceinline__ void init(int tid, uint32_t row_stride_bytes) {
        row0 = tid / CHUNKS;
        chunk = tid % CHUNKS;
        row_bytes = row_stride_bytes;
        goff = (uint32_t)row0 * row_stride_bytes + chunk * 16;
        kw = row0 * SM::K_STRIDE + chunk * 16;
        vw = row0 * SM::V_STRIDE + chunk * 16;
    }
    // Loads go through a buffer resource that covers exactly the valid rows of the tile: rows
    // past the end of a history read as zero (and get zero weight later), with no address
    // clamping in the loop.  voffset = the thread's constant offset, soffset = uniform.
    // STREAM: the data is read once by this workgroup and by nobody else (GDPA keys/values):
    // non-temporal loads keep it from displacing useful lines in the caches.  Not at D = 32: a row piece is then
    // half a 128-byte line, the other half belongs to the neighbouring head, and a streaming load fetches the
    // whole line for one use (measured on the bench batch: 2.06 GB fetched against 1.80 GB with plain loads, which
    // the neighbouring head's workgroup can hit in L2 when it runs on the same XCD; the operands are 1.2 GB).
    template <bool STREAM>
    __device__ __forceinline__ void load(u32x4 (&st)[LOADS], const char* __restrict__ tile_base, int rows_valid) const {
        const int rows = rows_valid < KT ? rows_valid : KT;
        const int bytes = (rows - 1) * (int)row_bytes + D * 2;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)tile_base, 0, bytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff, i * ROWS_PER_LOAD * row_bytes, STREAM && D != 32 ? 2 : 0);
    }
    __device__ __forceinline__ void store(char* ldsK, char* ldsV, const u32x4 (&ks)[LOADS], const u32x4 (&vs)[LOADS]) const {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) *(u32x4*)(ldsK + kw + i * ROWS_PER_LOAD * SM::K_STRIDE) = ks[i];
#pragma unroll
        for (int i = 0; i < LOADS; ++i) *(u32x4*)(ldsV + vw + i * ROWS_PER_LOAD * SM::V_STRIDE) = vs[i];
    }
};

// One work item.  q_row0 / nq_wg: first query row (global) and query count of the workgroup's tile.
// KS > 1 (with NW = 1): the workgroup has KS waves that own the SAME queries and take the key tiles of the
// item in turn (wave s: tiles s, s + KS, ...), each with its own tile buffers and no barrier in the key loop;
// their partial results are merged in LDS at the end, in wave order.  For launches with few work items, where
// one wave per item would leave the time to the longest history.
template <int D, int NQB, int NW, int ACT, int AHEAD, int KS>
__device__ __forceinline__ void attn_fwd_item(const AttnParams& p, char* lds, int h, int64_t q_row0, int nq_wg,
                                              int64_t k0, int n_kv) {
    using SM = FwdSmem<D>;
    using CT = CoopTile<D, NW>;
    static_assert(KS == 1 || NW == 1, "key splitting is for single-wave query groups");
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16;  // contraction steps of S^T = K Q^T
    constexpr int DB = D / 32;  // 32-channel blocks of O^T
    constexpr int QW = 32 * NQB;  // queries per wave
    // (the thread index goes through an opaque move per item: what is derived from it is computed where the item
    // uses it, and not kept in registers across the loop of a persistent launch for all six score functions)
    int tid_wg = threadIdx.x;
    asm volatile("" : "+v"(tid_wg));
    const int split = KS > 1 ? __builtin_amdgcn_readfirstlane(tid_wg >> 6) : 0;  // this wave's turn in the key tiles
    const int tid = KS > 1 ? (tid_wg & 63) : tid_wg;
    constexpr int LDS_BYTES = SM::bytes(KS);  // of one query-owning group of waves
    char* const lds_all = lds;
    lds += split * LDS_BYTES;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const bf16_t* Q = (const bf16_t*)p.q;
    const char* K = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* V = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);

    // this wave's queries
    const int q_lo_w = wave * QW;
    int nq = nq_wg - q_lo_w;
    nq = nq < 0 ? 0 : (nq > QW ? QW : nq);
    const bool wave_active = nq > 0;
    const int kt_end = (n_kv + KT - 1) / KT;  // key tiles of the item
    const int n_local = kt_end > split ? (kt_end - split + KS - 1) / KS : 0;  // ... of this wave: split + i*KS

    CT ct;
    ct.init(tid, row_bytes);
    // LDS read offsets of this lane.  K fragment of contraction step kc (A operand: row r,
    // channels 16*kc + 8g ..): kr + 32*kc.  V^T fragment of channel block db for the keys in
    // registers 8c..8c+7 of the score layout (keys 16c + 4g + 0..3 and 16c + 8 + 4g + 0..3): two
    // transposing reads at vr + 64*db + 16c rows (+ 8 rows); in each, the 16 lanes of a group
    // address a 4 (keys) x 16 (channels) block - lane s points at key s/4, channels 4*(s%4) .. -
    // and lane i receives channel i of the four keys.
    const int kr = r * SM::K_STRIDE + g * 16;
    const int vr = (4 * g + ((lane & 15) >> 2)) * SM::V_STRIDE + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // Q^T fragments (B operand): column = query 32*qb + r, contraction = channels 16*kc + 8g..
    // The workgroup's query tile is fetched with whole-row coalesced loads (rows past the tile
    // read as zero), staged in LDS in the K-tile row layout, and each wave picks its fragments.
    constexpr int QT = QW * NW;
    constexpr int Q_LOADS = QT * CT::CHUNKS / (64 * NW);
    static_assert(QT * SM::K_STRIDE <= LDS_BYTES, "query tile must fit the tile buffers");
    bf16x8 qf[NQB][KC];
    {
        const char* qbase = (const char*)(Q + q_src_row(p, q_row0) * hd + (int64_t)h * D);
        const __amdgpu_buffer_rsrc_t qrsrc =
            __builtin_amdgcn_make_buffer_rsrc((void*)qbase, 0, (nq_wg - 1) * (int)row_bytes + D * 2, 0x00020000);
        u32x4 qst[Q_LOADS];
#pragma unroll
        for (int i = 0; i < Q_LOADS; ++i)
            qst[i] = __builtin_amdgcn_raw_buffer_load_b128(qrsrc, ct.goff, i * CT::ROWS_PER_LOAD * row_bytes, 0);
#pragma unroll
        for (int i = 0; i < Q_LOADS; ++i) *(u32x4*)(lds + ct.kw + i * CT::ROWS_PER_LOAD * SM::K_STRIDE) = qst[i];
        if (NW > 1) __syncthreads();
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int kc = 0; kc < KC; ++kc)
                qf[qb][kc] = *(const bf16x8*)(lds + (q_lo_w + 32 * qb) * SM::K_STRIDE + kr + 32 * kc);
        if (NW > 1) __syncthreads();  // the tile buffers are reused for K/V from here on
    }

    // key k is visible iff (unsigned)k <= key_span (every key of the history; none if it is empty)
    const int key_lo = n_kv > 0 ? 0 : 0x3fffffff;
    const unsigned key_span = n_kv > 0 ? (unsigned)(n_kv - 1) : 0u;

    f32x16 oacc[DB][NQB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][qb][v] = 0.f;
    float m_ref[NQB], l_run[NQB];  // softmax: reference maximum (log2 units) and running sum
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) { m_ref[qb] = -INFINITY; l_run[qb] = 0.f; }
    const float sc = SOFTMAX ? p.scale * LOG2E : p.scale;

    // AHEAD tiles ahead of the one being consumed are in flight in registers (AHEAD register sets,
    // used in turn): one tile costs a full memory round trip, so a wave that walks its history alone
    // moves AHEAD tiles per round trip.
    static_assert(AHEAD == 1 || AHEAD % 2 == 0, "the LDS double buffer alternates with the tile index");
    u32x4 kst[AHEAD][CT::LOADS], vst[AHEAD][CT::LOADS];
    auto fetch = [&](u32x4 (&ks)[CT::LOADS], u32x4 (&vs)[CT::LOADS], int i) {
        const int kt = split + i * KS;
        if (kt < kt_end) {
            const int rows = n_kv - kt * KT;
            ct.template load<true>(ks, K + kt * tile_bytes, rows);
            ct.template load<true>(vs, V + kt * tile_bytes, rows);
        }
    };
    auto compute = [&](const char* ldsK, const char* ldsV, int i) {
        if (!wave_active) return;
        const int kt = split + i * KS;
        // ---- S^T = K Q^T
        f32x16 sacc[NQB];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[qb][v] = 0.f;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 a = *(const bf16x8*)(ldsK + kr + 32 * kc);
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) sacc[qb] = mfma32(a, qf[qb][kc], sacc[qb]);
        }
        // ---- score function, masking, packing
        const int key_base = kt * KT;
        const bool need_mask = key_base + KT > n_kv;  // only the last tile of a history has invisible keys
        bf16x8 pf[NQB][2];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
            score_to_weights<ACT, DB, NQB>(sacc[qb], need_mask, (unsigned)(key_base + 4 * g - key_lo), key_span, sc, m_ref[qb],
                                           l_run[qb], oacc, qb, pf[qb]);
        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const char* src = ldsV + vr + 64 * db + c * 16 * SM::V_STRIDE;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src + 8 * SM::V_STRIDE));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const bf16x8 a = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) oacc[db][qb] = mfma32(a, pf[qb][c], oacc[db][qb]);
            }
        }
    };
    auto step = [&](u32x4 (&ks)[CT::LOADS], u32x4 (&vs)[CT::LOADS], int i, int buf) {
        char* ldsK = lds + (KS > 1 ? 0 : buf) * SM::BUF_BYTES;
        char* ldsV = ldsK + SM::K_TILE;
        ct.store(ldsK, ldsV, ks, vs);
        // the tile is complete in LDS; every wave is also done with the other buffer (the tile before)
        if (NW > 1) __syncthreads();
        fetch(ks, vs, i + AHEAD);
        compute(ldsK, ldsV, i);
    };
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) fetch(kst[j], vst[j], j);
    if (AHEAD == 1) {
        for (int i = 0; i < n_local; i += 2) {
            step(kst[0], vst[0], i, 0);
            if (i + 1 < n_local) step(kst[0], vst[0], i + 1, 1);
        }
    } else {
        for (int i = 0; i < n_local; i += AHEAD) {
#pragma unroll
            for (int j = 0; j < AHEAD; ++j)
                if (i + j < n_local) step(kst[j], vst[j], i + j, j & 1);
        }
    }

    if (KS > 1) {
        // ---- merge of the KS partial results (wave 0 collects, in wave order): every other wave leaves its
        // accumulators, lane by lane, in its own idle tile buffers, with the softmax reference and sum
        constexpr int STAT = DB * NQB * 4 * 1024;  // byte offset of the statistics behind the accumulators
        static_assert(STAT + NQB * 2 * 256 <= LDS_BYTES, "partial results must fit the tile buffers");
        if (split > 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        f32x4 x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = oacc[db][qb][4 * vg + e];
                        *(f32x4*)(lds + ((db * NQB + qb) * 4 + vg) * 1024 + lane * 16) = x;
                    }
            if (SOFTMAX) {
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) {
                    *(float*)(lds + STAT + (2 * qb) * 256 + lane * 4) = m_ref[qb];
                    *(float*)(lds + STAT + (2 * qb + 1) * 256 + lane * 4) = l_run[qb];
                }
            }
        }
        __syncthreads();
        if (split > 0) return;
        for (int w = 1; w < KS; ++w) {
            const char* part = lds_all + w * LDS_BYTES;
            float cw[NQB];
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                cw[qb] = 1.f;
                if (SOFTMAX) {
                    const float mw = *(const float*)(part + STAT + (2 * qb) * 256 + lane * 4);
                    const float lw = *(const float*)(part + STAT + (2 * qb + 1) * 256 + lane * 4);
                    const float m_new = fmaxf(m_ref[qb], mw);
                    const float c0 = m_ref[qb] == -INFINITY ? 0.f : fast_exp2(m_ref[qb] - m_new);
                    cw[qb] = mw == -INFINITY ? 0.f : fast_exp2(mw - m_new);
                    l_run[qb] = l_run[qb] * c0 + lw * cw[qb];
                    m_ref[qb] = m_new;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= c0;
                }
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        const f32x4 x = *(const f32x4*)(part + ((db * NQB + qb) * 4 + vg) * 1024 + lane * 16);
#pragma unroll
                        for (int e = 0; e < 4; ++e) oacc[db][qb][4 * vg + e] = fmaf(x[e], cw[qb], oacc[db][qb][4 * vg + e]);
                    }
        }
    }

    // ---- epilogue: lane holds query 32*qb + r, channels 32*db + 8*(v/4) + 4g + (v%4).  The wave
    // transposes its O tile through LDS (its own region of the now idle tile buffers) and
    // writes whole rows, 16 bytes per lane.
    if (NW > 1) __syncthreads();  // every wave is done with the K/V tiles
    if (!wave_active) return;
    char* stage = lds + wave * (QW * SM::K_STRIDE);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int qi = 32 * qb + r;  // inside this wave's block
        float inv = 1.f;
        if (SOFTMAX) {
            const float l_tot = halves_sum(l_run[qb]);
            inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            if (p.lse && g == 0 && qi < nq)
                p.lse[(int64_t)h * p.total_q + q_row0 + q_lo_w + qi] =
                    l_tot > 0.f ? (m_ref[qb] + __builtin_amdgcn_logf(l_tot)) * (1.f / LOG2E) : -INFINITY;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                bf16x4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (bf16_t)(oacc[db][qb][4 * vg + e] * inv);
                *(bf16x4*)(stage + qi * SM::K_STRIDE + (32 * db + 8 * vg + 4 * g) * 2) = out;
            }
    }
    {
        bf16_t* obase = (bf16_t*)p.o + (q_row0 + q_lo_w) * hd + (int64_t)h * D;
        constexpr int O_STORES = QW * CT::CHUNKS / 64;
        const int chunk = lane % CT::CHUNKS, rsub = lane / CT::CHUNKS;
#pragma unroll
        for (int i = 0; i < O_STORES; ++i) {
            const int row = i * (64 / CT::CHUNKS) + rsub;
            const u32x4 val = *(const u32x4*)(stage + row * SM::K_STRIDE + chunk * 16);
            if (row < nq) __builtin_nontemporal_store(val, (u32x4*)(obase + row * hd + chunk * 8));  // written once, not read back
        }
    }
}

template <int D, int NQB, int NW, int AHEAD, int KS>
__device__ __forceinline__ void attn_fwd_dispatch(const AttnParams& p, char* lds, int act, int h, int64_t q_row0,
                                                  int nq, int64_t k0, int n_kv) {
    switch (act) {
    case KUNLUN_ACT_SOFTMAX: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_SOFTMAX, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    case KUNLUN_ACT_IDENTITY: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_IDENTITY, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    case KUNLUN_ACT_RELU: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_RELU, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    case KUNLUN_ACT_GELU: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_GELU, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    case KUNLUN_ACT_GELU_TANH: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_GELU_TANH, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    case KUNLUN_ACT_SILU: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_SILU, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    default: attn_fwd_item<D, NQB, NW, KUNLUN_ACT_GELU_POLY, AHEAD, KS>(p, lds, h, q_row0, nq, k0, n_kv); break;
    }
}

// GDPA / cross attention: work items = (example, query tile, head), examples in scheduler order (longest
// history first).  Item i belongs to "lane" i % 8: consecutive entries (example, query tile) go to consecutive
// lanes and each lane walks through all heads of its entries - on a grid of one workgroup per item, where
// workgroup i runs on XCD i % 8, every L2 so sees all address residues modulo the token stride H*D*2 (one head
// per XCD would use only a fraction of the L2 channels).
// With a work counter (p.queue: launches with more items than resident workgroups) the launch is persistent:
// as many workgroups as fit the device, each starts with the item of its index and then takes the next
// unclaimed one, which is the dispatcher's longest-first list scheduling without its cost (measured on the
// jagged benchmark batch: with cheap score functions the dispatcher kept a third of the workgroup slots empty).
// The counter is asked for the next item while the current one starts.
template <int D, int NQB, int NW, int OCC, int AHEAD, int KS>
__global__ __launch_bounds__(64 * NW * KS, OCC) void gdpa_fwd_mfma_kernel(AttnParams p, int n_qtiles, int n_items) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];  // KS * FwdSmem<D>::bytes(KS) bytes
    constexpr int QT = 32 * NQB * NW;
    // hand-over word for the next item: the last word of the tile buffers, dead between items
    volatile int* const next_word = (volatile int*)(lds + KS * FwdSmem<D>::bytes(KS) - 4);
    const int64_t n_entries = (int64_t)p.B * n_qtiles;
    int item = blockIdx.x;
    while (item < n_items) {
        int claimed = 0;
        if (KS == 1 && p.queue && threadIdx.x == 0) claimed = atomicAdd(p.queue, 1);
        const int slot = item & 7;
        const int64_t j = item >> 3;
        const int h = (int)(j % p.H);
        const int64_t e = (j / p.H) * 8 + slot;
        if (e < n_entries) {
            const int qt = (int)(e % n_qtiles);
            const int b = p.order ? p.order[e / n_qtiles] : (int)(e / n_qtiles);
            const int64_t qb0 = q_begin(p, b);
            const int64_t nq_all = q_end(p, b) - qb0;
            const int64_t q_first = (int64_t)qt * QT;
            if (q_first < nq_all) {
                const int nq = (int)((nq_all - q_first) < QT ? (nq_all - q_first) : QT);
                const int64_t k0 = p.kv_off[b];
                const int n_kv = p.kv_off[b + 1] - (int)k0;
                attn_fwd_dispatch<D, NQB, NW, AHEAD, KS>(p, lds, p.head_act[h], h, qb0 + q_first, nq, k0, n_kv);
            }
        }
        if (KS > 1 || !p.queue) break;
        __syncthreads();  // the item's last LDS reads (output rows) are done
        if (threadIdx.x == 0) *next_word = claimed + (int)gridDim.x;
        __syncthreads();
        item = __builtin_amdgcn_readfirstlane(*next_word);  // (next written by the second key tile of the next item, behind barriers)
    }
}

bool mfma_fwd_supported(const AttnParams& p, int dtype) {
    if (dtype != KUNLUN_BF16 || (p.d != 32 && p.d != 64 && p.d != 128)) return false;
    // the online softmax takes the row maximum before scaling: it needs scale > 0
    // (other scales are served by the generic kernels)
    for (int h = 0; h < p.H; ++h)
        if (p.head_act[h] == KUNLUN_ACT_SOFTMAX && !(p.scale > 0.f)) return false;
    return true;
}

template <int D, int NQB, int NW, int OCC, int AHEAD, int KS = 1>
static hipError_t launch_gdpa(const AttnParams& p, hipStream_t stream) {
    constexpr int QT = 32 * NQB * NW;
    constexpr int bytes = KS * FwdSmem<D>::bytes(KS);
    auto kern = gdpa_fwd_mfma_kernel<D, NQB, NW, OCC, AHEAD, KS>;
    if (bytes > 64 * 1024) {
        // once per process (thread-safe initialisation of a function-local static); not a stream operation
        static const hipError_t raised = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (raised != hipSuccess) return raised;
    }
    const int n_qtiles = (p.max_q + QT - 1) / QT;
    const int64_t n_items = (((int64_t)p.B * n_qtiles + 7) / 8) * 8 * p.H;
    int64_t grid = n_items;
    if (KS == 1 && p.queue) {
        // workgroups of this kernel that fit the device (once per process, like the attribute above)
        static const int per_cu = [&] {
            int n = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)kern, 64 * NW * KS, bytes) != hipSuccess || n < 1) n = 1;
            return n;
        }();
        const int64_t resident = (int64_t)per_cu * compute_units();
        if (grid > resident) grid = resident;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NW * KS), bytes, stream, p, n_qtiles, (int)n_items);
    return hipGetLastError();
}

bool mfma_fwd_is_qtiled(const AttnParams& p) { return p.windowed || p.max_q > 64; }

hipError_t launch_mfma_fwd(const AttnParams& p, hipStream_t stream) {
    // 32 queries per wave, up to 255 registers per wave, two or three waves per SIMD.
    // Query-tiled launches use 128-query tiles (4 waves): fewer K/V tile loads per query.
    if (mfma_fwd_is_qtiled(p)) return launch_mfma_fwd_qtiled(p, stream);
    // Up to 32 queries per example = one wave per (example, head).  With few work items (every wave has a SIMD to
    // itself) the longest history and the score function of a single wave would set the time: four waves (two at
    // d = 128) then share the key tiles of an item.  (cfg2, GELU: 48 -> 40 us cold; the floor of that launch -
    // identity scores - is 37 us for its 156 MB.)
    const bool few_items = (int64_t)p.B * p.H <= 2048;
    if (p.max_q <= 32) {
        if (p.d == 128) return few_items ? launch_gdpa<128, 1, 1, 2, 1, 2>(p, stream) : launch_gdpa<128, 1, 1, 2, 1>(p, stream);
        if (p.d == 64) return few_items ? launch_gdpa<64, 1, 1, 2, 2, 4>(p, stream) : launch_gdpa<64, 1, 1, 2, 2>(p, stream);
        return few_items ? launch_gdpa<32, 1, 1, 2, 2, 4>(p, stream) : launch_gdpa<32, 1, 1, 2, 2>(p, stream);
    }
    return p.d == 128 ? launch_gdpa<128, 1, 2, 2, 2>(p, stream)
           : p.d == 64 ? launch_gdpa<64, 1, 2, 2, 2>(p, stream) : launch_gdpa<32, 1, 2, 2, 2>(p, stream);
}

}  // namespace kunlun
