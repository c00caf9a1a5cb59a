// bf16 matrix-core backward in two passes, for the shapes the fused backward kernel does not
// take: sliding-window self-attention (Eq. (sliding window)) and GDPA / softmax attention with
// more than 64 queries per example (the PFFN direction of Eq. (GDPA): sequence tokens are the
// queries).  Scores are recomputed tile by tile in both passes; nothing of score size is stored.
//
//   pass A (dQ):     one workgroup per (example, head, 128-query tile), the mirror image of the
//                    forward kernel: each wave owns 32 queries (Q^T and dO^T fragments in
//                    registers) and the waves stream the K/V tiles of the tile's key range;
//                        S^T = K Q^T,  dP^T = V dO^T,  dS^T in registers,  dQ^T += K^T dS^T.
//   pass B (dK, dV): one workgroup per (example, head, 128-key tile): each wave owns 32 keys
//                    (K^T and V^T fragments in registers) and the waves stream the Q/dO tiles of
//                    the queries that see those keys;
//                        S = Q K^T,  dP = dO V^T,  P and dS in registers (one key per lane),
//                        dV^T += dO^T P,  dK^T += Q^T dS.
// In both passes the score tile comes out of the first contraction with the owned dimension
// on the lanes, so the packed registers are directly the B operand of the second contraction
// and the streamed operand is read transposed from LDS (ds_read_b64_tr_b16).
// Softmax heads use the forward LSE and delta = rowsum(dO * O), computed once by a small
// kernel into the workspace.
#include "mfma_tile.h"

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

// Cooperative loads of a 32-row tile of a [tokens, H, D] tensor by 64*NW threads (whole rows
// coalesce); rows past `rows_valid` read as zero through the buffer resource.
template <int D, int NW>
struct TileIO {
    using PT = PadTiles<D>;
    static constexpr int CHUNKS = D / 8;
    static constexpr int SLOTS = KT * CHUNKS;
    static constexpr int LOADS = SLOTS / (64 * NW);
    static constexpr int ROWS_PER_LOAD = 64 * NW / CHUNKS;
    static_assert(LOADS >= 1 && SLOTS % (64 * NW) == 0, "tile does not split evenly over the workgroup");
    uint32_t goff, row_bytes;
    int w_row, w_tr;

    __device__ __forceinline__ void init(int tid, uint32_t row_stride_bytes) {
        const int row0 = tid / CHUNKS, chunk = tid % CHUNKS;
        row_bytes = row_stride_bytes;
        goff = (uint32_t)row0 * row_stride_bytes + chunk * 16;
        w_row = row0 * PT::ROW_STRIDE + chunk * 16;
        w_tr = row0 * PT::TR_STRIDE + chunk * 16;
    }
    __device__ __forceinline__ void load(u32x4 (&st)[LOADS], const char* __restrict__ tile_base, int rows_valid) const {
        const int rows = rows_valid < KT ? rows_valid : KT;
        const int bytes = (rows - 1) * (int)row_bytes + D * 2;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)tile_base, 0, bytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < LOADS; ++i) st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff, i * ROWS_PER_LOAD * row_bytes, 0);
    }
    __device__ __forceinline__ void store_row(char* lds, const u32x4 (&st)[LOADS]) const {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) *(u32x4*)(lds + w_row + i * ROWS_PER_LOAD * PT::ROW_STRIDE) = st[i];
    }
    __device__ __forceinline__ void store_tr(char* lds, const u32x4 (&st)[LOADS]) const {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) *(u32x4*)(lds + w_tr + i * ROWS_PER_LOAD * PT::TR_STRIDE) = st[i];
    }
};

// Stage a tile of up to 32*NW rows (global rows row0.., head h) into LDS in the row layout
// (whole-row coalesced loads, zero rows past n_rows).  Caller synchronises.
template <int D, int NW>
__device__ __forceinline__ void stage_rows(char* lds, const bf16_t* tensor, int64_t row0, int n_rows, int h, int H,
                                           const TileIO<D, NW>& io) {
    using PT = PadTiles<D>;
    using IO = TileIO<D, NW>;
    constexpr int N_LOADS = 32 * NW * IO::CHUNKS / (64 * NW);
    const char* base = (const char*)(tensor + (row0 * H + h) * D);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (n_rows - 1) * (int)io.row_bytes + D * 2, 0x00020000);
    u32x4 st[N_LOADS];
#pragma unroll
    for (int i = 0; i < N_LOADS; ++i)
        st[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, io.goff, i * IO::ROWS_PER_LOAD * io.row_bytes, 0);
#pragma unroll
    for (int i = 0; i < N_LOADS; ++i) *(u32x4*)(lds + io.w_row + i * IO::ROWS_PER_LOAD * PT::ROW_STRIDE) = st[i];
}

// A wave's 32 x D fp32 result tile in the C layout (lane: column r = row of the output tensor,
// registers: channels 32*db + 8*(v/4) + 4g + v%4) -> bf16 rows of a [tokens, H, D] tensor,
// transposed through the wave's own LDS region and written 16 bytes per lane.
template <int D>
__device__ __forceinline__ void store_tile_rows(char* stage, const f32x16 (&acc)[D / 32], bf16_t* out_rows, int64_t hd,
                                                int n_rows, int lane) {
    using PT = PadTiles<D>;
    constexpr int CHUNKS = D / 8;
    const int r = lane & 31, g = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            bf16x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (bf16_t)acc[db][4 * vg + e];
            *(bf16x4*)(stage + r * PT::ROW_STRIDE + (32 * db + 8 * vg + 4 * g) * 2) = out;
        }
    const int chunk = lane % CHUNKS, rsub = lane / CHUNKS;
#pragma unroll
    for (int i = 0; i < 32 * CHUNKS / 64; ++i) {
        const int row = i * (64 / CHUNKS) + rsub;
        const u32x4 val = *(const u32x4*)(stage + row * PT::ROW_STRIDE + chunk * 16);
        if (row < n_rows) *(u32x4*)(out_rows + row * hd + chunk * 8) = val;
    }
}

// The transposed fragment (A operand) of channel block db for the 16 tile rows that the C
// layout puts in registers 8c .. 8c+7 (rows 16c + 4g + 0..3 and 16c + 8 + 4g + 0..3).
template <int D>
__device__ __forceinline__ bf16x8 tr_frag(const char* tile, int vr, int db, int c) {
    using PT = PadTiles<D>;
    const char* src = tile + vr + 64 * db + c * 16 * PT::TR_STRIDE;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src + 8 * PT::TR_STRIDE));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// ------------------------------------------------------------------ pass A: dQ

template <int D>
struct DqSmem {
    using PT = PadTiles<D>;
    static constexpr int BUF = 2 * PT::ROW_TILE + PT::TR_TILE;  // K rows | K for transposed reads | V rows
    static constexpr int TOTAL = 2 * BUF;
};

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void bwd_dq_item(const AttnParams& p, const float* __restrict__ delta_ws, char* lds, int h,
                                            int64_t q_row0, int nq_wg, int64_t t0_wg, int64_t k0, int n_kv) {
    using PT = PadTiles<D>;
    using IO = TileIO<D, NW>;
    using SM = DqSmem<D>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16, DB = D / 32;
    static_assert(32 * NW * PT::ROW_STRIDE <= SM::TOTAL, "query tile must fit the tile buffers");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* K = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* V = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);

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

    IO io;
    io.init(tid, row_bytes);
    const int kr = r * PT::ROW_STRIDE + g * 16;
    const int vr = (4 * g + ((lane & 15) >> 2)) * PT::TR_STRIDE + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // Q^T and dO^T fragments of this wave's queries (B operands), via LDS
    bf16x8 qf[KC], dof[KC];
    stage_rows<D, NW>(lds, (const bf16_t*)p.q, q_row0, nq_wg, h, p.H, io);
    __syncthreads();
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[kc] = *(const bf16x8*)(lds + q_lo_w * PT::ROW_STRIDE + kr + 32 * kc);
    __syncthreads();
    stage_rows<D, NW>(lds, (const bf16_t*)p.d_o, q_row0, nq_wg, h, p.H, io);
    __syncthreads();
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) dof[kc] = *(const bf16x8*)(lds + q_lo_w * PT::ROW_STRIDE + kr + 32 * kc);
    __syncthreads();

    // this lane's query: softmax statistics and visible key range
    float lse2 = INFINITY, delta = 0.f;
    if (SOFTMAX && r < nq) {
        const int64_t idx = (int64_t)h * p.total_q + q_row0 + q_lo_w + r;
        lse2 = p.lse[idx] * LOG2E_T;
        delta = delta_ws[idx];
    }
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

    u32x4 kst[IO::LOADS], vst[IO::LOADS];
    auto fetch = [&](int kt) {
        if (kt < kt_end) {
            io.load(kst, K + kt * tile_bytes, n_kv - kt * KT);
            io.load(vst, V + kt * tile_bytes, n_kv - kt * KT);
        }
    };
    fetch(kt_begin);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        char* ldsK = lds + ((kt - kt_begin) & 1) * SM::BUF;
        char* ldsKt = ldsK + PT::ROW_TILE;
        char* ldsV = ldsKt + PT::TR_TILE;
        io.store_row(ldsK, kst);
        io.store_tr(ldsKt, kst);
        io.store_row(ldsV, vst);
        __syncthreads();  // tile kt complete; every wave is done with the other buffer
        fetch(kt + 1);
        if (!wave_active || kt < w_begin || kt >= w_end) continue;
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 ka = *(const bf16x8*)(ldsK + kr + 32 * kc);
            const bf16x8 va = *(const bf16x8*)(ldsV + kr + 32 * kc);
            sacc = mfma32(ka, qf[kc], sacc);
            dpacc = mfma32(va, dof[kc], dpacc);
        }
        // dS^T in registers (lane: query, registers: keys of the tile)
        const unsigned rel0 = (unsigned)(kt * KT + 4 * g - key_lo);
        float dsv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float s = sacc[v] * sc;
            float ds;
            if (SOFTMAX) {
                ds = fast_exp2(s - lse2) * (dpacc[v] - delta) * p.scale;
            } else {
                float val, der;
                act_fast_vd<ACT>(s, val, der);
                ds = dpacc[v] * der * p.scale;
            }
            const bool ok = rel0 + (unsigned)(8 * (v >> 2) + (v & 3)) <= key_span;
            dsv[v] = ok ? ds : 0.f;
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
            for (int c = 0; c < 2; ++c) dqacc[db] = mfma32(tr_frag<D>(ldsKt, vr, db, c), dsf[c], dqacc[db]);
    }
    __syncthreads();  // every wave is done with the tile buffers
    if (!wave_active) return;
    store_tile_rows<D>(lds + wave * PT::ROW_TILE, dqacc, (bf16_t*)p.dq + (q_row0 + q_lo_w) * hd + (int64_t)h * D, hd, nq,
                       lane);
}

// ------------------------------------------------------------------ pass B: dK, dV

template <int D>
struct DkvSmem {
    using PT = PadTiles<D>;
    static constexpr int STATS = 256;  // lse (log2 units) and delta of the 32 queries of a tile
    static constexpr int BUF = 2 * PT::ROW_TILE + 2 * PT::TR_TILE + STATS;  // Q rows | Q tr | dO rows | dO tr | stats
    static constexpr int TOTAL = 2 * BUF;
};

template <int D, int NW, int ACT, bool WINDOWED>
__device__ __forceinline__ void bwd_dkdv_item(const AttnParams& p, const float* __restrict__ delta_ws, char* lds, int h,
                                              int64_t k_row0, int nk_wg, int kpos0_wg, int64_t q0, int nq_all) {
    using PT = PadTiles<D>;
    using IO = TileIO<D, NW>;
    using SM = DkvSmem<D>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16, DB = D / 32;
    static_assert(32 * NW * PT::ROW_STRIDE <= SM::TOTAL, "key tile must fit the tile buffers");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const char* Q = (const char*)((const bf16_t*)p.q + (q0 * p.H + h) * D);
    const char* DO = (const char*)((const bf16_t*)p.d_o + (q0 * p.H + h) * D);

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

    IO io;
    io.init(tid, row_bytes);
    const int kr = r * PT::ROW_STRIDE + g * 16;
    const int vr = (4 * g + ((lane & 15) >> 2)) * PT::TR_STRIDE + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // K^T and V^T fragments of this wave's keys (B operands: column = key r), via LDS
    bf16x8 kf[KC], vf[KC];
    stage_rows<D, NW>(lds, (const bf16_t*)p.k, k_row0, nk_wg, h, p.H, io);
    __syncthreads();
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) kf[kc] = *(const bf16x8*)(lds + k_lo_w * PT::ROW_STRIDE + kr + 32 * kc);
    __syncthreads();
    stage_rows<D, NW>(lds, (const bf16_t*)p.v, k_row0, nk_wg, h, p.H, io);
    __syncthreads();
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) vf[kc] = *(const bf16x8*)(lds + k_lo_w * PT::ROW_STRIDE + kr + 32 * kc);
    __syncthreads();

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

    u32x4 qst[IO::LOADS], dst[IO::LOADS];
    float st_lse = INFINITY, st_delta = 0.f;
    auto fetch = [&](int qt) {
        if (qt < qt_end) {
            io.load(qst, Q + qt * tile_bytes, nq_all - qt * KT);
            io.load(dst, DO + qt * tile_bytes, nq_all - qt * KT);
            if (SOFTMAX && tid < KT) {
                const int qi = qt * KT + tid;
                st_lse = INFINITY;  // weight exp2(s - inf) = 0 for rows past the end
                st_delta = 0.f;
                if (qi < nq_all) {
                    const int64_t idx = (int64_t)h * p.total_q + q0 + qi;
                    st_lse = p.lse[idx] * LOG2E_T;
                    st_delta = delta_ws[idx];
                }
            }
        }
    };
    fetch(qt_begin);
    for (int qt = qt_begin; qt < qt_end; ++qt) {
        char* ldsQ = lds + ((qt - qt_begin) & 1) * SM::BUF;
        char* ldsQt = ldsQ + PT::ROW_TILE;
        char* ldsDO = ldsQt + PT::TR_TILE;
        char* ldsDOt = ldsDO + PT::ROW_TILE;
        float* stats = (float*)(ldsDOt + PT::TR_TILE);
        io.store_row(ldsQ, qst);
        io.store_tr(ldsQt, qst);
        io.store_row(ldsDO, dst);
        io.store_tr(ldsDOt, dst);
        if (SOFTMAX && tid < KT) { stats[tid] = st_lse; stats[KT + tid] = st_delta; }
        __syncthreads();  // tile qt complete; every wave is done with the other buffer
        fetch(qt + 1);
        if (!wave_active || qt < w_begin || qt >= w_end) continue;
        // S = Q K^T and dP = dO V^T: lane = key column, registers = queries of the tile
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 qa = *(const bf16x8*)(ldsQ + kr + 32 * kc);
            const bf16x8 da = *(const bf16x8*)(ldsDO + kr + 32 * kc);
            sacc = mfma32(qa, kf[kc], sacc);
            dpacc = mfma32(da, vf[kc], dpacc);
        }
        const unsigned rel0 = (unsigned)(qt * KT + 4 * g - q_lo);
        float pv[16], dsv[16];
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            f32x4 lse4 = {0.f, 0.f, 0.f, 0.f}, del4 = {0.f, 0.f, 0.f, 0.f};
            if (SOFTMAX) {
                lse4 = *(const f32x4*)(stats + 8 * vg + 4 * g);
                del4 = *(const f32x4*)(stats + KT + 8 * vg + 4 * g);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = 4 * vg + e;
                const float s = sacc[v] * sc;
                float val, ds;
                if (SOFTMAX) {
                    val = fast_exp2(s - lse4[e]);
                    ds = val * (dpacc[v] - del4[e]) * p.scale;
                } else {
                    float der;
                    act_fast_vd<ACT>(s, val, der);
                    ds = dpacc[v] * der * p.scale;
                }
                const bool ok = rel0 + (unsigned)(8 * vg + e) <= q_span;
                pv[v] = ok ? val : 0.f;
                dsv[v] = ok ? ds : 0.f;
            }
        }
        bf16x8 pf[2], dsf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) { pf[c][e] = (bf16_t)pv[8 * c + e]; dsf[c][e] = (bf16_t)dsv[8 * c + e]; }
        // dV^T += dO^T P and dK^T += Q^T dS (contraction over the queries of the tile)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                dvacc[db] = mfma32(tr_frag<D>(ldsDOt, vr, db, c), pf[c], dvacc[db]);
                dkacc[db] = mfma32(tr_frag<D>(ldsQt, vr, db, c), dsf[c], dkacc[db]);
            }
    }
    __syncthreads();  // every wave is done with the tile buffers
    if (!wave_active) return;
    char* stage = lds + wave * PT::ROW_TILE;
    store_tile_rows<D>(stage, dvacc, (bf16_t*)p.dv + (k_row0 + k_lo_w) * hd + (int64_t)h * D, hd, nk, lane);
    store_tile_rows<D>(stage, dkacc, (bf16_t*)p.dk + (k_row0 + k_lo_w) * hd + (int64_t)h * D, hd, nk, lane);
}

// ------------------------------------------------------------------ kernels

// items = (example, head, tile) in that order, cut into 8 contiguous ranges, one per XCD
// (workgroup i runs on XCD i % 8); tile_start[b] = number of tiles before example b.
__device__ __forceinline__ bool locate_item(const int32_t* __restrict__ tile_start, int B, int H, int& b, int& h, int& t) {
    const int64_t n_items = (int64_t)tile_start[B] * H;
    const int64_t per_xcd = (n_items + 7) / 8;
    const int xcd = blockIdx.x & 7;
    const int64_t slot = blockIdx.x >> 3;
    if (slot >= per_xcd) return false;
    const int64_t item = xcd * per_xcd + slot;
    if (item >= n_items) return false;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)tile_start[mid] * H <= item) lo = mid; else hi = mid - 1;
    }
    b = lo;
    const int nt = tile_start[b + 1] - tile_start[b];
    const int64_t rem = item - (int64_t)tile_start[b] * H;
    h = (int)(rem / nt);
    t = (int)(rem % nt);
    return true;
}

#define KUNLUN_ACT_SWITCH(ACTV, CALL)                                   \
    switch (ACTV) {                                                     \
    case KUNLUN_ACT_SOFTMAX: { constexpr int A = KUNLUN_ACT_SOFTMAX; CALL; } break;     \
    case KUNLUN_ACT_IDENTITY: { constexpr int A = KUNLUN_ACT_IDENTITY; CALL; } break;   \
    case KUNLUN_ACT_RELU: { constexpr int A = KUNLUN_ACT_RELU; CALL; } break;           \
    case KUNLUN_ACT_GELU: { constexpr int A = KUNLUN_ACT_GELU; CALL; } break;           \
    case KUNLUN_ACT_GELU_TANH: { constexpr int A = KUNLUN_ACT_GELU_TANH; CALL; } break; \
    default: { constexpr int A = KUNLUN_ACT_SILU; CALL; } break;                        \
    }

template <int D, int NW, bool WINDOWED>
__global__ __launch_bounds__(64 * NW, 2) void bwd_dq_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                            const float* __restrict__ delta_ws) {
    __shared__ __attribute__((aligned(1024))) char lds[DqSmem<D>::TOTAL];
    int b, h, qt;
    if (!locate_item(tile_start, p.B, p.H, b, h, qt)) return;
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
__global__ __launch_bounds__(64 * NW, 2) void bwd_dkdv_kernel(AttnParams p, const int32_t* __restrict__ tile_start,
                                                              const float* __restrict__ delta_ws) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];  // DkvSmem<D>::TOTAL bytes (above 64 KB at D = 128)
    int b, h, kt;
    if (!locate_item(tile_start, p.B, p.H, b, h, kt)) return;
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

// Exclusive prefix sum of ceil(len_b / tile) over the examples (off == null: dense_len rows each).
__global__ __launch_bounds__(1024) void bwd_tile_prefix_kernel(const int32_t* __restrict__ off, int dense_len, int B,
                                                               int tile, int32_t* __restrict__ tile_start) {
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
        run += tiles_of(b);
    }
    if (tid == 1023) tile_start[B] = part[1023];
}

bool mfma_bwd_tiled_supported(const AttnParams& p, int dtype) {
    return dtype == KUNLUN_BF16 && (p.d == 64 || p.d == 128);
}

size_t mfma_bwd_tiled_workspace(int B, int H, int64_t total_q) {
    return 2 * align_up((size_t)(B + 1) * sizeof(int32_t), 256) + align_up((size_t)H * total_q * sizeof(float), 256);
}

template <int D, bool WINDOWED>
static hipError_t launch_tiled(const AttnParams& p, char* ws, bool any_softmax, hipStream_t stream) {
    constexpr int NW = 4, TILE = 32 * NW;
    const size_t pre = align_up((size_t)(p.B + 1) * sizeof(int32_t), 256);
    int32_t* q_tiles = (int32_t*)ws;
    int32_t* k_tiles = (int32_t*)(ws + pre);
    float* delta = (float*)(ws + 2 * pre);
    if (any_softmax && p.total_q > 0) {
        const int64_t threads = p.total_q * p.H * (D / 8);
        hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                           (const bf16_t*)p.o, (const bf16_t*)p.d_o, delta, p.total_q, p.H);
    }
    if (p.total_q > 0) {
        hipLaunchKernelGGL(bwd_tile_prefix_kernel, dim3(1), dim3(1024), 0, stream, p.q_off, p.max_q, p.B, TILE, q_tiles);
        const int64_t per_xcd = ((p.total_q / TILE + p.B) * p.H + 7) / 8;
        hipLaunchKernelGGL((bwd_dq_kernel<D, NW, WINDOWED>), dim3((unsigned)(per_xcd * 8)), dim3(64 * NW), 0, stream, p,
                           q_tiles, delta);
    }
    if (p.total_kv > 0) {
        hipLaunchKernelGGL(bwd_tile_prefix_kernel, dim3(1), dim3(1024), 0, stream, p.kv_off, 0, p.B, TILE, k_tiles);
        const int64_t per_xcd = ((p.total_kv / TILE + p.B) * p.H + 7) / 8;
        auto kern = bwd_dkdv_kernel<D, NW, WINDOWED>;
        constexpr int lds_bytes = DkvSmem<D>::TOTAL;
        if (lds_bytes > 64 * 1024) {
            static bool raised = false;  // once per process; not a stream operation
            if (!raised) {
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e != hipSuccess) return e;
                raised = true;
            }
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(64 * NW), lds_bytes, stream, p, k_tiles, delta);
    }
    return hipGetLastError();
}

hipError_t launch_mfma_bwd_tiled(const AttnParams& p, void* workspace_tail, bool any_softmax, hipStream_t stream) {
    char* ws = (char*)workspace_tail;
    if (p.windowed) return p.d == 128 ? launch_tiled<128, true>(p, ws, true, stream) : launch_tiled<64, true>(p, ws, true, stream);
    return p.d == 128 ? launch_tiled<128, false>(p, ws, any_softmax, stream) : launch_tiled<64, false>(p, ws, any_softmax, stream);
}

}  // namespace kunlun
