// Fused bf16 matrix-core backward for GDPA / softmax attention at head dimension 128 with 33..64
// queries per example (the seed/context direction at its largest): dQ, dK, dV of <O, dO>.
//
// One workgroup of 4 wavefronts = one (example, head).  The waves form two PAIRS; a pair takes
// every second 32-key tile of the history, and inside a pair the work of a tile is split
// without any duplicated arithmetic:
//     wave w of the pair owns query block w (32 queries):
//         S^T = K Q_w^T,  dP^T = V dO_w^T           (Q_w^T, dO_w^T fragments live in registers)
//         P_w^T, dS_w^T in registers;  dQ_w^T += K^T dS_w^T
//         bf16 copies of P_w, dS_w go to the pair's [query][key] LDS tiles
//     then wave w owns channel half w (64 channels) of the key gradients:
//         dV^T[half w] = dO^T[half w] P,   dK^T[half w] = Q^T[half w] dS   (all 64 queries)
// Each wave so needs 64 (not 128) dQ accumulators and half of the score registers: the kernel
// fits 256 registers and two workgroups (2 x 80 KB of LDS) share a compute unit - two waves
// per SIMD whose memory, LDS and matrix-core latencies overlap.  The price is three workgroup
// barriers per tile.  dK/dV tiles are transposed through the dead K/V tiles and stored as whole
// rows; the dQ partial sums of the two pairs are added in LDS in a fixed order.
#include "mfma_tile.h"

namespace kunlun {

constexpr float LOG2E_P = 1.4426950408889634f;

struct PairSmem {
    static constexpr int D = 128;
    static constexpr int Q_BYTES = 64 * D * 2;          // Q tile, and dO tile
    static constexpr int TILE_BYTES = KT * D * 2;       // K tile, V tile
    static constexpr int P_BYTES = 64 * KT * 2;         // P tile, dS tile ([query][key])
    static constexpr int PAIR_BYTES = 2 * TILE_BYTES + 2 * P_BYTES;
    static constexpr int TOTAL = 2 * Q_BYTES + 2 * PAIR_BYTES;   // 80 KB
    static constexpr int REDUCE_BYTES = 2 * 64 * D * 4;           // dQ partials of the two pairs
    static_assert(REDUCE_BYTES <= TOTAL, "dQ reduction scratch must fit");
};

__device__ __forceinline__ int pp_offset(int row, int byte_in_row) {  // P / dS tile, chunk swizzled by the row
    return row * 64 + ((((byte_in_row >> 4) ^ (row >> 2)) & 3) << 4) + (byte_in_row & 15);
}
__device__ __forceinline__ int pr_offset(int row, int chunk) {        // fp32 [query][128] reduction scratch
    return row * 512 + ((chunk ^ (row & 31)) << 4);
}

template <int ACT>
__device__ __forceinline__ void attn_bwd_pair_item(const AttnParams& p, char* smem, int h, int64_t q_row0, int nq,
                                                   int64_t k0, int n_kv) {
    constexpr int D = 128;
    using L = TileLayout<D>;
    using SM = PairSmem;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16;
    // (the thread index goes through an opaque move per item: everything derived from it is then computed where the
    // item uses it, instead of being kept in registers across the persistent loop for all six score functions)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (scalar: the tile descriptors below depend on it)
    const int pair = wave >> 1, w = wave & 1;     // w: query block owned in the score phase, channel half in the dK/dV phase
    const int ptid = tid & 127;                   // thread index inside the pair
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;
    const bf16_t* Qg = (const bf16_t*)p.q + q_src_row(p, q_row0) * hd + (int64_t)h * D;
    const bf16_t* DOg = (const bf16_t*)p.d_o + q_row0 * hd + (int64_t)h * D;
    const char* Kg = (const char*)((const bf16_t*)p.k + (k0 * p.H + h) * D);
    const char* Vg = (const char*)((const bf16_t*)p.v + (k0 * p.H + h) * D);
    char* DKg = (char*)((bf16_t*)p.dk + (k0 * p.H + h) * D);
    char* DVg = (char*)((bf16_t*)p.dv + (k0 * p.H + h) * D);

    char* ldsQ = smem;
    char* ldsDO = smem + SM::Q_BYTES;
    char* pbase = smem + 2 * SM::Q_BYTES + pair * SM::PAIR_BYTES;
    char* ldsK = pbase;
    char* ldsV = pbase + SM::TILE_BYTES;
    char* ldsP = pbase + 2 * SM::TILE_BYTES;
    char* ldsDS = ldsP + SM::P_BYTES;

    // ---- prologue: Q and dO of the item into LDS (rows past nq read as zero: they add nothing
    // to dK, dV and their dQ rows are never stored)
    {
        const __amdgpu_buffer_rsrc_t qr = __builtin_amdgcn_make_buffer_rsrc((void*)Qg, 0, (nq - 1) * (int)row_bytes + D * 2, 0x00020000);
        const __amdgpu_buffer_rsrc_t dr = __builtin_amdgcn_make_buffer_rsrc((void*)DOg, 0, (nq - 1) * (int)row_bytes + D * 2, 0x00020000);
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // 64 rows x 16 chunks over 256 threads
            const int row = i * 16 + (tid >> 4), ch = tid & 15;
            const u32x4 qv = __builtin_amdgcn_raw_buffer_load_b128(qr, (uint32_t)row * row_bytes + ch * 16, 0, 0);
            const u32x4 dv = __builtin_amdgcn_raw_buffer_load_b128(dr, (uint32_t)row * row_bytes + ch * 16, 0, 0);
            *(u32x4*)(ldsQ + L::u_offset(row, ch * 16)) = qv;
            *(u32x4*)(ldsDO + L::u_offset(row, ch * 16)) = dv;
        }
    }
    // softmax statistics of this lane's query (block w): lse in log2 units, delta = <dO, O>
    float lse2 = INFINITY, delta = 0.f;
    if (SOFTMAX) {
        const bf16_t* Og = (const bf16_t*)p.o + q_row0 * hd + (int64_t)h * D;
        const int qi = 32 * w + r;
        if (qi < nq) {
            lse2 = p.lse[(int64_t)h * p.total_q + q_row0 + qi] * LOG2E_P;
            float acc = 0.f;
            for (int c = 0; c < D / 16; ++c) {  // this lane half covers channels g*64 ..
                const bf16x8 a = *(const bf16x8*)(DOg + qi * hd + g * (D / 2) + c * 8);
                const bf16x8 b = *(const bf16x8*)(Og + qi * hd + g * (D / 2) + c * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)b[e], acc);
            }
            delta = acc;
        }
        delta = halves_sum(delta);
    }
    __syncthreads();

    // ---- everything that depends only on the lane (LDS byte offsets)
    const int s16 = lane & 15, hi16 = (lane >> 4) & 1;
    // All swizzles are XORs on the 16-byte chunk index, so "the same place, kc / db / vg chunks
    // further" is one XOR with a constant: one base offset per access pattern is kept.
    const int rr0 = L::u_offset(r, g * 16);  // row fragment: row r, channels 16*kc + 8g ..  -> rr0 ^ (kc << 5)
    // Q_w^T fragments (B operand of S^T) stay in registers; dO_w^T fragments are re-read per tile
    // (both resident would not fit 256 registers)
    bf16x8 qf[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
        qf[kc] = *(const bf16x8*)(ldsQ + w * 32 * L::ROW_BYTES + (rr0 ^ (kc << 5)));
    }
    const int colb = (16 * hi16 + 4 * (s16 & 3)) * 2;  // transposing reads: 4 rows x 16 columns per 16 lanes
    const int ktA = L::u_offset(4 * g + (s16 >> 2), colb);       // K^T: keys 16c + 4g + 0..3, channel block db -> ^ (db << 6)
    const int ktB = L::u_offset(8 + 4 * g + (s16 >> 2), colb);   //      keys 16c + 8 + 4g + 0..3
    const int qtA = L::u_offset(8 * g + (s16 >> 2), colb + 128 * w);      // Q^T, dO^T: queries 16j + 8g + 0..3, half w
    const int qtB = L::u_offset(8 * g + 4 + (s16 >> 2), colb + 128 * w);  //            queries 16j + 8g + 4..7
    const int ptA = pp_offset(8 * g + (s16 >> 2), colb);
    const int ptB = pp_offset(8 * g + 4 + (s16 >> 2), colb);
    const int pw0 = pp_offset(32 * w + r, 8 * g);  // P / dS writes: query 32*w + r, keys 8*vg + 4g ..  -> ^ (vg << 4)
    // K/V tile traffic of the pair: 128 threads, 4 chunks of 16 bytes each per tensor
    const int lrow = ptid >> 4, lch = ptid & 15;   // rows lrow + 8*i
    const uint32_t goff = (uint32_t)lrow * row_bytes + lch * 16;
    int uw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) uw[i] = L::u_offset(lrow + 8 * i, lch * 16);
    const int st_w = L::u_offset(r, 8 * w * 16 + 8 * g);  // staging write: key r, first chunk of channel half w
    auto tr_read = [](const char* a, const char* b) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, b));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    f32x16 dqacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) dqacc[db][v] = 0.f;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float sc = SOFTMAX ? p.scale * LOG2E_P : p.scale;

    const int n_tiles = (n_kv + KT - 1) / KT;
    const int n_iter = (n_tiles + 1) / 2;  // both pairs run the same number of rounds (barriers are workgroup-wide)
    u32x4 kst[4], vst[4];
    auto fetch = [&](int kt) {
        if (kt < n_tiles) {
            const int rows = (n_kv - kt * KT) < KT ? (n_kv - kt * KT) : KT;
            const int bytes = (rows - 1) * (int)row_bytes + D * 2;
            const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc((void*)(Kg + kt * tile_bytes), 0, bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc((void*)(Vg + kt * tile_bytes), 0, bytes, 0x00020000);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kst[i] = __builtin_amdgcn_raw_buffer_load_b128(kr, goff, 8 * i * row_bytes, 2);
                vst[i] = __builtin_amdgcn_raw_buffer_load_b128(vr, goff, 8 * i * row_bytes, 2);
            }
        }
    };
    fetch(pair);
    if (pair < n_tiles) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(u32x4*)(ldsK + uw[i]) = kst[i];
            *(u32x4*)(ldsV + uw[i]) = vst[i];
        }
    }
    for (int it = 0; it < n_iter; ++it) {
        const int kt = 2 * it + pair;
        const bool active = kt < n_tiles;
        __syncthreads();  // (1) K/V tiles complete
        fetch(kt + 2);
        bf16x8 dsf[2];
        if (active) {
            // ---- S^T = K Q_w^T and dP^T = V dO_w^T
            f32x16 sacc, dpacc;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                const bf16x8 ka = *(const bf16x8*)(ldsK + (rr0 ^ (kc << 5)));
                const bf16x8 va = *(const bf16x8*)(ldsV + (rr0 ^ (kc << 5)));
                sacc = mfma32(ka, qf[kc], kc == 0 ? zero16 : sacc);
                dpacc = mfma32(va, *(const bf16x8*)(ldsDO + w * 32 * L::ROW_BYTES + (rr0 ^ (kc << 5))), kc == 0 ? zero16 : dpacc);
            }
            // ---- P_w^T, dS_w^T in registers; bf16 copies to the pair's P / dS tiles
            const int key_base = kt * KT;
            const unsigned keys_left = (unsigned)(n_kv - key_base - 4 * g);
            float pv[16], dsv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float s = sacc[v] * sc;
                float val, der;
                if (SOFTMAX) {
                    val = fast_exp2(s - lse2);
                    dsv[v] = val * (dpacc[v] - delta) * p.scale;
                } else {
                    act_fast_vd<ACT>(s, val, der);
                    dsv[v] = dpacc[v] * der * p.scale;
                }
                pv[v] = val;
            }
            if (key_base + KT > n_kv) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const bool ok = (unsigned)(8 * (v >> 2) + (v & 3)) < keys_left;
                    pv[v] = ok ? pv[v] : 0.f;
                    dsv[v] = ok ? dsv[v] : 0.f;
                }
            }
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e) dsf[c][e] = (bf16_t)dsv[8 * c + e];
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                bf16x4 pk, dk4;
#pragma unroll
                for (int e = 0; e < 4; ++e) { pk[e] = (bf16_t)pv[4 * vg + e]; dk4[e] = (bf16_t)dsv[4 * vg + e]; }
                *(bf16x4*)(ldsP + (pw0 ^ (vg << 4))) = pk;
                *(bf16x4*)(ldsDS + (pw0 ^ (vg << 4))) = dk4;
            }
            // ---- dQ_w^T += K^T dS_w^T
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 a = tr_read(ldsK + c * 16 * L::ROW_BYTES + (ktA ^ (db << 6)), ldsK + c * 16 * L::ROW_BYTES + (ktB ^ (db << 6)));
                    dqacc[db] = mfma32(a, dsf[c], dqacc[db]);
                }
        }
        __syncthreads();  // (2) P and dS of both query blocks are in LDS; K and V tiles are dead
        if (active) {
            // ---- dV^T = dO^T P and dK^T = Q^T dS for channel half w, over all 64 queries
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                const char* src = which == 0 ? ldsDO : ldsQ;
                const char* wt = which == 0 ? ldsP : ldsDS;
                char* stage = which == 0 ? ldsV : ldsK;
                bf16x8 bfrag[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) bfrag[j] = tr_read(wt + j * 16 * 64 + ptA, wt + j * 16 * 64 + ptB);
#pragma unroll
                for (int d2 = 0; d2 < 2; ++d2) {
                    f32x16 acc;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const bf16x8 a = tr_read(src + j * 16 * L::ROW_BYTES + (qtA ^ (d2 << 6)), src + j * 16 * L::ROW_BYTES + (qtB ^ (d2 << 6)));
                        acc = mfma32(a, bfrag[j], j == 0 ? zero16 : acc);
                    }
                    // lane: key r, channels 32*(2w + d2) + 8*vg + 4g + 0..3  -> staging tile (same swizzle as the K/V tiles)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        bf16x4 out;
#pragma unroll
                        for (int e = 0; e < 4; ++e) out[e] = (bf16_t)acc[4 * vg + e];
                        *(bf16x4*)(stage + (st_w ^ ((4 * d2 + vg) << 4))) = out;
                    }
                }
            }
        }
        __syncthreads();  // (3) both channel halves of dV^T and dK^T are staged
        if (active) {
            const int key_base = kt * KT;
            const int rows = (n_kv - key_base) < KT ? (n_kv - key_base) : KT;
            const int out_bytes = (rows - 1) * (int)row_bytes + D * 2;
            const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc((void*)(DVg + key_base * (int64_t)row_bytes), 0, out_bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc((void*)(DKg + key_base * (int64_t)row_bytes), 0, out_bytes, 0x00020000);
            // Whole rows, 16 bytes per lane; rows past the history are dropped.  A thread stores exactly the staging
            // chunks that it fills with the next K/V tile, so the tile goes into LDS right here, behind the read of
            // the chunk (LDS serves a wave in order) and without a barrier.  The order matters for more than the
            // barrier: a wait for the tile's loads also waits for every older memory operation, and at this point the
            // next older ones are the stores of the previous round, long complete - whereas after this round's
            // stores it would expose their whole write latency in every round.
            const bool next = kt + 2 < n_tiles;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 dvv = *(const u32x4*)(ldsV + uw[i]);
                const u32x4 dkv = *(const u32x4*)(ldsK + uw[i]);
                if (next) {
                    *(u32x4*)(ldsV + uw[i]) = vst[i];
                    *(u32x4*)(ldsK + uw[i]) = kst[i];
                }
                __builtin_amdgcn_raw_buffer_store_b128(dvv, vr, goff, 8 * i * row_bytes, 2);
                __builtin_amdgcn_raw_buffer_store_b128(dkv, kr, goff, 8 * i * row_bytes, 2);
            }
        }
    }

    // ---- dQ: wave (pair, w) holds the partial sum of query block w over its pair's tiles
    __syncthreads();
    {
        char* mine = smem + pair * (64 * D * 4);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                f32x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = dqacc[db][4 * vg + e];
                *(f32x4*)(mine + pr_offset(32 * w + r, (32 * db + 8 * vg + 4 * g) / 4)) = x;
            }
    }
    __syncthreads();
    bf16_t* DQg = (bf16_t*)p.dq + q_row0 * hd + (int64_t)h * D;
    for (int idx = tid; idx < 64 * (D / 8); idx += 256) {
        const int row = idx / (D / 8), c8 = idx % (D / 8);
        if (row >= nq) continue;
        f32x4 lo = *(const f32x4*)(smem + pr_offset(row, 2 * c8));
        f32x4 hi = *(const f32x4*)(smem + pr_offset(row, 2 * c8 + 1));
        lo += *(const f32x4*)(smem + 64 * D * 4 + pr_offset(row, 2 * c8));
        hi += *(const f32x4*)(smem + 64 * D * 4 + pr_offset(row, 2 * c8 + 1));
        bf16x8 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) { out[e] = (bf16_t)lo[e]; out[4 + e] = (bf16_t)hi[e]; }
        *(bf16x8*)(DQg + row * hd + c8 * 8) = out;
    }
}

// Work items = (example, head), examples in scheduler order (longest history first), all heads of eight examples
// before the next eight.  With a work counter (p.queue; launches with more items than resident workgroups) the
// launch is persistent: two workgroups per compute unit, each starts with the item of its index and then takes
// the next unclaimed one - the same longest-first list scheduling as the hardware dispatcher performs on a grid
// of one workgroup per item, without its cost: measured on the jagged benchmark batch, the dispatcher kept only
// 60-90 % of the workgroup slots occupied once the items became short.  The counter is asked for the next item
// while the current one starts, so its round trip is never waited for.
__global__ __launch_bounds__(256, 2) void gdpa_bwd_pair_kernel(AttnParams p, int n_items) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int D = 128;
    // hand-over word for the next item: the last word of the second pair's dS tile, dead between items
    volatile int* const next_word = (volatile int*)(smem + PairSmem::TOTAL - 4);
    int item = blockIdx.x;
    while (item < n_items) {
        int claimed = 0;
        if (p.queue && threadIdx.x == 0) claimed = atomicAdd(p.queue, 1);
        const int slot = item & 7;
        const int64_t j = item >> 3;
        const int h = (int)(j % p.H);
        const int64_t e = (j / p.H) * 8 + slot;
        if (e < p.B) {
            const int b = p.order ? p.order[e] : (int)e;
            const int64_t q0 = q_begin(p, b);
            const int nq = (int)(q_end(p, b) - q0);
            const int64_t k0 = p.kv_off[b];
            const int n_kv = p.kv_off[b + 1] - (int)k0;
            if (nq <= 0) {  // no query sees these keys: their gradients are zero
                const int64_t hd = (int64_t)p.H * D;
                const u32x4 z = {0, 0, 0, 0};
                for (int idx = threadIdx.x; idx < n_kv * (D / 8); idx += 256) {
                    const int row = idx / (D / 8), c8 = idx % (D / 8);
                    *(u32x4*)((bf16_t*)p.dk + (k0 + row) * hd + (int64_t)h * D + c8 * 8) = z;
                    *(u32x4*)((bf16_t*)p.dv + (k0 + row) * hd + (int64_t)h * D + c8 * 8) = z;
                }
            } else {
                switch (p.head_act[h]) {
                case KUNLUN_ACT_SOFTMAX: attn_bwd_pair_item<KUNLUN_ACT_SOFTMAX>(p, smem, h, q0, nq, k0, n_kv); break;
                case KUNLUN_ACT_IDENTITY: attn_bwd_pair_item<KUNLUN_ACT_IDENTITY>(p, smem, h, q0, nq, k0, n_kv); break;
                case KUNLUN_ACT_RELU: attn_bwd_pair_item<KUNLUN_ACT_RELU>(p, smem, h, q0, nq, k0, n_kv); break;
                case KUNLUN_ACT_GELU: attn_bwd_pair_item<KUNLUN_ACT_GELU>(p, smem, h, q0, nq, k0, n_kv); break;
                case KUNLUN_ACT_GELU_TANH: attn_bwd_pair_item<KUNLUN_ACT_GELU_TANH>(p, smem, h, q0, nq, k0, n_kv); break;
                case KUNLUN_ACT_SILU: attn_bwd_pair_item<KUNLUN_ACT_SILU>(p, smem, h, q0, nq, k0, n_kv); break;
                default: attn_bwd_pair_item<KUNLUN_ACT_GELU_POLY>(p, smem, h, q0, nq, k0, n_kv); break;
                }
            }
        }
        if (!p.queue) break;
        __syncthreads();  // the item's last LDS reads (dQ sums) are done
        if (threadIdx.x == 0) *next_word = claimed + (int)gridDim.x;
        __syncthreads();
        item = __builtin_amdgcn_readfirstlane(*next_word);  // (next written in the first round of the next item, behind its barriers)
    }
}

hipError_t launch_mfma_bwd_pair(const AttnParams& p, hipStream_t stream) {
    constexpr int bytes = PairSmem::TOTAL;
    // once per process (initialisation of a function-local static is thread-safe); not a stream operation,
    // so a later call under graph capture launches only kernels
    static const hipError_t raised =
        hipFuncSetAttribute((const void*)gdpa_bwd_pair_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (raised != hipSuccess) return raised;
    const int64_t n_items = (((int64_t)p.B + 7) / 8) * 8 * p.H;
    const int64_t resident = 2 * (int64_t)compute_units();
    const unsigned grid = (unsigned)(p.queue && n_items > resident ? resident : n_items);
    hipLaunchKernelGGL(gdpa_bwd_pair_kernel, dim3(grid), dim3(256), bytes, stream, p, (int)n_items);
    return hipGetLastError();
}

}  // namespace kunlun
