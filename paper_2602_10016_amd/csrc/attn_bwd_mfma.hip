// bf16 matrix-core backward kernel for GDPA / softmax attention over jagged keys (gfx950):
// dQ, dK, dV of <O, dO>.  Scores are recomputed tile by tile; nothing of score size is ever
// stored (the block-wise backward of Sec. "Efficient Attention-Style Implementation").
//
// One workgroup of NW wavefronts = one work item = (example, head) with up to 32*NQB queries.
// Q and dO of the item stay in LDS (shared by the waves); the waves take the 32-key tiles of
// the history round-robin and never synchronise inside the key loop.  Per tile, per wave:
//     S^T  = K Q^T            dP^T = V dO^T                       (MFMA, keys x queries)
//     P^T  = f(S^T scale)     dS^T = dP^T * f'(S^T scale) * scale (registers; softmax:
//                                                  P = exp(s - lse), dS = P (dP - delta) scale)
//     dQ^T += K^T dS^T        (MFMA; dS^T straight from registers, K^T by transposing LDS reads)
//     dV^T  = dO^T P          dK^T = Q^T dS    (MFMA; P, dS go through a small LDS tile to change
//                                               from query-per-lane to key-per-lane layout)
// dK^T / dV^T tiles are transposed through LDS and written as whole rows.  dQ partial sums of
// the NW waves are added in LDS at the end of the item, in a fixed order (bit-reproducible).
#include "mfma_tile.h"

namespace kunlun {

constexpr float LOG2E_B = 1.4426950408889634f;

template <int D, int NQB, int NW>
struct BwdSmem {
    static constexpr int QROWS = 32 * NQB;
    static constexpr int Q_BYTES = QROWS * D * 2;
    static constexpr int TILE_BYTES = KT * D * 2;
    static constexpr int P_BYTES = QROWS * KT * 2;  // [query][key] bf16, 64 bytes per row
    static constexpr int WAVE_BYTES = 2 * TILE_BYTES + 2 * P_BYTES;
    static constexpr int TOTAL = 2 * Q_BYTES + NW * WAVE_BYTES;
    static constexpr int REDUCE_BYTES = NW * QROWS * D * 4;
    static_assert(REDUCE_BYTES <= TOTAL, "dQ reduction scratch must fit in the tile memory");
};

// P / dS tile: row = query, 4 chunks of 16 bytes (8 keys) per row, chunk index swizzled by the row.
__device__ __forceinline__ int p_offset(int row, int byte_in_row) {
    return row * 64 + ((((byte_in_row >> 4) ^ (row >> 2)) & 3) << 4) + (byte_in_row & 15);
}

// fp32 [query][channel] scratch of the dQ reduction: 16-byte chunks swizzled by the row.
template <int D>
__device__ __forceinline__ int r_offset(int row, int chunk) {
    return row * D * 4 + ((chunk ^ (row & (D / 4 - 1))) << 4);
}

template <int D, int NQB, int NW, int ACT>
__device__ __forceinline__ void attn_bwd_item(const AttnParams& p, char* smem, int h, int64_t q_row0, int nq,
                                              int64_t k0, int n_kv) {
    using L = TileLayout<D>;
    using SM = BwdSmem<D, NQB, NW>;
    constexpr bool SOFTMAX = ACT == KUNLUN_ACT_SOFTMAX;
    constexpr int KC = D / 16;
    constexpr int DB = D / 32;
    constexpr int QROWS = SM::QROWS;
    constexpr int QCH = QROWS / 16;  // 16-query contraction chunks
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, g = lane >> 5;
    const int64_t hd = (int64_t)p.H * D;
    const bf16_t* Qg = (const bf16_t*)p.q + q_src_row(p, q_row0) * hd + (int64_t)h * D;
    const bf16_t* DOg = (const bf16_t*)p.d_o + q_row0 * hd + (int64_t)h * D;
    const bf16_t* Kg = (const bf16_t*)p.k + (k0 * p.H + h) * D;
    const bf16_t* Vg = (const bf16_t*)p.v + (k0 * p.H + h) * D;
    bf16_t* DKg = (bf16_t*)p.dk + (k0 * p.H + h) * D;
    bf16_t* DVg = (bf16_t*)p.dv + (k0 * p.H + h) * D;

    char* ldsQ = smem;
    char* ldsDO = smem + SM::Q_BYTES;
    char* wbase = smem + 2 * SM::Q_BYTES + wave * SM::WAVE_BYTES;
    char* ldsK = wbase;
    char* ldsV = wbase + SM::TILE_BYTES;
    char* ldsP = wbase + 2 * SM::TILE_BYTES;
    char* ldsDS = ldsP + SM::P_BYTES;

    // ---- prologue: Q and dO of the item into LDS; rows past nq are zero (they then add
    // nothing to dK, dV, and their dQ rows are never stored)
    for (int idx = tid; idx < QROWS * L::CHUNKS; idx += 64 * NW) {
        const int row = idx / L::CHUNKS, ch = idx % L::CHUNKS;
        u32x4 qv = {0, 0, 0, 0}, dv = {0, 0, 0, 0};
        if (row < nq) {
            qv = *(const u32x4*)(Qg + row * hd + ch * 8);
            dv = *(const u32x4*)(DOg + row * hd + ch * 8);
        }
        *(u32x4*)(ldsQ + L::u_offset(row, ch * 16)) = qv;
        *(u32x4*)(ldsDO + L::u_offset(row, ch * 16)) = dv;
    }
    // softmax statistics of this lane's query columns: lse (log2 units) and delta = <dO, O>
    float lse2[NQB], delta[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) { lse2[qb] = 0.f; delta[qb] = 0.f; }
    if (SOFTMAX) {
        const bf16_t* Og = (const bf16_t*)p.o + q_row0 * hd + (int64_t)h * D;
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            const int qi = 32 * qb + r;
            if (qi < nq) {
                lse2[qb] = p.lse[(int64_t)h * p.total_q + q_row0 + qi] * LOG2E_B;
                float acc = 0.f;
                for (int c = 0; c < D / 16; ++c) {  // this lane half covers channels g*D/2 ..
                    const bf16x8 a = *(const bf16x8*)(DOg + qi * hd + g * (D / 2) + c * 8);
                    const bf16x8 b = *(const bf16x8*)(Og + qi * hd + g * (D / 2) + c * 8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)b[e], acc);
                }
                delta[qb] = acc;
            } else {
                lse2[qb] = INFINITY;  // weight exp2(s - inf) = 0
            }
            delta[qb] = halves_sum(delta[qb]);
        }
    }
    if (NW > 1) __syncthreads();
    else __builtin_amdgcn_s_waitcnt(0);

    f32x16 dqacc[DB][NQB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) dqacc[db][qb][v] = 0.f;

    const int n_tiles = (n_kv + KT - 1) / KT;
    const float sc = SOFTMAX ? p.scale * LOG2E_B : p.scale;
    const uint32_t row_bytes = (uint32_t)(hd * 2);
    const int64_t tile_bytes = (int64_t)KT * row_bytes;

    // ---- everything that depends only on the lane, computed once per item (LDS byte offsets;
    // "A"/"B" = the two transposing reads of one 8-element fragment)
    const int s16 = lane & 15, hi16 = (lane >> 4) & 1;
    const int chunk = lane % L::CHUNKS, rsub = lane / L::CHUNKS;
    const uint32_t goff = (uint32_t)rsub * row_bytes + chunk * 16;  // this lane's chunk in a global tile
    int uw[L::LOADS];   // the same chunk in a swizzled LDS tile, per load
#pragma unroll
    for (int i = 0; i < L::LOADS; ++i) uw[i] = L::u_offset(i * L::ROWS_PER_LOAD + rsub, chunk * 16);
    int rr[KC];         // row fragment (row r, channels 16*kc + 8g ..); rows r + 32*qb add a constant
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) rr[kc] = L::u_offset(r, (2 * kc + g) * 16);
    int ktA[DB], ktB[DB], qtA[DB], qtB[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        const int colb = (32 * db + 16 * hi16 + 4 * (s16 & 3)) * 2;
        ktA[db] = L::u_offset(4 * g + (s16 >> 2), colb);          // K^T: keys 16c + 4g + 0..3 (+ 16c rows)
        ktB[db] = L::u_offset(8 + 4 * g + (s16 >> 2), colb);      //      keys 16c + 8 + 4g + 0..3
        qtA[db] = L::u_offset(8 * g + (s16 >> 2), colb);          // Q^T, dO^T: queries 16j + 8g + 0..3
        qtB[db] = L::u_offset(8 * g + 4 + (s16 >> 2), colb);      //            queries 16j + 8g + 4..7
    }
    const int ptA = p_offset(8 * g + (s16 >> 2), (16 * hi16 + 4 * (s16 & 3)) * 2);  // P, dS: like Q^T
    const int ptB = p_offset(8 * g + 4 + (s16 >> 2), (16 * hi16 + 4 * (s16 & 3)) * 2);
    int pw[4];          // P / dS writes: query r (+ 32*qb rows), keys 8*vg + 4g ..
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) pw[vg] = p_offset(r, (8 * vg + 4 * g) * 2);
    // dK^T / dV^T staging: padded rows (2D + 16 bytes) over the dead K and V tiles
    constexpr int ST_STRIDE = 2 * D + 16;
    static_assert(KT * ST_STRIDE <= 2 * SM::TILE_BYTES, "staging must fit the K and V tiles");
    const int st_w = r * ST_STRIDE + 8 * g;
    const int st_r = rsub * ST_STRIDE + chunk * 16;
    auto tr_read = [](const char* a, const char* b) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, b));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // K/V tile loads: buffer resource over the valid rows of the tile (rows past the end of the
    // history read as zero), non-temporal
    auto fetch = [&](u32x4 (&ks)[L::LOADS], u32x4 (&vs)[L::LOADS], int kt) {
        const int rows = (n_kv - kt * KT) < KT ? (n_kv - kt * KT) : KT;
        const int bytes = (rows - 1) * (int)row_bytes + D * 2;
        const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)Kg + kt * tile_bytes), 0, bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)Vg + kt * tile_bytes), 0, bytes, 0x00020000);
#pragma unroll
        for (int i = 0; i < L::LOADS; ++i) {
            // (streaming loads, except at D = 32: a row piece is then half a 128-byte line, which a streaming load
            // fetches whole for one use)
            ks[i] = __builtin_amdgcn_raw_buffer_load_b128(kr, goff, i * L::ROWS_PER_LOAD * row_bytes, D != 32 ? 2 : 0);
            vs[i] = __builtin_amdgcn_raw_buffer_load_b128(vr, goff, i * L::ROWS_PER_LOAD * row_bytes, D != 32 ? 2 : 0);
        }
    };
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    u32x4 kst[L::LOADS], vst[L::LOADS];
    if (wave < n_tiles) fetch(kst, vst, wave);
    for (int kt = wave; kt < n_tiles; kt += NW) {
#pragma unroll
        for (int i = 0; i < L::LOADS; ++i) {
            *(u32x4*)(ldsK + uw[i]) = kst[i];
            *(u32x4*)(ldsV + uw[i]) = vst[i];
        }
        if (kt + NW < n_tiles) fetch(kst, vst, kt + NW);
        // ---- S^T = K Q^T and dP^T = V dO^T
        f32x16 sacc[NQB], dpacc[NQB];
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            const bf16x8 ka = *(const bf16x8*)(ldsK + rr[kc]);
            const bf16x8 va = *(const bf16x8*)(ldsV + rr[kc]);
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                const bf16x8 qf = *(const bf16x8*)(ldsQ + qb * 32 * L::ROW_BYTES + rr[kc]);
                const bf16x8 df = *(const bf16x8*)(ldsDO + qb * 32 * L::ROW_BYTES + rr[kc]);
                sacc[qb] = mfma32(ka, qf, kc == 0 ? zero16 : sacc[qb]);
                dpacc[qb] = mfma32(va, df, kc == 0 ? zero16 : dpacc[qb]);
            }
        }
        // ---- P^T, dS^T in registers; bf16 copies to the P / dS tiles ([query][key])
        const int key_base = kt * KT;
        const bool need_mask = key_base + KT > n_kv;
        const unsigned keys_left = (unsigned)(n_kv - key_base - 4 * g);  // key 8*(v/4) + (v%4) + 4g < n_kv - key_base
        bf16x8 dsf[NQB][2];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            float pv[16], dsv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float s = sacc[qb][v] * sc;
                float val, der;
                if (SOFTMAX) {
                    val = fast_exp2(s - lse2[qb]);
                    dsv[v] = val * (dpacc[qb][v] - delta[qb]) * p.scale;
                } else {
                    act_fast_vd<ACT>(s, val, der);
                    dsv[v] = dpacc[qb][v] * der * p.scale;
                }
                pv[v] = val;
            }
            if (need_mask) {
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
                for (int e = 0; e < 8; ++e) dsf[qb][c][e] = (bf16_t)dsv[8 * c + e];
            // registers 4*vg .. 4*vg+3 hold keys 8*vg + 4g + 0..3 of query 32*qb + r
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                bf16x4 pk, dk4;
#pragma unroll
                for (int e = 0; e < 4; ++e) { pk[e] = (bf16_t)pv[4 * vg + e]; dk4[e] = (bf16_t)dsv[4 * vg + e]; }
                *(bf16x4*)(ldsP + qb * 32 * 64 + pw[vg]) = pk;
                *(bf16x4*)(ldsDS + qb * 32 * 64 + pw[vg]) = dk4;
            }
        }
        // ---- dQ^T += K^T dS^T  (keys in the register order of the C layout)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const bf16x8 a = tr_read(ldsK + c * 16 * L::ROW_BYTES + ktA[db], ldsK + c * 16 * L::ROW_BYTES + ktB[db]);
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) dqacc[db][qb] = mfma32(a, dsf[qb][c], dqacc[db][qb]);
            }
        }
        // ---- dV^T = dO^T P and dK^T = Q^T dS (contraction over queries, natural order)
        bf16x8 pb[QCH], dsb[QCH];
#pragma unroll
        for (int j = 0; j < QCH; ++j) {
            pb[j] = tr_read(ldsP + j * 16 * 64 + ptA, ldsP + j * 16 * 64 + ptB);
            dsb[j] = tr_read(ldsDS + j * 16 * 64 + ptA, ldsDS + j * 16 * 64 + ptB);
        }
        const int rows = (n_kv - key_base) < KT ? (n_kv - key_base) : KT;
        const int out_bytes = (rows - 1) * (int)row_bytes + D * 2;
        char* stage = ldsK;  // K and V tiles are dead from here on
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const char* src = which == 0 ? ldsDO : ldsQ;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                f32x16 acc;
#pragma unroll
                for (int j = 0; j < QCH; ++j) {
                    const bf16x8 a = tr_read(src + j * 16 * L::ROW_BYTES + qtA[db], src + j * 16 * L::ROW_BYTES + qtB[db]);
                    acc = mfma32(a, which == 0 ? pb[j] : dsb[j], j == 0 ? zero16 : acc);
                }
                // lane: key r, channels 32*db + 8*vg + 4g + 0..3
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    bf16x4 out;
#pragma unroll
                    for (int e = 0; e < 4; ++e) out[e] = (bf16_t)acc[4 * vg + e];
                    *(bf16x4*)(stage + st_w + (32 * db + 8 * vg) * 2) = out;
                }
            }
            // whole rows out, 16 bytes per lane; the buffer resource drops rows past the history
            char* dst = (char*)(which == 0 ? DVg : DKg) + key_base * (int64_t)row_bytes;
            const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc((void*)dst, 0, out_bytes, 0x00020000);
#pragma unroll
            for (int i = 0; i < L::LOADS; ++i) {
                const u32x4 val = *(const u32x4*)(stage + st_r + i * L::ROWS_PER_LOAD * ST_STRIDE);
                __builtin_amdgcn_raw_buffer_store_b128(val, orsrc, goff, i * L::ROWS_PER_LOAD * row_bytes, 2);
            }
        }
    }

    // ---- dQ: add the partial sums of the waves in LDS, write rows as bf16
    if (NW > 1) __syncthreads();
    char* red = smem;
    {
        char* mine = red + wave * (QROWS * D * 4);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = dqacc[db][qb][4 * vg + e];
                    const int chunk = (32 * db + 8 * vg + 4 * g) / 4;
                    *(f32x4*)(mine + r_offset<D>(32 * qb + r, chunk)) = x;
                }
    }
    if (NW > 1) __syncthreads();
    else __builtin_amdgcn_s_waitcnt(0);
    bf16_t* DQg = (bf16_t*)p.dq + q_row0 * hd + (int64_t)h * D;
    for (int idx = tid; idx < QROWS * (D / 8); idx += 64 * NW) {
        const int row = idx / (D / 8), c8 = idx % (D / 8);
        if (row >= nq) continue;
        f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const char* part = red + w * (QROWS * D * 4);
            lo += *(const f32x4*)(part + r_offset<D>(row, 2 * c8));
            hi += *(const f32x4*)(part + r_offset<D>(row, 2 * c8 + 1));
        }
        bf16x8 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) { out[e] = (bf16_t)lo[e]; out[4 + e] = (bf16_t)hi[e]; }
        *(bf16x8*)(DQg + row * hd + c8 * 8) = out;
    }
}

// one workgroup per (example, head), examples in scheduler order (longest history first).
template <int D, int NQB, int NW>
__global__ __launch_bounds__(64 * NW) void gdpa_bwd_mfma_kernel(AttnParams p) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // workgroup i runs on XCD i % 8: consecutive examples go to consecutive XCDs, and each
    // XCD walks through all heads of its examples (all L2 channels stay in use)
    const int xcd = blockIdx.x & 7;
    const int64_t j = blockIdx.x >> 3;
    const int h = (int)(j % p.H);
    const int64_t e = (j / p.H) * 8 + xcd;
    if (e >= p.B) return;
    const int b = p.order ? p.order[e] : (int)e;
    const int64_t q0 = q_begin(p, b);
    const int nq = (int)(q_end(p, b) - q0);
    const int64_t k0 = p.kv_off[b];
    const int n_kv = p.kv_off[b + 1] - (int)k0;
    if (nq <= 0) {
        // no query sees these keys: their gradients are zero
        const int64_t hd = (int64_t)p.H * D;
        const u32x4 z = {0, 0, 0, 0};
        for (int idx = threadIdx.x; idx < n_kv * (D / 8); idx += 64 * NW) {
            const int row = idx / (D / 8), c8 = idx % (D / 8);
            *(u32x4*)((bf16_t*)p.dk + (k0 + row) * hd + (int64_t)h * D + c8 * 8) = z;
            *(u32x4*)((bf16_t*)p.dv + (k0 + row) * hd + (int64_t)h * D + c8 * 8) = z;
        }
        return;
    }
    switch (p.head_act[h]) {
    case KUNLUN_ACT_SOFTMAX: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_SOFTMAX>(p, smem, h, q0, nq, k0, n_kv); break;
    case KUNLUN_ACT_IDENTITY: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_IDENTITY>(p, smem, h, q0, nq, k0, n_kv); break;
    case KUNLUN_ACT_RELU: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_RELU>(p, smem, h, q0, nq, k0, n_kv); break;
    case KUNLUN_ACT_GELU: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_GELU>(p, smem, h, q0, nq, k0, n_kv); break;
    case KUNLUN_ACT_GELU_TANH: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_GELU_TANH>(p, smem, h, q0, nq, k0, n_kv); break;
    case KUNLUN_ACT_SILU: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_SILU>(p, smem, h, q0, nq, k0, n_kv); break;
    default: attn_bwd_item<D, NQB, NW, KUNLUN_ACT_GELU_POLY>(p, smem, h, q0, nq, k0, n_kv); break;
    }
}

bool mfma_bwd_supported(const AttnParams& p, int dtype) {
    return dtype == KUNLUN_BF16 && (p.d == 32 || p.d == 64 || p.d == 128) && p.max_q >= 1 && p.max_q <= 64;
}

size_t mfma_bwd_workspace_tail(int, int, int, int, int64_t) { return 0; }

template <int D, int NQB, int NW>
static hipError_t launch_bwd(const AttnParams& p, hipStream_t stream) {
    constexpr int bytes = BwdSmem<D, NQB, NW>::TOTAL;
    auto kern = gdpa_bwd_mfma_kernel<D, NQB, NW>;
    if (bytes > 64 * 1024) {
        // raise the kernel's dynamic LDS limit once per process (initialisation of a function-local
        // static is thread-safe; not a stream operation, so a later call under graph capture
        // launches only kernels)
        static const hipError_t raised =
            hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (raised != hipSuccess) return raised;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)((((int64_t)p.B + 7) / 8) * 8 * p.H)), dim3(64 * NW), bytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_mfma_bwd(const AttnParams& p, void*, hipStream_t stream) {
    const bool one_block = p.max_q <= 32;
    if (p.d == 128) return one_block ? launch_bwd<128, 1, 4>(p, stream) : launch_mfma_bwd_pair(p, stream);
    if (p.d == 32) return one_block ? launch_bwd<32, 1, 4>(p, stream) : launch_bwd<32, 2, 4>(p, stream);
    // d = 64: two waves per (example, head) keep the LDS footprint small when there are many items;
    // with few items (less than about two per SIMD) the longest history sets the time, and four
    // waves walk it twice as fast
    const bool few_items = (int64_t)p.B * p.H <= 2048;
    if (few_items) return one_block ? launch_bwd<64, 1, 4>(p, stream) : launch_bwd<64, 2, 4>(p, stream);
    return one_block ? launch_bwd<64, 1, 2>(p, stream) : launch_bwd<64, 2, 2>(p, stream);
}

}  // namespace kunlun
