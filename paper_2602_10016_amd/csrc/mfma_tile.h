// Building blocks of the bf16 matrix-core kernels for gfx950 (CDNA4), wave64.
//
// Matrix instruction used throughout: v_mfma_f32_32x32x16_bf16, D(32x32) += A(32x16) B(16x32).
// Register layouts (lane l, r = l % 32, g = l / 32):
//   A operand: row r,    contraction indices 8g .. 8g+7   (8 bf16 = 4 VGPRs)
//   B operand: column r, contraction indices 8g .. 8g+7
//   D/C      : column r, rows 8*(v/4) + 4g + (v%4) for v = 0..15
// The kernels compute the TRANSPOSED score tile S^T = K Q^T (keys x queries), so that every
// lane owns one query column: the 16 scores a lane holds belong to one query, row-wise
// softmax statistics reduce inside a lane plus one exchange between the two lane halves,
// and the packed P^T registers are directly the B operand of O^T += V^T P^T (contraction
// over keys, in whatever key order the C layout has - the A operand V^T is read in the
// same order).  V^T fragments come from row-major V tiles in LDS through the gfx950
// transposing LDS read (ds_read_b64_tr_b16).
#pragma once
#include "common.h"

namespace kunlun {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int KT = 32;  // keys per tile

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// A 32-row tile of a [tokens, H, D] bf16 tensor, held row-major in LDS (D*2 bytes per row,
// no padding) with XOR swizzles that keep both access patterns free of bank conflicts.
template <int D>
struct TileLayout {
    static_assert(D == 32 || D == 64 || D == 128, "head dimensions of the matrix-core kernels");
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int TILE_BYTES = KT * ROW_BYTES;
    static constexpr int CHUNKS = D / 8;        // 16-byte chunks per row
    static constexpr int ROWS_PER_LOAD = 64 / CHUNKS;
    static constexpr int LOADS = KT / ROWS_PER_LOAD;  // 16-byte loads per lane per tile

    // K tiles: read as A operand (lane: row r, chunk 2*kc+g).  16 consecutive rows must hit
    // 16 different chunk positions.
    __device__ static __forceinline__ int k_offset(int row, int chunk) {
        const int x = (D == 128) ? (row & 15) : (D == 64) ? ((row >> 1) & 7) : ((row >> 2) & 3);
        return row * ROW_BYTES + ((chunk ^ x) << 4);
    }
    // V tiles: read with the transposing LDS read, 4 consecutive rows x 64 bytes per 32 lanes.
    // The four rows must sit in four different 64-byte bank groups (D = 32: a row IS 64 bytes).
    __device__ static __forceinline__ int v_offset(int row, int byte_in_row) {
        const int x = (D == 128) ? (row & 3) : (D == 64) ? ((row >> 1) & 1) : 0;
        return row * ROW_BYTES + ((((byte_in_row >> 6) ^ x)) << 6) + (byte_in_row & 63);
    }
    // Tiles that are read BOTH ways (backward pass: K, Q, dO): one swizzle that satisfies both
    // conditions above.  D = 128: chunk ^= 4*(row%4) + (row/4)%4;  D = 64: chunk ^= bit-reversed
    // (row/2)%8;  D = 32: chunk ^= (row/4)%4.
    __device__ static __forceinline__ int u_swizzle(int row) {
        if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
        if (D == 32) return (row >> 2) & 3;
        const int x = (row >> 1) & 7;
        return ((x & 1) << 2) | (x & 2) | ((x >> 2) & 1);
    }
    __device__ static __forceinline__ int u_offset(int row, int byte_in_row) {
        return row * ROW_BYTES + ((((byte_in_row >> 4) ^ u_swizzle(row))) << 4) + (byte_in_row & 15);
    }
};

// Global -> register staging of one 32-row tile: lane l fetches 16 bytes of row
// i*ROWS_PER_LOAD + l/CHUNKS, chunk l%CHUNKS, for i = 0..LOADS-1 (whole rows coalesced).
// Rows past `rows_valid` are clamped to the last valid row (their weights are masked to 0).
// Non-temporal: the rows are read once and by this wave only.
template <int D>
__device__ __forceinline__ void load_tile_regs(u32x4 (&st)[TileLayout<D>::LOADS], const bf16_t* __restrict__ base,
                                               int64_t row_stride, int rows_valid, int lane) {
    using L = TileLayout<D>;
    const int chunk = lane % L::CHUNKS;
    const int rsub = lane / L::CHUNKS;
#pragma unroll
    for (int i = 0; i < L::LOADS; ++i) {
        int row = i * L::ROWS_PER_LOAD + rsub;
        row = row < rows_valid ? row : rows_valid - 1;
        st[i] = __builtin_nontemporal_load((const u32x4*)(base + row * row_stride + chunk * 8));
    }
}

template <int D>
__device__ __forceinline__ void store_k_tile(char* lds, const u32x4 (&st)[TileLayout<D>::LOADS], int lane) {
    using L = TileLayout<D>;
    const int chunk = lane % L::CHUNKS;
    const int rsub = lane / L::CHUNKS;
#pragma unroll
    for (int i = 0; i < L::LOADS; ++i) {
        const int row = i * L::ROWS_PER_LOAD + rsub;
        *(u32x4*)(lds + L::k_offset(row, chunk)) = st[i];
    }
}

template <int D>
__device__ __forceinline__ void store_v_tile(char* lds, const u32x4 (&st)[TileLayout<D>::LOADS], int lane) {
    using L = TileLayout<D>;
    const int chunk = lane % L::CHUNKS;
    const int rsub = lane / L::CHUNKS;
#pragma unroll
    for (int i = 0; i < L::LOADS; ++i) {
        const int row = i * L::ROWS_PER_LOAD + rsub;
        *(u32x4*)(lds + L::v_offset(row, chunk * 16)) = st[i];
    }
}

// A operand from a K-layout tile: row r, contraction indices 16*kc + 8g .. +7.
template <int D>
__device__ __forceinline__ bf16x8 read_k_frag(const char* lds, int kc, int r, int g) {
    return *(const bf16x8*)(lds + TileLayout<D>::k_offset(r, 2 * kc + g));
}

// A operand V^T (row = channel 32*db + r, contraction over keys) for the 16 keys that the
// C layout of a score tile puts in registers 8c .. 8c+7:
//   elements 0..3 = keys 16c + 4g + 0..3, elements 4..7 = keys 16c + 8 + 4g + 0..3.
// Each half is one transposing read: the 16 lanes of a group address a 4 (keys) x 16
// (channels) block - lane s points at key s/4, channels 4*(s%4) .. +3 - and lane i receives
// channel i of the four keys.
template <int D>
__device__ __forceinline__ bf16x8 read_vt_frag(const char* lds, int db, int c, int lane) {
    const int g = lane >> 5;
    const int s = lane & 15;
    const int col = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int key0 = 16 * c + 4 * g + (s >> 2);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, lds + TileLayout<D>::v_offset(key0, col * 2)));
    const s16x4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, lds + TileLayout<D>::v_offset(key0 + 8, col * 2)));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// ---- the same accessors for tiles in the two-way ("u") swizzle ----
template <int D>
__device__ __forceinline__ void store_u_tile(char* lds, const u32x4 (&st)[TileLayout<D>::LOADS], int lane) {
    using L = TileLayout<D>;
    const int chunk = lane % L::CHUNKS;
    const int rsub = lane / L::CHUNKS;
#pragma unroll
    for (int i = 0; i < L::LOADS; ++i) {
        const int row = i * L::ROWS_PER_LOAD + rsub;
        *(u32x4*)(lds + L::u_offset(row, chunk * 16)) = st[i];
    }
}

// A (or B) operand: row `row`, contraction indices 16*kc + 8g .. +7 along the row.
template <int D>
__device__ __forceinline__ bf16x8 read_u_frag(const char* lds, int kc, int row, int g) {
    return *(const bf16x8*)(lds + TileLayout<D>::u_offset(row, (2 * kc + g) * 16));
}

// Transposed operand from a row-major tile: for this lane, column col0 + (lane%32) and the
// rows rowA .. rowA+3 (elements 0..3) and rowB .. rowB+3 (elements 4..7).  OFFSET(row, byte)
// gives the LDS byte offset of an element.  rowA, rowB must be multiples of 4.
template <typename OFFSET>
__device__ __forceinline__ bf16x8 read_tr_frag(const char* lds, OFFSET offset, int rowA, int rowB, int col0, int lane) {
    const int s = lane & 15;
    const int col = col0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, lds + offset(rowA + (s >> 2), col * 2)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, lds + offset(rowB + (s >> 2), col * 2)));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Value of x in the lane 32 further (or 32 back), paired with the lane's own: the gfx950
// half-wave swap is a VALU operation, where a shuffle would take an LDS round trip.
// Returns both values in an order that depends on the lane half; use for symmetric reductions.
__device__ __forceinline__ void both_halves(float x, float& a, float& b) {
    unsigned u = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // r[0] = {low half, low half}, r[1] = {high, high}
    unsigned r0 = r[0], r1 = r[1];
    a = __builtin_bit_cast(float, r0);
    b = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float halves_max(float x) { float a, b; both_halves(x, a, b); return fmaxf(a, b); }
__device__ __forceinline__ float halves_sum(float x) { float a, b; both_halves(x, a, b); return a + b; }

// Key index (inside a 32-key tile) of register v of the score C layout for lane half g.
__device__ __forceinline__ int c_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

// ---- fast score functions (bf16 path: results are rounded to bf16 right after) ----
// Hardware exp2 / rcp (about 1 ulp); everything else is plain ALU work, per the remark of
// App. "GDPA and Fused PFFN Kernel" that without softmax the transcendental unit becomes
// the bottleneck and should be relieved by ALU arithmetic.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Phi(-|x|) = 0.5 erfc(|x|/sqrt 2) through the rational-times-Gaussian form of Abramowitz &
// Stegun 7.1.26 (absolute error <= 1.5e-7 in erf, so <= 7.5e-8 in Phi; evaluating the lower
// tail directly avoids the cancellation of 1 - erf).  Also returns gauss = exp(-x^2/2).
__device__ __forceinline__ float phi_neg_abs(float x, float& gauss) {
    const float z = fabsf(x) * 0.70710678118654752f;
    const float t = fast_rcp(fmaf(0.3275911f, z, 1.f));
    gauss = fast_exp2(x * x * -0.72134752044448170f);  // exp(-x^2/2) = 2^(-x^2 log2(e)/2)
    float poly = fmaf(t, 1.061405429f, -1.453152027f);
    poly = fmaf(t, poly, 1.421413741f);
    poly = fmaf(t, poly, -0.284496736f);
    poly = fmaf(t, poly, 0.254829592f);
    return 0.5f * poly * t * gauss;
}

template <int ACT>
__device__ __forceinline__ float act_fast(float x) {
    if constexpr (ACT == KUNLUN_ACT_IDENTITY) return x;
    if constexpr (ACT == KUNLUN_ACT_RELU) return fmaxf(x, 0.f);
    if constexpr (ACT == KUNLUN_ACT_GELU) {
        float gauss;
        const float q = phi_neg_abs(x, gauss);
        return x * (x < 0.f ? q : 1.f - q);
    }
    if constexpr (ACT == KUNLUN_ACT_GELU_TANH) {
        // 0.5 x (1 + tanh u) = x / (1 + exp(-2u))
        const float u2 = x * fmaf(x * x, 0.044715f * 1.5957691216057308f, 1.5957691216057308f);
        return x * fast_rcp(1.f + fast_exp2(u2 * -1.4426950408889634f));
    }
    if constexpr (ACT == KUNLUN_ACT_SILU) return x * fast_rcp(1.f + fast_exp2(x * -1.4426950408889634f));
    if constexpr (ACT == KUNLUN_ACT_GELU_POLY) {
        float slope;  // (unused here: the compiler drops its arithmetic)
        return x * gelu_poly_cdf(x, slope);
    }
    return 0.f;
}

// value and derivative together (backward)
template <int ACT>
__device__ __forceinline__ void act_fast_vd(float x, float& val, float& der) {
    if constexpr (ACT == KUNLUN_ACT_IDENTITY) { val = x; der = 1.f; }
    if constexpr (ACT == KUNLUN_ACT_RELU) { val = fmaxf(x, 0.f); der = x > 0.f ? 1.f : 0.f; }
    if constexpr (ACT == KUNLUN_ACT_GELU) {
        float gauss;
        const float q = phi_neg_abs(x, gauss);
        const float cdf = x < 0.f ? q : 1.f - q;
        val = x * cdf;
        der = fmaf(x * 0.39894228040143268f, gauss, cdf);
    }
    if constexpr (ACT == KUNLUN_ACT_GELU_TANH) {
        const float x2 = x * x;
        const float u2 = x * fmaf(x2, 0.044715f * 1.5957691216057308f, 1.5957691216057308f);
        const float sg = fast_rcp(1.f + fast_exp2(u2 * -1.4426950408889634f));  // sigmoid(2u)
        const float du2 = fmaf(x2, 3.f * 0.044715f * 1.5957691216057308f, 1.5957691216057308f);
        val = x * sg;
        der = fmaf(x * sg * (1.f - sg), du2, sg);
    }
    if constexpr (ACT == KUNLUN_ACT_SILU) {
        const float sg = fast_rcp(1.f + fast_exp2(x * -1.4426950408889634f));
        val = x * sg;
        der = fmaf(x * sg, 1.f - sg, sg);
    }
    if constexpr (ACT == KUNLUN_ACT_GELU_POLY) {
        float slope;
        const float cdf = gelu_poly_cdf(x, slope);
        val = x * cdf;
        der = fmaf(x, slope, cdf);
    }
}

}  // namespace kunlun
