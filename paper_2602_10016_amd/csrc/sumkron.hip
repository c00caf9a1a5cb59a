// SumKronLinear, Eq. (SumKronLinear) of Sec. "Hierarchical Seed Pooling" (stage 3):
//     Y_b = sum_{i=1..k} Z_i^T X_b W_i ,   X_b [S, D], Z_i [S, T], W_i [D, D], Y_b [T, D].
// Unlike the attention operators this one is a dense contraction with weights shared by the
// whole batch (about 570 flop per byte of X at the paper's S=256, T=32, D=384, k=8): it belongs
// on the matrix cores.  It is evaluated as two GEMMs with a bf16 intermediate in the workspace:
//     stage 1, per example:  U_b [T, k*D]  with  U_b[t, i*D + c] = sum_s Z_i[s, t] X_b[s, c]
//                            = rows (i, t) of  Zt [k*T, S] * X_b [S, D],  Zt = all Z_i transposed
//     stage 2, whole batch:  Y [B*T, D] = U [B*T, k*D] * Wcat [k*D, D],   Wcat = the W_i stacked
// Both run the same kernel: C = A * B for row-major bf16 operands, fp32 accumulation,
// 256 x 128 (or 128 x 128) output tiles, K in steps of 32 through a ring of three LDS stages filled by
// buffer-load-to-LDS (lds_ring.h).  The kernel computes the transposed tile C^T = B^T A^T: B^T
// fragments come from the row-major B tile through transposing LDS reads, A^T fragments are
// plain row reads of the A tile, and every lane ends up owning one row of C with consecutive
// columns in consecutive registers, which packs into whole bf16 rows for the store.
// Other shapes and fp32 take two plain kernels (one thread per output element).
#include "lds_ring.h"

namespace kunlun {

constexpr int GN = 128, GK = 32;  // output tile columns and K step; tile rows = 64 * MB (template)

// C = op(A) op(B).  An operand is stored either with the contraction index along its rows
// ("row form": A as [M, K], B as [N, K]) or across them ("column form": A as [K, M], B as [K, N]);
// the forward uses A row / B column (the usual row-major product), the gradients also the other
// two mixes.  The contraction index may run over several slabs of the operands (k_inner values
// per slab, slab strides a_kslab / b_kslab): sums over the batch are contractions of this kind.
// With `partial` set the K steps are cut into `splits` ranges, workgroup (split, tile) writes its
// fp32 partial tile into partial[split][M][N], and a second kernel adds the partial sums in a
// fixed order (bit-reproducible) and rounds once.
struct GemmArgs {
    const bf16_t* a;      // row form: row m of a batch at a + batch*a_batch + (m % a_mod)*a_lo + (m / a_mod)*a_hi, K contiguous
                          // column form: [K, M] with row stride lda
    const bf16_t* b;      // column form: [K, N] with row stride ldb;  row form: [N, K] with row stride ldb
    bf16_t* c;            // partial == null: row m of a batch -> c + batch*c_batch + (m % c_mod)*c_lo + (m / c_mod)*c_hi, N contiguous values
    float* partial;       // non-null: [splits][M][N] fp32 partial sums instead of c
    int64_t a_batch, b_batch, c_batch, c_lo, c_hi, a_lo, a_hi, a_kslab, b_kslab;
    int lda, ldb, c_mod, a_mod;
    uint32_t a_span;      // row form: bytes from a tile's lowest row offset that its rows may span (an upper bound)
    int M, N, K, k_inner; // N % 128 == 0, k_inner % 32 == 0, K = slabs * k_inner; any M >= 1 (column-form A: M % tile rows == 0)
    int splits, steps_per_split;
    int tiles_per_unit;   // workgroups that share a streamed operand (kept on one XCD, back to back)
    int n_tiles, m_tiles, batches;
    int unit_is_batch;    // 1: unit = batch (tiles = m_tiles*n_tiles), 0: unit = m tile (tiles = n_tiles)
};

template <int MB>  // 32-row blocks per wave: the workgroup tile has 64*MB rows (2 x 2 waves)
struct GemmSmem {
    static constexpr int GM = 64 * MB;
    static constexpr int A_TILE = GM * GK * 2;  // row form: GM rows x 64 bytes, chunk ^= (row / 4) % 4; column form: GM/128 tiles like B
    static constexpr int B_TILE = GK * GN * 2;  // column form: 32 rows x 256 bytes, V swizzle of TileLayout<128>; row form: 128 rows x 64 bytes
    static constexpr int STAGE = A_TILE + B_TILE;
    static constexpr int TOTAL = 3 * STAGE;
    static constexpr int OUT_STRIDE = 64 * 2 + 16;  // a wave's output block goes out 64 rows x 64 columns at a time, padded rows
    static constexpr int PART_STRIDE = 64 * 4 + 16; // fp32 partial tiles: 32 rows x 64 columns at a time
    static_assert(4 * 64 * OUT_STRIDE <= TOTAL, "output staging must fit");
    static_assert(4 * 32 * PART_STRIDE <= TOTAL, "partial-sum staging must fit");
};

// 64-byte rows (32 contraction values) of a row-form tile
__device__ __forceinline__ int a_tile_offset(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }

template <int MB, bool A_COLS, bool B_ROWS>  // A_COLS: A in column form;  B_ROWS: B in row form
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(GemmArgs p) {
    using SM = GemmSmem<MB>;
    constexpr int GM = SM::GM;
    constexpr int A_LOADS = GM / 64;  // A-tile load instructions per wave (row form: 16 rows each; column form: 4 rows of 128 columns each)
    __shared__ __attribute__((aligned(1024))) char lds[SM::TOTAL];
    using L = TileLayout<128>;
    using ColDma = TileDma<128, 4, SWZ_V>;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    int split = 0, in_unit;
    int64_t unit;
    if (p.partial) {
        // split-K: consecutive workgroups (= consecutive XCDs) take the K ranges of one output tile
        split = (int)(blockIdx.x % p.splits);
        const int64_t rest = blockIdx.x / p.splits;
        in_unit = (int)(rest % p.tiles_per_unit);
        unit = rest / p.tiles_per_unit;
    } else {
        // workgroup i runs on XCD i % 8: the workgroups of a unit follow each other on one XCD
        const int xcd = blockIdx.x & 7;
        const int64_t j = blockIdx.x >> 3;
        in_unit = (int)(j % p.tiles_per_unit);
        unit = (j / p.tiles_per_unit) * 8 + xcd;
    }
    int batch, mt, nt;
    if (p.unit_is_batch) {
        if (unit >= p.batches) return;
        batch = (int)unit; mt = in_unit / p.n_tiles; nt = in_unit % p.n_tiles;
    } else {
        if (unit >= p.m_tiles) return;
        batch = 0; mt = (int)unit; nt = in_unit;
    }
    const int m0 = mt * GM, n0 = nt * GN;
    const int rows_valid = p.M - m0 < GM ? p.M - m0 : GM;
    const uint32_t lda_b = (uint32_t)p.lda * 2, ldb_b = (uint32_t)p.ldb * 2;
    const uint32_t lds0 = lds_address(lds);
    const int steps_per_slab = p.k_inner / GK;
    const int n_total = p.K / GK;
    const int ks0 = split * p.steps_per_split;
    const int ks1 = ks0 + p.steps_per_split < n_total ? ks0 + p.steps_per_split : n_total;
    const int n_steps = ks1 - ks0;

    // ---- tile transport.  Row form: 16 rows x 64 bytes per load instruction, per-lane offsets fixed,
    // the K step moves the uniform offset.  Column form: 4 rows x 256 bytes per instruction (TileDma).
    auto row_of_a = [&](int m) { return (int64_t)(m % p.a_mod) * p.a_lo + (int64_t)(m / p.a_mod) * p.a_hi; };
    const int64_t a_row0 = A_COLS ? 0 : (int64_t)(m0 / p.a_mod) * p.a_hi;  // a lower bound of the tile's row offsets (a_lo, a_hi >= 0)
    const char* A = (const char*)(p.a + batch * p.a_batch + (A_COLS ? (int64_t)m0 : a_row0));
    const char* Bm = (const char*)(p.b + batch * p.b_batch + (B_ROWS ? (int64_t)n0 * p.ldb : (int64_t)n0));
    uint32_t a_voff[A_LOADS], b_voff[2];
    if (!A_COLS) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int row = (wave * A_LOADS + i) * 16 + lane / 4, pos = lane % 4;
            const int src_row = row < rows_valid ? row : rows_valid - 1;  // rows past M re-read the last one (never stored)
            a_voff[i] = (uint32_t)((row_of_a(m0 + src_row) - a_row0) * 2) + ((pos ^ ((row >> 2) & 3)) << 4);
        }
    }
    if (B_ROWS) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = (wave * 2 + i) * 16 + lane / 4, pos = lane % 4;
            b_voff[i] = (uint32_t)row * ldb_b + ((pos ^ ((row >> 2) & 3)) << 4);
        }
    }
    ColDma cdma_a, cdma_b;
    if (A_COLS) cdma_a.init(lane, wave, lda_b);
    if (!B_ROWS) cdma_b.init(lane, wave, ldb_b);
    auto issue = [&](int ks, int stage) {
        const uint32_t dst = lds0 + stage * SM::STAGE;
        const int slab = ks / steps_per_slab, kin = ks % steps_per_slab;
        if (A_COLS) {
            const char* src = A + (slab * p.a_kslab + (int64_t)kin * GK * p.lda) * 2;
#pragma unroll
            for (int t = 0; t < GM / 128; ++t) cdma_a.issue(src + t * 256, GK, dst + t * 8192);
        } else {
            const u32x4 rsrc = make_rsrc_words(A + slab * p.a_kslab * 2, p.a_span);
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
                load_to_lds_b128(rsrc, a_voff[i], (uint32_t)kin * (GK * 2), dst + (wave * A_LOADS + i) * 1024);
        }
        if (B_ROWS) {
            const u32x4 rsrc = make_rsrc_words(Bm + slab * p.b_kslab * 2, (uint32_t)(GN - 1) * ldb_b + (uint32_t)p.k_inner * 2);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                load_to_lds_b128(rsrc, b_voff[i], (uint32_t)kin * (GK * 2), dst + SM::A_TILE + (wave * 2 + i) * 1024);
        } else {
            cdma_b.issue(Bm + (slab * p.b_kslab + (int64_t)kin * GK * p.ldb) * 2, GK, dst + SM::A_TILE);
        }
    };
    constexpr int LOADS_PER_STEP = A_LOADS + 2;
    static_assert(ColDma::IPW == 2, "a 32 x 128 column-form tile is two load instructions per wave");
    if (n_steps > 0) issue(ks0, 0);
    if (n_steps > 1) issue(ks0 + 1, 1);

    // ---- wave (wm, wn) owns the (32*MB) x 64 block at rows 32*MB*wm, columns 64*wn of the tile.
    // The kernel computes C^T = B^T A^T: the matrix instruction's A operand is a B^T fragment (row =
    // column n of C, contraction k = 16c + 8g + 0..7), its B operand an A^T fragment (column = row m of
    // C).  From a row-form tile a fragment is one 16-byte read of the row (rows 32 apart share the
    // swizzle: + 32*64 bytes per block; ^ (c << 5) for k step c); from a column-form tile it is two
    // transposing reads (4 contraction rows each; + 16 rows per k step c; ^ (block << 6) for the
    // next 32 columns).
    const int wm = wave >> 1, wn = wave & 1;
    const int s16 = lane & 15, hi16 = (lane >> 4) & 1;
    int b_rd[2], a_rd[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        b_rd[half] = B_ROWS ? 0 : L::v_offset(8 * g + 4 * half + (s16 >> 2), (64 * wn + 16 * hi16 + 4 * (s16 & 3)) * 2);
        const int col = 32 * MB * wm;  // first column (= row of C) of the wave inside the A tile
        a_rd[half] = A_COLS ? (col / 128) * 8192 + L::v_offset(8 * g + 4 * half + (s16 >> 2), (col % 128 + 16 * hi16 + 4 * (s16 & 3)) * 2) : 0;
    }
    if (B_ROWS) b_rd[0] = a_tile_offset(64 * wn + r, g);
    if (!A_COLS) a_rd[0] = a_tile_offset(32 * MB * wm + r, g);
    auto tr2 = [](const char* a, const char* b) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, b));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    f32x16 acc[2][MB];  // [nb][mb]
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

    int stage = 0;
    for (int i = 0; i < n_steps; ++i) {
        if (i + 1 < n_steps) wait_vmcnt<LOADS_PER_STEP>();
        else wait_vmcnt<0>();
        __syncthreads();  // step i complete; every wave is done with the stage of step i-1
        if (i + 2 < n_steps) issue(ks0 + i + 2, stage == 0 ? 2 : stage - 1);
        const char* sa = lds + stage * SM::STAGE;
        const char* sb = sa + SM::A_TILE;
        stage = stage == 2 ? 0 : stage + 1;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            bf16x8 af[MB], bf[2];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (A_COLS) af[mb] = tr2(sa + c * 16 * 256 + (a_rd[0] ^ (mb << 6)), sa + c * 16 * 256 + (a_rd[1] ^ (mb << 6)));
                else af[mb] = *(const bf16x8*)(sa + mb * 32 * 64 + (a_rd[0] ^ (c << 5)));
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                if (B_ROWS) bf[nb] = *(const bf16x8*)(sb + nb * 32 * 64 + (b_rd[0] ^ (c << 5)));
                else bf[nb] = tr2(sb + c * 16 * 256 + (b_rd[0] ^ (nb << 6)), sb + c * 16 * 256 + (b_rd[1] ^ (nb << 6)));
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma32(bf[nb], af[mb], acc[nb][mb]);
        }
    }

    // ---- epilogue: lane holds row m = 32*MB*wm + 32*mb + r, columns 64*wn + 32*nb + 8*(v/4) + 4g + (v%4)
    __syncthreads();  // every wave is done with the ring
    if (p.partial) {
        // fp32 partial tile: 32 rows of the wave's block at a time through its own padded staging rows
        char* out = lds + wave * (32 * SM::PART_STRIDE);
        float* pb = p.partial + ((int64_t)split * p.M) * p.N + n0 + 64 * wn;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    f32x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = acc[nb][mb][4 * vg + e];
                    *(f32x4*)(out + r * SM::PART_STRIDE + (32 * nb + 8 * vg + 4 * g) * 4) = o4;
                }
            // 16 lanes x 16 bytes per row, 4 rows per pass
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = i * 4 + lane / 16, ch = lane % 16;
                const int m = m0 + 32 * MB * wm + 32 * mb + row;
                const f32x4 val = *(const f32x4*)(out + row * SM::PART_STRIDE + ch * 16);
                if (m < p.M) *(f32x4*)(pb + (int64_t)m * p.N + ch * 4) = val;
            }
        }
        return;
    }
    // bf16 rows: 64 rows of the wave's block at a time through its own padded staging rows, whole rows out
    char* out = lds + wave * (64 * SM::OUT_STRIDE);
    bf16_t* cb = p.c + batch * p.c_batch + n0 + 64 * wn;
#pragma unroll
    for (int half = 0; half < MB / 2; ++half) {
#pragma unroll
        for (int mb2 = 0; mb2 < 2; ++mb2)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)acc[nb][2 * half + mb2][4 * vg + e];
                    *(bf16x4*)(out + (32 * mb2 + r) * SM::OUT_STRIDE + (32 * nb + 8 * vg + 4 * g) * 2) = o4;
                }
        // 8 lanes x 16 bytes per row, 8 rows per pass (the staging rows are private to the wave)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = i * 8 + lane / 8, ch = lane % 8;
            const int m = m0 + 32 * MB * wm + 64 * half + row;
            const u32x4 val = *(const u32x4*)(out + row * SM::OUT_STRIDE + ch * 16);
            if (m < p.M) *(u32x4*)(cb + (int64_t)(m % p.c_mod) * p.c_lo + (int64_t)(m / p.c_mod) * p.c_hi + ch * 8) = val;
        }
    }
}

// out[(m / r_mod)*r_hi + (m % r_mod)*r_lo + n*r_n] = sum over the splits of partial[split][m][n].
// 32 consecutive outputs x 8 ranges of splits per workgroup: every thread adds its range in split
// order, then the 8 range sums are added in range order (a fixed order: bit-reproducible).
template <typename T_>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, T_* __restrict__ out, int splits,
                                                            int M, int N, int r_mod, int64_t r_lo, int64_t r_hi, int64_t r_n) {
    __shared__ float part[8][32];
    const int col = threadIdx.x & 31, range = threadIdx.x >> 5;
    const int64_t idx = (int64_t)blockIdx.x * 32 + col;
    const int64_t mn = (int64_t)M * N;
    const int per = (splits + 7) / 8;
    const int s0 = range * per, s1 = s0 + per < splits ? s0 + per : splits;
    float acc = 0.f;
    if (idx < mn) {
        int s = s0;
        for (; s + 4 <= s1; s += 4) {
            const float a = partial[(int64_t)s * mn + idx], b = partial[(int64_t)(s + 1) * mn + idx];
            const float c = partial[(int64_t)(s + 2) * mn + idx], d = partial[(int64_t)(s + 3) * mn + idx];
            acc = (((acc + a) + b) + c) + d;
        }
        for (; s < s1; ++s) acc += partial[(int64_t)s * mn + idx];
    }
    part[range][col] = acc;
    __syncthreads();
    if (range != 0 || idx >= mn) return;
    float total = part[0][col];
#pragma unroll
    for (int i = 1; i < 8; ++i) total += part[i][col];
    const int m = (int)(idx / N), n = (int)(idx % N);
    out[(int64_t)(m / r_mod) * r_hi + (int64_t)(m % r_mod) * r_lo + (int64_t)n * r_n] = from_float<T_>(total);
}

// zt[(i*T + t)*S + s] = z[(i*S + s)*T + t]
__global__ __launch_bounds__(256) void transpose_z_kernel(const bf16_t* __restrict__ z, bf16_t* __restrict__ zt, int k, int S,
                                                          int T) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)k * S * T) return;
    const int s = (int)(idx % S);
    const int t = (int)((idx / S) % T);
    const int i = (int)(idx / ((int64_t)S * T));
    zt[idx] = z[((int64_t)i * S + s) * T + t];
}

// ---- plain kernels (fp32, or shapes the tiled kernel does not take): one thread per output element; sums and the
// intermediate U in fp64, so that the only rounding of an fp32 result is the final one
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_stage1_plain(const T_* __restrict__ x, const T_* __restrict__ z,
                                                            double* __restrict__ u, int B, int S, int T, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // ((b*T + t)*k + i)*D + c
    if (idx >= (int64_t)B * T * k * D) return;
    const int c = (int)(idx % D);
    const int i = (int)((idx / D) % k);
    const int t = (int)((idx / ((int64_t)D * k)) % T);
    const int64_t b = idx / ((int64_t)D * k * T);
    double acc = 0.0;
    for (int s = 0; s < S; ++s) acc += (double)to_float(z[((int64_t)i * S + s) * T + t]) * (double)to_float(x[(b * S + s) * D + c]);
    u[idx] = acc;
}
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_stage2_plain(const double* __restrict__ u, const T_* __restrict__ w,
                                                            T_* __restrict__ y, int64_t rows, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // row*D + e, row = b*T + t
    if (idx >= rows * D) return;
    const int e = (int)(idx % D);
    const int64_t row = idx / D;
    double acc = 0.0;
    for (int jc = 0; jc < k * D; ++jc) acc += u[row * (int64_t)k * D + jc] * (double)to_float(w[(int64_t)jc * D + e]);
    y[idx] = from_float<T_>((float)acc);
}

bool sumkron_tiled_supported(int S, int T, int D, int k, int dtype) {
    return dtype == KUNLUN_BF16 && D % GN == 0 && S % GK == 0 && T >= 1 && k >= 1;
}
// the gradient GEMMs also contract over (t, i) and over (b, t), and one has S as its column count
bool sumkron_bwd_tiled_supported(int B, int S, int T, int D, int k, int dtype) {
    return sumkron_tiled_supported(S, T, D, k, dtype) && S % GN == 0 && ((int64_t)T * k) % GK == 0 && ((int64_t)B * T) % GK == 0;
}

size_t sumkron_workspace(int B, int S, int T, int D, int k, int dtype) {
    if (sumkron_fused_supported(S, T, D, k, dtype)) return sumkron_fused_workspace(S, T, D, k);
    if (sumkron_tiled_supported(S, T, D, k, dtype))
        return align_up((size_t)k * T * S * 2, 256) + align_up((size_t)B * T * k * D * 2, 256);
    return align_up((size_t)B * T * k * D * sizeof(double), 256);
}

static unsigned gemm_grid(int64_t units, int tiles_per_unit) { return (unsigned)(((units + 7) / 8) * 8 * tiles_per_unit); }

// K steps per split so that about `target` workgroups run, none with fewer than 4 steps
static void plan_splits(int64_t tiles, int n_steps, int target, int& splits, int& steps_per_split) {
    if (n_steps < 1) { splits = 1; steps_per_split = 1; return; }
    int64_t want = target / (tiles > 0 ? tiles : 1);
    if (want > n_steps / 4) want = n_steps / 4;
    if (want < 1) want = 1;
    steps_per_split = (int)((n_steps + want - 1) / want);
    splits = (n_steps + steps_per_split - 1) / steps_per_split;
}
// workgroups aimed at: the dW contraction is matrix-core-bound (two workgroups per compute unit, two rounds),
// the dZ contraction streams X and G once and writes 128 KB of partial sums per workgroup (one round)
constexpr int SPLIT_TARGET_DW = 1024, SPLIT_TARGET_DZ = 512;

static bool gemm_is_tall(int M, bool a_cols) { return a_cols ? M % 256 == 0 : (M % 256 == 0 || M >= 1024); }
static int64_t gemm_tiles(int M, int N, int batches, bool a_cols) {
    const int gm = gemm_is_tall(M, a_cols) ? 256 : 128;
    return (int64_t)((M + gm - 1) / gm) * (N / GN) * batches;
}

// 256-row tiles (16 MFMAs per wave between two barriers) when the rows fill them, else 128-row tiles.
// g.splits == 0: one split.  Plain row-major row-form A: a_mod = 1, a_lo = 0, a_hi = row stride.
template <bool A_COLS, bool B_ROWS>
static void launch_gemm(GemmArgs g, hipStream_t stream) {
    const bool tall = gemm_is_tall(g.M, A_COLS);
    const int gm = tall ? 256 : 128;
    g.m_tiles = (g.M + gm - 1) / gm;
    g.n_tiles = g.N / GN;
    g.tiles_per_unit = g.unit_is_batch ? g.m_tiles * g.n_tiles : g.n_tiles;
    if (g.k_inner == 0) g.k_inner = g.K;
    if (g.splits <= 1) { g.splits = 1; g.steps_per_split = g.K / GK; }
    if (!A_COLS) {
        const int64_t rows = g.a_mod < gm ? g.a_mod : gm;
        g.a_span = (uint32_t)(((rows - 1) * g.a_lo + (gm / g.a_mod + 1) * g.a_hi + g.k_inner) * 2);
    }
    const int64_t units = g.unit_is_batch ? g.batches : g.m_tiles;
    const dim3 grid(g.partial ? (unsigned)(units * g.tiles_per_unit * g.splits) : gemm_grid(units, g.tiles_per_unit));
    if (tall) hipLaunchKernelGGL((gemm_bf16_kernel<4, A_COLS, B_ROWS>), grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL((gemm_bf16_kernel<2, A_COLS, B_ROWS>), grid, dim3(256), 0, stream, g);
}

// U_b rows (i, t) = Zt [k*T, S] * X_b [S, D], stored as U[b][t][i*D + c]
static void launch_stage1(const bf16_t* x, const bf16_t* z, bf16_t* zt, bf16_t* u, int B, int S, int T, int D, int k,
                          hipStream_t stream) {
    const int64_t nz = (int64_t)k * S * T;
    hipLaunchKernelGGL(transpose_z_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, stream, z, zt, k, S, T);
    GemmArgs g1 = {};
    g1.a = zt; g1.a_batch = 0; g1.a_mod = 1; g1.a_hi = S;
    g1.b = x; g1.b_batch = (int64_t)S * D; g1.ldb = D;
    g1.c = u; g1.c_batch = (int64_t)T * k * D; g1.c_mod = T; g1.c_lo = (int64_t)k * D; g1.c_hi = D;
    g1.M = k * T; g1.N = D; g1.K = S;
    g1.batches = B; g1.unit_is_batch = 1;
    launch_gemm<false, false>(g1, stream);
}

hipError_t launch_sumkron(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k,
                          int dtype, void* workspace, hipStream_t stream) {
    if (sumkron_fused_supported(S, T, D, k, dtype)) return launch_sumkron_fused(x, z, w, y, B, S, T, D, k, workspace, stream);
    if (sumkron_tiled_supported(S, T, D, k, dtype)) {
        bf16_t* zt = (bf16_t*)workspace;
        bf16_t* u = (bf16_t*)((char*)workspace + align_up((size_t)k * T * S * 2, 256));
        launch_stage1((const bf16_t*)x, (const bf16_t*)z, zt, u, B, S, T, D, k, stream);
        GemmArgs g2 = {};  // Y [B*T, D] = U [B*T, k*D] * Wcat [k*D, D]
        g2.a = u; g2.a_batch = 0; g2.a_mod = 1; g2.a_hi = (int64_t)k * D;
        g2.b = (const bf16_t*)w; g2.b_batch = 0; g2.ldb = D;
        g2.c = (bf16_t*)y; g2.c_batch = 0; g2.c_mod = 1; g2.c_lo = 0; g2.c_hi = D;
        g2.M = B * T; g2.N = D; g2.K = k * D;
        g2.batches = 1; g2.unit_is_batch = 0;
        launch_gemm<false, false>(g2, stream);
        return hipGetLastError();
    }
    double* u = (double*)workspace;
    const int64_t n1 = (int64_t)B * T * k * D, n2 = (int64_t)B * T * D;
    if (dtype == KUNLUN_BF16) {
        hipLaunchKernelGGL(sumkron_stage1_plain<bf16_t>, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, stream,
                           (const bf16_t*)x, (const bf16_t*)z, u, B, S, T, D, k);
        hipLaunchKernelGGL(sumkron_stage2_plain<bf16_t>, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, stream, u,
                           (const bf16_t*)w, (bf16_t*)y, (int64_t)B * T, D, k);
    } else {
        hipLaunchKernelGGL(sumkron_stage1_plain<float>, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, stream,
                           (const float*)x, (const float*)z, u, B, S, T, D, k);
        hipLaunchKernelGGL(sumkron_stage2_plain<float>, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, stream, u,
                           (const float*)w, (float*)y, (int64_t)B * T, D, k);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ backward
// With U_b = [Z_1^T X_b | ... | Z_k^T X_b]  (T x kD)  and  G_b = [dY_b W_1^T | ... | dY_b W_k^T]  (T x kD):
//     dX_b = sum_i Z_i G_{b,i}          dW_i = sum_b U_{b,i}^T dY_b          dZ_i = sum_b X_b G_{b,i}^T
// (the chain rule applied to Eq. (SumKronLinear)).  Five GEMMs of the kernel above; the two sums over
// the batch are split-K contractions with fp32 partial sums.

// zc[s*(T*k) + t*k + i] = z[(i*S + s)*T + t]
__global__ __launch_bounds__(256) void interleave_z_kernel(const bf16_t* __restrict__ z, bf16_t* __restrict__ zc, int k, int S,
                                                           int T) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)k * S * T) return;
    const int i = (int)(idx % k);
    const int t = (int)((idx / k) % T);
    const int s = (int)(idx / ((int64_t)k * T));
    zc[idx] = z[((int64_t)i * S + s) * T + t];
}

template <typename T_>
__global__ __launch_bounds__(256) void fill_zero_kernel(T_* __restrict__ p, int64_t n) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < n) p[idx] = from_float<T_>(0.f);
}

// plain kernels: one thread per output element; every sum and the intermediates in fp64;
// u and gq are [B*T][k][D] fp64
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_g_plain(const T_* __restrict__ dy, const T_* __restrict__ w, double* __restrict__ gq,
                                                       int64_t rows, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (row*k + i)*D + c
    if (idx >= rows * k * D) return;
    const int c = (int)(idx % D);
    const int i = (int)((idx / D) % k);
    const int64_t row = idx / ((int64_t)D * k);
    double acc = 0.0;
    for (int e = 0; e < D; ++e) acc += (double)to_float(dy[row * D + e]) * (double)to_float(w[((int64_t)i * D + c) * D + e]);
    gq[idx] = acc;
}
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_dx_plain(const T_* __restrict__ z, const double* __restrict__ gq, T_* __restrict__ dx,
                                                        int B, int S, int T, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (b*S + s)*D + c
    if (idx >= (int64_t)B * S * D) return;
    const int c = (int)(idx % D);
    const int s = (int)((idx / D) % S);
    const int64_t b = idx / ((int64_t)D * S);
    double acc = 0.0;
    for (int i = 0; i < k; ++i)
        for (int t = 0; t < T; ++t)
            acc += (double)to_float(z[((int64_t)i * S + s) * T + t]) * gq[(((b * T + t) * k) + i) * D + c];
    dx[idx] = from_float<T_>((float)acc);
}
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_dw_plain(const double* __restrict__ u, const T_* __restrict__ dy, T_* __restrict__ dw,
                                                        int64_t rows, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (i*D + c)*D + e
    if (idx >= (int64_t)k * D * D) return;
    const int e = (int)(idx % D);
    const int c = (int)((idx / D) % D);
    const int i = (int)(idx / ((int64_t)D * D));
    double acc = 0.0;
    for (int64_t row = 0; row < rows; ++row) acc += u[(row * k + i) * D + c] * (double)to_float(dy[row * D + e]);
    dw[idx] = from_float<T_>((float)acc);
}
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_dz_plain(const T_* __restrict__ x, const double* __restrict__ gq, T_* __restrict__ dz,
                                                        int B, int S, int T, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (i*S + s)*T + t
    if (idx >= (int64_t)k * S * T) return;
    const int t = (int)(idx % T);
    const int s = (int)((idx / T) % S);
    const int i = (int)(idx / ((int64_t)T * S));
    double acc = 0.0;
    for (int64_t b = 0; b < B; ++b)
        for (int c = 0; c < D; ++c) acc += (double)to_float(x[(b * S + s) * D + c]) * gq[(((b * T + t) * k) + i) * D + c];
    dz[idx] = from_float<T_>((float)acc);
}

struct BwdLayout {
    size_t zt, zc, u, gq, partial, total;
    int dw_splits, dw_steps, dz_splits, dz_steps;
};
static BwdLayout sumkron_bwd_layout(int B, int S, int T, int D, int k, int dtype) {
    BwdLayout l = {};
    const size_t ukd = (size_t)B * T * k * D;
    if (!sumkron_bwd_tiled_supported(B, S, T, D, k, dtype)) {
        l.u = 0;
        l.gq = align_up(ukd * sizeof(double), 256);
        l.total = l.gq + align_up(ukd * sizeof(double), 256);
        return l;
    }
    l.zt = 0;
    l.zc = l.zt + align_up((size_t)k * T * S * 2, 256);
    l.u = l.zc + align_up((size_t)k * T * S * 2, 256);
    l.gq = l.u + align_up(ukd * 2, 256);
    l.partial = l.gq + align_up(ukd * 2, 256);
    plan_splits(gemm_tiles(k * D, D, 1, true), (int)((int64_t)B * T / GK), SPLIT_TARGET_DW, l.dw_splits, l.dw_steps);
    plan_splits(gemm_tiles(k * T, S, 1, false), (int)((int64_t)B * D / GK), SPLIT_TARGET_DZ, l.dz_splits, l.dz_steps);
    const size_t p1 = (size_t)l.dw_splits * k * D * D * sizeof(float), p2 = (size_t)l.dz_splits * k * T * S * sizeof(float);
    l.total = l.partial + align_up(p1 > p2 ? p1 : p2, 256);
    return l;
}
size_t sumkron_bwd_workspace(int B, int S, int T, int D, int k, int dtype) { return sumkron_bwd_layout(B, S, T, D, k, dtype).total; }

template <typename T_>
static void launch_bwd_plain(const T_* x, const T_* z, const T_* w, const T_* dy, T_* dx, T_* dz, T_* dw, int B, int S, int T,
                             int D, int k, double* u, double* gq, hipStream_t stream) {
    const int64_t rows = (int64_t)B * T, n1 = rows * k * D;
    auto blocks = [](int64_t n) { return dim3((unsigned)((n + 255) / 256)); };
    hipLaunchKernelGGL(sumkron_stage1_plain<T_>, blocks(n1), dim3(256), 0, stream, x, z, u, B, S, T, D, k);
    hipLaunchKernelGGL(sumkron_g_plain<T_>, blocks(n1), dim3(256), 0, stream, dy, w, gq, rows, D, k);
    hipLaunchKernelGGL(sumkron_dx_plain<T_>, blocks((int64_t)B * S * D), dim3(256), 0, stream, z, gq, dx, B, S, T, D, k);
    hipLaunchKernelGGL(sumkron_dw_plain<T_>, blocks((int64_t)k * D * D), dim3(256), 0, stream, u, dy, dw, rows, D, k);
    hipLaunchKernelGGL(sumkron_dz_plain<T_>, blocks((int64_t)k * S * T), dim3(256), 0, stream, x, gq, dz, B, S, T, D, k);
}

hipError_t launch_sumkron_bwd(const void* x, const void* z, const void* w, const void* dy, void* dx, void* dz, void* dw, int B,
                              int S, int T, int D, int k, int dtype, void* workspace, hipStream_t stream) {
    const int64_t nz = (int64_t)k * S * T, nw = (int64_t)k * D * D;
    auto blocks = [](int64_t n) { return dim3((unsigned)((n + 255) / 256)); };
    if (B == 0) {  // no example: the weight gradients are zero
        if (dtype == KUNLUN_BF16) {
            hipLaunchKernelGGL(fill_zero_kernel<bf16_t>, blocks(nz), dim3(256), 0, stream, (bf16_t*)dz, nz);
            hipLaunchKernelGGL(fill_zero_kernel<bf16_t>, blocks(nw), dim3(256), 0, stream, (bf16_t*)dw, nw);
        } else {
            hipLaunchKernelGGL(fill_zero_kernel<float>, blocks(nz), dim3(256), 0, stream, (float*)dz, nz);
            hipLaunchKernelGGL(fill_zero_kernel<float>, blocks(nw), dim3(256), 0, stream, (float*)dw, nw);
        }
        return hipGetLastError();
    }
    const BwdLayout l = sumkron_bwd_layout(B, S, T, D, k, dtype);
    char* ws = (char*)workspace;
    if (!sumkron_bwd_tiled_supported(B, S, T, D, k, dtype)) {
        if (dtype == KUNLUN_BF16)
            launch_bwd_plain<bf16_t>((const bf16_t*)x, (const bf16_t*)z, (const bf16_t*)w, (const bf16_t*)dy, (bf16_t*)dx,
                                     (bf16_t*)dz, (bf16_t*)dw, B, S, T, D, k, (double*)(ws + l.u), (double*)(ws + l.gq), stream);
        else
            launch_bwd_plain<float>((const float*)x, (const float*)z, (const float*)w, (const float*)dy, (float*)dx, (float*)dz,
                                    (float*)dw, B, S, T, D, k, (double*)(ws + l.u), (double*)(ws + l.gq), stream);
        return hipGetLastError();
    }
    bf16_t* zt = (bf16_t*)(ws + l.zt);
    bf16_t* zc = (bf16_t*)(ws + l.zc);
    bf16_t* u = (bf16_t*)(ws + l.u);
    bf16_t* gq = (bf16_t*)(ws + l.gq);
    float* partial = (float*)(ws + l.partial);
    const int kD = k * D;
    launch_stage1((const bf16_t*)x, (const bf16_t*)z, zt, u, B, S, T, D, k, stream);
    hipLaunchKernelGGL(interleave_z_kernel, blocks(nz), dim3(256), 0, stream, (const bf16_t*)z, zc, k, S, T);
    {   // G [B*T, k*D] = dY [B*T, D] * Wstack^T,  Wstack [k*D, D] = w as it is stored (row form)
        GemmArgs g = {};
        g.a = (const bf16_t*)dy; g.a_mod = 1; g.a_hi = D;
        g.b = (const bf16_t*)w; g.ldb = D;
        g.c = gq; g.c_mod = 1; g.c_hi = kD;
        g.M = B * T; g.N = kD; g.K = D;
        g.batches = 1; g.unit_is_batch = 0;
        launch_gemm<false, true>(g, stream);
    }
    {   // dX_b [S, D] = Zc [S, T*k] * G_b viewed as [T*k, D]  (row t*k + i of the view = G_b[t, i*D ..])
        GemmArgs g = {};
        g.a = zc; g.a_batch = 0; g.a_mod = 1; g.a_hi = (int64_t)T * k;
        g.b = gq; g.b_batch = (int64_t)T * kD; g.ldb = D;
        g.c = (bf16_t*)dx; g.c_batch = (int64_t)S * D; g.c_mod = 1; g.c_hi = D;
        g.M = S; g.N = D; g.K = T * k;
        g.batches = B; g.unit_is_batch = 1;
        launch_gemm<false, false>(g, stream);
    }
    {   // dW stacked [k*D, D] = U^T dY: contraction over the B*T rows of U [B*T, k*D] (column form) and dY [B*T, D]
        GemmArgs g = {};
        g.a = u; g.lda = kD;
        g.b = (const bf16_t*)dy; g.ldb = D;
        g.partial = partial; g.splits = l.dw_splits; g.steps_per_split = l.dw_steps;
        g.M = kD; g.N = D; g.K = B * T;
        g.batches = 1; g.unit_is_batch = 0;
        launch_gemm<true, false>(g, stream);
        hipLaunchKernelGGL(splitk_reduce_kernel<bf16_t>, dim3((unsigned)((nw + 31) / 32)), dim3(256), 0, stream, partial, (bf16_t*)dw, l.dw_splits, kD, D,
                           1, (int64_t)0, (int64_t)D, (int64_t)1);
    }
    {   // dZ^T stacked [k*T, S]: row (i, t), column s = sum over (b, c) of G[b, t, i*D + c] X[b, s, c]
        GemmArgs g = {};
        g.a = gq; g.a_mod = T; g.a_lo = kD; g.a_hi = D; g.a_kslab = (int64_t)T * kD;
        g.b = (const bf16_t*)x; g.ldb = D; g.b_kslab = (int64_t)S * D;
        g.partial = partial; g.splits = l.dz_splits; g.steps_per_split = l.dz_steps;
        g.M = k * T; g.N = S; g.K = B * D; g.k_inner = D;
        g.batches = 1; g.unit_is_batch = 0;
        launch_gemm<false, true>(g, stream);
        hipLaunchKernelGGL(splitk_reduce_kernel<bf16_t>, dim3((unsigned)((nz + 31) / 32)), dim3(256), 0, stream, partial, (bf16_t*)dz, l.dz_splits, k * T, S,
                           T, (int64_t)1, (int64_t)S * T, (int64_t)T);
    }
    return hipGetLastError();
}

}  // namespace kunlun
