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

struct GemmArgs {
    const bf16_t* a;      // [batch][M, K], row stride lda
    const bf16_t* b;      // [batch][K, N], row stride ldb
    bf16_t* c;            // row m of a batch -> c + batch*c_batch + (m % c_mod)*c_lo + (m / c_mod)*c_hi, N contiguous values
    int64_t a_batch, b_batch, c_batch, c_lo, c_hi;
    int lda, ldb, c_mod;
    int M, N, K;          // N % 128 == 0, K % 32 == 0; any M >= 1
    int tiles_per_unit;   // workgroups that share a streamed operand (kept on one XCD, back to back)
    int n_tiles, m_tiles, batches;
    int unit_is_batch;    // 1: unit = batch (tiles = m_tiles*n_tiles), 0: unit = m tile (tiles = n_tiles)
};

template <int MB>  // 32-row blocks per wave: the workgroup tile has 64*MB rows (2 x 2 waves)
struct GemmSmem {
    static constexpr int GM = 64 * MB;
    static constexpr int A_TILE = GM * GK * 2;  // GM rows x 64 bytes, chunk ^= (row / 4) % 4
    static constexpr int B_TILE = GK * GN * 2;  // 32 rows x 256 bytes, V swizzle of TileLayout<128>
    static constexpr int STAGE = A_TILE + B_TILE;
    static constexpr int TOTAL = 3 * STAGE;
    static constexpr int OUT_STRIDE = 64 * 2 + 16;  // a wave's output block goes out 64 rows x 64 columns at a time, padded rows
    static_assert(4 * 64 * OUT_STRIDE <= TOTAL, "output staging must fit");
};

__device__ __forceinline__ int a_tile_offset(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }

template <int MB>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(GemmArgs p) {
    using SM = GemmSmem<MB>;
    constexpr int GM = SM::GM;
    constexpr int A_LOADS = GM / 64;  // A-tile load instructions (16 rows each) per wave
    __shared__ __attribute__((aligned(1024))) char lds[SM::TOTAL];
    using L = TileLayout<128>;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    // workgroup i runs on XCD i % 8: the workgroups of a unit follow each other on one XCD
    const int xcd = blockIdx.x & 7;
    const int64_t j = blockIdx.x >> 3;
    const int in_unit = (int)(j % p.tiles_per_unit);
    const int64_t unit = (j / p.tiles_per_unit) * 8 + xcd;
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
    const char* A = (const char*)(p.a + batch * p.a_batch + (int64_t)m0 * p.lda);
    const char* B = (const char*)(p.b + batch * p.b_batch + n0);
    const uint32_t lda_b = (uint32_t)p.lda * 2, ldb_b = (uint32_t)p.ldb * 2;
    const uint32_t lds0 = lds_address(lds);

    // ---- tile transport: A tile GM/16 load instructions (16 rows each), B tile 8 (4 rows each), split over the waves
    uint32_t a_voff[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int row = (wave * A_LOADS + i) * 16 + lane / 4, pos = lane % 4;
        const int src_row = row < rows_valid ? row : rows_valid - 1;  // rows past M re-read the last one (never stored)
        a_voff[i] = (uint32_t)src_row * lda_b + ((pos ^ ((row >> 2) & 3)) << 4);
    }
    const u32x4 a_rsrc = make_rsrc_words(A, (uint32_t)(rows_valid - 1) * lda_b + (uint32_t)p.K * 2);
    TileDma<128, 4, SWZ_V> bdma;
    bdma.init(lane, wave, ldb_b);
    auto issue = [&](int ks, int stage) {
        const uint32_t dst = lds0 + stage * SM::STAGE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            load_to_lds_b128(a_rsrc, a_voff[i], (uint32_t)ks * (GK * 2), dst + (wave * A_LOADS + i) * 1024);
        bdma.issue(B + (int64_t)ks * GK * ldb_b, GK, dst + SM::A_TILE);
    };
    constexpr int LOADS_PER_STEP = A_LOADS + TileDma<128, 4, SWZ_V>::IPW;
    const int n_steps = p.K / GK;
    issue(0, 0);
    if (n_steps > 1) issue(1, 1);

    // ---- wave (wm, wn) owns the (32*MB) x 64 block at rows 32*MB*wm, columns 64*wn of the tile
    const int wm = wave >> 1, wn = wave & 1;
    // B^T fragment (A operand: row = column n of C, contraction k = 16c + 8g + 0..7): two transposing reads
    const int s16 = lane & 15, hi16 = (lane >> 4) & 1;
    int bt_rd[2];
#pragma unroll
    for (int half = 0; half < 2; ++half)
        bt_rd[half] = SM::A_TILE + L::v_offset(8 * g + 4 * half + (s16 >> 2), (64 * wn + 16 * hi16 + 4 * (s16 & 3)) * 2);
    // A^T fragment (B operand: column = row m of C, contraction k = 16c + 8g + 0..7): one 16-byte read of row m
    // (rows 32 apart share the swizzle: + 32*64 bytes per block mb; ^ (c << 5) for k step c)
    const int a_rd = a_tile_offset(32 * MB * wm + r, g);

    f32x16 acc[2][MB];  // [nb][mb]
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

    int stage = 0;
    for (int ks = 0; ks < n_steps; ++ks) {
        if (ks + 1 < n_steps) wait_vmcnt<LOADS_PER_STEP>();
        else wait_vmcnt<0>();
        __syncthreads();  // step ks complete; every wave is done with the stage of step ks-1
        if (ks + 2 < n_steps) issue(ks + 2, stage == 0 ? 2 : stage - 1);
        const char* st = lds + stage * SM::STAGE;
        stage = stage == 2 ? 0 : stage + 1;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            bf16x8 af[MB], bf[2];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) af[mb] = *(const bf16x8*)(st + mb * 32 * 64 + (a_rd ^ (c << 5)));
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                // column block nb of the wave = 64-byte group 2*wn + nb of the B tile row: XOR on bit 6
                const char* base = st + c * 16 * L::ROW_BYTES;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, base + (bt_rd[0] ^ (nb << 6))));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, base + (bt_rd[1] ^ (nb << 6))));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                bf[nb] = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma32(bf[nb], af[mb], acc[nb][mb]);
        }
    }

    // ---- epilogue: lane holds row m = 32*MB*wm + 32*mb + r, columns 64*wn + 32*nb + 8*(v/4) + 4g + (v%4);
    // 64 rows of the wave's block at a time through its own padded staging rows, whole rows out
    __syncthreads();  // every wave is done with the ring
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

// ---- plain kernels (fp32, or shapes the tiled kernel does not take): one thread per output element
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_stage1_plain(const T_* __restrict__ x, const T_* __restrict__ z,
                                                            float* __restrict__ u, int B, int S, int T, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // ((b*T + t)*k + i)*D + c
    if (idx >= (int64_t)B * T * k * D) return;
    const int c = (int)(idx % D);
    const int i = (int)((idx / D) % k);
    const int t = (int)((idx / ((int64_t)D * k)) % T);
    const int64_t b = idx / ((int64_t)D * k * T);
    float acc = 0.f;
    for (int s = 0; s < S; ++s) acc = fmaf(to_float(z[((int64_t)i * S + s) * T + t]), to_float(x[(b * S + s) * D + c]), acc);
    u[idx] = acc;
}
template <typename T_>
__global__ __launch_bounds__(256) void sumkron_stage2_plain(const float* __restrict__ u, const T_* __restrict__ w,
                                                            T_* __restrict__ y, int64_t rows, int D, int k) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // row*D + e, row = b*T + t
    if (idx >= rows * D) return;
    const int e = (int)(idx % D);
    const int64_t row = idx / D;
    float acc = 0.f;
    for (int jc = 0; jc < k * D; ++jc) acc = fmaf(u[row * (int64_t)k * D + jc], to_float(w[(int64_t)jc * D + e]), acc);
    y[idx] = from_float<T_>(acc);
}

bool sumkron_tiled_supported(int S, int T, int D, int k, int dtype) {
    return dtype == KUNLUN_BF16 && D % GN == 0 && S % GK == 0 && T >= 1 && k >= 1;
}

size_t sumkron_workspace(int B, int S, int T, int D, int k, int dtype) {
    if (sumkron_tiled_supported(S, T, D, k, dtype))
        return align_up((size_t)k * T * S * 2, 256) + align_up((size_t)B * T * k * D * 2, 256);
    return align_up((size_t)B * T * k * D * sizeof(float), 256);
}

static unsigned gemm_grid(int64_t units, int tiles_per_unit) { return (unsigned)(((units + 7) / 8) * 8 * tiles_per_unit); }

// 256-row tiles (16 MFMAs per wave between two barriers) when the rows fill them, else 128-row tiles
static void launch_gemm(GemmArgs g, hipStream_t stream) {
    const bool tall = g.M % 256 == 0 || g.M >= 1024;
    const int gm = tall ? 256 : 128;
    g.m_tiles = (g.M + gm - 1) / gm;
    g.tiles_per_unit = g.unit_is_batch ? g.m_tiles * g.n_tiles : g.n_tiles;
    const unsigned grid = gemm_grid(g.unit_is_batch ? g.batches : g.m_tiles, g.tiles_per_unit);
    if (tall) hipLaunchKernelGGL(gemm_bf16_kernel<4>, dim3(grid), dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(gemm_bf16_kernel<2>, dim3(grid), dim3(256), 0, stream, g);
}

hipError_t launch_sumkron(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k,
                          int dtype, void* workspace, hipStream_t stream) {
    if (sumkron_tiled_supported(S, T, D, k, dtype)) {
        bf16_t* zt = (bf16_t*)workspace;
        bf16_t* u = (bf16_t*)((char*)workspace + align_up((size_t)k * T * S * 2, 256));
        const int64_t nz = (int64_t)k * S * T;
        hipLaunchKernelGGL(transpose_z_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, stream, (const bf16_t*)z, zt, k,
                           S, T);
        GemmArgs g1 = {};  // U_b rows (i, t) = Zt [k*T, S] * X_b [S, D], stored as U[b][t][i*D + c]
        g1.a = zt; g1.a_batch = 0; g1.lda = S;
        g1.b = (const bf16_t*)x; g1.b_batch = (int64_t)S * D; g1.ldb = D;
        g1.c = u; g1.c_batch = (int64_t)T * k * D; g1.c_mod = T; g1.c_lo = (int64_t)k * D; g1.c_hi = D;
        g1.M = k * T; g1.N = D; g1.K = S;
        g1.n_tiles = D / GN; g1.batches = B; g1.unit_is_batch = 1;
        launch_gemm(g1, stream);
        GemmArgs g2 = {};  // Y [B*T, D] = U [B*T, k*D] * Wcat [k*D, D]
        g2.a = u; g2.a_batch = 0; g2.lda = k * D;
        g2.b = (const bf16_t*)w; g2.b_batch = 0; g2.ldb = D;
        g2.c = (bf16_t*)y; g2.c_batch = 0; g2.c_mod = 1; g2.c_lo = 0; g2.c_hi = D;
        g2.M = B * T; g2.N = D; g2.K = k * D;
        g2.n_tiles = D / GN; g2.batches = 1; g2.unit_is_batch = 0;
        launch_gemm(g2, stream);
        return hipGetLastError();
    }
    float* u = (float*)workspace;
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

}  // namespace kunlun
