// SumKronLinear forward as ONE kernel, Eq. (SumKronLinear) of Sec. "Hierarchical Seed Pooling" (stage 3):
//     Y_b = sum_i Z_i^T X_b W_i ,   X_b [S, D], Z_i [S, T], W_i [D, D], Y_b [T, D],  T = 32.
// The intermediate U_{b,i} = Z_i^T X_b never leaves the compute unit.  The operator has the shape of the
// attention kernels: per 32-channel block of X,
//     stage 1   U^T_{b,i}[c, t] = sum_s X_b[s, c] Z_i[s, t]      ("scores": rows = channels c of the block, columns = t)
//     stage 2   Y^T_b[n, t]    += sum_c W_i[c, n] U^T_{b,i}[c, t]  ("values": W_i^T, summed over (i, c))
// and as there the transposed first product leaves every lane with one column t and 16 rows c of a 32 x 32 tile,
// which - rounded to bf16 - is directly the B operand of the second product, provided that its A operand (W_i^T)
// is read in the same order of c; X^T comes from the row-major X rows through transposing LDS reads.
//
// A workgroup of 8 waves works on FOUR examples at a time (persistent: groups blockIdx.x, + gridDim.x, ...):
//   stage 1: wave i owns factor Z_i and forms U^T_{e,i} of the block for the four examples, S/16 steps each, A
//            fragments from the X blocks in LDS, B fragments (Z_i) in registers;
//   the packed results go, register image by register image, into an LDS exchange buffer (64 KB);
//   stage 2: wave (g, h) owns the output channels [D/4 * g, D/4 * (g + 1)) of the examples 2h and 2h + 1 (2 * D/128
//            accumulator tiles that live for the whole group): the U^T fragments come from the exchange buffer, the
//            W fragments straight from global memory, three fragment steps ahead of their use, each used for both
//            examples.
// What sets the shape: W (2.4 MB) is read by every workgroup for every group of examples, so the L2 traffic per example
// is W / (examples that share a fragment load).  With two examples per workgroup and one per wave the kernel was bound
// by exactly that (2.4 GB at the 12 TB/s the L2s sustained: 192 us); two examples per wave need twice the accumulators,
// and the registers for them are those of the Z fragments, which are therefore re-read from L2 for every step (dead
// during stage 2) - a third of the W traffic that is saved.
// W is prepared once per call in fragment order: the 64 x 16 bytes that the lanes of a wave need for one MFMA are
// 1 KB contiguous (read the other way - 16 bytes per lane from 32 different rows - every load touched 32 cache
// lines and the kernel ran at a third of its speed).  Z likewise transposed, in the c order of the register layout.
// X blocks of the next step are fetched into registers at the end of stage 2 (last, so that no wait for a W fragment
// covers them) and stored to LDS as soon as stage 1 has read the old ones.
// Per example: 3840 MFMAs of 32x32x16 (the 126 MFLOP of the operator), X read once.
#include "lds_ring.h"

namespace kunlun {

constexpr int SKF_T = 32;       // output tokens per example (columns of Z_i)
constexpr int SKF_CB = 32;      // channels of X per step
constexpr int SKF_WAVES = 8;
constexpr int SKF_EX = 4;       // examples per workgroup step

// position p of a 16-group holds channel perm(p): lane half g of a B fragment owns {4g..4g+3, 8+4g..8+4g+3}
__host__ __device__ inline int skf_perm(int p) { return (p & 3) + 4 * (p >> 3) + 8 * ((p >> 2) & 1); }

// zt[(i*T + t)*S + 16q + p] = z[(i*S + 16q + perm(p))*T + t]
__global__ __launch_bounds__(256) void skf_prepare_z_kernel(const bf16_t* __restrict__ z, bf16_t* __restrict__ zt, int k, int S, int T) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)k * S * T) return;
    const int sp = (int)(idx % S);
    const int t = (int)((idx / S) % T);
    const int i = (int)(idx / ((int64_t)S * T));
    const int s = (sp & ~15) + skf_perm(sp & 15);
    zt[idx] = z[((int64_t)i * S + s) * T + t];
}
// Fragment order: fragment (i, channel block cb of 32, output block nb of 32, half cc) holds, for lane (r, g) and
// q = 0..7, w[i][c = 32*cb + 16*cc + perm(8g + q)][n = 32*nb + r]; 512 values per fragment, lane-major.
__global__ __launch_bounds__(256) void skf_prepare_w_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int k, int D) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)k * D * D) return;
    const int q = (int)(idx & 7), lane = (int)((idx >> 3) & 63), cc = (int)((idx >> 9) & 1);
    const int64_t rest = idx >> 10;  // (i * D/32 + cb) * D/32 + nb
    const int nb = (int)(rest % (D / 32));
    const int cb = (int)((rest / (D / 32)) % (D / 32));
    const int i = (int)(rest / ((int64_t)(D / 32) * (D / 32)));
    const int c = 32 * cb + 16 * cc + skf_perm(8 * (lane >> 5) + q);
    const int n = 32 * nb + (lane & 31);
    wp[idx] = w[((int64_t)i * D + c) * D + n];
}

template <int NBW, int S>  // D = 128 * NBW output / input channels; S rows of X per example (128 or 256)
__global__ __launch_bounds__(64 * SKF_WAVES, 1) void sumkron_fused_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ zt,
                                                                          const bf16_t* __restrict__ wp, bf16_t* __restrict__ y,
                                                                          int B, int k) {
    using L = TileLayout<SKF_CB>;  // 32-row tiles of 32 channels, the layout of the transposing reads
    constexpr int D = 128 * NBW;
    constexpr int KS = S / 16;                  // contraction steps of stage 1
    constexpr int NCB = D / SKF_CB;             // channel blocks of X
    constexpr int XBYTES = S * SKF_CB * 2;      // one example's block
        constexpr int FRAG = 1024;                  // a packed B fragment: 64 lanes x 16 bytes
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    char* const ldsX = lds;                          // [example][S/32 tiles][32 rows x 64 bytes]
    char* const ldsU = lds + SKF_EX * XBYTES;        // [example][factor 8][half 2] fragments

    int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int ng = wave & 3, eh = wave >> 2;    // stage 2: channel group and pair of examples

    // ---- stage-1 B fragments: column t = r of Z_wave, rows in the fragment order (prepared); re-read for every step
    bf16x8 zf[KS];
    auto load_z = [&]() {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            zf[ks] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
            if (wave < k) zf[ks] = *(const bf16x8*)(zt + ((int64_t)wave * SKF_T + r) * S + 16 * ks + 8 * g);
        }
        asm volatile("" ::: "memory");
    };
    // transposing reads of an X tile: see the V^T reads of the attention kernels
    const int xrd = L::v_offset(4 * g + ((lane & 15) >> 2), (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);

    // ---- X transport: wave e < 4 sends the block of example e straight into LDS (buffer-load-to-LDS, 16 rows of 64
    // bytes per instruction; 32-channel rows need no swizzle).  The loads are issued right after stage 1 has read the
    // old blocks, by the four waves that the SIMDs favour anyway (the older wave of each SIMD finishes stage 2 with
    // time to spare), and no registers carry them.
    const uint32_t x_voff = (uint32_t)(lane >> 2) * (uint32_t)(D * 2) + (lane & 3) * 16;
    const uint32_t ldsX0 = lds_address(ldsX);
    auto send_x = [&](int64_t group, int cb) {
        if (wave >= SKF_EX) return;
        int64_t b = group * SKF_EX + wave;
        b = b < B ? b : B - 1;  // (a missing example re-reads the last one; its results are never stored)
        u32x4 rsrc = make_rsrc_words(x + (b * S) * D + cb * SKF_CB, (uint32_t)(S - 1) * (D * 2) + SKF_CB * 2);
#pragma unroll
        for (int q = 0; q < 4; ++q) rsrc[q] = __builtin_amdgcn_readfirstlane(rsrc[q]);
        const uint32_t dst = __builtin_amdgcn_readfirstlane(ldsX0 + wave * XBYTES);
#pragma unroll
        for (int j = 0; j < S / 16; ++j) load_to_lds_b128(rsrc, x_voff, (uint32_t)j * 16 * (D * 2), dst + j * 1024);
    };

    const int64_t n_groups = ((int64_t)B + SKF_EX - 1) / SKF_EX;
    int64_t group = blockIdx.x;
    if (group >= n_groups) return;
    send_x(group, 0);
    load_z();
    wait_vmcnt<0>();
    // W fragments travel three fragment steps ahead of their use in a ring of four register sets that runs on from
    // one step into the next (W does not depend on the group): the first three steps of all
    const int kp = (k + 1) & ~1;                                  // factors rounded up to whole pairs
    constexpr int64_t wfactor = (int64_t)D * D;                   // values per factor
    constexpr int64_t wblock = (int64_t)(D / 32) * 2 * 512;       // values per channel block of a factor
    const bf16_t* const wlane = wp + (int64_t)NBW * ng * 2 * 512 + lane * 8;
    bf16x8 wq[4][NBW];
    auto issue = [&](int cb, int i, int cc, bf16x8 (&dst)[NBW]) {
        // factor i of block cb; i >= kp: factor i - kp of the next block (past the last real factor: it once more, unused)
        const bool next = i >= kp;
        int ii = next ? i - kp : i;
        ii = ii < k ? ii : k - 1;
        const int cbb = next ? (cb + 1 < NCB ? cb + 1 : 0) : cb;
        const bf16_t* src = wlane + cbb * wblock + ii * wfactor + cc * 512;
#pragma unroll
        for (int j = 0; j < NBW; ++j) dst[j] = *(const bf16x8*)(src + j * 2 * 512);
        asm volatile("" ::: "memory");
    };
    issue(0, 0, 0, wq[0]);
    issue(0, 0, 1, wq[1]);
    issue(0, 1, 0, wq[2]);
    for (; group < n_groups; group += gridDim.x) {
        f32x16 yacc[2][NBW];
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int j = 0; j < NBW; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) yacc[e][j][v] = 0.f;
        for (int cb = 0; cb < NCB; ++cb) {
            __syncthreads();  // (A) this step's X blocks are in LDS; the exchange buffer is free
            // ---- stage 1: U^T_{e, wave} of the block, example by example.  Every MFMA needs a fresh A fragment from LDS:
            // the fragments are requested four MFMAs ahead (left to the compiler they were read one at a time, each
            // MFMA behind the full latency of its own read)
            if (wave < k) {
                constexpr int AHEAD = 4, TOTAL = SKF_EX * KS;
                bf16x8 af[AHEAD];
                auto read_a = [&](int idx, bf16x8& dst) {
                    const int e = idx / KS, ks = idx % KS;
                    const char* src = ldsX + e * XBYTES + (ks >> 1) * L::TILE_BYTES + (ks & 1) * 16 * L::ROW_BYTES + xrd;
                    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src));
                    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, src + 8 * L::ROW_BYTES));
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    dst = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
                    asm volatile("" ::: "memory");
                };
#pragma unroll
                for (int q = 0; q < AHEAD; ++q) read_a(q, af[q]);
                f32x16 uacc;
#pragma unroll
                for (int idx = 0; idx < TOTAL; ++idx) {
                    const int e = idx / KS, ks = idx % KS;
                    if (ks == 0) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) uacc[v] = 0.f;
                    }
                    const bf16x8 a = af[idx % AHEAD];
                    if (idx + AHEAD < TOTAL) read_a(idx + AHEAD, af[idx % AHEAD]);
                    uacc = mfma32(a, zf[ks], uacc);
                    if (ks == KS - 1) {
#pragma unroll
                        for (int cc = 0; cc < 2; ++cc) {
                            bf16x8 pk;
#pragma unroll
                            for (int q = 0; q < 8; ++q) pk[q] = (bf16_t)uacc[8 * cc + q];
                            *(bf16x8*)(ldsU + (((e * 8 + wave) * 2 + cc) * FRAG) + lane * 16) = pk;
                        }
                    }
                }
            }
            __syncthreads();  // (B) every U^T fragment of the step is in the exchange buffer; the X blocks are dead
            {   // the next step's blocks set out
                const bool same = cb + 1 < NCB;
                const int64_t ng_ = same ? group : group + gridDim.x;
                if (ng_ < n_groups) send_x(ng_, same ? cb + 1 : 0);
            }
            // ---- stage 2: Y^T_e[channels of group ng] += W_i^T[.., block] U^T_{e, i} over all factors, e = 2 eh, 2 eh + 1.  A
            // factor has two fragment steps cc (halves of the block) of NBW W fragments each; the fragments travel three
            // steps ahead of their use in a ring of four register sets, and the empty statements keep the compiler from
            // sinking the loads to their use (it would then wait for every single one).  The Z fragments of the next
            // stage 1 are requested behind the last factor, the X blocks of the step after the next at the very end.
            {
                // the U^T fragments of both examples for step (i, cc): requested one step ahead of their use
                bf16x8 ubq[2][2];
                auto fetch_u = [&](int i, int cc, bf16x8 (&dst)[2]) {
                    i = i < k ? i : k - 1;
                    dst[0] = *(const bf16x8*)(ldsU + ((((2 * eh) * 8 + i) * 2 + cc) * FRAG) + lane * 16);
                    dst[1] = *(const bf16x8*)(ldsU + ((((2 * eh + 1) * 8 + i) * 2 + cc) * FRAG) + lane * 16);
                };
                auto compute = [&](const bf16x8 (&ub)[2], const bf16x8 (&wa)[NBW]) {
#pragma unroll
                    for (int j = 0; j < NBW; ++j) {
                        yacc[0][j] = mfma32(wa[j], ub[0], yacc[0][j]);
                        yacc[1][j] = mfma32(wa[j], ub[1], yacc[1][j]);
                    }
                };
                fetch_u(0, 0, ubq[0]);
                for (int i0 = 0; i0 < k; i0 += 2) {
                    const bool two = i0 + 1 < k;
                    issue(cb, i0 + 1, 1, wq[3]);
                    fetch_u(i0, 1, ubq[1]);
                    compute(ubq[0], wq[0]);
                    issue(cb, i0 + 2, 0, wq[0]);
                    fetch_u(i0 + 1, 0, ubq[0]);
                    compute(ubq[1], wq[1]);
                    issue(cb, i0 + 2, 1, wq[1]);
                    fetch_u(i0 + 1, 1, ubq[1]);
                    if (two) compute(ubq[0], wq[2]);
                    issue(cb, i0 + 3, 0, wq[2]);
                    fetch_u(i0 + 2, 0, ubq[0]);
                    if (two) compute(ubq[1], wq[3]);
                }
            }
            // the X blocks have landed: they are older than every W fragment, and at most the three fragment steps
            // requested for the next block are still on their way
            wait_vmcnt<3 * NBW>();
        }
        // ---- output: lane holds column t = r of Y^T, rows n = 32*(NBW*ng + j) + 8*(v/4) + 4g + v%4
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int64_t b = group * SKF_EX + 2 * eh + e;
            if (b < B) {
                bf16_t* yrow = y + (b * SKF_T + r) * D + 32 * NBW * ng + 4 * g;
#pragma unroll
                for (int j = 0; j < NBW; ++j)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        bf16x4 out;
#pragma unroll
                        for (int q = 0; q < 4; ++q) out[q] = (bf16_t)yacc[e][j][4 * vg + q];
                        *(bf16x4*)(yrow + 32 * j + 8 * vg) = out;
                    }
            }
        }
    }
}

bool sumkron_fused_supported(int S, int T, int D, int k, int dtype) {
    return dtype == KUNLUN_BF16 && T == SKF_T && (S == 128 || S == 256) && D % 128 == 0 && D >= 128 && D <= 384 && k >= 1 && k <= SKF_WAVES;
}

size_t sumkron_fused_workspace(int S, int T, int D, int k) {
    return align_up((size_t)k * T * S * 2, 256) + align_up((size_t)k * D * D * 2, 256);
}

template <int NBW, int S>
static hipError_t launch_skf(const bf16_t* x, const bf16_t* zt, const bf16_t* wp, bf16_t* y, int B, int k, hipStream_t stream) {
    constexpr int bytes = SKF_EX * S * SKF_CB * 2 + SKF_EX * 8 * 2 * 1024;
    auto kern = sumkron_fused_kernel<NBW, S>;
    // once per process (thread-safe initialisation of a function-local static); not a stream operation
    static const hipError_t raised = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (raised != hipSuccess) return raised;
    const int64_t n_groups = ((int64_t)B + SKF_EX - 1) / SKF_EX;
    const int64_t resident = compute_units();
    hipLaunchKernelGGL(kern, dim3((unsigned)(n_groups < resident ? n_groups : resident)), dim3(64 * SKF_WAVES), bytes, stream, x, zt, wp, y, B, k);
    return hipGetLastError();
}

// workspace: sumkron_fused_workspace(...) bytes (prepared Z, prepared W)
hipError_t launch_sumkron_fused(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k, void* workspace,
                                hipStream_t stream) {
    bf16_t* zt = (bf16_t*)workspace;
    bf16_t* wp = (bf16_t*)((char*)workspace + align_up((size_t)k * T * S * 2, 256));
    const int64_t nz = (int64_t)k * S * T, nw = (int64_t)k * D * D;
    hipLaunchKernelGGL(skf_prepare_z_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, stream, (const bf16_t*)z, zt, k, S, T);
    hipLaunchKernelGGL(skf_prepare_w_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, stream, (const bf16_t*)w, wp, k, D);
    const bf16_t* xb = (const bf16_t*)x;
    bf16_t* yb = (bf16_t*)y;
    const int nbw = D / 128;
#define KUNLUN_SKF(NBW_) (S == 256 ? launch_skf<NBW_, 256>(xb, zt, wp, yb, B, k, stream) : launch_skf<NBW_, 128>(xb, zt, wp, yb, B, k, stream))
    switch (nbw) {
    case 1: return KUNLUN_SKF(1);
    case 2: return KUNLUN_SKF(2);
    default: return KUNLUN_SKF(3);  // (D = 512 does not fit the registers of a wave: the two-GEMM path takes it)
    }
#undef KUNLUN_SKF
}

}  // namespace kunlun
