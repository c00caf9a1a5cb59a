// Measurement aids, no part of any operator: plain streaming kernels that move the bytes of an attention call
// without its arithmetic, to calibrate what the memory system sustains (a) for a read : write mix and (b) for the
// access pattern of the jagged calls - one independent walker per (example, head), each reading and writing the
// d-channel pieces of consecutive token rows of its own history.
#include "common.h"

namespace kunlun {

// ---- streaming probe: what this memory system sustains for a given read : write mix (calibration of the HBM
// roof that the attention calls are held against).  Block b handles the 16 KB segment b of every stream: `reads`
// (1..3) streams are read with non-temporal loads and combined, the result is written to `out` when `write` is
// set, else folded into a value that is never stored.  The fastest of the access patterns tried on this device.
template <int NR, bool WRITE>
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4_t* __restrict__ a, const u32x4_t* __restrict__ b,
                                                           const u32x4_t* __restrict__ c, u32x4_t* __restrict__ out, size_t n16) {
    const size_t s0 = (size_t)blockIdx.x * 1024;
    u32x4_t acc = {0, 0, 0, 0};
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const size_t j = s0 + u * 256 + threadIdx.x;
        if (j < n16) {
            v[u] = __builtin_nontemporal_load(a + j);
            if (NR > 1) v[u] ^= __builtin_nontemporal_load(b + j);
            if (NR > 2) v[u] ^= __builtin_nontemporal_load(c + j);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const size_t j = s0 + u * 256 + threadIdx.x;
        if (j < n16) {
            if (WRITE) __builtin_nontemporal_store(v[u], out + j);
            else acc ^= v[u];
        }
    }
    if (!WRITE && acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u) out[threadIdx.x] = acc;  // (keeps the loads alive)
}

hipError_t launch_stream_probe(const void* a, const void* b, const void* c, void* out, size_t bytes, int reads, int write,
                               hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const dim3 grid((unsigned)((n16 + 1023) / 1024)), block(256);
    const u32x4_t *pa = (const u32x4_t*)a, *pb = (const u32x4_t*)b, *pc = (const u32x4_t*)c;
    u32x4_t* po = (u32x4_t*)out;
    if (write) {
        if (reads == 1) hipLaunchKernelGGL((stream_probe_kernel<1, true>), grid, block, 0, stream, pa, pb, pc, po, n16);
        else if (reads == 2) hipLaunchKernelGGL((stream_probe_kernel<2, true>), grid, block, 0, stream, pa, pb, pc, po, n16);
        else hipLaunchKernelGGL((stream_probe_kernel<3, true>), grid, block, 0, stream, pa, pb, pc, po, n16);
    } else {
        if (reads == 1) hipLaunchKernelGGL((stream_probe_kernel<1, false>), grid, block, 0, stream, pa, pb, pc, po, n16);
        else if (reads == 2) hipLaunchKernelGGL((stream_probe_kernel<2, false>), grid, block, 0, stream, pa, pb, pc, po, n16);
        else hipLaunchKernelGGL((stream_probe_kernel<3, false>), grid, block, 0, stream, pa, pb, pc, po, n16);
    }
    return hipGetLastError();
}


// ---- jagged probe.  Work items = (example, head) in the scheduler's order, handed out by the work counter to a
// persistent launch, exactly as in the attention kernels.  A workgroup walks its item in steps of 4 * (256 / CH)
// rows (CH = 16-byte chunks of a d-channel piece), two steps of loads in flight; x = a, y = b ^ c (what is read
// of them): writes = 1 stores x ^ y to out_a, writes = 2 stores x to out_a and y to out_b, writes = 0 folds
// everything into a value that goes nowhere.
template <int CH, int NR, int NWR>
__global__ __launch_bounds__(256) void jagged_probe_kernel(const char* __restrict__ a, const char* __restrict__ b,
                                                           const char* __restrict__ c, char* __restrict__ out_a,
                                                           char* __restrict__ out_b, const int32_t* __restrict__ order,
                                                           const int32_t* __restrict__ off, int B, int H, int32_t* queue,
                                                           int n_items) {
    extern __shared__ char smem[];  // sized by the launcher to set the number of resident workgroups
    constexpr int RP = 256 / CH;    // rows per load instruction
    constexpr int STEP = 4 * RP;
    const int tid = threadIdx.x, row = tid / CH, ch = tid % CH;
    const size_t row_bytes = (size_t)H * CH * 16;
    u32x4_t sink = {0, 0, 0, 0};
    int item = blockIdx.x;
    while (item < n_items) {
        int claimed = 0;
        if (tid == 0) claimed = atomicAdd(queue, 1);
        const int h = (item >> 3) % H, e = ((item >> 3) / H) * 8 + (item & 7);
        if (e < B) {
            const int ex = order[e];
            const int r0 = off[ex], n = off[ex + 1] - r0;
            const size_t base = (size_t)r0 * row_bytes + ((size_t)h * CH + ch) * 16;
            const int steps = (n + STEP - 1) / STEP;
            u32x4_t x[2][4], y[2][4];
            auto fetch = [&](int t, u32x4_t* xs, u32x4_t* ys) {
                if (t >= steps) return;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int r = t * STEP + i * RP + row;
                    r = r < n ? r : n - 1;  // (rows past the end re-read the last row; they are never stored)
                    const size_t o = base + (size_t)r * row_bytes;
                    xs[i] = __builtin_nontemporal_load((const u32x4_t*)(a + o));
                    if (NR > 1) ys[i] = __builtin_nontemporal_load((const u32x4_t*)(b + o));
                    if (NR > 2) ys[i] ^= __builtin_nontemporal_load((const u32x4_t*)(c + o));
                }
            };
            auto drain = [&](int t, u32x4_t* xs, u32x4_t* ys) {
                if (t >= steps) return;
                u32x4_t xv[4], yv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { xv[i] = xs[i]; yv[i] = NR > 1 ? ys[i] : (u32x4_t){0, 0, 0, 0}; }
                fetch(t + 2, xs, ys);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = t * STEP + i * RP + row;
                    const size_t o = base + (size_t)r * row_bytes;
                    if (NWR == 0) sink ^= xv[i] ^ yv[i];
                    if (NWR == 1 && r < n) __builtin_nontemporal_store(xv[i] ^ yv[i], (u32x4_t*)(out_a + o));
                    if (NWR == 2 && r < n) {
                        __builtin_nontemporal_store(xv[i], (u32x4_t*)(out_a + o));
                        __builtin_nontemporal_store(yv[i], (u32x4_t*)(out_b + o));
                    }
                }
            };
            if (n > 0) {
                fetch(0, x[0], y[0]);
                fetch(1, x[1], y[1]);
                for (int t = 0; t < steps; t += 2) {
                    drain(t, x[0], y[0]);
                    drain(t + 1, x[1], y[1]);
                }
            }
        }
        __syncthreads();
        if (tid == 0) *(volatile int*)smem = claimed + (int)gridDim.x;
        __syncthreads();
        item = __builtin_amdgcn_readfirstlane(*(volatile int*)smem);
        __syncthreads();
    }
    if (NWR == 0 && sink[0] == 0x9e3779b9u && sink[1] == 0x7f4a7c15u) queue[1 + (tid & 31)] = (int32_t)sink[2];  // (keeps the loads alive)
}

template <int CH, int NR, int NWR>
static hipError_t launch_jagged_probe_t(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* order,
                                        const int32_t* off, int B, int H, int32_t* queue, int wgs_per_cu, hipStream_t stream) {
    auto kern = jagged_probe_kernel<CH, NR, NWR>;
    // the LDS request sets how many workgroups a compute unit holds (160 KB each); the kernel uses four bytes of it
    const int lds = (160 * 1024 / wgs_per_cu) & ~1023;
    static const hipError_t raised = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (raised != hipSuccess) return raised;
    const int n_items = (B + 7) / 8 * 8 * H;
    const int64_t resident = (int64_t)wgs_per_cu * compute_units();
    const unsigned grid = (unsigned)(n_items < resident ? n_items : resident);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, (const char*)a, (const char*)b, (const char*)c, (char*)out_a,
                       (char*)out_b, order, off, B, H, queue, n_items);
    return hipGetLastError();
}

template <int CH>
static hipError_t launch_jagged_probe_ch(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* order,
                                         const int32_t* off, int B, int H, int32_t* queue, int reads, int writes, int wgs_per_cu,
                                         hipStream_t s) {
#define KUNLUN_JP(NR, NWR) launch_jagged_probe_t<CH, NR, NWR>(a, b, c, out_a, out_b, order, off, B, H, queue, wgs_per_cu, s)
    switch (reads * 3 + writes) {
    case 3: return KUNLUN_JP(1, 0);
    case 4: return KUNLUN_JP(1, 1);
    case 6: return KUNLUN_JP(2, 0);
    case 7: return KUNLUN_JP(2, 1);
    case 8: return KUNLUN_JP(2, 2);
    case 9: return KUNLUN_JP(3, 0);
    case 10: return KUNLUN_JP(3, 1);
    case 11: return KUNLUN_JP(3, 2);
    default: return hipErrorInvalidValue;
    }
#undef KUNLUN_JP
}

hipError_t launch_jagged_probe(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* order,
                               const int32_t* off, int B, int H, int d, int32_t* queue, int reads, int writes, int wgs_per_cu,
                               hipStream_t s) {
    if (d == 128) return launch_jagged_probe_ch<16>(a, b, c, out_a, out_b, order, off, B, H, queue, reads, writes, wgs_per_cu, s);
    if (d == 64) return launch_jagged_probe_ch<8>(a, b, c, out_a, out_b, order, off, B, H, queue, reads, writes, wgs_per_cu, s);
    return launch_jagged_probe_ch<4>(a, b, c, out_a, out_b, order, off, B, H, queue, reads, writes, wgs_per_cu, s);
}

}  // namespace kunlun
