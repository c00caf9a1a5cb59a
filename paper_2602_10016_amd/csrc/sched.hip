// Offsets-driven work ordering (the software tile scheduler of App. "GDPA and Fused PFFN
// Kernel": sequence-length metadata decides the order in which work items are issued, so
// that the long histories start first and the short ones fill the tail).
//
// One workgroup sorts the examples by history length, longest first, with a counting sort
// over NBINS length buckets.  The attention kernels launch one workgroup per
// (example, head, query tile) in that order; the hardware dispatcher hands them to compute
// units as slots free up, which is longest-processing-time-first list scheduling.
// Results never depend on the order: each work item is computed by exactly one wavefront.
#include "common.h"

namespace kunlun {

constexpr int NBINS = 2048;
constexpr int SCHED_THREADS = 1024;

__global__ __launch_bounds__(SCHED_THREADS) void schedule_kernel(const int32_t* __restrict__ kv_off, int B,
                                                                  int max_kv, int32_t* __restrict__ order,
                                                                  int32_t* __restrict__ counters) {
    __shared__ int hist[NBINS];
    __shared__ int scan[NBINS];
    const int tid = threadIdx.x;
    if (tid < (int)(WS_HEADER_BYTES / sizeof(int32_t))) counters[tid] = 0;
    for (int i = tid; i < NBINS; i += SCHED_THREADS) hist[i] = 0;
    __syncthreads();
    const int64_t span = (int64_t)max_kv + 1;
    auto bin_of = [&](int b) {
        int64_t len = (int64_t)kv_off[b + 1] - kv_off[b];
        int64_t x = len * NBINS / span;
        if (x > NBINS - 1) x = NBINS - 1;
        if (x < 0) x = 0;
        return NBINS - 1 - (int)x;  // bin 0 = longest
    };
    for (int b = tid; b < B; b += SCHED_THREADS) atomicAdd(&hist[bin_of(b)], 1);
    __syncthreads();
    // exclusive scan of hist (Hillis-Steele over NBINS entries, two per thread)
    for (int i = tid; i < NBINS; i += SCHED_THREADS) scan[i] = hist[i];
    __syncthreads();
    for (int off = 1; off < NBINS; off <<= 1) {
        int v0 = 0, v1 = 0;
        const int i0 = tid, i1 = tid + SCHED_THREADS;
        if (i0 >= off) v0 = scan[i0 - off];
        if (i1 >= off) v1 = scan[i1 - off];
        __syncthreads();
        scan[i0] += v0;
        scan[i1] += v1;
        __syncthreads();
    }
    // scan is inclusive; bucket start = scan - hist.  Reuse hist as the running cursor.
    for (int i = tid; i < NBINS; i += SCHED_THREADS) hist[i] = scan[i] - hist[i];
    __syncthreads();
    for (int b = tid; b < B; b += SCHED_THREADS) {
        const int pos = atomicAdd(&hist[bin_of(b)], 1);
        order[pos] = b;
    }
}

// Debug aid: counts the ways in which an offsets array breaks the contract (offsets[0] = 0, lengths in
// [0, max_len], offsets[B] = total); one workgroup, deterministic.
__global__ __launch_bounds__(SCHED_THREADS) void check_offsets_kernel(const int32_t* __restrict__ off, int B, int64_t total,
                                                                       int max_len, int32_t* __restrict__ violations) {
    __shared__ int bad[SCHED_THREADS];
    const int tid = threadIdx.x;
    int n = 0;
    for (int b = tid; b < B; b += SCHED_THREADS) {
        const int64_t len = (int64_t)off[b + 1] - off[b];
        n += (len < 0 || len > max_len) ? 1 : 0;
    }
    if (tid == 0) n += (off[0] != 0 ? 1 : 0) + ((int64_t)off[B] != total ? 1 : 0);
    bad[tid] = n;
    __syncthreads();
    for (int s = SCHED_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) bad[tid] += bad[tid + s];
        __syncthreads();
    }
    if (tid == 0) *violations = bad[0];
}

hipError_t launch_check_offsets(const int32_t* off, int B, int64_t total, int max_len, int32_t* violations, hipStream_t stream) {
    hipLaunchKernelGGL(check_offsets_kernel, dim3(1), dim3(SCHED_THREADS), 0, stream, off, B, total, max_len, violations);
    return hipGetLastError();
}

// MI355X has 256 compute units.
bool schedule_is_moot(int64_t workgroups, int wgs_per_cu) { return workgroups <= (int64_t)wgs_per_cu * 256; }

hipError_t launch_schedule(const int32_t* kv_off, int B, int max_kv, int32_t* order, int32_t* counters, hipStream_t stream) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(SCHED_THREADS), 0, stream, kv_off, B, max_kv, order, counters);
    return hipGetLastError();
}

int compute_units() {
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;  // MI355X
        return cus;
    }();
    return n;
}

}  // namespace kunlun

namespace kunlun {

// ---- gradient of batch-shared seed queries (Sec. "Hierarchical Seed Pooling", stage 1: the learnable seeds are
// shared by all examples, so their gradient is the sum of the per-example query gradients).  No atomics: the
// order of every addition is fixed by (group, example), so the result does not depend on the launch.
// V consecutive elements per thread (16-byte loads when the row length allows it); the additions of one element
// happen in example order whatever V is.
template <typename T, int V>
__global__ __launch_bounds__(256) void seed_grad_group_kernel(const T* __restrict__ rows, float* __restrict__ partial, int B,
                                                              int64_t n_elems) {
    typedef T vec_t __attribute__((ext_vector_type(V)));
    const int64_t n = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V;
    const int group = blockIdx.y;
    if (n >= n_elems) return;
    const int b0 = group * SEED_GROUP, b1 = b0 + SEED_GROUP < B ? b0 + SEED_GROUP : B;
    float acc[V];
#pragma unroll
    for (int q = 0; q < V; ++q) acc[q] = 0.f;
#pragma unroll 4
    for (int b = b0; b < b1; ++b) {
        const vec_t x = *(const vec_t*)(rows + (int64_t)b * n_elems + n);
#pragma unroll
        for (int q = 0; q < V; ++q) acc[q] += to_float((T)x[q]);
    }
#pragma unroll
    for (int q = 0; q < V; ++q) partial[(int64_t)group * n_elems + n + q] = acc[q];
}
template <typename T>
__global__ __launch_bounds__(256) void seed_grad_final_kernel(const float* __restrict__ partial, T* __restrict__ d_e, int groups,
                                                              int64_t n_elems) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= n_elems) return;
    float acc = 0.f;
    for (int g = 0; g < groups; ++g) acc += partial[(int64_t)g * n_elems + n];
    d_e[n] = from_float<T>(acc);
}

hipError_t launch_seed_grad_sum(const void* rows, void* d_e, float* partial, int B, int64_t n_elems, int dtype, hipStream_t stream) {
    if (n_elems <= 0) return hipSuccess;
    const int groups = (B + SEED_GROUP - 1) / SEED_GROUP;
    const dim3 grid2((unsigned)((n_elems + 255) / 256));
    auto grid1 = [&](int v) { return dim3((unsigned)((n_elems / v + 255) / 256), (unsigned)groups); };
    if (dtype == KUNLUN_FP32) {
        if (n_elems % 4 == 0 && (reinterpret_cast<uintptr_t>(rows) % 16 == 0))
            hipLaunchKernelGGL((seed_grad_group_kernel<float, 4>), grid1(4), dim3(256), 0, stream, (const float*)rows, partial, B, n_elems);
        else
            hipLaunchKernelGGL((seed_grad_group_kernel<float, 1>), grid1(1), dim3(256), 0, stream, (const float*)rows, partial, B, n_elems);
        hipLaunchKernelGGL(seed_grad_final_kernel<float>, grid2, dim3(256), 0, stream, partial, (float*)d_e, groups, n_elems);
    } else {
        if (n_elems % 8 == 0 && (reinterpret_cast<uintptr_t>(rows) % 16 == 0))
            hipLaunchKernelGGL((seed_grad_group_kernel<bf16_t, 8>), grid1(8), dim3(256), 0, stream, (const bf16_t*)rows, partial, B, n_elems);
        else
            hipLaunchKernelGGL((seed_grad_group_kernel<bf16_t, 1>), grid1(1), dim3(256), 0, stream, (const bf16_t*)rows, partial, B, n_elems);
        hipLaunchKernelGGL(seed_grad_final_kernel<bf16_t>, grid2, dim3(256), 0, stream, partial, (bf16_t*)d_e, groups, n_elems);
    }
    return hipGetLastError();
}

}  // namespace kunlun
