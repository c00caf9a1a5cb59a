// Shared declarations of the Kunlun attention kernels (device side) and their host launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kunlun.h"

namespace kunlun {

typedef __bf16 bf16_t;

// Everything a kernel needs, passed by value as the single kernel argument.
struct AttnParams {
    const void* q;
    const void* k;
    const void* v;
    void* o;           // forward output, or the forward result read by the softmax backward
    float* lse;        // [H, total_q]; may be null in the forward pass
    const void* d_o;   // backward only
    void* dq;
    void* dk;
    void* dv;
    const int32_t* q_off;   // null: dense queries, max_q rows per example
    const int32_t* kv_off;
    const int32_t* order;   // examples, longest history first (written by the scheduler kernel); null: 0..B-1
    int32_t* queue;         // work counter of a persistent launch (zeroed by the scheduler kernel); null: one item per workgroup
    int B, H, d, max_q, max_kv;
    int64_t total_q, total_kv;
    float scale;
    int windowed, left, right;  // sliding window (self-attention); left/right < 0: unbounded
    int q_shared;               // 1: q holds ONE block of max_q rows that every example uses (batch-shared seed queries)
    uint8_t head_act[KUNLUN_MAX_HEADS];
};

// Workspace layout (bytes from the start of the caller's workspace).
constexpr size_t WS_HEADER_BYTES = 256;  // counters
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// kunlun_gdpa_fwd with one more argument: launch = false validates only (nothing enqueued, no device touched).
int gdpa_fwd_checked(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                     const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv,
                     float scale, int act, const int32_t* head_act, int dtype, void* workspace, size_t workspace_bytes,
                     void* stream, bool launch, bool q_shared);

// Gradient of batch-shared seed queries: d_e[n] = sum over the B examples of rows[b * n_elems + n] (rows: the
// per-example query gradients, `dtype` elements), in a fixed order - examples in groups of SEED_GROUP, each group
// summed in example order into an fp32 partial sum, the partial sums added in group order, rounded once.
constexpr int SEED_GROUP = 32;
inline size_t seed_grad_rows_bytes(int64_t total_q, int H, int d, int dtype) {
    return align_up((size_t)total_q * H * d * (dtype == KUNLUN_FP32 ? 4 : 2), 256);
}
inline size_t seed_grad_partial_bytes(int B, int64_t n_elems) {
    return align_up((size_t)((B + SEED_GROUP - 1) / SEED_GROUP) * n_elems * sizeof(float), 256);
}
hipError_t launch_seed_grad_sum(const void* rows, void* d_e, float* partial, int B, int64_t n_elems, int dtype, hipStream_t stream);

// ---- launchers (each enqueues on `stream`, returns the hipError_t of the launch) ----
// Sorts the examples by length (longest first) into order[B] and zeroes the WS_HEADER_BYTES of work counters at
// `counters` (the start of the workspace) for the persistent kernels that follow on the stream.
hipError_t launch_schedule(const int32_t* kv_off, int B, int max_kv, int32_t* order, int32_t* counters, hipStream_t stream);
// Compute units of the current device (cached per process).
int compute_units();
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
hipError_t launch_stream_probe(const void* a, const void* b, const void* c, void* out, size_t bytes, int reads, int write,
                               hipStream_t stream);
// x = a, y = b ^ c over the d-channel pieces of every (example, head) item (bf16 rows of H * d channels), items in
// `order`, handed out by `queue`; writes: 0 none, 1 out_a = x ^ y, 2 out_a = x and out_b = y (writes = 2 needs reads >= 2)
hipError_t launch_jagged_probe(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* order,
                               const int32_t* off, int B, int H, int d, int32_t* queue, int reads, int writes, int wgs_per_cu,
                               hipStream_t stream);
hipError_t launch_check_offsets(const int32_t* off, int B, int64_t total, int max_len, int32_t* violations, hipStream_t stream);
// True when the launch is so small that every workgroup is resident at once (wgs_per_cu = how
// many workgroups of the kernel fit one compute unit): the issue order then has no effect and
// the sorting kernel is skipped.
bool schedule_is_moot(int64_t workgroups, int wgs_per_cu);
hipError_t launch_scalar_fwd(const AttnParams& p, int dtype, hipStream_t stream);
hipError_t launch_scalar_bwd(const AttnParams& p, int dtype, hipStream_t stream);
bool mfma_fwd_supported(const AttnParams& p, int dtype);
hipError_t launch_mfma_fwd(const AttnParams& p, hipStream_t stream);
// True when the forward launch walks query tiles (window op, or more than 64 queries per
// example): the workspace then holds query-tile prefix sums instead of the sorted example order.
bool mfma_fwd_is_qtiled(const AttnParams& p);
// p.order points at tile_table_bytes(B, total_q) bytes (tile_map.h): prefix sums, then the example of every query tile
hipError_t launch_mfma_fwd_qtiled(const AttnParams& p, hipStream_t stream);
// Sliding window with a bounded, narrow window and many (sequence, head) items: one workgroup walks one item,
// its waves rotate through the query blocks (attn_swa_band_mfma.hip).  p.order: sequences, longest first.
bool swa_band_applies(const AttnParams& p);
hipError_t launch_swa_band_fwd(const AttnParams& p, hipStream_t stream);
bool mfma_bwd_supported(const AttnParams& p, int dtype);
hipError_t launch_mfma_bwd(const AttnParams& p, void* workspace_tail, hipStream_t stream);
size_t mfma_bwd_workspace_tail(int B, int H, int d, int max_q, int64_t total_q);
// d = 128 with 33..64 queries per example: wave pairs share each key tile (two workgroups per compute unit).
hipError_t launch_mfma_bwd_pair(const AttnParams& p, hipStream_t stream);
// Two-pass matrix-core backward (sliding window, or more than 64 queries per example).
bool mfma_bwd_tiled_supported(const AttnParams& p, int dtype);
size_t mfma_bwd_tiled_workspace(int B, int H, int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, bool windowed);
hipError_t launch_mfma_bwd_tiled(const AttnParams& p, void* workspace_tail, bool any_softmax, hipStream_t stream);

// SumKronLinear (two tiled GEMMs with a bf16 intermediate, or plain fp32 kernels)
size_t sumkron_workspace(int B, int S, int T, int D, int k, int dtype);
// One-kernel forward for T = 32, S in {128, 256}, D in {128, 256, 384}, k <= 8 (sumkron_fused.hip)
bool sumkron_fused_supported(int S, int T, int D, int k, int dtype);
size_t sumkron_fused_workspace(int S, int T, int D, int k);
hipError_t launch_sumkron_fused(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k, void* workspace,
                                hipStream_t stream);
hipError_t launch_sumkron(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k,
                          int dtype, void* workspace, hipStream_t stream);
bool sumkron_bwd_tiled_supported(int B, int S, int T, int D, int k, int dtype);
size_t sumkron_bwd_workspace(int B, int S, int T, int D, int k, int dtype);
hipError_t launch_sumkron_bwd(const void* x, const void* z, const void* w, const void* dy, void* dx, void* dz, void* dw, int B,
                              int S, int T, int D, int k, int dtype, void* workspace, hipStream_t stream);

#ifdef __HIPCC__
// ---- device helpers ----

__device__ __forceinline__ int64_t q_begin(const AttnParams& p, int b) {
    return p.q_off ? (int64_t)p.q_off[b] : (int64_t)b * p.max_q;
}
__device__ __forceinline__ int64_t q_end(const AttnParams& p, int b) {
    return p.q_off ? (int64_t)p.q_off[b + 1] : (int64_t)(b + 1) * p.max_q;
}
// Row of the q tensor that holds query `row` (a row of o, d_o, dq and lse, numbered over the whole batch): the
// same row, unless the batch shares one block of max_q seed queries (dense queries then: example b owns rows
// b * max_q ..), where it is the row's position inside its example.
__device__ __forceinline__ int64_t q_src_row(const AttnParams& p, int64_t row) { return p.q_shared ? row % p.max_q : row; }

// Largest b in [0, B) with off[b] <= row (rows of empty examples are skipped naturally).
__device__ __forceinline__ int find_example(const int32_t* off, int B, int64_t row) {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if ((int64_t)off[mid] <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// The polynomial GELU of include/kunlun.h: cdf(x) = 1/2 + t q(t^2), t = x clamped to [-C, C], and the slope of
// the cdf (0 outside (-C, C)).  Plain fused multiply-adds, no transcendental (App. "GDPA and Fused PFFN Kernel").
constexpr float GELU_POLY_C = 3.875f;
__device__ __forceinline__ float gelu_poly_cdf(float x, float& slope) {
    constexpr float A0 = 3.9862210505e-01f, A1 = -6.5595134356e-02f, A2 = 9.2376422360e-03f, A3 = -9.1053389233e-04f,
                    A4 = 5.8010079080e-05f, A5 = -2.1110704002e-06f, A6 = 3.2949778488e-08f;
    const float t = __builtin_amdgcn_fmed3f(x, -GELU_POLY_C, GELU_POLY_C);
    const float u = t * t;
    float q = fmaf(u, A6, A5);
    q = fmaf(u, q, A4);
    q = fmaf(u, q, A3);
    q = fmaf(u, q, A2);
    q = fmaf(u, q, A1);
    q = fmaf(u, q, A0);
    float dq = fmaf(u, 6.f * A6, 5.f * A5);  // q'(u)
    dq = fmaf(u, dq, 4.f * A4);
    dq = fmaf(u, dq, 3.f * A3);
    dq = fmaf(u, dq, 2.f * A2);
    dq = fmaf(u, dq, A1);
    slope = (x > -GELU_POLY_C && x < GELU_POLY_C) ? fmaf(2.f * u, dq, q) : 0.f;
    return fmaf(t, q, 0.5f);
}

// Exact score functions (fp32 path): definitions as in include/kunlun.h.
template <int ACT>
__device__ __forceinline__ float act_exact(float x) {
    if constexpr (ACT == KUNLUN_ACT_IDENTITY) return x;
    if constexpr (ACT == KUNLUN_ACT_RELU) return x > 0.f ? x : 0.f;
    if constexpr (ACT == KUNLUN_ACT_GELU) return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    if constexpr (ACT == KUNLUN_ACT_GELU_TANH) {
        float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
        return 0.5f * x * (1.f + tanhf(u));
    }
    if constexpr (ACT == KUNLUN_ACT_SILU) return x / (1.f + expf(-x));
    if constexpr (ACT == KUNLUN_ACT_GELU_POLY) {
        float slope;
        return x * gelu_poly_cdf(x, slope);
    }
    return 0.f;
}

template <int ACT>
__device__ __forceinline__ float act_deriv_exact(float x) {
    if constexpr (ACT == KUNLUN_ACT_IDENTITY) return 1.f;
    if constexpr (ACT == KUNLUN_ACT_RELU) return x > 0.f ? 1.f : 0.f;
    if constexpr (ACT == KUNLUN_ACT_GELU) {
        float cdf = 0.5f * (1.f + erff(x * 0.70710678118654752f));
        float pdf = 0.39894228040143268f * expf(-0.5f * x * x);
        return cdf + x * pdf;
    }
    if constexpr (ACT == KUNLUN_ACT_GELU_TANH) {
        float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
        float t = tanhf(u);
        float du = 0.79788456080286536f * (1.f + 3.f * 0.044715f * x * x);
        return 0.5f * (1.f + t) + 0.5f * x * (1.f - t * t) * du;
    }
    if constexpr (ACT == KUNLUN_ACT_SILU) {
        float s = 1.f / (1.f + expf(-x));
        return s + x * s * (1.f - s);
    }
    if constexpr (ACT == KUNLUN_ACT_GELU_POLY) {
        float slope;
        const float cdf = gelu_poly_cdf(x, slope);
        return fmaf(x, slope, cdf);
    }
    return 0.f;
}

__device__ __forceinline__ float act_exact_rt(int act, float x) {
    switch (act) {
    case KUNLUN_ACT_IDENTITY: return act_exact<KUNLUN_ACT_IDENTITY>(x);
    case KUNLUN_ACT_RELU: return act_exact<KUNLUN_ACT_RELU>(x);
    case KUNLUN_ACT_GELU: return act_exact<KUNLUN_ACT_GELU>(x);
    case KUNLUN_ACT_GELU_TANH: return act_exact<KUNLUN_ACT_GELU_TANH>(x);
    case KUNLUN_ACT_SILU: return act_exact<KUNLUN_ACT_SILU>(x);
    default: return act_exact<KUNLUN_ACT_GELU_POLY>(x);
    }
}
__device__ __forceinline__ float act_deriv_exact_rt(int act, float x) {
    switch (act) {
    case KUNLUN_ACT_IDENTITY: return act_deriv_exact<KUNLUN_ACT_IDENTITY>(x);
    case KUNLUN_ACT_RELU: return act_deriv_exact<KUNLUN_ACT_RELU>(x);
    case KUNLUN_ACT_GELU: return act_deriv_exact<KUNLUN_ACT_GELU>(x);
    case KUNLUN_ACT_GELU_TANH: return act_deriv_exact<KUNLUN_ACT_GELU_TANH>(x);
    case KUNLUN_ACT_SILU: return act_deriv_exact<KUNLUN_ACT_SILU>(x);
    default: return act_deriv_exact<KUNLUN_ACT_GELU_POLY>(x);
    }
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { return (bf16_t)x; }
#endif  // __HIPCC__

}  // namespace kunlun
