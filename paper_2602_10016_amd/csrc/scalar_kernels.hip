// Generic (non matrix-core) kernels: fp32 storage and arithmetic, or any head dimension
// the MFMA kernels do not tile.  One wavefront per output row; lanes run over keys for the
// score dot products and over channels for the weighted sums.  Exact transcendental
// functions.  These kernels serve the fp32 data type and the head dimensions other than 32, 64
// and 128; the bf16 hot path lives in attn_fwd_mfma.hip (streaming forward), attn_fwd_ring_mfma.hip
// (query-tiled forward: sliding window, long query sequences), attn_bwd_pair_mfma.hip /
// attn_bwd_mfma.hip (fused backward) and attn_bwd_tiled_mfma.hip (two-pass and few-keys backward).
//
// Forward: Eq. (GDPA) and softmax attention (Eq. (PMA), Eq. (seed-level attention),
// Eq. (sliding window)).  Backward: gradients of <O, dO>, scores recomputed per row.
#include "common.h"

namespace kunlun {

constexpr int MAX_D = 256;
constexpr int CH = MAX_D / 64;  // channel registers per lane

template <typename T>
__device__ __forceinline__ float row_dot(const float* __restrict__ a_lds, const T* __restrict__ row, int d) {
    float acc = 0.f;
    for (int c = 0; c < d; ++c) acc = fmaf(a_lds[c], to_float(row[c]), acc);
    return acc;
}

__device__ __forceinline__ void window_keys(const AttnParams& p, int64_t t, int64_t n_kv, int64_t& lo, int64_t& hi) {
    lo = 0;
    hi = n_kv - 1;
    if (p.windowed) {
        if (p.left >= 0 && t - p.left > lo) lo = t - p.left;
        if (p.right >= 0 && t + p.right < hi) hi = t + p.right;
    }
}

// One wavefront per (query row, head).
template <typename T>
__global__ __launch_bounds__(64) void scalar_fwd_kernel(AttnParams p) {
    __shared__ float sq[MAX_D];
    __shared__ float sp[64];
    const int lane = threadIdx.x;
    const int64_t item = blockIdx.x;
    const int64_t row = item / p.H;
    const int h = (int)(item % p.H);
    const int d = p.d;
    const int64_t hd = (int64_t)p.H * d;
    const int b = p.q_off ? find_example(p.q_off, p.B, row) : (int)(row / p.max_q);
    const int64_t t = row - q_begin(p, b);
    const int64_t k0 = p.kv_off[b];
    const int64_t n_kv = (int64_t)p.kv_off[b + 1] - k0;
    const int act = p.head_act[h];
    const T* Q = (const T*)p.q;
    const T* K = (const T*)p.k;
    const T* V = (const T*)p.v;
    T* O = (T*)p.o;

    for (int c = lane; c < d; c += 64) sq[c] = to_float(Q[q_src_row(p, row) * hd + (int64_t)h * d + c]);
    __syncthreads();

    int64_t lo, hi;
    window_keys(p, t, n_kv, lo, hi);
    float acc[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) acc[i] = 0.f;
    float m = -INFINITY, l = 0.f;

    for (int64_t base = lo; base <= hi; base += 64) {
        const int64_t j = base + lane;
        const bool valid = j <= hi;
        float s = -INFINITY;
        if (valid) s = p.scale * row_dot(sq, K + (k0 + j) * hd + (int64_t)h * d, d);
        float pj;
        if (act == KUNLUN_ACT_SOFTMAX) {
            const float m_new = fmaxf(m, wave_max(s));  // finite: the chunk holds at least one key
            const float corr = expf(m - m_new);         // exp(-inf) = 0 on the first chunk
            pj = valid ? expf(s - m_new) : 0.f;
            l = l * corr + wave_sum(pj);
#pragma unroll
            for (int i = 0; i < CH; ++i) acc[i] *= corr;
            m = m_new;
        } else {
            pj = valid ? act_exact_rt(act, s) : 0.f;
        }
        sp[lane] = pj;
        __syncthreads();
        const int nk = (int)((hi - base + 1) < 64 ? (hi - base + 1) : 64);
        for (int jj = 0; jj < nk; ++jj) {
            const float w = sp[jj];
            const T* vrow = V + (k0 + base + jj) * hd + (int64_t)h * d;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int c = lane + 64 * i;
                if (c < d) acc[i] = fmaf(w, to_float(vrow[c]), acc[i]);
            }
        }
        __syncthreads();
    }
    const bool softmax = act == KUNLUN_ACT_SOFTMAX;
    const float inv = (softmax && l > 0.f) ? 1.f / l : 1.f;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        if (c < d) O[row * hd + (int64_t)h * d + c] = from_float<T>(softmax ? acc[i] * inv : acc[i]);
    }
    if (softmax && p.lse && lane == 0) p.lse[(int64_t)h * p.total_q + row] = (lo <= hi) ? m + logf(l) : -INFINITY;
}

// dQ: one wavefront per (query row, head).
template <typename T>
__global__ __launch_bounds__(64) void scalar_bwd_dq_kernel(AttnParams p) {
    __shared__ float sq[MAX_D];
    __shared__ float sdo[MAX_D];
    __shared__ float sds[64];
    const int lane = threadIdx.x;
    const int64_t item = blockIdx.x;
    const int64_t row = item / p.H;
    const int h = (int)(item % p.H);
    const int d = p.d;
    const int64_t hd = (int64_t)p.H * d;
    const int b = p.q_off ? find_example(p.q_off, p.B, row) : (int)(row / p.max_q);
    const int64_t t = row - q_begin(p, b);
    const int64_t k0 = p.kv_off[b];
    const int64_t n_kv = (int64_t)p.kv_off[b + 1] - k0;
    const int act = p.head_act[h];
    const bool softmax = act == KUNLUN_ACT_SOFTMAX;
    const T* Q = (const T*)p.q;
    const T* K = (const T*)p.k;
    const T* V = (const T*)p.v;
    const T* DO = (const T*)p.d_o;
    const T* O = (const T*)p.o;
    T* DQ = (T*)p.dq;
    const int64_t qbase = row * hd + (int64_t)h * d;

    float part = 0.f;
    for (int c = lane; c < d; c += 64) {
        sq[c] = to_float(Q[q_src_row(p, row) * hd + (int64_t)h * d + c]);
        sdo[c] = to_float(DO[qbase + c]);
        if (softmax) part = fmaf(sdo[c], to_float(O[qbase + c]), part);
    }
    const float delta = softmax ? wave_sum(part) : 0.f;
    const float lse = softmax ? p.lse[(int64_t)h * p.total_q + row] : 0.f;
    __syncthreads();

    int64_t lo, hi;
    window_keys(p, t, n_kv, lo, hi);
    float acc[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) acc[i] = 0.f;
    for (int64_t base = lo; base <= hi; base += 64) {
        const int64_t j = base + lane;
        float ds = 0.f;
        if (j <= hi) {
            const int64_t kb = (k0 + j) * hd + (int64_t)h * d;
            const float s = p.scale * row_dot(sq, K + kb, d);
            const float dp = row_dot(sdo, V + kb, d);
            ds = softmax ? expf(s - lse) * (dp - delta) * p.scale : dp * act_deriv_exact_rt(act, s) * p.scale;
        }
        sds[lane] = ds;
        __syncthreads();
        const int nk = (int)((hi - base + 1) < 64 ? (hi - base + 1) : 64);
        for (int jj = 0; jj < nk; ++jj) {
            const float w = sds[jj];
            const T* krow = K + (k0 + base + jj) * hd + (int64_t)h * d;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int c = lane + 64 * i;
                if (c < d) acc[i] = fmaf(w, to_float(krow[c]), acc[i]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        if (c < d) DQ[qbase + c] = from_float<T>(acc[i]);
    }
}

// dK, dV: one wavefront per (key row, head); runs over the queries that see this key.
template <typename T>
__global__ __launch_bounds__(64) void scalar_bwd_dkdv_kernel(AttnParams p) {
    __shared__ float sk[MAX_D];
    __shared__ float sv[MAX_D];
    __shared__ float sp[64];
    __shared__ float sds[64];
    const int lane = threadIdx.x;
    const int64_t item = blockIdx.x;
    const int64_t krow_id = item / p.H;
    const int h = (int)(item % p.H);
    const int d = p.d;
    const int64_t hd = (int64_t)p.H * d;
    const int b = find_example(p.kv_off, p.B, krow_id);
    const int64_t j = krow_id - p.kv_off[b];  // key position inside its example
    const int64_t q0 = q_begin(p, b);
    const int64_t n_q = q_end(p, b) - q0;
    const int act = p.head_act[h];
    const bool softmax = act == KUNLUN_ACT_SOFTMAX;
    const T* Q = (const T*)p.q;
    const T* K = (const T*)p.k;
    const T* V = (const T*)p.v;
    const T* DO = (const T*)p.d_o;
    const T* O = (const T*)p.o;
    const int64_t kbase = krow_id * hd + (int64_t)h * d;

    for (int c = lane; c < d; c += 64) {
        sk[c] = to_float(K[kbase + c]);
        sv[c] = to_float(V[kbase + c]);
    }
    __syncthreads();

    // queries t with t - left <= j <= t + right
    int64_t lo = 0, hi = n_q - 1;
    if (p.windowed) {
        if (p.right >= 0 && j - p.right > lo) lo = j - p.right;
        if (p.left >= 0 && j + p.left < hi) hi = j + p.left;
    }
    float acck[CH], accv[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) acck[i] = accv[i] = 0.f;
    for (int64_t base = lo; base <= hi; base += 64) {
        const int64_t i_q = base + lane;
        float pw = 0.f, ds = 0.f;
        if (i_q <= hi) {
            const int64_t qb = (q0 + i_q) * hd + (int64_t)h * d;
            const int64_t qsrc = q_src_row(p, q0 + i_q) * hd + (int64_t)h * d;
            const float s = p.scale * row_dot(sk, Q + qsrc, d);
            const float dp = row_dot(sv, DO + qb, d);
            if (softmax) {
                float delta = 0.f;
                for (int c = 0; c < d; ++c) delta = fmaf(to_float(DO[qb + c]), to_float(O[qb + c]), delta);
                pw = expf(s - p.lse[(int64_t)h * p.total_q + q0 + i_q]);
                ds = pw * (dp - delta) * p.scale;
            } else {
                pw = act_exact_rt(act, s);
                ds = dp * act_deriv_exact_rt(act, s) * p.scale;
            }
        }
        sp[lane] = pw;
        sds[lane] = ds;
        __syncthreads();
        const int nq = (int)((hi - base + 1) < 64 ? (hi - base + 1) : 64);
        for (int ii = 0; ii < nq; ++ii) {
            const float wp = sp[ii], wds = sds[ii];
            const int64_t qb = (q0 + base + ii) * hd + (int64_t)h * d;
            const int64_t qsb = q_src_row(p, q0 + base + ii) * hd + (int64_t)h * d;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int c = lane + 64 * i;
                if (c < d) {
                    acck[i] = fmaf(wds, to_float(Q[qsb + c]), acck[i]);
                    accv[i] = fmaf(wp, to_float(DO[qb + c]), accv[i]);
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        if (c < d) {
            ((T*)p.dk)[kbase + c] = from_float<T>(acck[i]);
            ((T*)p.dv)[kbase + c] = from_float<T>(accv[i]);
        }
    }
}

hipError_t launch_scalar_fwd(const AttnParams& p, int dtype, hipStream_t stream) {
    const int64_t items = p.total_q * p.H;
    if (items == 0) return hipSuccess;
    if (dtype == KUNLUN_FP32)
        hipLaunchKernelGGL(scalar_fwd_kernel<float>, dim3((unsigned)items), dim3(64), 0, stream, p);
    else
        hipLaunchKernelGGL(scalar_fwd_kernel<bf16_t>, dim3((unsigned)items), dim3(64), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_scalar_bwd(const AttnParams& p, int dtype, hipStream_t stream) {
    const int64_t qi = p.total_q * p.H, ki = p.total_kv * p.H;
    if (qi > 0) {
        if (dtype == KUNLUN_FP32)
            hipLaunchKernelGGL(scalar_bwd_dq_kernel<float>, dim3((unsigned)qi), dim3(64), 0, stream, p);
        else
            hipLaunchKernelGGL(scalar_bwd_dq_kernel<bf16_t>, dim3((unsigned)qi), dim3(64), 0, stream, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ki > 0) {
        if (dtype == KUNLUN_FP32)
            hipLaunchKernelGGL(scalar_bwd_dkdv_kernel<float>, dim3((unsigned)ki), dim3(64), 0, stream, p);
        else
            hipLaunchKernelGGL(scalar_bwd_dkdv_kernel<bf16_t>, dim3((unsigned)ki), dim3(64), 0, stream, p);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace kunlun
