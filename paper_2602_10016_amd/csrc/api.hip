// C ABI of the library (see include/kunlun.h): argument validation on the host, then the
// scheduler kernel and the attention kernels are enqueued on the caller's stream.  Nothing
// here allocates, synchronises or keeps state.
#include <cmath>
#include <cstring>

#include "common.h"
#include "tile_map.h"

using namespace kunlun;

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_common(int B, int H, int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, float scale,
                 int dtype) {
    if (B < 0 || H <= 0 || d <= 0 || max_q < 0 || max_kv < 0 || total_q < 0 || total_kv < 0) return KUNLUN_ERR_SHAPE;
    if (total_q >= (int64_t)1 << 31 || total_kv >= (int64_t)1 << 31) return KUNLUN_ERR_SHAPE;  // int32 offsets
    if (dtype != KUNLUN_BF16 && dtype != KUNLUN_FP32) return KUNLUN_ERR_UNSUPPORTED;
    if (H > KUNLUN_MAX_HEADS || d > 256 || d % 8 != 0) return KUNLUN_ERR_UNSUPPORTED;
    if (!std::isfinite(scale)) return KUNLUN_ERR_UNSUPPORTED;
    if (total_q * (int64_t)H >= (int64_t)1 << 31 || total_kv * (int64_t)H >= (int64_t)1 << 31)
        return KUNLUN_ERR_UNSUPPORTED;  // one workgroup per (row, head) must fit a 1-D grid
    return KUNLUN_OK;
}

int fill_acts(AttnParams& p, int H, int act, const int32_t* head_act, bool& any_softmax) {
    any_softmax = false;
    for (int h = 0; h < H; ++h) {
        const int a = head_act ? head_act[h] : act;
        if (a < KUNLUN_ACT_SOFTMAX || a > KUNLUN_ACT_GELU_POLY) return KUNLUN_ERR_UNSUPPORTED;
        p.head_act[h] = (uint8_t)a;
        any_softmax |= a == KUNLUN_ACT_SOFTMAX;
    }
    return KUNLUN_OK;
}

size_t order_bytes(int B) { return align_up((size_t)(B + 1) * sizeof(int32_t), 256); }

int gdpa_bwd_checked(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o, void* dq,
                     void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, int B, int H, int d, int max_q,
                     int max_kv, int64_t total_q, int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype,
                     void* workspace, size_t workspace_bytes, void* stream, bool q_shared);

}  // namespace

extern "C" {

size_t kunlun_workspace_bytes(int op, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                              int64_t total_kv) {
    if (B < 0 || H <= 0 || d <= 0 || max_q < 0 || max_kv < 0 || total_q < 0 || total_kv < 0) return 0;
    switch (op) {
    case KUNLUN_OP_GDPA_FWD:
    case KUNLUN_OP_SWA_FWD:
    case KUNLUN_OP_SEED_FWD:
        return WS_HEADER_BYTES + tile_table_bytes(B, total_q);
    case KUNLUN_OP_SEED_BWD:  // + the per-example query gradients (at most 4 bytes per element) and the partial sums over the batch
        return kunlun_workspace_bytes(KUNLUN_OP_GDPA_BWD, B, H, d, max_q, max_kv, total_q, total_kv) +
               seed_grad_rows_bytes(total_q, H, d, KUNLUN_FP32) + seed_grad_partial_bytes(B, (int64_t)max_q * H * d);
    case KUNLUN_OP_GDPA_BWD:
    case KUNLUN_OP_SWA_BWD:
        return WS_HEADER_BYTES + order_bytes(B) +
               mfma_bwd_tiled_workspace(B, H, d, max_q, max_kv, total_q, total_kv, op == KUNLUN_OP_SWA_BWD);
    default:
        return 0;
    }
}

size_t kunlun_sumkron_workspace_bytes(int B, int S, int T, int D, int k, int dtype) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0 || (dtype != KUNLUN_BF16 && dtype != KUNLUN_FP32)) return 0;
    return sumkron_workspace(B, S, T, D, k, dtype) + 256;
}

int kunlun_sumkron_fwd(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k,
                       int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0) return KUNLUN_ERR_SHAPE;
    if (dtype != KUNLUN_BF16 && dtype != KUNLUN_FP32) return KUNLUN_ERR_UNSUPPORTED;
    // 32-bit index arithmetic inside a row block of the kernels
    if ((int64_t)k * D > (1 << 20) || (int64_t)k * T > (1 << 20) || S > (1 << 20) || D % 8 != 0) return KUNLUN_ERR_UNSUPPORTED;
    if ((int64_t)B * T >= (1ll << 31) || (int64_t)B * S >= (1ll << 31)) return KUNLUN_ERR_UNSUPPORTED;
    if (B == 0) return KUNLUN_OK;
    if (!x || !z || !w || !y) return KUNLUN_ERR_NULL;
    if (!aligned(x, 16) || !aligned(z, 16) || !aligned(w, 16) || !aligned(y, 16)) return KUNLUN_ERR_ALIGN;
    if (!workspace || workspace_bytes < kunlun_sumkron_workspace_bytes(B, S, T, D, k, dtype)) return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;
    const hipError_t e = launch_sumkron(x, z, w, y, B, S, T, D, k, dtype, workspace, (hipStream_t)stream);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

size_t kunlun_sumkron_bwd_workspace_bytes(int B, int S, int T, int D, int k, int dtype) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0 || (dtype != KUNLUN_BF16 && dtype != KUNLUN_FP32)) return 0;
    return sumkron_bwd_workspace(B, S, T, D, k, dtype) + 256;
}

int kunlun_sumkron_bwd(const void* x, const void* z, const void* w, const void* dy, void* dx, void* dz, void* dw, int B, int S,
                       int T, int D, int k, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0) return KUNLUN_ERR_SHAPE;
    if (dtype != KUNLUN_BF16 && dtype != KUNLUN_FP32) return KUNLUN_ERR_UNSUPPORTED;
    // 32-bit index arithmetic inside a row block of the kernels, and 32-bit row / contraction counts
    if ((int64_t)k * D > (1 << 20) || (int64_t)k * T > (1 << 20) || S > (1 << 20) || D % 8 != 0) return KUNLUN_ERR_UNSUPPORTED;
    if ((int64_t)B * T >= (1ll << 31) || (int64_t)B * D >= (1ll << 31) || (int64_t)B * S >= (1ll << 31)) return KUNLUN_ERR_UNSUPPORTED;
    if (!z || !w || !dz || !dw) return KUNLUN_ERR_NULL;
    if (B > 0 && (!x || !dy || !dx)) return KUNLUN_ERR_NULL;
    if (!aligned(x, 16) || !aligned(z, 16) || !aligned(w, 16) || !aligned(dy, 16) || !aligned(dx, 16) || !aligned(dz, 16) ||
        !aligned(dw, 16))
        return KUNLUN_ERR_ALIGN;
    if (B > 0) {
        if (!workspace || workspace_bytes < kunlun_sumkron_bwd_workspace_bytes(B, S, T, D, k, dtype)) return KUNLUN_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;
    }
    const hipError_t e = launch_sumkron_bwd(x, z, w, dy, dx, dz, dw, B, S, T, D, k, dtype, workspace, (hipStream_t)stream);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

int kunlun_check_offsets(const int32_t* offsets, int B, int64_t total, int max_len, int32_t* violations, void* stream) {
    if (B < 0 || total < 0 || max_len < 0) return KUNLUN_ERR_SHAPE;
    if (!offsets || !violations) return KUNLUN_ERR_NULL;
    if (!aligned(offsets, 4) || !aligned(violations, 4)) return KUNLUN_ERR_ALIGN;
    const hipError_t e = launch_check_offsets(offsets, B, total, max_len, violations, (hipStream_t)stream);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

int kunlun_stream_probe(const void* a, const void* b, const void* c, void* out, size_t bytes, int reads, int write, void* stream) {
    if (reads < 1 || reads > 3 || (write != 0 && write != 1)) return KUNLUN_ERR_UNSUPPORTED;
    if (bytes % 16 != 0) return KUNLUN_ERR_SHAPE;
    if (bytes == 0) return KUNLUN_OK;
    if (!a || (reads > 1 && !b) || (reads > 2 && !c) || !out) return KUNLUN_ERR_NULL;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(c, 16) || !aligned(out, 16)) return KUNLUN_ERR_ALIGN;
    if (!write && bytes < 4096) return KUNLUN_ERR_SHAPE;  // `out` must hold 4 KiB even when nothing is written
    const hipError_t e = launch_stream_probe(a, b, c, out, bytes, reads, write, (hipStream_t)stream);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

int kunlun_jagged_stream_probe(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* offsets,
                               int B, int H, int d, int max_len, int64_t total, int reads, int writes, int workgroups_per_cu,
                               void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 0 || H < 1 || H > KUNLUN_MAX_HEADS || max_len < 0 || total < 0) return KUNLUN_ERR_SHAPE;
    if (d != 32 && d != 64 && d != 128) return KUNLUN_ERR_UNSUPPORTED;
    if (reads < 1 || reads > 3 || writes < 0 || writes > 2 || (writes == 2 && reads < 2)) return KUNLUN_ERR_UNSUPPORTED;
    if (workgroups_per_cu < 1 || workgroups_per_cu > 8) return KUNLUN_ERR_UNSUPPORTED;
    if ((size_t)total * H * d * 2 > ((size_t)1 << 40)) return KUNLUN_ERR_SHAPE;
    if (B == 0 || total == 0) return KUNLUN_OK;
    if (!offsets || !a || (reads > 1 && !b) || (reads > 2 && !c) || (writes > 0 && !out_a) || (writes > 1 && !out_b)) return KUNLUN_ERR_NULL;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(c, 16) || !aligned(out_a, 16) || !aligned(out_b, 16)) return KUNLUN_ERR_ALIGN;
    if (!workspace || workspace_bytes < WS_HEADER_BYTES + order_bytes(B)) return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    int32_t* queue = (int32_t*)workspace;
    int32_t* order = (int32_t*)((char*)workspace + WS_HEADER_BYTES);
    hipError_t e = launch_schedule(offsets, B, max_len, order, queue, s);
    if (e == hipSuccess) e = launch_jagged_probe(a, b, c, out_a, out_b, order, offsets, B, H, d, queue, reads, writes, workgroups_per_cu, s);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

const char* kunlun_strerror(int status) {
    switch (status) {
    case KUNLUN_OK: return "ok";
    case KUNLUN_ERR_NULL: return "a required pointer is NULL";
    case KUNLUN_ERR_SHAPE: return "negative or inconsistent sizes";
    case KUNLUN_ERR_UNSUPPORTED: return "unsupported dtype, activation, head count or head dimension";
    case KUNLUN_ERR_ALIGN: return "a pointer is not aligned as required";
    case KUNLUN_ERR_WORKSPACE: return "workspace missing or too small";
    case KUNLUN_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
    }
}

int kunlun_gdpa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                    const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                    int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return kunlun::gdpa_fwd_checked(q, k, v, o, lse, q_offsets, kv_offsets, B, H, d, max_q, max_kv, total_q, total_kv, scale, act,
                                    head_act, dtype, workspace, workspace_bytes, stream, true, false);
}

int kunlun_seed_attn_fwd(const void* e_seed, const void* k, const void* v, void* o, float* lse, const int32_t* kv_offsets, int B,
                         int H, int d, int n_seeds, int max_kv, int64_t total_kv, float scale, int act, const int32_t* head_act,
                         int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_seeds < 0 || B < 0) return KUNLUN_ERR_SHAPE;
    return kunlun::gdpa_fwd_checked(e_seed, k, v, o, lse, nullptr, kv_offsets, B, H, d, n_seeds, max_kv, (int64_t)B * n_seeds,
                                    total_kv, scale, act, head_act, dtype, workspace, workspace_bytes, stream, true, true);
}

}  // extern "C"

// The forward entry point proper.  launch = false: validation only (every check of the entry point, nothing
// enqueued, no device touched).
int kunlun::gdpa_fwd_checked(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                             const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                             int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* workspace,
                             size_t workspace_bytes, void* stream, bool launch, bool q_shared) {
    int rc = check_common(B, H, d, max_q, max_kv, total_q, total_kv, scale, dtype);
    if (rc != KUNLUN_OK) return rc;
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    bool any_softmax;
    rc = fill_acts(p, H, act, head_act, any_softmax);
    if (rc != KUNLUN_OK) return rc;
    if (!q_offsets && (int64_t)B * max_q != total_q) return KUNLUN_ERR_SHAPE;
    if (B == 0 || total_q == 0) return KUNLUN_OK;
    if (!q || !o || !kv_offsets) return KUNLUN_ERR_NULL;
    if (total_kv > 0 && (!k || !v)) return KUNLUN_ERR_NULL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lse, 4) ||
        !aligned(q_offsets, 4) || !aligned(kv_offsets, 4))
        return KUNLUN_ERR_ALIGN;
    if (!workspace || workspace_bytes < kunlun_workspace_bytes(KUNLUN_OP_GDPA_FWD, B, H, d, max_q, max_kv, total_q, total_kv))
        return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;
    if (!launch) return KUNLUN_OK;

    p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse;
    p.q_off = q_offsets; p.kv_off = kv_offsets;
    p.B = B; p.H = H; p.d = d; p.max_q = max_q; p.max_kv = max_kv;
    p.total_q = total_q; p.total_kv = total_kv; p.scale = scale;
    p.windowed = 0; p.left = -1; p.right = -1;
    p.q_shared = q_shared ? 1 : 0;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (mfma_fwd_supported(p, dtype)) {
        int32_t* order = (int32_t*)((char*)workspace + WS_HEADER_BYTES);
        const int64_t wgs = (int64_t)B * H * ((max_q + 63) / 64);
        if (mfma_fwd_is_qtiled(p)) {
            p.order = order;  // holds the query-tile prefix sums
        } else if (schedule_is_moot(wgs, 4)) {  // every forward kernel fits 4 workgroups per compute unit
            p.order = nullptr;
        } else {
            p.order = order;
            p.queue = (int32_t*)workspace;
            e = launch_schedule(kv_offsets, B, max_kv, order, p.queue, s);
            if (e != hipSuccess) return KUNLUN_ERR_LAUNCH;
        }
        e = launch_mfma_fwd(p, s);
    } else {
        e = launch_scalar_fwd(p, dtype, s);
    }
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

extern "C" {

int kunlun_gdpa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                    void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, int B, int H,
                    int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, float scale, int act,
                    const int32_t* head_act, int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    return gdpa_bwd_checked(q, k, v, o, lse, d_o, dq, dk, dv, q_offsets, kv_offsets, B, H, d, max_q, max_kv, total_q, total_kv,
                            scale, act, head_act, dtype, workspace, workspace_bytes, stream, false);
}

int kunlun_seed_attn_bwd(const void* e_seed, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                         void* d_e, void* dk, void* dv, const int32_t* kv_offsets, int B, int H, int d, int n_seeds, int max_kv,
                         int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (n_seeds < 0 || B < 0) return KUNLUN_ERR_SHAPE;
    return gdpa_bwd_checked(e_seed, k, v, o, lse, d_o, d_e, dk, dv, nullptr, kv_offsets, B, H, d, n_seeds, max_kv,
                            (int64_t)B * n_seeds, total_kv, scale, act, head_act, dtype, workspace, workspace_bytes, stream, true);
}

}  // extern "C"

namespace {
// kunlun_gdpa_bwd proper.  q_shared: q is one block of max_q seed rows used by every example and dq receives the
// gradient of that block, the sum over the batch of the per-example query gradients (which go to the workspace).
int gdpa_bwd_checked(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                     void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, int B, int H,
                     int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, float scale, int act,
                     const int32_t* head_act, int dtype, void* workspace, size_t workspace_bytes, void* stream, bool q_shared) {
    int rc = check_common(B, H, d, max_q, max_kv, total_q, total_kv, scale, dtype);
    if (rc != KUNLUN_OK) return rc;
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    bool any_softmax;
    rc = fill_acts(p, H, act, head_act, any_softmax);
    if (rc != KUNLUN_OK) return rc;
    if (!q_offsets && (int64_t)B * max_q != total_q) return KUNLUN_ERR_SHAPE;
    if (B == 0 || (total_q == 0 && total_kv == 0)) return KUNLUN_OK;
    if (!kv_offsets) return KUNLUN_ERR_NULL;
    if (total_q > 0 && (!q || !d_o || !dq)) return KUNLUN_ERR_NULL;
    if (total_kv > 0 && (!k || !v || !dk || !dv)) return KUNLUN_ERR_NULL;
    if (any_softmax && total_q > 0 && (!o || !lse)) return KUNLUN_ERR_NULL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(d_o, 16) ||
        !aligned(dq, 16) || !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lse, 4) || !aligned(q_offsets, 4) ||
        !aligned(kv_offsets, 4))
        return KUNLUN_ERR_ALIGN;
    const size_t base_bytes = kunlun_workspace_bytes(KUNLUN_OP_GDPA_BWD, B, H, d, max_q, max_kv, total_q, total_kv);
    if (!workspace || workspace_bytes < (q_shared ? kunlun_workspace_bytes(KUNLUN_OP_SEED_BWD, B, H, d, max_q, max_kv, total_q, total_kv)
                                                  : base_bytes))
        return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;

    p.q = q; p.k = k; p.v = v; p.o = const_cast<void*>(o); p.lse = const_cast<float*>(lse); p.d_o = d_o;
    p.dq = dq; p.dk = dk; p.dv = dv;
    p.q_off = q_offsets; p.kv_off = kv_offsets;
    p.B = B; p.H = H; p.d = d; p.max_q = max_q; p.max_kv = max_kv;
    p.total_q = total_q; p.total_kv = total_kv; p.scale = scale;
    p.windowed = 0; p.left = -1; p.right = -1;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    // shared seed queries: the kernels leave the per-example query gradients in the workspace (behind what the
    // call needs anyway); the sum over the batch follows below
    char* const dq_all = (char*)workspace + base_bytes;
    const size_t dq_all_bytes = seed_grad_rows_bytes(total_q, H, d, dtype);
    if (q_shared) {
        p.q_shared = 1;
        p.dq = dq_all;
    }
    if (mfma_bwd_supported(p, dtype)) {
        int32_t* order = (int32_t*)((char*)workspace + WS_HEADER_BYTES);
        if (schedule_is_moot((int64_t)B * H, d == 128 ? (max_q > 32 ? 2 : 1) : 4)) {  // workgroups of the kernel per compute unit
            p.order = nullptr;
        } else {
            p.order = order;
            p.queue = (int32_t*)workspace;
            e = launch_schedule(kv_offsets, B, max_kv, order, p.queue, s);
            if (e != hipSuccess) return KUNLUN_ERR_LAUNCH;
        }
        e = launch_mfma_bwd(p, (char*)workspace + WS_HEADER_BYTES + order_bytes(B), s);
    } else if (mfma_bwd_tiled_supported(p, dtype)) {
        e = launch_mfma_bwd_tiled(p, (char*)workspace + WS_HEADER_BYTES + order_bytes(B), any_softmax, s);
    } else {
        e = launch_scalar_bwd(p, dtype, s);
    }
    if (e == hipSuccess && q_shared && total_q > 0)
        e = launch_seed_grad_sum(dq_all, dq, (float*)(dq_all + dq_all_bytes), B, (int64_t)max_q * H * d, dtype, s);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}
}  // namespace

extern "C" {

int kunlun_swa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* offsets, int B,
                   int H, int d, int max_len, int64_t total, int window_left, int window_right, float scale,
                   int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_common(B, H, d, max_len, max_len, total, total, scale, dtype);
    if (rc != KUNLUN_OK) return rc;
    if (B == 0 || total == 0) return KUNLUN_OK;
    if (!q || !k || !v || !o || !offsets) return KUNLUN_ERR_NULL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(lse, 4) ||
        !aligned(offsets, 4))
        return KUNLUN_ERR_ALIGN;
    if (!workspace || workspace_bytes < kunlun_workspace_bytes(KUNLUN_OP_SWA_FWD, B, H, d, max_len, max_len, total, total))
        return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;

    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    for (int h = 0; h < H; ++h) p.head_act[h] = KUNLUN_ACT_SOFTMAX;
    p.q = q; p.k = k; p.v = v; p.o = o; p.lse = lse;
    p.q_off = offsets; p.kv_off = offsets;
    p.B = B; p.H = H; p.d = d; p.max_q = max_len; p.max_kv = max_len;
    p.total_q = total; p.total_kv = total; p.scale = scale;
    p.windowed = 1;
    // a reach of max_len or more covers every sequence: treated as unbounded, which also keeps the kernels'
    // 32-bit window arithmetic (position + reach) far from overflow
    p.left = (window_left < 0 || window_left >= max_len) ? -1 : window_left;
    p.right = (window_right < 0 || window_right >= max_len) ? -1 : window_right;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (mfma_fwd_supported(p, dtype) && swa_band_applies(p)) {
        int32_t* order = (int32_t*)((char*)workspace + WS_HEADER_BYTES);  // sequences, longest first
        p.queue = (int32_t*)workspace;
        e = launch_schedule(offsets, B, max_len, order, p.queue, s);
        if (e != hipSuccess) return KUNLUN_ERR_LAUNCH;
        p.order = order;
        e = launch_swa_band_fwd(p, s);
    } else if (mfma_fwd_supported(p, dtype)) {
        p.order = (int32_t*)((char*)workspace + WS_HEADER_BYTES);  // holds the query-tile prefix sums
        e = launch_mfma_fwd(p, s);
    } else {
        e = launch_scalar_fwd(p, dtype, s);
    }
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

int kunlun_swa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                   void* dq, void* dk, void* dv, const int32_t* offsets, int B, int H, int d, int max_len,
                   int64_t total, int window_left, int window_right, float scale, int dtype, void* workspace,
                   size_t workspace_bytes, void* stream) {
    int rc = check_common(B, H, d, max_len, max_len, total, total, scale, dtype);
    if (rc != KUNLUN_OK) return rc;
    if (B == 0 || total == 0) return KUNLUN_OK;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !offsets) return KUNLUN_ERR_NULL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(d_o, 16) ||
        !aligned(dq, 16) || !aligned(dk, 16) || !aligned(dv, 16) || !aligned(lse, 4) || !aligned(offsets, 4))
        return KUNLUN_ERR_ALIGN;
    if (!workspace || workspace_bytes < kunlun_workspace_bytes(KUNLUN_OP_SWA_BWD, B, H, d, max_len, max_len, total, total))
        return KUNLUN_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return KUNLUN_ERR_ALIGN;

    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    for (int h = 0; h < H; ++h) p.head_act[h] = KUNLUN_ACT_SOFTMAX;
    p.q = q; p.k = k; p.v = v; p.o = const_cast<void*>(o); p.lse = const_cast<float*>(lse); p.d_o = d_o;
    p.dq = dq; p.dk = dk; p.dv = dv;
    p.q_off = offsets; p.kv_off = offsets;
    p.B = B; p.H = H; p.d = d; p.max_q = max_len; p.max_kv = max_len;
    p.total_q = total; p.total_kv = total; p.scale = scale;
    p.windowed = 1;
    // a reach of max_len or more covers every sequence: treated as unbounded, which also keeps the kernels'
    // 32-bit window arithmetic (position + reach) far from overflow
    p.left = (window_left < 0 || window_left >= max_len) ? -1 : window_left;
    p.right = (window_right < 0 || window_right >= max_len) ? -1 : window_right;
    hipError_t e;
    if (mfma_bwd_tiled_supported(p, dtype))
        e = launch_mfma_bwd_tiled(p, (char*)workspace + WS_HEADER_BYTES + order_bytes(B), true, (hipStream_t)stream);
    else  // one wavefront per gradient row: dQ rows over their windows, then dK/dV rows
        e = launch_scalar_bwd(p, dtype, (hipStream_t)stream);
    return e == hipSuccess ? KUNLUN_OK : KUNLUN_ERR_LAUNCH;
}

}  // extern "C"
