/*
 * kunlun.h - C ABI of the Kunlun attention library for AMD Instinct MI355X (gfx950).
 *
 * The attention operators of the Kunlun architecture (arXiv 2602.10016) as fused, jagged-aware
 * GPU kernels:
 *
 *   kunlun_gdpa_fwd  Generalized Dot-Product Attention, Eq. (GDPA) of Sec. "Multi-Head
 *                    PFFN with Generalized Dot-Product Attention" and the per-head line of
 *                    Alg. "Generalized Dot-Product Attention":
 *                        O_h = Act_h(Q_h K_h^T * scale) V_h ,  scale = 1/tau,
 *                    with an element-wise score function per head and no normaliser; and,
 *                    with KUNLUN_ACT_SOFTMAX, the multi-head attention of Eq. (PMA) and of
 *                    Eq. (seed-level attention) in Sec. "Hierarchical Seed Pooling":
 *                        O_h = softmax(Q_h K_h^T * scale) V_h .
 *   kunlun_gdpa_bwd  Gradient of <O, dO> with respect to Q, K, V of the above (the fused
 *                    backward pass that Sec. "Efficient Attention-Style Implementation" and
 *                    App. "GDPA and Fused PFFN Kernel" describe: scores are recomputed
 *                    tile by tile, no score-sized tensor is stored).
 *   kunlun_seed_attn_fwd / _bwd  The same with one block of seed queries shared by the whole batch
 *                    (Sec. "Hierarchical Seed Pooling", stage 1) and its gradient summed over the batch.
 *   kunlun_swa_fwd   Sliding-window self-attention, Eq. (sliding window) of Sec. "Sliding
 *                    Window Attention": query t attends to keys [t-left, t+right] of its
 *                    own sequence under softmax.
 *   kunlun_swa_bwd   Gradient of <O, dO> of the same with respect to Q, K, V.
 *   kunlun_sumkron_fwd  SumKronLinear, Eq. (SumKronLinear) of Sec. "Hierarchical Seed Pooling"
 *                    (stage 3: compression of the S pooled seeds to T tokens):
 *                        Y_b = sum_{i=1..k} Z_i^T X_b W_i .
 *   kunlun_sumkron_bwd  Gradient of <Y, dY> of the same with respect to X, Z_i and W_i.
 *
 * Jagged layout.  A batch holds B examples.  Tensors are packed "tokens, heads, channels":
 *   Q  [total_q,  H, d]      O, dO, dQ like Q
 *   K,V[total_kv, H, d]      dK, dV like K
 *   LSE[H, total_q] float    (softmax mode only)
 * row-major and contiguous.  Example b owns key rows kv_offsets[b] .. kv_offsets[b+1]-1 and
 * query rows q_offsets[b] .. q_offsets[b+1]-1; with q_offsets == NULL every example owns
 * exactly max_q query rows (b*max_q ..).  Keys of other examples are never read for example
 * b and contribute exactly nothing.  An example without keys gets zero output rows (and
 * LSE = -inf, zero gradients).
 *
 * Memory.  q, k, v, o, lse, d_o, dq, dk, dv, *_offsets and workspace are DEVICE pointers;
 * head_act is a HOST pointer.  The caller owns every buffer.  The library allocates
 * nothing, keeps no state between calls and never synchronises: kernels are enqueued on
 * `stream` (a hipStream_t, NULL = default stream) and the call returns at once.  Tensor
 * pointers must be 16-byte aligned.  `workspace` must hold at least
 * kunlun_workspace_bytes(...) bytes, 256-byte aligned; its contents are scratch (work
 * lists, counters, partial results) and calls that share a workspace must be ordered on
 * one stream.  Offsets are trusted: offsets[0] = 0, non-decreasing, offsets[B] = total.
 *
 * Data types.  KUNLUN_BF16: bf16 storage, fp32 accumulation, outputs rounded to nearest
 * even; the two contractions run on the matrix cores when d is 32, 64 or 128.  KUNLUN_FP32:
 * fp32 storage and arithmetic throughout.  Supported d: multiples of 8 up to 256.
 *
 * Errors.  Every entry point validates its arguments on the host before anything is
 * enqueued and returns a kunlun_status (0 = OK, negative = error); nothing is launched on
 * error.  No exceptions, no abort.
 */
#ifndef KUNLUN_H_
#define KUNLUN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KUNLUN_OK = 0,
    KUNLUN_ERR_NULL = -1,        /* a required pointer is NULL */
    KUNLUN_ERR_SHAPE = -2,       /* negative or inconsistent sizes */
    KUNLUN_ERR_UNSUPPORTED = -3, /* unknown dtype / activation, unsupported d or H */
    KUNLUN_ERR_ALIGN = -4,       /* a pointer is not aligned as required */
    KUNLUN_ERR_WORKSPACE = -5,   /* workspace missing or too small */
    KUNLUN_ERR_LAUNCH = -6       /* the HIP runtime refused a launch */
} kunlun_status;

typedef enum { KUNLUN_BF16 = 0, KUNLUN_FP32 = 1 } kunlun_dtype;

/* Score functions (Eq. (GDPA): one activation per head).  gelu(x) = x * Phi(x) (erf form); gelu_tanh is the
 * tanh approximation 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))); silu(x) = x / (1 + exp(-x)).
 * gelu_poly is a GELU without a transcendental (App. "GDPA and Fused PFFN Kernel": without softmax the
 * special-function unit becomes the limiter, to be relieved by plain arithmetic), DEFINED as
 *     gelu_poly(x) = x * (1/2 + t q(t^2)),   t = min(max(x, -C), C),   C = 3.875,
 *     q(u) = 3.9862210505e-01 - 6.5595134356e-02 u + 9.2376422360e-03 u^2 - 9.1053389233e-04 u^3
 *            + 5.8010079080e-05 u^4 - 2.1110704002e-06 u^5 + 3.2949778488e-08 u^6
 * (C q(C^2) = 1/2: exactly 0 below -C, exactly x above C).  |gelu_poly(x) - gelu(x)| <= 3e-4 and
 * |gelu_poly(x) / x - Phi(x)| <= 8e-5 for every x: below the bf16 rounding of any weight above 0.15.  Its
 * derivative is that of this function (1/2 + t q + x (q + 2 t^2 q') inside (-C, C); 0 or 1 outside). */
typedef enum {
    KUNLUN_ACT_SOFTMAX = 0,
    KUNLUN_ACT_IDENTITY = 1,
    KUNLUN_ACT_RELU = 2,
    KUNLUN_ACT_GELU = 3,
    KUNLUN_ACT_GELU_TANH = 4,
    KUNLUN_ACT_SILU = 5,
    KUNLUN_ACT_GELU_POLY = 6
} kunlun_act;

typedef enum {
    KUNLUN_OP_GDPA_FWD = 0,
    KUNLUN_OP_GDPA_BWD = 1,
    KUNLUN_OP_SWA_FWD = 2,
    KUNLUN_OP_SWA_BWD = 3,
    KUNLUN_OP_SEED_FWD = 4,
    KUNLUN_OP_SEED_BWD = 5
} kunlun_op;

#define KUNLUN_MAX_HEADS 64

/*
 * Forward GDPA / multi-head attention over jagged keys (Eq. (GDPA); Eq. (PMA), Eq.
 * (seed-level attention) with KUNLUN_ACT_SOFTMAX).
 *   q, k, v      in,  device, `dtype` elements, layouts above
 *   o            out, device, like q; every row of every example is written
 *   lse          out, device, float [H, total_q], may be NULL; written for softmax heads only
 *   q_offsets    in,  device int32 [B+1] or NULL (dense queries: max_q rows per example)
 *   kv_offsets   in,  device int32 [B+1]
 *   max_q,max_kv upper bounds on the per-example query / key counts: they size work lists and
 *                select kernels, the true counts come from the offsets and must not exceed them
 *                (results are undefined if they do); total_q, total_kv: row counts of q and k
 *   scale        multiplies the dot products (1/tau for GDPA, 1/sqrt(d) for softmax)
 *   act          kunlun_act used by every head unless head_act is given
 *   head_act     in, HOST int32 [H] or NULL: per-head kunlun_act ("Act_h")
 * B == 0 or total_q == 0 is legal and does nothing.
 */
int kunlun_gdpa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                    const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                    int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * kunlun_gdpa_fwd for callers that cannot allocate device memory - code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc - and therefore cannot provide a workspace.  Same arguments, same kernels
 * and bit-identical results, but no workspace: the work lists go into a fixed array of
 * KUNLUN_STATIC_SCRATCH_BYTES of device memory that is part of the library image (each GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing and enqueues kernels only (no
 * memset: nothing in the array has to start at zero).
 *   Limit: kunlun_workspace_bytes(KUNLUN_OP_GDPA_FWD, ...) of the call must not exceed
 *   KUNLUN_STATIC_SCRATCH_BYTES (about 4 (2 B + total_q / 128) + 1 KiB: e.g. B = 100 000 examples of 64 queries);
 *   larger calls return KUNLUN_ERR_WORKSPACE and enqueue nothing.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams,
 *   or graphs that hold such calls replayed concurrently) race on it - order them, or use kunlun_gdpa_fwd with
 *   separate workspaces.
 *   The first call on a device looks the array's address up (hipGetSymbolAddress, once per device, under a
 *   mutex): make that first call outside stream capture.  The device that is current at the call must be the
 *   device of `stream` and of the tensors.
 * Other errors as for kunlun_gdpa_fwd; the address lookup failing gives KUNLUN_ERR_LAUNCH.
 */
#define KUNLUN_STATIC_SCRATCH_BYTES (1 << 20)
int kunlun_gdpa_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* q_offsets,
                           const int32_t* kv_offsets, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                           int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* stream);

/*
 * Backward of kunlun_gdpa_fwd: dq, dk, dv (out, device, shaped like q, k, v, fully
 * overwritten) from q, k, v and the upstream gradient d_o (in, device, like q).
 * With p the weight of a (query, key) pair and dp = <dO_row, V_row>:
 *     dV += p dO;   activation heads: ds = dp Act'(s) scale;
 *     softmax heads: ds = p (dp - rowsum(dO * O)) scale;   dQ += ds K;   dK += ds Q.
 * o and lse (in, device) are the forward outputs; they are read for softmax heads only and
 * may be NULL when no head uses softmax.  Other arguments as in kunlun_gdpa_fwd.
 */
int kunlun_gdpa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                    void* dq, void* dk, void* dv, const int32_t* q_offsets, const int32_t* kv_offsets, int B, int H,
                    int d, int max_q, int max_kv, int64_t total_q, int64_t total_kv, float scale, int act,
                    const int32_t* head_act, int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Seed-level attention with batch-shared seeds (Sec. "Hierarchical Seed Pooling", stage 1: the learnable seed
 * embeddings "are shared across all samples in the batch"; Eq. (seed-level attention): H_seed = MHA(Norm(E_seed),
 * S, S)).  The same computation as kunlun_gdpa_fwd with n_seeds dense queries per example, except that the
 * queries are ONE block
 *   e_seed   in, device, [n_seeds, H, d]   the projected (and normalised) seed queries, used by every example
 * instead of a [B * n_seeds, H, d] tensor that repeats it B times; o (out, [B * n_seeds, H, d]) and lse
 * ([H, B * n_seeds]) are per example as before.  act = KUNLUN_ACT_SOFTMAX is the paper's use; the other score
 * functions work as well.  Workspace: kunlun_workspace_bytes(KUNLUN_OP_SEED_FWD, B, H, d, n_seeds, max_kv,
 * B * n_seeds, total_kv).  The normalisation and the query projection of the seeds are the caller's: they act on
 * the n_seeds x d_model parameter once per step, before the per-head projection, not on anything per example.
 */
int kunlun_seed_attn_fwd(const void* e_seed, const void* k, const void* v, void* o, float* lse, const int32_t* kv_offsets, int B,
                         int H, int d, int n_seeds, int max_kv, int64_t total_kv, float scale, int act, const int32_t* head_act,
                         int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of kunlun_seed_attn_fwd.  dk, dv as in kunlun_gdpa_bwd;
 *   d_e   out, device, [n_seeds, H, d]   gradient of the shared seed queries = the sum over the B examples of the
 *         per-example query gradients dQ_b (Eq. (seed-level attention) with shared E_seed, chain rule).
 * The dQ_b go to the workspace and are added in a fixed order (examples in groups of 32, each group in example
 * order, then the groups in order; fp32 sums, rounded once): no atomics, bit-reproducible.  o, lse, d_o:
 * [B * n_seeds, ...] as in kunlun_gdpa_bwd.  Workspace: kunlun_workspace_bytes(KUNLUN_OP_SEED_BWD, ... as above).
 */
int kunlun_seed_attn_bwd(const void* e_seed, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                         void* d_e, void* dk, void* dv, const int32_t* kv_offsets, int B, int H, int d, int n_seeds, int max_kv,
                         int64_t total_kv, float scale, int act, const int32_t* head_act, int dtype, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * Sliding-window softmax self-attention over jagged sequences (Eq. (sliding window)).
 * q, k, v, o share `offsets` (device int32 [B+1]) and have `total` rows.  The query at
 * position t of a sequence of length L sees keys max(0, t-window_left) ..
 * min(L-1, t+window_right); a negative bound means unbounded on that side, so (-1, -1) is
 * full attention and (-1, 0) causal attention.  The equation's symmetric window of size w is
 * (w, w); "the previous W tokens including itself" is (W-1, 0).  lse: float [H, total] or NULL.
 */
int kunlun_swa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* offsets, int B,
                   int H, int d, int max_len, int64_t total, int window_left, int window_right, float scale,
                   int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of kunlun_swa_fwd (Eq. (sliding window)): dq, dk, dv (out, device, shaped like q,
 * fully overwritten) from q, k, v, the forward results o and lse (in, device, both required)
 * and the upstream gradient d_o.  With p = exp(s - lse) the weight of an in-window (query,
 * key) pair and dp = <dO_row, V_row>:  dV += p dO;  ds = p (dp - rowsum(dO * O)) scale;
 * dQ += ds K;  dK += ds Q.  A key collects contributions from the queries t with
 * t - window_left <= key <= t + window_right.  Other arguments as in kunlun_swa_fwd.
 */
int kunlun_swa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* d_o,
                   void* dq, void* dk, void* dv, const int32_t* offsets, int B, int H, int d, int max_len,
                   int64_t total, int window_left, int window_right, float scale, int dtype, void* workspace,
                   size_t workspace_bytes, void* stream);

/* Bytes of workspace that a call of `op` (kunlun_op) with these sizes needs.  Returns 0 for
 * an unknown op or negative sizes.  For the sliding-window ops pass max_len as max_q and
 * max_kv and total as total_q and total_kv; for the seed ops n_seeds as max_q and B * n_seeds as total_q. */
size_t kunlun_workspace_bytes(int op, int B, int H, int d, int max_q, int max_kv, int64_t total_q,
                              int64_t total_kv);

/*
 * SumKronLinear forward (Eq. (SumKronLinear)):  Y[b] = sum_i Z[i]^T X[b] W[i].
 *   x  in,  device, [B, S, D]   the S pooled seed vectors of every example
 *   z  in,  device, [k, S, T]   sequence-side factors Z_i
 *   w  in,  device, [k, D, D]   embedding-side factors W_i (applied from the right: rows = input channel)
 *   y  out, device, [B, T, D]   fully overwritten
 * all row-major, contiguous, `dtype` elements, 16-byte aligned.  KUNLUN_BF16: both contractions on
 * the matrix cores with fp32 accumulation when D is a multiple of 128 and S a multiple of 32 (the
 * intermediate Z_i^T X_b is rounded to bf16 once) - in ONE kernel that keeps the intermediate on the
 * compute unit when T = 32, S is 128 or 256, D <= 384 and k <= 8 (the paper's S = 256, T = 32, D = 384,
 * k = 8 among them), else as two matrix products through the workspace; other shapes and KUNLUN_FP32
 * take plain kernels that keep every intermediate and sum in fp64.  workspace: device, at least kunlun_sumkron_workspace_bytes(...) bytes, 256-byte aligned.
 * B == 0 is legal and does nothing.  Errors as for the other entry points.
 */
int kunlun_sumkron_fwd(const void* x, const void* z, const void* w, void* y, int B, int S, int T, int D, int k,
                       int dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace that kunlun_sumkron_fwd needs for these sizes (0 for invalid sizes). */
size_t kunlun_sumkron_workspace_bytes(int B, int S, int T, int D, int k, int dtype);

/*
 * SumKronLinear backward: the gradients of <Y, dY> for Y of Eq. (SumKronLinear),
 *     dX[b] = sum_i Z[i] dY[b] W[i]^T,   dZ[i] = sum_b X[b] W[i] dY[b]^T,   dW[i] = sum_b X[b]^T Z[i] dY[b].
 *   x, z, w  in, device, as in kunlun_sumkron_fwd
 *   dy  in,  device, [B, T, D]   gradient with respect to Y
 *   dx  out, device, [B, S, D];  dz out, device, [k, S, T];  dw out, device, [k, D, D]   fully overwritten
 * KUNLUN_BF16: five matrix-core contractions with fp32 accumulation when, in addition to the forward
 * conditions, S is a multiple of 128 and T*k and B*T are multiples of 32; Z_i^T X_b and dY_b W_i^T are
 * recomputed and rounded to bf16 once, the two sums over the batch are accumulated in fp32 partial
 * sums that are added in a fixed order (results are bit-reproducible).  Other shapes and KUNLUN_FP32
 * take plain fp32 kernels.  workspace: device, at least kunlun_sumkron_bwd_workspace_bytes(...) bytes,
 * 256-byte aligned.  B == 0 is legal: dz and dw are set to zero.  Errors as for the other entry points.
 */
int kunlun_sumkron_bwd(const void* x, const void* z, const void* w, const void* dy, void* dx, void* dz, void* dw, int B, int S,
                       int T, int D, int k, int dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace that kunlun_sumkron_bwd needs for these sizes (0 for invalid sizes). */
size_t kunlun_sumkron_bwd_workspace_bytes(int B, int S, int T, int D, int k, int dtype);

/*
 * Debug aid for the jagged layout ("Offsets are trusted" above: the operators do not check them).  Enqueues
 * one small kernel that counts the violations of the contract - offsets[0] != 0, offsets[B] != total, an
 * example shorter than 0 or longer than max_len - into *violations (out, device, one int32; 0 = the array is
 * fine).  offsets: in, device int32 [B+1].  Asynchronous like every other call: read *violations after the
 * stream has been synchronised.  Errors as for the other entry points.
 */
int kunlun_check_offsets(const int32_t* offsets, int B, int64_t total, int max_len, int32_t* violations, void* stream);

/*
 * Measurement aid, no part of any operator: one plain streaming kernel with the read : write mix of an attention
 * call, to calibrate what the device's memory system sustains for that mix (the HBM roof the calls' achieved GB/s are
 * held against: reads only for the forward over a long history, 1 : 1 for the backward, 3 : 1 for the sliding
 * window).  Reads `reads` (1..3) of the device buffers a, b, c (`bytes` each, a multiple of 16; unused ones may be
 * NULL) and, with write = 1, writes their XOR to out (device, `bytes`); with write = 0 nothing is written, but out
 * must still be a device buffer of at least 4 KiB.  Traffic of a call: (reads + write) * bytes.  Enqueued on
 * `stream`; errors as for the other entry points.
 */
int kunlun_stream_probe(const void* a, const void* b, const void* c, void* out, size_t bytes, int reads, int write, void* stream);

/*
 * The same aid for the access pattern of the jagged attention calls, whose memory traffic is not one sweep over
 * contiguous buffers but one independent walk per (example, head): work items in the scheduler's order (longest
 * first) on a persistent launch of workgroups_per_cu (1..8) workgroups per compute unit, as in the attention
 * kernels; a workgroup walks the token rows of its item and moves, per row, the d-channel piece of its head.
 * a, b, c, out_a, out_b: device, bf16 [total, H, d] (d in {32, 64, 128}), 16-byte aligned; offsets: device int32
 * [B + 1] as for the attention calls (lengths <= max_len, offsets[B] = total).  reads (1..3) of a, b, c are read;
 * with x = a and y = b ^ c (of what is read; bitwise), writes = 0 stores nothing, writes = 1 stores x ^ y to
 * out_a, writes = 2 (needs reads >= 2) stores x to out_a and y to out_b; unused pointers may be NULL.  Rows and
 * heads outside the items are never touched.  Traffic of a call: (reads + writes) * total * H * d * 2 bytes.
 * workspace: device, 256-byte aligned, at least 256 + 4 * (B + 1) rounded up to a multiple of 256 bytes (issue
 * order and work counter; contents undefined afterwards).  Enqueued on `stream`; errors as for the other entry
 * points.  Read-only forward over a history: reads = 2; its backward (K, V in, dK, dV out): reads = 2,
 * writes = 2; sliding-window forward (Q, K, V in, O out): reads = 3, writes = 1.
 */
int kunlun_jagged_stream_probe(const void* a, const void* b, const void* c, void* out_a, void* out_b, const int32_t* offsets,
                               int B, int H, int d, int max_len, int64_t total, int reads, int writes, int workgroups_per_cu,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Static, human-readable text for a kunlun_status. */
const char* kunlun_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* KUNLUN_H_ */
