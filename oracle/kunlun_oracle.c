/*
 * CPU oracle for the Kunlun attention operators.  TEST INFRASTRUCTURE ONLY:
 * it defines what the GPU library must compute and is never part of the
 * product path.  It shares no code, header, table or helper with the HIP
 * library.
 *
 * Everything is fp64, straight loops over (example, head, query, key, channel)
 * with no blocking, no online softmax and no reordering: each function is the
 * definition of the operator written out.
 *
 *   - GDPA, activation mode  : paper Eq. (GDPA) in Sec. "Multi-Head PFFN with
 *       Generalized Dot-Product Attention", and the per-head line of Alg.
 *       "Generalized Dot-Product Attention":
 *           O_h = Act_h(Q_h K_h^T / tau) V_h         (no normaliser but 1/tau)
 *   - GDPA, softmax mode     : multi-head attention as used by PMA (Eq. PMA)
 *       and by stage 2 of Hierarchical Seed Pooling (Eq. seed-level attention):
 *           O_h = softmax(Q_h K_h^T * scale) V_h
 *   - sliding-window attention: Eq. (sliding window) in Sec. "Sliding Window
 *       Attention": query t sees keys in [t-left, t+right], clipped to its own
 *       sequence; softmax over that set.
 *   - backward: the analytic gradient of <O, dO> with respect to Q, K, V.
 *   - SumKronLinear          : Eq. (SumKronLinear) in Sec. "Hierarchical Seed
 *       Pooling", stage 3 (and the last line of Alg. "Hierarchical Seed Pooling"):
 *           Y_b = sum_{i=1..k} Z_i^T X_b W_i ,  Z_i [S, T], W_i [D, D], X_b [S, D]
 *       written as the quadruple sum over (i, s, c) per output element, and the
 *       analytic gradient of <Y, dY> with respect to X, Z, W.
 *
 * Layout ("THD"): Q [total_q, H, d], K and V [total_kv, H, d], O like Q, all
 * row-major doubles; LSE [H, total_q].  Example b owns query rows
 * q_off[b]..q_off[b+1]-1 (or b*max_q.. if q_off is NULL: every example has
 * max_q rows) and key rows kv_off[b]..kv_off[b+1]-1.
 *
 * Conventions fixed where the paper is silent: keys outside an example
 * contribute exactly nothing; an example with no keys gives zero output rows
 * and LSE = -inf; window bounds < 0 mean unbounded on that side.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ACT_SOFTMAX = 0, ACT_IDENTITY = 1, ACT_RELU = 2, ACT_GELU = 3, ACT_GELU_TANH = 4, ACT_SILU = 5, ACT_GELU_POLY = 6 };

static const double SQRT_2_OVER_PI = 0.79788456080286535587989211986876;
static const double INV_SQRT_2 = 0.70710678118654752440084436210485;
static const double INV_SQRT_2PI = 0.39894228040143267793994605993438;

/* The polynomial GELU (a score function without a transcendental, after the remark of App. "GDPA and Fused
 * PFFN Kernel" that without softmax the special-function unit limits the kernel):
 *     gelu_poly(x) = x * cdf(x),  cdf(x) = 1/2 + t * q(t^2),  t = x clamped to [-C, C],  q of degree 6.
 * The coefficients ARE the definition of this score function (they are an odd near-minimax fit of Phi - 1/2
 * on [-C, C] under the side condition C q(C^2) = 1/2, so that the tails are exactly 0 and exactly x);
 * the pins hold it within 8e-5 of Phi and 3e-4 of x Phi(x). */
static const double GELU_POLY_C = 3.875;
static const double GELU_POLY_Q[7] = {3.9862210505e-01,  -6.5595134356e-02, 9.2376422360e-03, -9.1053389233e-04,
                                      5.8010079080e-05,  -2.1110704002e-06, 3.2949778488e-08};
/* cdf(x) of the polynomial GELU and its derivative (0 outside [-C, C]). */
static double gelu_poly_cdf(double x, double* slope) {
    const double t = x < -GELU_POLY_C ? -GELU_POLY_C : (x > GELU_POLY_C ? GELU_POLY_C : x);
    const double u = t * t;
    double q = 0.0, dq = 0.0; /* q(u) and q'(u) */
    for (int i = 6; i >= 0; --i) q = q * u + GELU_POLY_Q[i];
    for (int i = 6; i >= 1; --i) dq = dq * u + i * GELU_POLY_Q[i];
    *slope = (x > -GELU_POLY_C && x < GELU_POLY_C) ? q + 2.0 * u * dq : 0.0;
    return 0.5 + t * q;
}

/* Element-wise score functions, exact definitions. */
static double act_value(int act, double x) {
    switch (act) {
    case ACT_IDENTITY: return x;
    case ACT_RELU: return x > 0.0 ? x : 0.0;
    case ACT_GELU: return x * 0.5 * (1.0 + erf(x * INV_SQRT_2));
    case ACT_GELU_TANH: {
        double u = SQRT_2_OVER_PI * (x + 0.044715 * x * x * x);
        return 0.5 * x * (1.0 + tanh(u));
    }
    case ACT_SILU: return x / (1.0 + exp(-x));
    case ACT_GELU_POLY: {
        double slope;
        return x * gelu_poly_cdf(x, &slope);
    }
    default: return NAN;
    }
}

/* d/dx of the above, closed forms (relu'(0) = 0). */
static double act_deriv(int act, double x) {
    switch (act) {
    case ACT_IDENTITY: return 1.0;
    case ACT_RELU: return x > 0.0 ? 1.0 : 0.0;
    case ACT_GELU: {
        double cdf = 0.5 * (1.0 + erf(x * INV_SQRT_2));
        double pdf = INV_SQRT_2PI * exp(-0.5 * x * x);
        return cdf + x * pdf;
    }
    case ACT_GELU_TANH: {
        double u = SQRT_2_OVER_PI * (x + 0.044715 * x * x * x);
        double t = tanh(u);
        double du = SQRT_2_OVER_PI * (1.0 + 3.0 * 0.044715 * x * x);
        return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * du;
    }
    case ACT_SILU: {
        double s = 1.0 / (1.0 + exp(-x));
        return s + x * s * (1.0 - s);
    }
    case ACT_GELU_POLY: {
        double slope;
        const double cdf = gelu_poly_cdf(x, &slope);
        return cdf + x * slope;
    }
    default: return NAN;
    }
}

static int64_t row_begin(const int32_t* off, int b, int max_rows) {
    return off ? (int64_t)off[b] : (int64_t)b * max_rows;
}
static int64_t row_end(const int32_t* off, int b, int max_rows) {
    return off ? (int64_t)off[b + 1] : (int64_t)(b + 1) * max_rows;
}

/* Key range of query i (position relative to its example) among n_kv keys.
 * windowed == 0: every key of the example.  Returns an empty range as lo > hi. */
static void key_range(int windowed, int left, int right, int64_t i, int64_t n_kv, int64_t* lo, int64_t* hi) {
    *lo = 0;
    *hi = n_kv - 1;
    if (windowed) {
        if (left >= 0 && i - left > *lo) *lo = i - left;
        if (right >= 0 && i + right < *hi) *hi = i + right;
    }
}

static int head_activation(int act, const int32_t* head_act, int h) { return head_act ? head_act[h] : act; }

/*
 * Forward.  For each example b, head h and query row i:
 *     s_j = scale * <Q[i,h,:], K[j,h,:]>     for j in the key set of i
 *     activation mode: O[i,h,:] = sum_j Act_h(s_j) V[j,h,:]
 *     softmax mode   : O[i,h,:] = sum_j exp(s_j - m) / Z * V[j,h,:],
 *                      m = max_j s_j, Z = sum_j exp(s_j - m), LSE = m + log Z
 * lse may be NULL.  Returns 0, or -1 on an unknown activation.
 */
static int attention_forward(const double* q, const double* k, const double* v, double* o, double* lse,
                             const int32_t* q_off, const int32_t* kv_off, int B, int H, int d, int max_q,
                             int64_t total_q, double scale, int act, const int32_t* head_act, int windowed,
                             int left, int right) {
    for (int h = 0; h < H; ++h) {
        int a = head_activation(act, head_act, h);
        if (a < ACT_SOFTMAX || a > ACT_GELU_POLY) return -1;
    }
    const int64_t hd = (int64_t)H * d;
    int64_t max_kv = 1;
    for (int b = 0; b < B; ++b) {
        int64_t n = (int64_t)kv_off[b + 1] - kv_off[b];
        if (n > max_kv) max_kv = n;
    }
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)max_kv);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int b = 0; b < B; ++b) {
            for (int h = 0; h < H; ++h) {
                const int a = head_activation(act, head_act, h);
                const int64_t q0 = row_begin(q_off, b, max_q), q1 = row_end(q_off, b, max_q);
                const int64_t k0 = kv_off[b], n_kv = (int64_t)kv_off[b + 1] - kv_off[b];
                for (int64_t i = 0; i < q1 - q0; ++i) {
                    const double* qi = q + (q0 + i) * hd + (int64_t)h * d;
                    double* oi = o + (q0 + i) * hd + (int64_t)h * d;
                    for (int c = 0; c < d; ++c) oi[c] = 0.0;
                    int64_t lo, hi;
                    key_range(windowed, left, right, i, n_kv, &lo, &hi);
                    if (lo > hi) {
                        if (lse) lse[(int64_t)h * total_q + q0 + i] = -INFINITY;
                        continue;
                    }
                    for (int64_t j = lo; j <= hi; ++j) {
                        const double* kj = k + (k0 + j) * hd + (int64_t)h * d;
                        double dot = 0.0;
                        for (int c = 0; c < d; ++c) dot += qi[c] * kj[c];
                        s[j] = scale * dot;
                    }
                    if (a == ACT_SOFTMAX) {
                        double m = s[lo];
                        for (int64_t j = lo + 1; j <= hi; ++j) m = s[j] > m ? s[j] : m;
                        double z = 0.0;
                        for (int64_t j = lo; j <= hi; ++j) z += exp(s[j] - m);
                        for (int64_t j = lo; j <= hi; ++j) {
                            const double p = exp(s[j] - m) / z;
                            const double* vj = v + (k0 + j) * hd + (int64_t)h * d;
                            for (int c = 0; c < d; ++c) oi[c] += p * vj[c];
                        }
                        if (lse) lse[(int64_t)h * total_q + q0 + i] = m + log(z);
                    } else {
                        for (int64_t j = lo; j <= hi; ++j) {
                            const double p = act_value(a, s[j]);
                            const double* vj = v + (k0 + j) * hd + (int64_t)h * d;
                            for (int c = 0; c < d; ++c) oi[c] += p * vj[c];
                        }
                        if (lse) lse[(int64_t)h * total_q + q0 + i] = 0.0;
                    }
                }
            }
        }
        free(s);
    }
    return 0;
}

/*
 * Backward of f = <O, dO>.  With p_j the weight of key j for query i and
 * dp_j = <dO[i,h,:], V[j,h,:]>:
 *     dV[j] += p_j dO[i]
 *     activation mode: ds_j = dp_j * Act_h'(s_j) * scale
 *     softmax mode   : ds_j = p_j (dp_j - sum_l p_l dp_l) * scale
 *     dQ[i] += ds_j K[j],   dK[j] += ds_j Q[i]
 * dq, dk, dv are overwritten.  Every (b, h) owns disjoint slices of all three.
 */
static int attention_backward(const double* q, const double* k, const double* v, const double* d_o, double* dq,
                              double* dk, double* dv, const int32_t* q_off, const int32_t* kv_off, int B, int H,
                              int d, int max_q, int64_t total_q, int64_t total_kv, double scale, int act,
                              const int32_t* head_act, int windowed, int left, int right) {
    for (int h = 0; h < H; ++h) {
        int a = head_activation(act, head_act, h);
        if (a < ACT_SOFTMAX || a > ACT_GELU_POLY) return -1;
    }
    const int64_t hd = (int64_t)H * d;
    memset(dq, 0, sizeof(double) * (size_t)(total_q * hd));
    memset(dk, 0, sizeof(double) * (size_t)(total_kv * hd));
    memset(dv, 0, sizeof(double) * (size_t)(total_kv * hd));
    int64_t max_kv = 1;
    for (int b = 0; b < B; ++b) {
        int64_t n = (int64_t)kv_off[b + 1] - kv_off[b];
        if (n > max_kv) max_kv = n;
    }
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)max_kv);
        double* p = (double*)malloc(sizeof(double) * (size_t)max_kv);
        double* dp = (double*)malloc(sizeof(double) * (size_t)max_kv);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int b = 0; b < B; ++b) {
            for (int h = 0; h < H; ++h) {
                const int a = head_activation(act, head_act, h);
                const int64_t q0 = row_begin(q_off, b, max_q), q1 = row_end(q_off, b, max_q);
                const int64_t k0 = kv_off[b], n_kv = (int64_t)kv_off[b + 1] - kv_off[b];
                for (int64_t i = 0; i < q1 - q0; ++i) {
                    const int64_t qrow = (q0 + i) * hd + (int64_t)h * d;
                    int64_t lo, hi;
                    key_range(windowed, left, right, i, n_kv, &lo, &hi);
                    if (lo > hi) continue;
                    for (int64_t j = lo; j <= hi; ++j) {
                        const int64_t krow = (k0 + j) * hd + (int64_t)h * d;
                        double dot = 0.0, dpj = 0.0;
                        for (int c = 0; c < d; ++c) {
                            dot += q[qrow + c] * k[krow + c];
                            dpj += d_o[qrow + c] * v[krow + c];
                        }
                        s[j] = scale * dot;
                        dp[j] = dpj;
                    }
                    double delta = 0.0;
                    if (a == ACT_SOFTMAX) {
                        double m = s[lo];
                        for (int64_t j = lo + 1; j <= hi; ++j) m = s[j] > m ? s[j] : m;
                        double z = 0.0;
                        for (int64_t j = lo; j <= hi; ++j) z += exp(s[j] - m);
                        for (int64_t j = lo; j <= hi; ++j) {
                            p[j] = exp(s[j] - m) / z;
                            delta += p[j] * dp[j];
                        }
                    } else {
                        for (int64_t j = lo; j <= hi; ++j) p[j] = act_value(a, s[j]);
                    }
                    for (int64_t j = lo; j <= hi; ++j) {
                        const int64_t krow = (k0 + j) * hd + (int64_t)h * d;
                        const double ds = (a == ACT_SOFTMAX) ? p[j] * (dp[j] - delta) * scale
                                                             : dp[j] * act_deriv(a, s[j]) * scale;
                        for (int c = 0; c < d; ++c) {
                            dv[krow + c] += p[j] * d_o[qrow + c];
                            dq[qrow + c] += ds * k[krow + c];
                            dk[krow + c] += ds * q[qrow + c];
                        }
                    }
                }
            }
        }
        free(s);
        free(p);
        free(dp);
    }
    return 0;
}

/* ---- exported entry points (doubles in, doubles out) ---- */

int oracle_gdpa_fwd(const double* q, const double* k, const double* v, double* o, double* lse,
                    const int32_t* q_off, const int32_t* kv_off, int B, int H, int d, int max_q, int64_t total_q,
                    double scale, int act, const int32_t* head_act) {
    return attention_forward(q, k, v, o, lse, q_off, kv_off, B, H, d, max_q, total_q, scale, act, head_act, 0, -1,
                             -1);
}

int oracle_gdpa_bwd(const double* q, const double* k, const double* v, const double* d_o, double* dq, double* dk,
                    double* dv, const int32_t* q_off, const int32_t* kv_off, int B, int H, int d, int max_q,
                    int64_t total_q, int64_t total_kv, double scale, int act, const int32_t* head_act) {
    return attention_backward(q, k, v, d_o, dq, dk, dv, q_off, kv_off, B, H, d, max_q, total_q, total_kv, scale, act,
                              head_act, 0, -1, -1);
}

/* Self-attention over jagged sequences: Q, K, V share one offsets array. */
int oracle_swa_fwd(const double* q, const double* k, const double* v, double* o, double* lse, const int32_t* off,
                   int B, int H, int d, int64_t total, int left, int right, double scale) {
    return attention_forward(q, k, v, o, lse, off, off, B, H, d, 0, total, scale, ACT_SOFTMAX, NULL, 1, left, right);
}

int oracle_swa_bwd(const double* q, const double* k, const double* v, const double* d_o, double* dq, double* dk,
                   double* dv, const int32_t* off, int B, int H, int d, int64_t total, int left, int right,
                   double scale) {
    return attention_backward(q, k, v, d_o, dq, dk, dv, off, off, B, H, d, 0, total, total, scale, ACT_SOFTMAX, NULL,
                              1, left, right);
}

/*
 * SumKronLinear, Eq. (SumKronLinear):  Y[b, t, e] = sum_i sum_s sum_c Z[i, s, t] * X[b, s, c] * W[i, c, e].
 * x [B, S, D], z [k, S, T], w [k, D, D], y [B, T, D], row-major doubles.  The sum is taken exactly
 * as written, one output element at a time (no intermediate Z^T X, no reordering).
 */
int oracle_sumkron_fwd(const double* x, const double* z, const double* w, double* y, int B, int S, int T, int D,
                       int k) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t)
            for (int e = 0; e < D; ++e) {
                double acc = 0.0;
                for (int i = 0; i < k; ++i)
                    for (int s = 0; s < S; ++s) {
                        const double zst = z[((int64_t)i * S + s) * T + t];
                        const double* xr = x + ((int64_t)b * S + s) * D;
                        const double* wc = w + (int64_t)i * D * D + e;
                        double inner = 0.0;
                        for (int c = 0; c < D; ++c) inner += xr[c] * wc[(int64_t)c * D];
                        acc += zst * inner;
                    }
                y[((int64_t)b * T + t) * D + e] = acc;
            }
    return 0;
}

/*
 * Gradient of <Y, dY> of the above:
 *   dX[b, s, c] = sum_i sum_t sum_e Z[i, s, t] * dY[b, t, e] * W[i, c, e]
 *   dZ[i, s, t] = sum_b sum_c sum_e X[b, s, c] * W[i, c, e] * dY[b, t, e]
 *   dW[i, c, e] = sum_b sum_s sum_t X[b, s, c] * Z[i, s, t] * dY[b, t, e]
 * each written out per output element.
 */
int oracle_sumkron_bwd(const double* x, const double* z, const double* w, const double* dy, double* dx, double* dz,
                       double* dw, int B, int S, int T, int D, int k) {
    if (B < 0 || S <= 0 || T <= 0 || D <= 0 || k <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int s = 0; s < S; ++s)
            for (int c = 0; c < D; ++c) {
                double acc = 0.0;
                for (int i = 0; i < k; ++i)
                    for (int t = 0; t < T; ++t) {
                        const double* dyr = dy + ((int64_t)b * T + t) * D;
                        const double* wr = w + ((int64_t)i * D + c) * D;
                        double inner = 0.0;
                        for (int e = 0; e < D; ++e) inner += dyr[e] * wr[e];
                        acc += z[((int64_t)i * S + s) * T + t] * inner;
                    }
                dx[((int64_t)b * S + s) * D + c] = acc;
            }
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int i = 0; i < k; ++i)
        for (int s = 0; s < S; ++s)
            for (int t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int b = 0; b < B; ++b) {
                    const double* xr = x + ((int64_t)b * S + s) * D;
                    const double* dyr = dy + ((int64_t)b * T + t) * D;
                    for (int c = 0; c < D; ++c) {
                        const double* wr = w + ((int64_t)i * D + c) * D;
                        double inner = 0.0;
                        for (int e = 0; e < D; ++e) inner += wr[e] * dyr[e];
                        acc += xr[c] * inner;
                    }
                }
                dz[((int64_t)i * S + s) * T + t] = acc;
            }
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int i = 0; i < k; ++i)
        for (int c = 0; c < D; ++c)
            for (int e = 0; e < D; ++e) {
                double acc = 0.0;
                for (int b = 0; b < B; ++b)
                    for (int s = 0; s < S; ++s) {
                        const double xv = x[((int64_t)b * S + s) * D + c];
                        double inner = 0.0;
                        for (int t = 0; t < T; ++t) inner += z[((int64_t)i * S + s) * T + t] * dy[((int64_t)b * T + t) * D + e];
                        acc += xv * inner;
                    }
                dw[((int64_t)i * D + c) * D + e] = acc;
            }
    return 0;
}

double oracle_act_value(int act, double x) { return act_value(act, x); }
double oracle_act_deriv(int act, double x) { return act_deriv(act, x); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
