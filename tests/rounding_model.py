"""A numpy fp64 model of the ONE lossy step of the bf16 kernels (the weights P, and dS in the backward, are rounded
to bf16 before the second contraction; everything else exact), for one (example, head) item.  Test infrastructure:
it explains the size of the GPU-vs-oracle differences on long sums (see tests/test_gpu_rounding_model.py).  Written
from Eq. (GDPA) / the softmax of Eq. (PMA) and their chain rule; imports neither the oracle nor the library."""
import numpy as np
from scipy.special import erf

from paper_2602_10016_amd.workloads import round_to_bf16

SOFTMAX, IDENTITY, RELU, GELU, GELU_TANH, SILU = range(6)
_C = np.sqrt(2.0 / np.pi)


def bf(x):
    return round_to_bf16(np.asarray(x, dtype=np.float32)).astype(np.float64)


def ulp_bf16(x):
    """Spacing of bf16 numbers at |x| (8 significant bits); the spacing of the smallest normal range below it."""
    a = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def act_value_deriv(act, s):
    if act == IDENTITY:
        return s, np.ones_like(s)
    if act == RELU:
        return np.maximum(s, 0.0), (s > 0).astype(np.float64)
    if act == GELU:
        cdf = 0.5 * (1.0 + erf(s / np.sqrt(2.0)))
        return s * cdf, cdf + s * np.exp(-0.5 * s * s) / np.sqrt(2.0 * np.pi)
    if act == GELU_TANH:
        u = _C * (s + 0.044715 * s ** 3)
        t = np.tanh(u)
        return 0.5 * s * (1.0 + t), 0.5 * (1.0 + t) + 0.5 * s * (1.0 - t * t) * _C * (1.0 + 3 * 0.044715 * s * s)
    if act == SILU:
        sg = 1.0 / (1.0 + np.exp(-s))
        return s * sg, sg + s * sg * (1.0 - sg)
    raise ValueError(act)


def forward_item(q, k, v, scale, act, rounded=True):
    """O of one (example, head) with an activation score function: O = bf16(P) V.  Also returns sum_j |p_j v_j|
    and an upper bound of max_j |p_j v_j| per output (for the accumulation and re-rounding allowances)."""
    p, _ = act_value_deriv(act, (q @ k.T) * scale)
    pr = bf(p) if rounded else p
    return pr @ v, np.abs(pr) @ np.abs(v), np.abs(pr).max(axis=1, keepdims=True) * np.abs(v).max(axis=0, keepdims=True)


def backward_item(q, k, v, d_o, scale, act, o=None, lse=None, rounded=True):
    """dQ, dK, dV of one (example, head): dV = bf16(P)^T dO, dQ = bf16(dS) K, dK = bf16(dS)^T Q.  Softmax heads take
    the forward results o and lse as the backward call does (P = exp(S - lse), delta = rowsum(dO * O)).
    Returns the three gradients and, for each, (sum of |terms|, bound of the largest |term|)."""
    s = (q @ k.T) * scale
    dp = d_o @ v.T
    if act == SOFTMAX:
        p = np.exp(s - lse[:, None])
        ds = p * (dp - (d_o * o).sum(axis=1, keepdims=True)) * scale
        # dp - delta cancels (exactly, when an example has one key): the fp32 rounding noise of the two sums is
        # relative to their uncancelled size, which is what the accumulation allowance of dQ / dK is built from
        ds_size = p * (np.abs(d_o) @ np.abs(v).T + np.abs(d_o * o).sum(axis=1, keepdims=True)) * abs(scale)
    else:
        p, der = act_value_deriv(act, s)
        ds = dp * der * scale
        ds_size = np.abs(ds)
    pr, dsr = (bf(p), bf(ds)) if rounded else (p, ds)
    ap, ads = np.abs(pr), np.abs(dsr)
    mx = lambda a, b: a.max(axis=1, keepdims=True) * b.max(axis=0, keepdims=True)
    return ((dsr @ k, dsr.T @ q, pr.T @ d_o),
            ((ds_size @ np.abs(k), mx(ads, np.abs(k))), (ds_size.T @ np.abs(q), mx(ads.T, np.abs(q))), (ap.T @ np.abs(d_o), mx(ap.T, np.abs(d_o)))))
