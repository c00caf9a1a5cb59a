"""ctypes front end of the C oracle: numpy float64 arrays in, numpy float64 arrays out.

Argument marshalling only; every number is computed by kunlun_oracle.c.
Layout: Q [total_q, H, d], K/V [total_kv, H, d], O like Q, LSE [H, total_q].
"""
import ctypes

import numpy as np

from .build import build

ACT_SOFTMAX, ACT_IDENTITY, ACT_RELU, ACT_GELU, ACT_GELU_TANH, ACT_SILU, ACT_GELU_POLY = range(7)

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _p(a, t=_dp):
    return None if a is None else a.ctypes.data_as(t)


def _check(q, k, v, H, d):
    assert q.ndim == 3 and k.ndim == 3 and v.ndim == 3, "expected [tokens, H, d]"
    assert q.shape[1:] == (H, d) and k.shape[1:] == (H, d) and v.shape == k.shape


class OracleLib:
    """One loaded build of kunlun_oracle.c.  The module-level functions below use the default
    build; tests that plant mistakes in a copy of the C source load that copy through this class."""

    def __init__(self, path):
        lib = ctypes.CDLL(path)
        lib.oracle_gdpa_fwd.argtypes = [_dp, _dp, _dp, _dp, _dp, _ip, _ip, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_int, _ip]
        lib.oracle_gdpa_bwd.argtypes = [_dp, _dp, _dp, _dp, _dp, _dp, _dp, _ip, _ip, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                        ctypes.c_int, _ip]
        lib.oracle_swa_fwd.argtypes = [_dp, _dp, _dp, _dp, _dp, _ip, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        lib.oracle_swa_bwd.argtypes = [_dp, _dp, _dp, _dp, _dp, _dp, _dp, _ip, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        lib.oracle_sumkron_fwd.argtypes = [_dp, _dp, _dp, _dp] + [ctypes.c_int] * 5
        lib.oracle_sumkron_bwd.argtypes = [_dp] * 7 + [ctypes.c_int] * 5
        lib.oracle_act_value.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.oracle_act_value.restype = ctypes.c_double
        lib.oracle_act_deriv.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.oracle_act_deriv.restype = ctypes.c_double
        self._lib = lib

    def gdpa_fwd(self, q, k, v, kv_offsets, scale, act, q_offsets=None, max_q=None, head_act=None):
        """Returns (O, LSE).  q_offsets=None: dense queries, max_q rows per example."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        H, d = q.shape[1], q.shape[2]
        _check(q, k, v, H, d)
        kvo, qo, ha = _i32(kv_offsets), _i32(q_offsets), _i32(head_act)
        B = kvo.size - 1
        if qo is None:
            assert max_q is not None and q.shape[0] == B * max_q
        else:
            assert qo.size == B + 1 and qo[-1] == q.shape[0]
            max_q = 0
        assert kvo[-1] == k.shape[0]
        o = np.empty_like(q)
        lse = np.empty((H, q.shape[0]), dtype=np.float64)
        rc = self._lib.oracle_gdpa_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), _p(qo, _ip), _p(kvo, _ip), B, H, d,
                                       int(max_q), q.shape[0], float(scale), int(act), _p(ha, _ip))
        if rc != 0:
            raise ValueError("oracle_gdpa_fwd: unknown activation")
        return o, lse

    def gdpa_bwd(self, q, k, v, d_o, kv_offsets, scale, act, q_offsets=None, max_q=None, head_act=None):
        """Returns (dQ, dK, dV), the gradient of <O, dO>."""
        q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
        H, d = q.shape[1], q.shape[2]
        _check(q, k, v, H, d)
        assert d_o.shape == q.shape
        kvo, qo, ha = _i32(kv_offsets), _i32(q_offsets), _i32(head_act)
        B = kvo.size - 1
        if qo is None:
            assert max_q is not None and q.shape[0] == B * max_q
        else:
            assert qo.size == B + 1 and qo[-1] == q.shape[0]
            max_q = 0
        assert kvo[-1] == k.shape[0]
        dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
        rc = self._lib.oracle_gdpa_bwd(_p(q), _p(k), _p(v), _p(d_o), _p(dq), _p(dk), _p(dv), _p(qo, _ip),
                                       _p(kvo, _ip), B, H, d, int(max_q), q.shape[0], k.shape[0], float(scale),
                                       int(act), _p(ha, _ip))
        if rc != 0:
            raise ValueError("oracle_gdpa_bwd: unknown activation")
        return dq, dk, dv

    def seed_attn_fwd(self, e_seed, k, v, kv_offsets, scale, act, head_act=None):
        """Seed-level attention with seeds shared across the batch (Sec. "Hierarchical Seed Pooling", stage 1;
        Eq. (seed-level attention)): every example uses the same n_seeds query rows.  Written out as the
        definition: the seed block repeated once per example, then the per-example attention.  Returns (O, LSE)."""
        e_seed = _f64(e_seed)
        B = _i32(kv_offsets).size - 1
        q = np.ascontiguousarray(np.tile(e_seed, (B, 1, 1)))
        return self.gdpa_fwd(q, k, v, kv_offsets, scale, act, max_q=e_seed.shape[0], head_act=head_act)

    def seed_attn_bwd(self, e_seed, k, v, d_o, kv_offsets, scale, act, head_act=None):
        """Gradient of <O, dO> of seed_attn_fwd: (dE, dK, dV), where dE is the sum over the examples of the
        per-example query gradients (the seeds are one shared parameter block)."""
        e_seed = _f64(e_seed)
        B = _i32(kv_offsets).size - 1
        q = np.ascontiguousarray(np.tile(e_seed, (B, 1, 1)))
        dq, dk, dv = self.gdpa_bwd(q, k, v, d_o, kv_offsets, scale, act, max_q=e_seed.shape[0], head_act=head_act)
        d_e = np.zeros_like(e_seed)
        for b in range(B):
            d_e += dq[b * e_seed.shape[0]:(b + 1) * e_seed.shape[0]]
        return d_e, dk, dv

    def swa_fwd(self, q, k, v, offsets, left, right, scale):
        """Sliding-window softmax self-attention; left/right < 0 means unbounded.  Returns (O, LSE)."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        H, d = q.shape[1], q.shape[2]
        _check(q, k, v, H, d)
        off = _i32(offsets)
        assert off[-1] == q.shape[0] == k.shape[0]
        o = np.empty_like(q)
        lse = np.empty((H, q.shape[0]), dtype=np.float64)
        self._lib.oracle_swa_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), _p(off, _ip), off.size - 1, H, d, q.shape[0],
                                 int(left), int(right), float(scale))
        return o, lse

    def swa_bwd(self, q, k, v, d_o, offsets, left, right, scale):
        q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
        H, d = q.shape[1], q.shape[2]
        _check(q, k, v, H, d)
        off = _i32(offsets)
        assert off[-1] == q.shape[0] == k.shape[0]
        dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
        self._lib.oracle_swa_bwd(_p(q), _p(k), _p(v), _p(d_o), _p(dq), _p(dk), _p(dv), _p(off, _ip), off.size - 1, H,
                                 d, q.shape[0], int(left), int(right), float(scale))
        return dq, dk, dv

    def sumkron_fwd(self, x, z, w):
        """SumKronLinear: x [B,S,D], z [k,S,T], w [k,D,D] -> y [B,T,D]."""
        x, z, w = _f64(x), _f64(z), _f64(w)
        B, S, D = x.shape
        k, S2, T = z.shape
        assert S2 == S and w.shape == (k, D, D)
        y = np.zeros((B, T, D), dtype=np.float64)
        rc = self._lib.oracle_sumkron_fwd(_p(x), _p(z), _p(w), _p(y), B, S, T, D, k)
        assert rc == 0
        return y

    def sumkron_bwd(self, x, z, w, dy):
        """Gradient of <Y, dY> with respect to x, z, w.  Returns (dx, dz, dw)."""
        x, z, w, dy = _f64(x), _f64(z), _f64(w), _f64(dy)
        B, S, D = x.shape
        k, S2, T = z.shape
        assert S2 == S and w.shape == (k, D, D) and dy.shape == (B, T, D)
        dx, dz, dw = np.zeros_like(x), np.zeros_like(z), np.zeros_like(w)
        rc = self._lib.oracle_sumkron_bwd(_p(x), _p(z), _p(w), _p(dy), _p(dx), _p(dz), _p(dw), B, S, T, D, k)
        assert rc == 0
        return dx, dz, dw

    def act_value(self, act, x):
        return self._lib.oracle_act_value(int(act), float(x))

    def act_deriv(self, act, x):
        return self._lib.oracle_act_deriv(int(act), float(x))

    def num_threads(self):
        return int(self._lib.oracle_num_threads())


_default = OracleLib(build())
gdpa_fwd = _default.gdpa_fwd
gdpa_bwd = _default.gdpa_bwd
seed_attn_fwd = _default.seed_attn_fwd
seed_attn_bwd = _default.seed_attn_bwd
swa_fwd = _default.swa_fwd
swa_bwd = _default.swa_bwd
sumkron_fwd = _default.sumkron_fwd
sumkron_bwd = _default.sumkron_bwd
act_value = _default.act_value
act_deriv = _default.act_deriv
num_threads = _default.num_threads
