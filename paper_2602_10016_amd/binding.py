"""Thin ctypes binding of libkunlun.so: argument marshalling only.

torch is used for device memory and the current HIP stream; every step of the operators
runs in the library's kernels.  Importing this module fails loudly when the library has not
been built (python -m paper_2602_10016_amd.build, or __graft_entry__.build()).
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkunlun.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python paper_2602_10016_amd/build.py). "
                      "There is no fallback implementation.")
_lib = ctypes.CDLL(LIB_PATH)

OK = 0
ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_ALIGN, ERR_WORKSPACE, ERR_LAUNCH = -1, -2, -3, -4, -5, -6
BF16, FP32 = 0, 1
ACT_SOFTMAX, ACT_IDENTITY, ACT_RELU, ACT_GELU, ACT_GELU_TANH, ACT_SILU = range(6)
OP_GDPA_FWD, OP_GDPA_BWD, OP_SWA_FWD, OP_SWA_BWD = 0, 1, 2, 3
EXPORTS = ["kunlun_gdpa_fwd", "kunlun_gdpa_bwd", "kunlun_swa_fwd", "kunlun_swa_bwd", "kunlun_workspace_bytes",
           "kunlun_sumkron_fwd", "kunlun_sumkron_workspace_bytes", "kunlun_sumkron_bwd", "kunlun_sumkron_bwd_workspace_bytes",
           "kunlun_check_offsets", "kunlun_strerror"]

_vp, _i, _i64, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_lib.kunlun_gdpa_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _i64, _f, _i, _vp, _i,
                                 _vp, _sz, _vp]
_lib.kunlun_gdpa_fwd.restype = _i
_lib.kunlun_gdpa_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64,
                                 _i64, _f, _i, _vp, _i, _vp, _sz, _vp]
_lib.kunlun_gdpa_bwd.restype = _i
_lib.kunlun_swa_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i64, _i, _i, _f, _i, _vp, _sz, _vp]
_lib.kunlun_swa_fwd.restype = _i
_lib.kunlun_swa_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i64, _i, _i, _f, _i, _vp,
                                _sz, _vp]
_lib.kunlun_swa_bwd.restype = _i
_lib.kunlun_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i, _i64, _i64]
_lib.kunlun_workspace_bytes.restype = _sz
_lib.kunlun_sumkron_fwd.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.kunlun_sumkron_fwd.restype = _i
_lib.kunlun_sumkron_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i]
_lib.kunlun_sumkron_workspace_bytes.restype = _sz
_lib.kunlun_sumkron_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.kunlun_sumkron_bwd.restype = _i
_lib.kunlun_sumkron_bwd_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i]
_lib.kunlun_sumkron_bwd_workspace_bytes.restype = _sz
_lib.kunlun_check_offsets.argtypes = [_vp, _i, _i64, _i, _vp, _vp]
_lib.kunlun_check_offsets.restype = _i
_lib.kunlun_strerror.argtypes = [_i]
_lib.kunlun_strerror.restype = ctypes.c_char_p


class KunlunError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"kunlun status {status}: {strerror(status)}")


def strerror(status: int) -> str:
    return _lib.kunlun_strerror(int(status)).decode()


def workspace_bytes(op, B, H, d, max_q, max_kv, total_q, total_kv) -> int:
    return int(_lib.kunlun_workspace_bytes(op, B, H, d, max_q, max_kv, total_q, total_kv))


def raw():
    """The ctypes library handle, for tests that call the C ABI with hand-made arguments."""
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return FP32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _head_act(head_act):
    if head_act is None:
        return None
    return (ctypes.c_int32 * len(head_act))(*[int(a) for a in head_act])


def _workspace(workspace, nbytes, device):
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace


def gdpa_fwd(q, k, v, kv_offsets, scale, act, *, q_offsets=None, max_q=None, max_kv, head_act=None, out=None,
             lse=None, want_lse=True, workspace=None, stream=None):
    """kunlun_gdpa_fwd.  q [total_q,H,d], k/v [total_kv,H,d] device tensors; returns (o, lse)."""
    total_q, H, d = q.shape
    total_kv = k.shape[0]
    B = kv_offsets.numel() - 1
    if q_offsets is None:
        assert max_q is not None
    elif max_q is None:
        raise ValueError("max_q is required with q_offsets")
    o = torch.empty_like(q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty((H, total_q), dtype=torch.float32, device=q.device)
    nbytes = workspace_bytes(OP_GDPA_FWD, B, H, d, max_q, max_kv, total_q, total_kv)
    ws = _workspace(workspace, nbytes, q.device)
    ha = _head_act(head_act)
    rc = _lib.kunlun_gdpa_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(q_offsets), _ptr(kv_offsets), B, H,
                              d, int(max_q), int(max_kv), total_q, total_kv, float(scale), int(act), ha,
                              _dtype_code(q), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return o, lse


def gdpa_bwd(q, k, v, d_o, kv_offsets, scale, act, *, o=None, lse=None, q_offsets=None, max_q=None, max_kv,
             head_act=None, workspace=None, stream=None):
    """kunlun_gdpa_bwd.  Returns (dq, dk, dv).  o and lse are the forward results (softmax heads)."""
    total_q, H, d = q.shape
    total_kv = k.shape[0]
    B = kv_offsets.numel() - 1
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nbytes = workspace_bytes(OP_GDPA_BWD, B, H, d, max_q, max_kv, total_q, total_kv)
    ws = _workspace(workspace, nbytes, q.device)
    ha = _head_act(head_act)
    rc = _lib.kunlun_gdpa_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                              _ptr(q_offsets), _ptr(kv_offsets), B, H, d, int(max_q), int(max_kv), total_q, total_kv,
                              float(scale), int(act), ha, _dtype_code(q), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return dq, dk, dv


def swa_fwd(q, k, v, offsets, window_left, window_right, scale, *, max_len, out=None, lse=None, want_lse=True,
            workspace=None, stream=None):
    """kunlun_swa_fwd.  q, k, v [total,H,d] share `offsets`; returns (o, lse)."""
    total, H, d = q.shape
    B = offsets.numel() - 1
    o = torch.empty_like(q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty((H, total), dtype=torch.float32, device=q.device)
    nbytes = workspace_bytes(OP_SWA_FWD, B, H, d, max_len, max_len, total, total)
    ws = _workspace(workspace, nbytes, q.device)
    rc = _lib.kunlun_swa_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(offsets), B, H, d, int(max_len),
                             total, int(window_left), int(window_right), float(scale), _dtype_code(q), _ptr(ws),
                             ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return o, lse


def swa_bwd(q, k, v, o, lse, d_o, offsets, window_left, window_right, scale, *, max_len, workspace=None,
            stream=None):
    """kunlun_swa_bwd.  o and lse are the results of swa_fwd.  Returns (dq, dk, dv)."""
    total, H, d = q.shape
    B = offsets.numel() - 1
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nbytes = workspace_bytes(OP_SWA_BWD, B, H, d, max_len, max_len, total, total)
    ws = _workspace(workspace, nbytes, q.device)
    rc = _lib.kunlun_swa_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                             _ptr(offsets), B, H, d, int(max_len), total, int(window_left), int(window_right),
                             float(scale), _dtype_code(q), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return dq, dk, dv


def sumkron_workspace_bytes(B, S, T, D, k, dtype=BF16) -> int:
    return int(_lib.kunlun_sumkron_workspace_bytes(B, S, T, D, k, dtype))


def sumkron_fwd(x, z, w, *, out=None, workspace=None, stream=None):
    """kunlun_sumkron_fwd.  x [B,S,D], z [k,S,T], w [k,D,D] device tensors; returns y [B,T,D]."""
    B, S, D = x.shape
    k, _, T = z.shape
    y = torch.empty((B, T, D), dtype=x.dtype, device=x.device) if out is None else out
    ws = _workspace(workspace, sumkron_workspace_bytes(B, S, T, D, k, _dtype_code(x)), x.device)
    rc = _lib.kunlun_sumkron_fwd(_ptr(x), _ptr(z), _ptr(w), _ptr(y), B, S, T, D, k, _dtype_code(x), _ptr(ws), ws.numel(),
                                 _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return y


def sumkron_bwd_workspace_bytes(B, S, T, D, k, dtype=BF16) -> int:
    return int(_lib.kunlun_sumkron_bwd_workspace_bytes(B, S, T, D, k, dtype))


def sumkron_bwd(x, z, w, dy, *, workspace=None, stream=None):
    """kunlun_sumkron_bwd.  x [B,S,D], z [k,S,T], w [k,D,D], dy [B,T,D] device tensors; returns (dx, dz, dw)."""
    B, S, D = x.shape
    k, _, T = z.shape
    dx, dz, dw = torch.empty_like(x), torch.empty_like(z), torch.empty_like(w)
    ws = _workspace(workspace, sumkron_bwd_workspace_bytes(B, S, T, D, k, _dtype_code(x)), x.device)
    rc = _lib.kunlun_sumkron_bwd(_ptr(x), _ptr(z), _ptr(w), _ptr(dy), _ptr(dx), _ptr(dz), _ptr(dw), B, S, T, D, k,
                                 _dtype_code(x), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return dx, dz, dw


def check_offsets(offsets, total, max_len, *, stream=None) -> int:
    """kunlun_check_offsets, then a synchronising read of the count (0 = the offsets obey the contract)."""
    out = torch.empty(1, dtype=torch.int32, device=offsets.device)
    rc = _lib.kunlun_check_offsets(_ptr(offsets), offsets.numel() - 1, int(total), int(max_len), _ptr(out), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return int(out.item())
