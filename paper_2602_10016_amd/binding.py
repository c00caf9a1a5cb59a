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
ACT_SOFTMAX, ACT_IDENTITY, ACT_RELU, ACT_GELU, ACT_GELU_TANH, ACT_SILU, ACT_GELU_POLY = range(7)
OP_GDPA_FWD, OP_GDPA_BWD, OP_SWA_FWD, OP_SWA_BWD, OP_SEED_FWD, OP_SEED_BWD = 0, 1, 2, 3, 4, 5
EXPORTS = ["kunlun_gdpa_fwd", "kunlun_gdpa_fwd_static", "kunlun_gdpa_bwd", "kunlun_seed_attn_fwd", "kunlun_seed_attn_bwd", "kunlun_swa_fwd", "kunlun_swa_bwd", "kunlun_workspace_bytes",
           "kunlun_sumkron_fwd", "kunlun_sumkron_workspace_bytes", "kunlun_sumkron_bwd", "kunlun_sumkron_bwd_workspace_bytes",
           "kunlun_check_offsets", "kunlun_stream_probe", "kunlun_jagged_stream_probe", "kunlun_strerror"]

_vp, _i, _i64, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_lib.kunlun_gdpa_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _i64, _f, _i, _vp, _i,
                                 _vp, _sz, _vp]
_lib.kunlun_gdpa_fwd.restype = _i
_lib.kunlun_gdpa_fwd_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _i64, _f, _i, _vp, _i, _vp]
_lib.kunlun_gdpa_fwd_static.restype = _i
STATIC_SCRATCH_BYTES = 1 << 20
_lib.kunlun_gdpa_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64,
                                 _i64, _f, _i, _vp, _i, _vp, _sz, _vp]
_lib.kunlun_gdpa_bwd.restype = _i
_lib.kunlun_seed_attn_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _f, _i, _vp, _i, _vp, _sz, _vp]
_lib.kunlun_seed_attn_fwd.restype = _i
_lib.kunlun_seed_attn_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _f, _i, _vp, _i,
                                      _vp, _sz, _vp]
_lib.kunlun_seed_attn_bwd.restype = _i
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
_lib.kunlun_stream_probe.argtypes = [_vp, _vp, _vp, _vp, _sz, _i, _i, _vp]
_lib.kunlun_stream_probe.restype = _i
_lib.kunlun_jagged_stream_probe.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i64, _i, _i, _i, _vp, _sz, _vp]
_lib.kunlun_jagged_stream_probe.restype = _i
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


def _check(name, t, *, dtype=None, shape=None, like=None, optional=False):
    """The C ABI sees plain pointers and trusts the layout, so a wrong dtype (int64 offsets read as int32), a
    strided view or a host tensor would be read as something else without any error.  Reject them here:
    TypeError for a wrong type or dtype, ValueError for a wrong layout, shape or device."""
    if t is None:
        if optional:
            return
        raise TypeError(f"{name}: a tensor is required")
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: expected a torch.Tensor, got {type(t).__name__}")
    want = like.dtype if (dtype is None and like is not None) else dtype
    if want is not None and t.dtype != want:
        raise TypeError(f"{name}: dtype {t.dtype}, expected {want}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous (got strides {tuple(t.stride())} for shape {tuple(t.shape)})")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")


def _on_device(**tensors):
    """Last check of every entry point (after types, layouts and shapes): all tensors on one HIP device."""
    dev = None
    for name, t in tensors.items():
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError(f"{name}: must be a CUDA (HIP) tensor, got device {t.device}")
        if dev is None:
            dev = t.device
        elif t.device != dev:
            raise ValueError(f"{name}: on {t.device}, expected {dev}")


# The operators trust their offsets and the length bounds max_q / max_kv / max_len (an under-estimate selects a kernel
# whose tiles are too small).  With KUNLUN_CHECK_OFFSETS=1 in the environment - or verify_offsets(True) - every call
# first runs kunlun_check_offsets on its offsets (one small kernel and a synchronising read per call: a debugging mode).
VERIFY_OFFSETS = os.environ.get("KUNLUN_CHECK_OFFSETS", "0") == "1"


def verify_offsets(on: bool = True) -> None:
    global VERIFY_OFFSETS
    VERIFY_OFFSETS = bool(on)


def _verify(name, offsets, total, max_len, stream):
    if not VERIFY_OFFSETS or offsets is None:
        return
    bad = check_offsets(offsets, total, max_len, stream=stream)
    if bad:
        raise ValueError(f"{name}: {bad} violation(s) of the contract offsets[0] = 0, 0 <= length <= {int(max_len)}, "
                         f"offsets[-1] = {int(total)}")


def _check_qkv(q, k, v):
    if not isinstance(q, torch.Tensor) or q.dim() != 3:
        raise ValueError("q: expected a [rows, H, d] tensor")
    _dtype_code(q)
    _check("q", q)
    H, d = q.shape[1], q.shape[2]
    if not isinstance(k, torch.Tensor) or k.dim() != 3:
        raise ValueError("k: expected a [rows, H, d] tensor")
    _check("k", k, like=q, shape=(k.shape[0], H, d))
    _check("v", v, like=q, shape=tuple(k.shape))


def _check_offsets(name, off, B=None, optional=False):
    if off is None and optional:
        return
    _check(name, off, dtype=torch.int32)
    if off.dim() != 1 or off.numel() < 1 or (B is not None and off.numel() != B + 1):
        raise ValueError(f"{name}: expected int32 [B+1]" + (f" with B = {B}" if B is not None else "") + f", got shape {tuple(off.shape)}")


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return FP32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _head_act(head_act, H):
    if head_act is None:
        return None
    if len(head_act) != H:
        raise ValueError(f"head_act: {len(head_act)} entries, expected one per head ({H})")
    return (ctypes.c_int32 * len(head_act))(*[int(a) for a in head_act])


def _workspace(workspace, nbytes, device):
    if workspace is None:
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    _check("workspace", workspace, dtype=torch.uint8)
    return workspace


def gdpa_fwd(q, k, v, kv_offsets, scale, act, *, q_offsets=None, max_q=None, max_kv, head_act=None, out=None,
             lse=None, want_lse=True, workspace=None, stream=None):
    """kunlun_gdpa_fwd.  q [total_q,H,d], k/v [total_kv,H,d] device tensors; returns (o, lse)."""
    _check_qkv(q, k, v)
    total_q, H, d = q.shape
    total_kv = k.shape[0]
    _check_offsets("kv_offsets", kv_offsets)
    B = kv_offsets.numel() - 1
    _check_offsets("q_offsets", q_offsets, B, optional=True)
    if max_q is None:
        raise ValueError("max_q is required (queries per example, or their upper bound with q_offsets)")
    o = torch.empty_like(q) if out is None else out
    _check("out", o, like=q, shape=tuple(q.shape))
    if lse is None and want_lse:
        lse = torch.empty((H, total_q), dtype=torch.float32, device=q.device)
    _check("lse", lse, dtype=torch.float32, like=None, shape=(H, total_q), optional=True)
    nbytes = workspace_bytes(OP_GDPA_FWD, B, H, d, max_q, max_kv, total_q, total_kv)
    ha = _head_act(head_act, H)
    ws = _workspace(workspace, nbytes, q.device)
    _on_device(q=q, k=k, v=v, kv_offsets=kv_offsets, q_offsets=q_offsets, out=o, lse=lse, workspace=ws)
    _verify("kv_offsets", kv_offsets, total_kv, max_kv, stream)
    _verify("q_offsets", q_offsets, total_q, max_q, stream)
    rc = _lib.kunlun_gdpa_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(q_offsets), _ptr(kv_offsets), B, H,
                              d, int(max_q), int(max_kv), total_q, total_kv, float(scale), int(act), ha,
                              _dtype_code(q), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return o, lse


def gdpa_fwd_static(q, k, v, kv_offsets, scale, act, *, out, lse=None, q_offsets=None, max_q, max_kv, head_act=None,
                    stream=None):
    """kunlun_gdpa_fwd_static: the forward call without a workspace and without any allocation - the caller
    passes the outputs (out, and lse for softmax heads); returns (out, lse)."""
    _check_qkv(q, k, v)
    total_q, H, d = q.shape
    _check_offsets("kv_offsets", kv_offsets)
    B = kv_offsets.numel() - 1
    _check_offsets("q_offsets", q_offsets, B, optional=True)
    _check("out", out, like=q, shape=tuple(q.shape))
    _check("lse", lse, dtype=torch.float32, shape=(H, total_q), optional=True)
    ha = _head_act(head_act, H)
    _on_device(q=q, k=k, v=v, kv_offsets=kv_offsets, q_offsets=q_offsets, out=out, lse=lse)
    _verify("kv_offsets", kv_offsets, k.shape[0], max_kv, stream)
    _verify("q_offsets", q_offsets, q.shape[0], max_q, stream)
    rc = _lib.kunlun_gdpa_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(q_offsets), _ptr(kv_offsets), B, H,
                                     d, int(max_q), int(max_kv), total_q, k.shape[0], float(scale), int(act), ha,
                                     _dtype_code(q), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return out, lse


def _grads(out, q, k, v):
    if out is None:
        return torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    dq, dk, dv = out
    _check("out[0] (dq)", dq, like=q, shape=tuple(q.shape))
    _check("out[1] (dk)", dk, like=q, shape=tuple(k.shape))
    _check("out[2] (dv)", dv, like=q, shape=tuple(v.shape))
    return dq, dk, dv


def gdpa_bwd(q, k, v, d_o, kv_offsets, scale, act, *, o=None, lse=None, q_offsets=None, max_q=None, max_kv,
             head_act=None, out=None, workspace=None, stream=None):
    """kunlun_gdpa_bwd.  Returns (dq, dk, dv) (written into the tensors of `out` when given).  o and lse are
    the forward results (read for softmax heads)."""
    _check_qkv(q, k, v)
    total_q, H, d = q.shape
    total_kv = k.shape[0]
    _check("d_o", d_o, like=q, shape=tuple(q.shape))
    _check("o", o, like=q, shape=tuple(q.shape), optional=True)
    _check("lse", lse, dtype=torch.float32, shape=(H, total_q), optional=True)
    _check_offsets("kv_offsets", kv_offsets)
    B = kv_offsets.numel() - 1
    _check_offsets("q_offsets", q_offsets, B, optional=True)
    if max_q is None:
        raise ValueError("max_q is required (queries per example, or their upper bound with q_offsets)")
    dq, dk, dv = _grads(out, q, k, v)
    nbytes = workspace_bytes(OP_GDPA_BWD, B, H, d, max_q, max_kv, total_q, total_kv)
    ha = _head_act(head_act, H)
    ws = _workspace(workspace, nbytes, q.device)
    _on_device(q=q, k=k, v=v, d_o=d_o, o=o, lse=lse, kv_offsets=kv_offsets, q_offsets=q_offsets, dq=dq, dk=dk, dv=dv,
               workspace=ws)
    _verify("kv_offsets", kv_offsets, total_kv, max_kv, stream)
    _verify("q_offsets", q_offsets, total_q, max_q, stream)
    rc = _lib.kunlun_gdpa_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                              _ptr(q_offsets), _ptr(kv_offsets), B, H, d, int(max_q), int(max_kv), total_q, total_kv,
                              float(scale), int(act), ha, _dtype_code(q), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return dq, dk, dv


def seed_attn_fwd(e_seed, k, v, kv_offsets, scale, act=ACT_SOFTMAX, *, max_kv, head_act=None, out=None, lse=None,
                  want_lse=True, workspace=None, stream=None):
    """kunlun_seed_attn_fwd.  e_seed [n_seeds,H,d] is shared by all examples; returns (o [B*n_seeds,H,d], lse)."""
    _check_qkv(e_seed, k, v)
    n_seeds, H, d = e_seed.shape
    _check_offsets("kv_offsets", kv_offsets)
    B = kv_offsets.numel() - 1
    total_q = B * n_seeds
    o = torch.empty((total_q, H, d), dtype=e_seed.dtype, device=e_seed.device) if out is None else out
    _check("out", o, like=e_seed, shape=(total_q, H, d))
    if lse is None and want_lse:
        lse = torch.empty((H, total_q), dtype=torch.float32, device=e_seed.device)
    _check("lse", lse, dtype=torch.float32, shape=(H, total_q), optional=True)
    ha = _head_act(head_act, H)
    ws = _workspace(workspace, workspace_bytes(OP_SEED_FWD, B, H, d, n_seeds, max_kv, total_q, k.shape[0]), e_seed.device)
    _on_device(e_seed=e_seed, k=k, v=v, kv_offsets=kv_offsets, out=o, lse=lse, workspace=ws)
    _verify("kv_offsets", kv_offsets, k.shape[0], max_kv, stream)
    rc = _lib.kunlun_seed_attn_fwd(_ptr(e_seed), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(kv_offsets), B, H, d, n_seeds,
                                   int(max_kv), k.shape[0], float(scale), int(act), ha, _dtype_code(e_seed), _ptr(ws), ws.numel(),
                                   _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return o, lse


def seed_attn_bwd(e_seed, k, v, d_o, kv_offsets, scale, act=ACT_SOFTMAX, *, o=None, lse=None, max_kv, head_act=None, out=None,
                  workspace=None, stream=None):
    """kunlun_seed_attn_bwd.  Returns (d_e [n_seeds,H,d], dk, dv); o and lse are the forward results."""
    _check_qkv(e_seed, k, v)
    n_seeds, H, d = e_seed.shape
    _check_offsets("kv_offsets", kv_offsets)
    B = kv_offsets.numel() - 1
    total_q = B * n_seeds
    _check("d_o", d_o, like=e_seed, shape=(total_q, H, d))
    _check("o", o, like=e_seed, shape=(total_q, H, d), optional=True)
    _check("lse", lse, dtype=torch.float32, shape=(H, total_q), optional=True)
    d_e, dk, dv = _grads(out, e_seed, k, v)
    ha = _head_act(head_act, H)
    ws = _workspace(workspace, workspace_bytes(OP_SEED_BWD, B, H, d, n_seeds, max_kv, total_q, k.shape[0]), e_seed.device)
    _on_device(e_seed=e_seed, k=k, v=v, d_o=d_o, o=o, lse=lse, kv_offsets=kv_offsets, d_e=d_e, dk=dk, dv=dv, workspace=ws)
    _verify("kv_offsets", kv_offsets, k.shape[0], max_kv, stream)
    rc = _lib.kunlun_seed_attn_bwd(_ptr(e_seed), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(d_e), _ptr(dk), _ptr(dv),
                                   _ptr(kv_offsets), B, H, d, n_seeds, int(max_kv), k.shape[0], float(scale), int(act), ha,
                                   _dtype_code(e_seed), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return d_e, dk, dv


def swa_fwd(q, k, v, offsets, window_left, window_right, scale, *, max_len, out=None, lse=None, want_lse=True,
            workspace=None, stream=None):
    """kunlun_swa_fwd.  q, k, v [total,H,d] share `offsets`; returns (o, lse)."""
    _check_qkv(q, k, v)
    total, H, d = q.shape
    if k.shape[0] != total:
        raise ValueError(f"k: {k.shape[0]} rows, expected {total} (self-attention: q, k, v share the offsets)")
    _check_offsets("offsets", offsets)
    B = offsets.numel() - 1
    o = torch.empty_like(q) if out is None else out
    _check("out", o, like=q, shape=tuple(q.shape))
    if lse is None and want_lse:
        lse = torch.empty((H, total), dtype=torch.float32, device=q.device)
    _check("lse", lse, dtype=torch.float32, shape=(H, total), optional=True)
    nbytes = workspace_bytes(OP_SWA_FWD, B, H, d, max_len, max_len, total, total)
    ws = _workspace(workspace, nbytes, q.device)
    _on_device(q=q, k=k, v=v, offsets=offsets, out=o, lse=lse, workspace=ws)
    _verify("offsets", offsets, total, max_len, stream)
    rc = _lib.kunlun_swa_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(offsets), B, H, d, int(max_len),
                             total, int(window_left), int(window_right), float(scale), _dtype_code(q), _ptr(ws),
                             ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return o, lse


def swa_bwd(q, k, v, o, lse, d_o, offsets, window_left, window_right, scale, *, max_len, out=None, workspace=None,
            stream=None):
    """kunlun_swa_bwd.  o and lse are the results of swa_fwd.  Returns (dq, dk, dv) (written into the tensors
    of `out` when given)."""
    _check_qkv(q, k, v)
    total, H, d = q.shape
    if k.shape[0] != total:
        raise ValueError(f"k: {k.shape[0]} rows, expected {total} (self-attention: q, k, v share the offsets)")
    _check("o", o, like=q, shape=tuple(q.shape))
    _check("d_o", d_o, like=q, shape=tuple(q.shape))
    _check("lse", lse, dtype=torch.float32, shape=(H, total))
    _check_offsets("offsets", offsets)
    B = offsets.numel() - 1
    dq, dk, dv = _grads(out, q, k, v)
    nbytes = workspace_bytes(OP_SWA_BWD, B, H, d, max_len, max_len, total, total)
    ws = _workspace(workspace, nbytes, q.device)
    _on_device(q=q, k=k, v=v, o=o, lse=lse, d_o=d_o, offsets=offsets, dq=dq, dk=dk, dv=dv, workspace=ws)
    _verify("offsets", offsets, q.shape[0], max_len, stream)
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
    _dtype_code(x)
    _check("x", x)
    if x.dim() != 3 or z.dim() != 3:
        raise ValueError("x: expected [B, S, D]; z: expected [k, S, T]")
    B, S, D = x.shape
    k, _, T = z.shape
    _check("z", z, like=x, shape=(k, S, T))
    _check("w", w, like=x, shape=(k, D, D))
    y = torch.empty((B, T, D), dtype=x.dtype, device=x.device) if out is None else out
    _check("out", y, like=x, shape=(B, T, D))
    ws = _workspace(workspace, sumkron_workspace_bytes(B, S, T, D, k, _dtype_code(x)), x.device)
    _on_device(x=x, z=z, w=w, out=y, workspace=ws)
    rc = _lib.kunlun_sumkron_fwd(_ptr(x), _ptr(z), _ptr(w), _ptr(y), B, S, T, D, k, _dtype_code(x), _ptr(ws), ws.numel(),
                                 _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return y


def sumkron_bwd_workspace_bytes(B, S, T, D, k, dtype=BF16) -> int:
    return int(_lib.kunlun_sumkron_bwd_workspace_bytes(B, S, T, D, k, dtype))


def sumkron_bwd(x, z, w, dy, *, workspace=None, stream=None):
    """kunlun_sumkron_bwd.  x [B,S,D], z [k,S,T], w [k,D,D], dy [B,T,D] device tensors; returns (dx, dz, dw)."""
    _dtype_code(x)
    _check("x", x)
    if x.dim() != 3 or z.dim() != 3:
        raise ValueError("x: expected [B, S, D]; z: expected [k, S, T]")
    B, S, D = x.shape
    k, _, T = z.shape
    _check("z", z, like=x, shape=(k, S, T))
    _check("w", w, like=x, shape=(k, D, D))
    _check("dy", dy, like=x, shape=(B, T, D))
    dx, dz, dw = torch.empty_like(x), torch.empty_like(z), torch.empty_like(w)
    ws = _workspace(workspace, sumkron_bwd_workspace_bytes(B, S, T, D, k, _dtype_code(x)), x.device)
    _on_device(x=x, z=z, w=w, dy=dy, workspace=ws)
    rc = _lib.kunlun_sumkron_bwd(_ptr(x), _ptr(z), _ptr(w), _ptr(dy), _ptr(dx), _ptr(dz), _ptr(dw), B, S, T, D, k,
                                 _dtype_code(x), _ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return dx, dz, dw


def stream_probe(a, b, c, out, reads, write, *, stream=None):
    """kunlun_stream_probe: one streaming pass over `reads` of the uint8 device buffers a, b, c (+ a write of out)."""
    for name, t in (("a", a), ("b", b), ("c", c), ("out", out)):
        _check(name, t, dtype=torch.uint8, optional=name in ("b", "c"))
    for name, t in (("b", b), ("c", c)):
        if t is not None and t.numel() != a.numel():
            raise ValueError(f"{name}: {t.numel()} bytes, expected {a.numel()}")
    if out.numel() < (a.numel() if write else 4096):
        raise ValueError(f"out: {out.numel()} bytes are too few")
    _on_device(a=a, b=b, c=c, out=out)
    rc = _lib.kunlun_stream_probe(_ptr(a), _ptr(b), _ptr(c), _ptr(out), a.numel(), int(reads), int(write), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)


def jagged_stream_probe(a, b, c, out_a, out_b, offsets, max_len, reads, writes, workgroups_per_cu, *, workspace=None,
                        stream=None):
    """kunlun_jagged_stream_probe: one walk per (example, head) over the rows of bf16 [total, H, d] tensors."""
    _check("a", a, dtype=torch.bfloat16)
    if a.dim() != 3:
        raise ValueError(f"a: expected [total, H, d], got shape {tuple(a.shape)}")
    for name, t in (("b", b), ("c", c), ("out_a", out_a), ("out_b", out_b)):
        _check(name, t, dtype=torch.bfloat16, shape=a.shape, optional=True)
    total, H, d = a.shape
    _check_offsets("offsets", offsets)
    B = offsets.numel() - 1
    need = 256 + (4 * (B + 1) + 255) // 256 * 256
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    _check("workspace", workspace, dtype=torch.uint8)
    _on_device(a=a, b=b, c=c, out_a=out_a, out_b=out_b, offsets=offsets, workspace=workspace)
    rc = _lib.kunlun_jagged_stream_probe(_ptr(a), _ptr(b), _ptr(c), _ptr(out_a), _ptr(out_b), _ptr(offsets), B, H, d, int(max_len),
                                         total, int(reads), int(writes), int(workgroups_per_cu), _ptr(workspace),
                                         workspace.numel(), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)


def check_offsets(offsets, total, max_len, *, stream=None) -> int:
    """kunlun_check_offsets, then a synchronising read of the count (0 = the offsets obey the contract)."""
    _check_offsets("offsets", offsets)
    _on_device(offsets=offsets)
    out = torch.empty(1, dtype=torch.int32, device=offsets.device)
    rc = _lib.kunlun_check_offsets(_ptr(offsets), offsets.numel() - 1, int(total), int(max_len), _ptr(out), _stream(stream))
    if rc != OK:
        raise KunlunError(rc)
    return int(out.item())
