"""torch.autograd.Function wrappers of the C-ABI entry points: the forward call and the backward call
of each operator tied together so that the operators can sit inside a PyTorch training graph.
Marshalling only - every computation runs in the HIP library (see binding.py).

    gdpa(q, k, v, kv_offsets, scale, act, ...)                -> o    Eq. (GDPA) / softmax attention, jagged
    sliding_window_attention(q, k, v, offsets, left, right, scale, max_len)   -> o    Eq. (sliding window)
    sumkron_linear(x, z, w)                                   -> y    Eq. (SumKronLinear)

Inputs must be contiguous device tensors (bf16 or fp32); offsets are int32 device tensors and carry
no gradient.  The incoming gradient is made contiguous before it is handed to the library.
"""
import torch

from . import binding as kb


class _GDPA(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, kv_offsets, scale, act, q_offsets, max_q, max_kv, head_act):
        acts = [act] if head_act is None else list(head_act)
        need_lse = any(a == kb.ACT_SOFTMAX for a in acts)
        o, lse = kb.gdpa_fwd(q, k, v, kv_offsets, scale, act, q_offsets=q_offsets, max_q=max_q, max_kv=max_kv,
                             head_act=head_act, want_lse=need_lse)
        ctx.save_for_backward(q, k, v, kv_offsets, q_offsets, o if need_lse else None, lse)
        ctx.args = (scale, act, max_q, max_kv, head_act)
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, kv_offsets, q_offsets, o, lse = ctx.saved_tensors
        scale, act, max_q, max_kv, head_act = ctx.args
        dq, dk, dv = kb.gdpa_bwd(q, k, v, d_o.contiguous(), kv_offsets, scale, act, o=o, lse=lse, q_offsets=q_offsets,
                                 max_q=max_q, max_kv=max_kv, head_act=head_act)
        return dq, dk, dv, None, None, None, None, None, None, None


def gdpa(q, k, v, kv_offsets, scale, act=kb.ACT_GELU, *, q_offsets=None, max_q=None, max_kv, head_act=None):
    """O_h = Act_h(Q_h K_h^T scale) V_h per example over jagged rows (act = ACT_SOFTMAX: softmax attention).
    q [total_q, H, d], k / v [total_kv, H, d]; without q_offsets every example has max_q queries."""
    return _GDPA.apply(q, k, v, kv_offsets, float(scale), int(act), q_offsets, max_q, int(max_kv), head_act)


class _SWA(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, offsets, left, right, scale, max_len):
        o, lse = kb.swa_fwd(q, k, v, offsets, left, right, scale, max_len=max_len)
        ctx.save_for_backward(q, k, v, offsets, o, lse)
        ctx.args = (left, right, scale, max_len)
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, offsets, o, lse = ctx.saved_tensors
        left, right, scale, max_len = ctx.args
        dq, dk, dv = kb.swa_bwd(q, k, v, o, lse, d_o.contiguous(), offsets, left, right, scale, max_len=max_len)
        return dq, dk, dv, None, None, None, None, None


def sliding_window_attention(q, k, v, offsets, left, right, scale, *, max_len):
    """Query t of a sequence attends to keys [t - left, t + right] of the same sequence (negative = unbounded)."""
    return _SWA.apply(q, k, v, offsets, int(left), int(right), float(scale), int(max_len))


class _SumKron(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, z, w):
        ctx.save_for_backward(x, z, w)
        return kb.sumkron_fwd(x, z, w)

    @staticmethod
    def backward(ctx, dy):
        x, z, w = ctx.saved_tensors
        return kb.sumkron_bwd(x, z, w, dy.contiguous())


def sumkron_linear(x, z, w):
    """Y_b = sum_i Z_i^T X_b W_i;  x [B, S, D], z [k, S, T], w [k, D, D] -> y [B, T, D]."""
    return _SumKron.apply(x, z, w)
