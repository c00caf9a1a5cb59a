"""The Python binding rejects tensors that the C ABI (plain pointers, trusted layout) would misread:
wrong dtype (int64 offsets would be read as int32 pairs), strided views, host tensors, wrong shapes.
Runs without a GPU: every rejection happens before the library is called."""
import pytest
import torch

from paper_2602_10016_amd import binding as kb

H, D = 2, 64


def qkv(rows_q=8, rows_k=12, dtype=torch.bfloat16):
    return (torch.zeros((rows_q, H, D), dtype=dtype), torch.zeros((rows_k, H, D), dtype=dtype),
            torch.zeros((rows_k, H, D), dtype=dtype))


def off(*vals, dtype=torch.int32):
    return torch.tensor(vals, dtype=dtype)


def test_host_tensors_are_rejected():
    q, k, v = qkv()
    with pytest.raises(ValueError, match="CUDA"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)


def test_int64_offsets_are_rejected_before_anything_else():
    q, k, v = qkv()
    with pytest.raises(TypeError, match="int32"):
        kb.gdpa_fwd(q, k, v, off(0, 12, dtype=torch.int64), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(TypeError, match="int32"):
        kb.swa_fwd(k, k, k, torch.cumsum(torch.tensor([0, 12]), 0), 3, 0, 1.0, max_len=12)
    with pytest.raises(TypeError, match="int32"):
        kb.check_offsets(off(0, 12, dtype=torch.int64), 12, 12)


def test_strided_views_are_rejected():
    q, k, v = qkv()
    fused = torch.zeros((12, 3, H, D), dtype=torch.bfloat16)     # a packed QKV projection
    with pytest.raises(ValueError, match="contiguous"):
        kb.gdpa_fwd(q, fused[:, 1], fused[:, 2], off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(ValueError, match="contiguous"):
        kb.gdpa_fwd(q.transpose(0, 1).transpose(0, 1)[::2], k, v, off(0, 12), 1.0, kb.ACT_GELU, max_q=4, max_kv=12)
    with pytest.raises(ValueError, match="contiguous"):
        kb.gdpa_bwd(q, k, v, torch.zeros((8, H, 2 * D), dtype=torch.bfloat16)[:, :, :D], off(0, 12), 1.0, kb.ACT_GELU,
                    max_q=8, max_kv=12)


def test_mixed_or_unsupported_dtypes_are_rejected():
    q, k, v = qkv()
    with pytest.raises(TypeError, match="dtype"):
        kb.gdpa_fwd(q, k.float(), v, off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(TypeError, match="unsupported dtype"):
        kb.gdpa_fwd(q.half(), k.half(), v.half(), off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(TypeError, match="dtype"):
        kb.gdpa_bwd(q, k, v, q.float(), off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(TypeError, match="dtype"):
        kb.swa_bwd(k, k, k, k, torch.zeros((H, 12), dtype=torch.float64), k, off(0, 12), 3, 0, 1.0, max_len=12)


def test_shapes_are_checked():
    q, k, v = qkv()
    with pytest.raises(ValueError, match="shape"):
        kb.gdpa_fwd(q, k, v[:10].contiguous(), off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(ValueError, match="shape"):
        kb.gdpa_fwd(q, k, torch.zeros((12, H, 32), dtype=torch.bfloat16), off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(ValueError, match=r"\[B\+1\]"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, q_offsets=off(0, 4, 8), max_q=8, max_kv=12)
    with pytest.raises(ValueError, match="shape"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12, out=torch.zeros((4, H, D), dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="shape"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_SOFTMAX, max_q=8, max_kv=12, lse=torch.zeros((8, H)))
    with pytest.raises(ValueError, match="one per head"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12, head_act=[3])
    with pytest.raises(ValueError, match="max_q"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, max_kv=12)
    with pytest.raises(ValueError, match="rows"):
        kb.swa_fwd(q, k, v, off(0, 8), 3, 0, 1.0, max_len=8)
    with pytest.raises(ValueError, match="shape"):
        kb.sumkron_fwd(torch.zeros((2, 32, 128), dtype=torch.bfloat16), torch.zeros((2, 16, 4), dtype=torch.bfloat16),
                       torch.zeros((2, 128, 128), dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="shape"):
        kb.sumkron_bwd(torch.zeros((2, 32, 128), dtype=torch.bfloat16), torch.zeros((2, 32, 4), dtype=torch.bfloat16),
                       torch.zeros((2, 128, 128), dtype=torch.bfloat16), torch.zeros((2, 4, 64), dtype=torch.bfloat16))


def test_non_tensor_arguments_are_rejected():
    q, k, v = qkv()
    with pytest.raises(TypeError, match="torch.Tensor"):
        kb.gdpa_fwd(q, k, v, [0, 12], 1.0, kb.ACT_GELU, max_q=8, max_kv=12)
    with pytest.raises(TypeError, match="uint8"):
        kb.gdpa_fwd(q, k, v, off(0, 12), 1.0, kb.ACT_GELU, max_q=8, max_kv=12, workspace=torch.zeros(1024))
