"""kunlun_gdpa_fwd_static (the forward entry point that takes no workspace and allocates nothing: its work lists
live in a fixed device array inside the library) against kunlun_gdpa_fwd, through the C ABI: bit-identical
outputs, on two calls in a row of which the second is smaller (the array keeps the first call's contents), on the
launch kinds that use the array differently - sorted issue order, no order at all, query-tile tables."""
import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import offsets_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def both(kb, wl, act, q_offsets=None, max_q=None, head_act=None):
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    kvo, qo = offsets_dev(wl.kv_offsets), offsets_dev(q_offsets)
    max_q = wl.Nq if max_q is None else max_q
    max_kv = max(wl.max_kv, 1)
    ref_o, ref_lse = kb.gdpa_fwd(q, k, v, kvo, wl.scale, act, q_offsets=qo, max_q=max_q, max_kv=max_kv, head_act=head_act)
    o = torch.full_like(q, float("nan"))
    lse = torch.full((wl.H, q.shape[0]), float("nan"), dtype=torch.float32, device="cuda")
    kb.gdpa_fwd_static(q, k, v, kvo, wl.scale, act, out=o, lse=lse, q_offsets=qo, max_q=max_q, max_kv=max_kv, head_act=head_act)
    torch.cuda.synchronize()
    # once more with the device's free memory watched (the very first launch of a kernel makes the runtime load
    # the library's code object, fixed array included, which is not the call's doing)
    o.fill_(float("nan"))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    kb.gdpa_fwd_static(q, k, v, kvo, wl.scale, act, out=o, lse=lse, q_offsets=qo, max_q=max_q, max_kv=max_kv, head_act=head_act)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
    assert torch.equal(o, ref_o), "outputs differ from kunlun_gdpa_fwd"
    acts = head_act if head_act is not None else [act] * wl.H
    for h, a in enumerate(acts):
        if a == 0:
            assert torch.equal(lse[h], ref_lse[h])


def test_two_calls_in_a_row_second_smaller(kb):
    # sorted issue order in the array (more workgroups than are resident at once), then a smaller batch
    # that is launched without any order: stale entries of the first call must not matter
    both(kb, W.make("cfg2", 1, B=600, H=4, d=64, Nq=32, lengths=("uniform", 0, 200), scale=0.1), 3)
    both(kb, W.make("cfg2", 2, B=40, H=4, d=64, Nq=32, lengths=("uniform", 0, 90), scale=0.1), 3)
    # again a sorted one, smaller than the first, softmax with per-head score functions
    both(kb, W.make("cfg2", 3, B=300, H=6, d=128, Nq=64, lengths=("uniform", 1, 150), scale=0.1), 0, head_act=[0, 3, 5, 0, 1, 2])


def test_query_tiled_launches_share_the_array(kb):
    # more than 64 queries per example: the array holds tile prefix sums and the tile -> example table
    rng = np.random.default_rng(5)
    for B, hi in ((30, 700), (9, 300)):
        lens_q = rng.integers(0, hi, size=B)
        wl = W.make("cfg2", B, B=B, H=2, d=64, Nq=1, lengths=("uniform", 0, 64), scale=0.2)
        q_off = W.offsets_from_lengths(lens_q)
        wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], 2, 64), dtype=np.float32) * 0.5)
        both(kb, wl, 3, q_offsets=q_off, max_q=int(lens_q.max()))
        both(kb, wl, 0, q_offsets=q_off, max_q=int(lens_q.max()))


def test_calls_beyond_the_fixed_array_are_refused(kb):
    B = 200_000   # the issue order alone needs 800 KB, the tile table as much again
    q = torch.zeros((B, 1, 32), dtype=torch.bfloat16, device="cuda")
    off = torch.arange(B + 1, dtype=torch.int32, device="cuda")
    assert kb.workspace_bytes(kb.OP_GDPA_FWD, B, 1, 32, 1, 1, B, B) > kb.STATIC_SCRATCH_BYTES
    with pytest.raises(kb.KunlunError) as e:
        kb.gdpa_fwd_static(q, q, q, off, 1.0, 3, out=torch.empty_like(q), max_q=1, max_kv=1)
    assert e.value.status == kb.ERR_WORKSPACE
