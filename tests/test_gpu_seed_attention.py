"""Seed-level attention with batch-shared seeds (kunlun_seed_attn_fwd / _bwd; Sec. "Hierarchical Seed Pooling",
stage 1, Eq. (seed-level attention)) against the CPU oracle, and against the per-example-queries entry points fed
with the seed block repeated once per example (same kernels: bit-identical O, dK, dV)."""
import math

import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import TOL, assert_close, assert_close_sums, assert_lse_close, offsets_dev, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def make_case(seed, B, H, d, n_seeds, lo, hi, dtype="bf16"):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(lo, hi + 1, size=B)
    lengths[rng.choice(B, size=min(2, B - 1), replace=False)] = 0
    wl = W.make("cfg5", seed, B=B, H=H, d=d, Nq=n_seeds, dtype=dtype, sigma=0.5 if dtype == "bf16" else 1.0,
                lengths=("list", lengths), scale=1 / math.sqrt(d))
    e = rng.standard_normal((n_seeds, H, d), dtype=np.float32) * np.float32(0.5 if dtype == "bf16" else 1.0)
    return wl, (W.round_to_bf16(e) if dtype == "bf16" else e)


# (B, H, d, n_seeds): 64 seeds at d = 128 (the fused pair backward), 32 and fewer (one query block), 256 seeds (the
# paper's S: query-tiled forward, two-pass backward), d = 32, a batch of several summation groups (32 examples each)
CASES = [(70, 4, 128, 64), (40, 4, 64, 32), (33, 2, 64, 20), (12, 2, 128, 256), (100, 3, 32, 8), (5, 2, 32, 130), (1, 2, 64, 16)]


@pytest.mark.parametrize("B,H,d,n_seeds", CASES)
@pytest.mark.parametrize("act", [0, 3])
def test_shared_seeds_forward_backward_vs_oracle(kb, oracle, B, H, d, n_seeds, act):
    wl, e = make_case(B + n_seeds, B, H, d, n_seeds, 1, 200)
    ed, k, v, d_o = to_dev(e, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16"), to_dev(wl.d_o, "bf16")
    kvo = offsets_dev(wl.kv_offsets)
    mk = max(wl.max_kv, 1)
    o, lse = kb.seed_attn_fwd(ed, k, v, kvo, wl.scale, act, max_kv=mk)
    out = (torch.full_like(ed, float("nan")), torch.full_like(k, float("nan")), torch.full_like(v, float("nan")))
    d_e, dk, dv = kb.seed_attn_bwd(ed, k, v, d_o, kvo, wl.scale, act, o=o, lse=lse, max_kv=mk, out=out)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.seed_attn_fwd(e, wl.k, wl.v, wl.kv_offsets, wl.scale, act)
    what = f"B={B} H={H} d={d} seeds={n_seeds} act={act}"
    assert_close(to_np(o), o_ref, TOL["bf16"], what + " O")
    if act == 0:
        assert_lse_close(to_np(lse), lse_ref, 1e-2)
    refs = oracle.seed_attn_bwd(e, wl.k, wl.v, wl.d_o, wl.kv_offsets, wl.scale, act)
    for got, ref, name in zip((d_e, dk, dv), refs, ("dE", "dK", "dV")):
        # dE sums B * L products with a bf16-rounded factor (and B bf16-rounded per-example gradients, which the
        # other tests hold to the element-wise criterion one by one, and whose exact fixed-order sum dE is shown
        # to be below): the criterion for long sums
        (assert_close_sums if name == "dE" else assert_close)(to_np(got), ref, TOL["bf16"], what + " " + name)
    # the same kernels as the per-example-queries entry points: bit-identical on the repeated seed block
    q_rep = ed.repeat(B, 1, 1).contiguous()
    o2, lse2 = kb.gdpa_fwd(q_rep, k, v, kvo, wl.scale, act, max_q=n_seeds, max_kv=mk)
    dq2, dk2, dv2 = kb.gdpa_bwd(q_rep, k, v, d_o, kvo, wl.scale, act, o=o2, lse=lse2, max_q=n_seeds, max_kv=mk)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)
    # and the seed gradient is the fp32 sum of their per-example query gradients (groups of 32 examples, in order)
    rows = dq2.float().view(B, -1)
    total = torch.zeros_like(rows[0])
    for g0 in range(0, B, 32):
        part = torch.zeros_like(rows[0])
        for b in range(g0, min(B, g0 + 32)):
            part = part + rows[b]
        total = total + part
    assert torch.equal(d_e.view(-1), total.to(torch.bfloat16)), "the sum over the batch is not the documented fixed-order sum"


def test_shared_seeds_per_head_score_functions_and_repeatability(kb, oracle):
    wl, e = make_case(7, 45, 6, 64, 48, 1, 150)
    head_act = [0, 3, 5, 2, 1, 4]
    ed, k, v, d_o = to_dev(e, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16"), to_dev(wl.d_o, "bf16")
    kvo = offsets_dev(wl.kv_offsets)
    o, lse = kb.seed_attn_fwd(ed, k, v, kvo, 0.1, 0, max_kv=wl.max_kv, head_act=head_act)
    a = kb.seed_attn_bwd(ed, k, v, d_o, kvo, 0.1, 0, o=o, lse=lse, max_kv=wl.max_kv, head_act=head_act)
    b = kb.seed_attn_bwd(ed, k, v, d_o, kvo, 0.1, 0, o=o, lse=lse, max_kv=wl.max_kv, head_act=head_act)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    o_ref, _ = oracle.seed_attn_fwd(e, wl.k, wl.v, wl.kv_offsets, 0.1, 0, head_act=head_act)
    assert_close(to_np(o), o_ref, TOL["bf16"], "per-head O")
    refs = oracle.seed_attn_bwd(e, wl.k, wl.v, wl.d_o, wl.kv_offsets, 0.1, 0, head_act=head_act)
    for got, ref, name in zip(a, refs, ("dE", "dK", "dV")):
        (assert_close_sums if name == "dE" else assert_close)(to_np(got), ref, TOL["bf16"], "per-head " + name)


def test_shared_seeds_fp32_generic_kernels(kb, oracle):
    wl, e = make_case(9, 37, 2, 40, 6, 1, 60, dtype="fp32")
    ed, k, v, d_o = to_dev(e, "fp32"), to_dev(wl.k, "fp32"), to_dev(wl.v, "fp32"), to_dev(wl.d_o, "fp32")
    kvo = offsets_dev(wl.kv_offsets)
    for act in (0, 3):
        o, lse = kb.seed_attn_fwd(ed, k, v, kvo, wl.scale, act, max_kv=wl.max_kv)
        d_e, dk, dv = kb.seed_attn_bwd(ed, k, v, d_o, kvo, wl.scale, act, o=o, lse=lse, max_kv=wl.max_kv)
        torch.cuda.synchronize()
        o_ref, _ = oracle.seed_attn_fwd(e, wl.k, wl.v, wl.kv_offsets, wl.scale, act)
        assert_close(to_np(o), o_ref, TOL["fp32"], "fp32 O")
        refs = oracle.seed_attn_bwd(e, wl.k, wl.v, wl.d_o, wl.kv_offsets, wl.scale, act)
        for got, ref, name in zip((d_e, dk, dv), refs, ("dE", "dK", "dV")):
            assert_close(to_np(got), ref, TOL["fp32"], "fp32 " + name)


def test_shared_seeds_empty_batch_and_histories(kb):
    e = torch.randn((4, 2, 64), device="cuda").to(torch.bfloat16)
    z = torch.zeros((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    off = torch.zeros(4, dtype=torch.int32, device="cuda")   # three examples without any key
    o, lse = kb.seed_attn_fwd(e, z, z, off, 0.3, 0, max_kv=1)
    d_e, _, _ = kb.seed_attn_bwd(e, z, z, torch.ones_like(o), off, 0.3, 0, o=o, lse=lse, max_kv=1)
    torch.cuda.synchronize()
    assert torch.all(o == 0) and torch.all(torch.isneginf(lse)) and torch.all(d_e == 0)
