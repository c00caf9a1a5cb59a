"""Sliding-window forward on the launches that take the one-workgroup-per-(sequence, head) kernel (bounded
window of 8 to 11 block-steps, at least 512 (sequence, head) items): full compare with the CPU oracle on ragged
batches, every supported head dimension, windows on both sides of the conditions, and bit-identity of the
examples' results when other examples change."""
import math

import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import TOL, assert_close, assert_lse_close, offsets_dev, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def ragged_lengths(rng, B, hi):
    lengths = rng.integers(1, hi + 1, size=B)
    special = [0, 1, 31, 32, 33, 63, 64, 65, 255, 256, 257, 287, 288, 289, hi]
    lengths[rng.choice(B, size=len(special), replace=False)] = special
    return lengths


def check(kb, oracle, B, H, d, hi, window, seed):
    rng = np.random.default_rng(seed)
    lengths = ragged_lengths(rng, B, hi)
    wl = W.make("cfg3", seed, B=B, H=H, d=d, lengths=("list", lengths))
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    o = torch.full_like(q, float("nan"))
    lse = torch.full((H, q.shape[0]), float("nan"), dtype=torch.float32, device="cuda")
    kb.swa_fwd(q, k, v, offsets_dev(wl.kv_offsets), window[0], window[1], wl.scale, max_len=hi, out=o, lse=lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o).all()), "an output row was left unwritten"
    o_ref, lse_ref = oracle.swa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, window[0], window[1], wl.scale)
    assert_close(to_np(o), o_ref, TOL["bf16"], f"swa band B={B} H={H} d={d} window={window}")
    assert_lse_close(to_np(lse), lse_ref, 1e-2)


# window -> block-steps c_l + c_r + 2: (255,0) 10, (128,127) 10, (200,40) 11, (100,100) 10, (224,0) 9, (192,0) 8,
# (288,0) 11; (160,0) 7 and (289,0) 12 are outside and take the query-tiled kernel
@pytest.mark.parametrize("window", [(255, 0), (128, 127), (200, 40), (100, 100), (224, 0), (192, 0), (288, 0), (1, 223), (160, 0), (289, 0)])
def test_band_windows_d128(kb, oracle, window):
    check(kb, oracle, 520, 4, 128, 700, window, seed=sum(window))


@pytest.mark.parametrize("d,H", [(64, 4), (32, 8), (128, 2)])
@pytest.mark.parametrize("window", [(255, 0), (96, 130)])
def test_band_head_dimensions(kb, oracle, d, H, window):
    check(kb, oracle, 2048 // H + 8, H, d, 400, window, seed=d + window[0])


@pytest.mark.parametrize("B,H", [(127, 4), (128, 4), (256, 2), (511, 1), (512, 1)])
def test_band_item_count_threshold(kb, oracle, B, H):
    """511 and 508 items take the query-tiled kernel, 512 the one-workgroup-per-item kernel."""
    check(kb, oracle, B, H, 128, 600, (255, 0), seed=B * H)


def test_band_many_short_sequences_and_empty_ones(kb, oracle):
    rng = np.random.default_rng(3)
    B, H, d = 2100, 1, 64
    lengths = rng.integers(0, 70, size=B)
    wl = W.make("cfg3", 4, B=B, H=H, d=d, lengths=("list", lengths))
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    o, lse = kb.swa_fwd(q, k, v, offsets_dev(wl.kv_offsets), 255, 0, wl.scale, max_len=70)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.swa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, 255, 0, wl.scale)
    assert_close(to_np(o), o_ref, TOL["bf16"], "short sequences")
    assert_lse_close(to_np(lse), lse_ref, 1e-2)


def test_band_sequences_are_isolated_and_repeatable(kb):
    rng = np.random.default_rng(5)
    B, H, d = 600, 4, 128
    lengths = rng.integers(1, 500, size=B)
    wl = W.make("cfg3", 6, B=B, H=H, d=d, lengths=("list", lengths))
    off = offsets_dev(wl.kv_offsets)
    run = lambda w: kb.swa_fwd(to_dev(w.q, "bf16"), to_dev(w.k, "bf16"), to_dev(w.v, "bf16"), off, 255, 0, w.scale, max_len=500)[0]
    a, a2 = run(wl), run(wl)
    torch.cuda.synchronize()
    assert torch.equal(a, a2)
    b = 77
    lo, hi = int(wl.kv_offsets[b]), int(wl.kv_offsets[b + 1])
    for t in (wl.q, wl.k, wl.v):
        t[:lo] = 3.0
        t[hi:] = -2.0
    c = run(wl)
    torch.cuda.synchronize()
    assert torch.equal(a[lo:hi], c[lo:hi])
