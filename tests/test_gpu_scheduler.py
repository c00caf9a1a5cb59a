"""The offsets-driven scheduler (App. "GDPA and Fused PFFN Kernel": tile scheduling from precomputed
sequence-length metadata, no empty tiles): its integer output, read back from the workspace, and full
parity on launches that take the scheduled path, on both sides of every dispatch threshold.

Workspace layout relied on here (csrc/common.h, csrc/tile_map.h): a 256-byte header, then
  streaming launches      int32 order[B]: the examples in issue order, longest history first by length
                          bucket floor(len * 2048 / (max_kv + 1)); the order inside a bucket is free
  query-tiled launches    int32 tile_start[B+1] (exclusive prefix sums of ceil(n_b / 128)), padded to 256
                          bytes, then int32 tile_example[tile] = example of every tile.
The sorting kernel runs only when the launch has more workgroups than are resident at once: forward more
than 1024 (example, head, 64-query tile) items; backward B*H above 1024 (d = 32, 64), 512 (d = 128, more than
32 queries) or 256 (d = 128, up to 32 queries).  B*H <= 2048 additionally selects the few-items kernels."""
import math

import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import TOL, assert_close, assert_lse_close, offsets_dev, to_dev, to_np

pytestmark = pytest.mark.gpu
NBINS = 2048


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def read_i32(ws, byte_offset, count):
    return ws[byte_offset:byte_offset + 4 * count].cpu().numpy().view(np.int32).copy()


def check_order(order, lengths, max_kv):
    B = len(lengths)
    assert np.array_equal(np.sort(order), np.arange(B)), "order is not a permutation of the examples"
    buckets = np.minimum(NBINS - 1, lengths[order].astype(np.int64) * NBINS // (max_kv + 1))
    assert np.all(np.diff(buckets) <= 0), "length buckets must never increase along the issue order"


def check_tile_tables(ws, counts, B, tile_rows=128):
    tiles = (np.asarray(counts, dtype=np.int64) + tile_rows - 1) // tile_rows
    start_ref = np.concatenate([[0], np.cumsum(tiles)]).astype(np.int32)
    start = read_i32(ws, 256, B + 1)
    np.testing.assert_array_equal(start, start_ref)
    pad = ((B + 1) * 4 + 255) // 256 * 256
    example = read_i32(ws, 256 + pad, int(start_ref[-1]))
    np.testing.assert_array_equal(example, np.repeat(np.arange(B, dtype=np.int32), tiles))


def make_lengths(rng, B, lo, hi, zeros=3):
    lengths = rng.integers(lo, hi + 1, size=B)
    lengths[rng.choice(B, size=zeros, replace=False)] = 0   # empty histories take part in the order too
    return lengths


# ---------------------------------------------------------------- the integer output, bit-exact

@pytest.mark.parametrize("B,H,d,Nq,max_kv", [(320, 4, 64, 32, 96), (1025, 2, 64, 8, 300), (2500, 1, 32, 16, 40), (3000, 1, 64, 64, 7),
                                             (140, 8, 128, 64, 4096)])
def test_forward_issue_order_is_a_length_sorted_permutation(kb, B, H, d, Nq, max_kv):
    rng = np.random.default_rng(B)
    lengths = make_lengths(rng, B, 1, max_kv)
    lengths[0] = max_kv                                    # the longest possible history: the first bucket
    wl = W.make("cfg2", B, B=B, H=H, d=d, Nq=Nq, lengths=("list", lengths))
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    nbytes = kb.workspace_bytes(kb.OP_GDPA_FWD, B, H, d, Nq, max_kv, q.shape[0], k.shape[0])
    ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
    kb.gdpa_fwd(q, k, v, offsets_dev(wl.kv_offsets), wl.scale, 3, max_q=Nq, max_kv=max_kv, workspace=ws)
    torch.cuda.synchronize()
    assert B * H * ((Nq + 63) // 64) > 1024, "the case must be large enough for the sorting kernel to run"
    check_order(read_i32(ws, 256, B), lengths, max_kv)


@pytest.mark.parametrize("B,H,d,Nq,max_kv", [(260, 4, 64, 32, 96), (65, 8, 128, 64, 200), (33, 8, 128, 24, 120), (2100, 1, 32, 40, 30)])
def test_backward_issue_order_is_a_length_sorted_permutation(kb, B, H, d, Nq, max_kv):
    rng = np.random.default_rng(B + 1)
    lengths = make_lengths(rng, B, 1, max_kv)
    wl = W.make("cfg5", B, B=B, H=H, d=d, Nq=Nq, lengths=("list", lengths))
    q, k, v, d_o = [to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.d_o)]
    nbytes = kb.workspace_bytes(kb.OP_GDPA_BWD, B, H, d, Nq, max_kv, q.shape[0], k.shape[0])
    ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
    kb.gdpa_bwd(q, k, v, d_o, offsets_dev(wl.kv_offsets), wl.scale, 3, max_q=Nq, max_kv=max_kv, workspace=ws)
    torch.cuda.synchronize()
    check_order(read_i32(ws, 256, B), lengths, max_kv)


@pytest.mark.parametrize("B,lo,hi", [(7, 0, 700), (1024, 0, 300), (1025, 0, 300), (2500, 0, 200), (4100, 0, 130)])
def test_query_tile_tables_are_exact_prefix_sums(kb, B, lo, hi):
    """Sliding-window launch: tile_start / tile_example of the query tiles, incl. empty sequences, sequences of
    exactly one tile, and more examples than the prefix kernel has threads (1024)."""
    rng = np.random.default_rng(B + 2)
    lengths = make_lengths(rng, B, lo, hi, zeros=min(3, B - 1))
    lengths[-1] = 128
    lengths[B // 2] = 129
    H, d = 1, 32
    off = W.offsets_from_lengths(lengths)
    T = int(off[-1])
    q = torch.randn((T, H, d), device="cuda").to(torch.bfloat16)
    nbytes = kb.workspace_bytes(kb.OP_SWA_FWD, B, H, d, hi, hi, T, T)
    ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
    kb.swa_fwd(q, q, q, offsets_dev(off), 20, 0, 0.2, max_len=max(hi, 129), workspace=ws)
    torch.cuda.synchronize()
    check_tile_tables(ws, lengths, B)


def test_query_tile_tables_of_dense_long_queries(kb):
    """GDPA with more than 64 dense queries per example: every example has ceil(Nq / 128) tiles."""
    B, H, d, Nq = 37, 2, 64, 300
    wl = W.make("cfg2", 3, B=B, H=H, d=d, Nq=Nq, lengths=("uniform", 0, 50))
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    nbytes = kb.workspace_bytes(kb.OP_GDPA_FWD, B, H, d, Nq, 50, q.shape[0], k.shape[0])
    ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
    kb.gdpa_fwd(q, k, v, offsets_dev(wl.kv_offsets), wl.scale, 3, max_q=Nq, max_kv=50, workspace=ws)
    torch.cuda.synchronize()
    check_tile_tables(ws, np.full(B, Nq), B)


# ---------------------------------------------------------------- full parity on the scheduled path

def fwd_case(kb, oracle, B, H, d, Nq, lo, hi, act, seed):
    rng = np.random.default_rng(seed)
    lengths = make_lengths(rng, B, lo, hi)
    wl = W.make("cfg2", seed, B=B, H=H, d=d, Nq=Nq, lengths=("list", lengths), scale=0.5 / math.sqrt(d))
    q, k, v = to_dev(wl.q, "bf16"), to_dev(wl.k, "bf16"), to_dev(wl.v, "bf16")
    o = torch.full_like(q, float("nan"))
    lse = torch.full((H, q.shape[0]), float("nan"), dtype=torch.float32, device="cuda")
    kb.gdpa_fwd(q, k, v, offsets_dev(wl.kv_offsets), wl.scale, act, max_q=Nq, max_kv=hi, out=o, lse=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.gdpa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, wl.scale, act, max_q=Nq)
    assert_close(to_np(o), o_ref, TOL["bf16"], f"fwd B={B} H={H} d={d} Nq={Nq} act={act}")
    if act == 0:
        assert_lse_close(to_np(lse), lse_ref, 1e-2)


# B*H*ceil(Nq/64): 1024 = all resident (no sorting kernel), above = scheduled; B*H 2048 / 2052: few-items switch
@pytest.mark.parametrize("B,H,d,Nq", [(256, 4, 64, 32), (257, 4, 64, 32), (320, 4, 64, 32), (512, 4, 64, 32), (513, 4, 64, 32),
                                      (128, 8, 128, 64), (129, 8, 128, 64), (140, 8, 128, 33),
                                      (257, 8, 128, 24), (130, 8, 128, 24),
                                      (330, 4, 32, 40), (520, 4, 32, 8)])
@pytest.mark.parametrize("act", [3, 0])
def test_forward_parity_around_the_dispatch_thresholds(kb, oracle, B, H, d, Nq, act):
    fwd_case(kb, oracle, B, H, d, Nq, 1, 96, act, seed=B + Nq)


def bwd_case(kb, oracle, B, H, d, Nq, lo, hi, act, seed):
    rng = np.random.default_rng(seed)
    lengths = make_lengths(rng, B, lo, hi)
    wl = W.make("cfg5", seed, B=B, H=H, d=d, Nq=Nq, lengths=("list", lengths), scale=0.5 / math.sqrt(d))
    q, k, v, d_o = [to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.d_o)]
    kvo = offsets_dev(wl.kv_offsets)
    o, lse = kb.gdpa_fwd(q, k, v, kvo, wl.scale, act, max_q=Nq, max_kv=hi)
    out = tuple(torch.full_like(t, float("nan")) for t in (q, k, v))
    dq, dk, dv = kb.gdpa_bwd(q, k, v, d_o, kvo, wl.scale, act, o=o, lse=lse, max_q=Nq, max_kv=hi, out=out)
    torch.cuda.synchronize()
    refs = oracle.gdpa_bwd(wl.q, wl.k, wl.v, wl.d_o, wl.kv_offsets, wl.scale, act, max_q=Nq)
    for got, ref, name in zip((dq, dk, dv), refs, ("dQ", "dK", "dV")):
        assert_close(to_np(got), ref, TOL["bf16"], f"bwd B={B} H={H} d={d} Nq={Nq} act={act} {name}")


# B*H against 1024 (d = 64, 32), 512 (d = 128, > 32 queries), 256 (d = 128, <= 32 queries); 2048: few-items switch
@pytest.mark.parametrize("B,H,d,Nq", [(256, 4, 64, 32), (260, 4, 64, 32), (512, 4, 64, 32), (516, 4, 64, 32), (300, 4, 64, 64), (520, 4, 64, 40),
                                      (64, 8, 128, 64), (65, 8, 128, 64), (90, 8, 128, 40),
                                      (32, 8, 128, 32), (33, 8, 128, 24),
                                      (260, 4, 32, 64), (520, 4, 32, 20)])
@pytest.mark.parametrize("act", [3, 0])
def test_backward_parity_around_the_dispatch_thresholds(kb, oracle, B, H, d, Nq, act):
    bwd_case(kb, oracle, B, H, d, Nq, 1, 96, act, seed=B + Nq + 1)


def test_many_more_examples_than_scheduler_threads(kb, oracle):
    """B = 5000 short examples: the sorting kernel and the prefix kernel walk several examples per thread."""
    fwd_case(kb, oracle, 5000, 1, 64, 8, 0, 40, 3, seed=77)
    bwd_case(kb, oracle, 5000, 1, 64, 8, 0, 40, 0, seed=78)


def test_offsets_verification_mode_rejects_a_length_above_the_bound(kb):
    """With verification switched on, the binding runs kunlun_check_offsets before a call: a max_kv below the longest
    history (which would select kernels by a wrong bound) is refused instead of computed."""
    wl = W.make("cfg2", 3, B=6, lengths=("uniform", 40, 90))
    q, k, v = (to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v))
    off = offsets_dev(wl.kv_offsets)
    kb.verify_offsets(True)
    try:
        kb.gdpa_fwd(q, k, v, off, wl.scale, kb.ACT_GELU, max_q=wl.Nq, max_kv=96)       # a true bound: fine
        with pytest.raises(ValueError):
            kb.gdpa_fwd(q, k, v, off, wl.scale, kb.ACT_GELU, max_q=wl.Nq, max_kv=32)   # an under-estimate
        bad = off.clone()
        bad[2] = bad[3] + 1                                                             # a negative length
        with pytest.raises(ValueError):
            kb.gdpa_fwd(q, k, v, bad, wl.scale, kb.ACT_GELU, max_q=wl.Nq, max_kv=96)
    finally:
        kb.verify_offsets(False)
