"""GPU parity: the HIP library (through the C ABI) against the CPU fp64 oracle, element by
element on the same seeded inputs.  bf16: max-abs/rel 2e-2; fp32: 1e-5 (see helpers.assert_close)."""
import math

import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import TOL, assert_close, assert_close_sums, assert_lse_close, offsets_dev, to_dev, to_np

pytestmark = pytest.mark.gpu

ACTS = {"softmax": 0, "identity": 1, "relu": 2, "gelu": 3, "gelu_tanh": 4, "silu": 5, "gelu_poly": 6}


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def run_gdpa_fwd(kb, wl, act, head_act=None, scale=None):
    dt = wl.dtype
    q, k, v = to_dev(wl.q, dt), to_dev(wl.k, dt), to_dev(wl.v, dt)
    o, lse = kb.gdpa_fwd(q, k, v, offsets_dev(wl.kv_offsets), wl.scale if scale is None else scale, act,
                         q_offsets=offsets_dev(wl.q_offsets), max_q=wl.meta.get("max_q", wl.Nq),
                         max_kv=max(wl.max_kv, 1), head_act=head_act)
    torch.cuda.synchronize()
    return to_np(o), to_np(lse)


def check_gdpa_fwd(kb, oracle, wl, act, head_act=None, scale=None):
    scale = wl.scale if scale is None else scale
    o, lse = run_gdpa_fwd(kb, wl, act, head_act, scale)
    o_ref, lse_ref = oracle.gdpa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, scale, act, q_offsets=wl.q_offsets,
                                     max_q=wl.Nq, head_act=head_act)
    assert_close(o, o_ref, TOL[wl.dtype], f"{wl.name} O act={act}")
    acts = head_act if head_act is not None else [act] * wl.H
    for h, a in enumerate(acts):
        if a == 0:
            assert_lse_close(lse[h], lse_ref[h], 1e-2 if wl.dtype == "bf16" else 1e-5, f"{wl.name} lse h={h}")


# ---------------- config 1: tiny fp32, dense ----------------

@pytest.mark.parametrize("act", list(ACTS))
def test_cfg1_fp32_forward(kb, oracle, act):
    wl = W.make("cfg1", 0, softmax=(act == "softmax"))
    check_gdpa_fwd(kb, oracle, wl, ACTS[act])
    check_gdpa_fwd(kb, oracle, wl, ACTS[act], scale=1 / math.sqrt(wl.d))


@pytest.mark.parametrize("act", ["softmax", "gelu", "silu", "gelu_tanh", "relu", "identity", "gelu_poly"])
def test_cfg1_fp32_backward(kb, oracle, act):
    wl = W.make("cfg1", 0, scale=1 / math.sqrt(32))
    check_gdpa_bwd(kb, oracle, wl, ACTS[act])


# ---------------- config 2: bf16 jagged GDPA forward ----------------

@pytest.mark.parametrize("act", ["gelu", "softmax"])
@pytest.mark.parametrize("seed", [0, 1])
def test_cfg2_forward(kb, oracle, act, seed):
    wl = W.make("cfg2", seed, softmax=(act == "softmax"))
    check_gdpa_fwd(kb, oracle, wl, ACTS[act])


# The weights P are rounded to bf16 before the second contraction (2^-9 relative per term), so
# the output error is about 2^-9 * sqrt(sum_j (p_j v_j)^2).  With 1/tau scaling that is far below
# the tolerance; the stress cases below use scores of order 1 and keep the histories short enough
# for the absolute clause of the criterion to stay meaningful.
@pytest.mark.parametrize("act", list(ACTS))
@pytest.mark.parametrize("strength,lengths", [(1.0, ("uniform", 8, 96)), (3.0, ("uniform", 1, 24))])
def test_cfg2_forward_all_activations_nonlinear_range(kb, oracle, act, strength, lengths):
    """scale = strength/sqrt(d) puts the scores where the activations are non-linear."""
    wl = W.make("cfg2", 2, B=48, lengths=lengths, scale=strength / math.sqrt(64))
    check_gdpa_fwd(kb, oracle, wl, ACTS[act])


RAGGED = [0, 1, 31, 32, 33, 63, 64, 65, 95, 97, 128, 1, 0, 200, 511, 3]


@pytest.mark.parametrize("d,Nq", [(64, 32), (64, 8), (64, 40), (64, 64), (128, 64), (128, 33), (128, 100), (128, 1), (64, 130), (32, 8), (32, 64),
                                  (32, 33), (32, 130)])
@pytest.mark.parametrize("act", ["gelu", "softmax"])
def test_ragged_tails_and_query_counts(kb, oracle, d, Nq, act):
    wl = W.make("cfg2", 3, B=len(RAGGED), H=3, d=d, Nq=Nq, lengths=("list", RAGGED), scale=0.5 / math.sqrt(d))
    check_gdpa_fwd(kb, oracle, wl, ACTS[act])


def test_per_head_activations(kb, oracle):
    head_act = [3, 0, 5, 2, 1, 4]
    wl = W.make("cfg2", 4, B=24, H=6, lengths=("uniform", 8, 96), scale=0.125)
    check_gdpa_fwd(kb, oracle, wl, 0, head_act=head_act)


def test_jagged_queries(kb, oracle):
    rng = np.random.default_rng(5)
    B, H, d = 12, 2, 64
    lens_q = rng.integers(0, 90, size=B)
    wl = W.make("cfg2", 5, B=B, H=H, d=d, Nq=1, lengths=("uniform", 0, 300), scale=0.15)
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = int(lens_q.max())
    for act in (3, 0):
        check_gdpa_fwd(kb, oracle, wl, act)


@pytest.mark.parametrize("d", [32, 64, 128])
def test_long_jagged_queries_few_keys(kb, oracle, d):
    """The PFFN direction of Eq. (GDPA): the sequence tokens are the queries, a few context
    tokens per example are keys and values (query-tiled launch)."""
    rng = np.random.default_rng(11)
    B, H = 10, 3
    lens_q = np.array([700, 1, 0, 128, 129, 255, 256, 257, 64, 400])
    lens_kv = np.array([16, 32, 8, 0, 64, 33, 1, 48, 64, 20])
    wl = W.make("cfg2", 12, B=B, H=H, d=d, Nq=1, lengths=("list", lens_kv), scale=0.5 / math.sqrt(d))
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = int(lens_q.max())
    check_gdpa_fwd(kb, oracle, wl, 3)
    check_gdpa_fwd(kb, oracle, wl, 0, head_act=[0, 5, 3])


def test_dense_long_queries(kb, oracle):
    wl = W.make("cfg2", 13, B=5, H=2, d=128, Nq=300, lengths=("list", [40, 0, 64, 7, 100]), scale=0.5 / math.sqrt(128))
    check_gdpa_fwd(kb, oracle, wl, 3)
    check_gdpa_fwd(kb, oracle, wl, 0)


def test_fp32_generic_path_jagged(kb, oracle):
    wl = W.make("cfg1", 6, B=9, H=3, d=40, Nq=5, lengths=("list", [0, 1, 63, 64, 65, 129, 300, 2, 77]),
                scale=1 / math.sqrt(40))
    for act in (3, 0, 5):
        check_gdpa_fwd(kb, oracle, wl, act)


def test_bf16_head_dim_32_and_generic_head_dims(kb, oracle):
    """d = 32 runs the matrix-core kernels; d = 40 and d = 8 (bf16) fall to the generic kernels."""
    for d in (32, 40, 8):
        wl = W.make("cfg2", 7, B=6, H=2, d=d, Nq=8, lengths=("list", [5, 0, 64, 100, 33, 1]), scale=0.3)
        check_gdpa_fwd(kb, oracle, wl, 3)


def test_examples_are_isolated_bit_exact(kb):
    """Changing other examples' keys/values leaves an example's output bit-identical."""
    wl = W.make("cfg2", 8, B=20, scale=0.125)
    o1, _ = run_gdpa_fwd(kb, wl, 3)
    b = 7
    lo, hi = wl.kv_offsets[b], wl.kv_offsets[b + 1]
    k2, v2 = wl.k.copy(), wl.v.copy()
    k2[:lo] = 3.0; k2[hi:] = -2.0; v2[:lo] = 5.0; v2[hi:] = 7.0
    wl.k, wl.v = k2, v2
    o2, _ = run_gdpa_fwd(kb, wl, 3)
    np.testing.assert_array_equal(o1[b * wl.Nq:(b + 1) * wl.Nq], o2[b * wl.Nq:(b + 1) * wl.Nq])


def test_repeatable_bit_exact(kb):
    wl = W.make("cfg2", 9, B=64)
    a, _ = run_gdpa_fwd(kb, wl, 0)
    b, _ = run_gdpa_fwd(kb, wl, 0)
    np.testing.assert_array_equal(a, b)


# ---------------- config 3: sliding window ----------------

def run_swa(kb, wl, window, scale=None):
    dt = wl.dtype
    q, k, v = to_dev(wl.q, dt), to_dev(wl.k, dt), to_dev(wl.v, dt)
    o, lse = kb.swa_fwd(q, k, v, offsets_dev(wl.kv_offsets), window[0], window[1],
                        wl.scale if scale is None else scale, max_len=max(wl.max_kv, 1))
    torch.cuda.synchronize()
    return to_np(o), to_np(lse)


def check_swa(kb, oracle, wl, window):
    o, lse = run_swa(kb, wl, window)
    o_ref, lse_ref = oracle.swa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, window[0], window[1], wl.scale)
    assert_close(o, o_ref, TOL[wl.dtype], f"{wl.name} swa O window={window}")
    assert_lse_close(lse, lse_ref, 1e-2 if wl.dtype == "bf16" else 1e-5)


def test_cfg3_sliding_window(kb, oracle):
    wl = W.make("cfg3", 0)
    check_swa(kb, oracle, wl, wl.window)


@pytest.mark.parametrize("window", [(255, 0), (0, 0), (3, 3), (50, 50), (100, 7), (31, 0), (32, 0), (64, 64), (-1, 0), (-1, -1), (0, -1), (1000, 1000)])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_swa_windows_and_ragged_lengths(kb, oracle, window, d):
    lens = [1, 0, 63, 64, 65, 127, 129, 300, 2, 777, 33]
    wl = W.make("cfg3", 1, B=len(lens), H=2, d=d, lengths=("list", lens))
    check_swa(kb, oracle, wl, window)


def test_swa_fp32_generic(kb, oracle):
    lens = [5, 70, 0, 131]
    wl = W.make("cfg3", 2, B=4, H=2, d=32, dtype="fp32", sigma=1.0, lengths=("list", lens))
    for window in [(3, 0), (2, 5), (-1, -1)]:
        check_swa(kb, oracle, wl, window)


def test_swa_window_covering_sequence_equals_full_attention(kb):
    lens = [40, 100, 257]
    wl = W.make("cfg3", 3, B=3, H=2, d=64, lengths=("list", lens))
    a, _ = run_swa(kb, wl, (256, 256))
    b, _ = run_swa(kb, wl, (-1, -1))
    np.testing.assert_array_equal(a, b)


def check_swa_bwd(kb, oracle, wl, window):
    dt = wl.dtype
    q, k, v, d_o = to_dev(wl.q, dt), to_dev(wl.k, dt), to_dev(wl.v, dt), to_dev(wl.d_o, dt)
    off = offsets_dev(wl.kv_offsets)
    ml = max(wl.max_kv, 1)
    o, lse = kb.swa_fwd(q, k, v, off, window[0], window[1], wl.scale, max_len=ml)
    dq, dk, dv = kb.swa_bwd(q, k, v, o, lse, d_o, off, window[0], window[1], wl.scale, max_len=ml)
    torch.cuda.synchronize()
    ref = oracle.swa_bwd(wl.q, wl.k, wl.v, wl.d_o, wl.kv_offsets, window[0], window[1], wl.scale)
    for got, r, name in zip((dq, dk, dv), ref, ("dQ", "dK", "dV")):
        assert_close(to_np(got), r, TOL[dt], f"swa bwd {name} window={window}")


@pytest.mark.parametrize("window", [(255, 0), (3, 3), (0, 0), (40, 7), (-1, 0), (-1, -1), (127, 128), (0, 200)])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("bf16", 32), ("fp32", 32)])
def test_swa_backward(kb, oracle, window, dtype, d):
    lens = [1, 0, 63, 64, 65, 130, 300, 2, 33, 513]
    sigma = 0.5 if dtype == "bf16" else 1.0
    wl = W.make("cfg3", 4, B=len(lens), H=2, d=d, dtype=dtype, sigma=sigma, lengths=("list", lens))
    check_swa_bwd(kb, oracle, wl, window)


def test_cfg3_sliding_window_backward(kb, oracle):
    wl = W.make("cfg3", 0, B=32)
    check_swa_bwd(kb, oracle, wl, wl.window)


# ---------------- config 5: backward ----------------

def check_gdpa_bwd(kb, oracle, wl, act, head_act=None, long_sums=False):
    """long_sums: dK and dV are sums over thousands of queries with scores of order one; the bf16 rounding of
    P / dS then adds up to an error that scales with the typical output, not with the output at hand (a CPU
    emulation of that rounding reproduces the GPU result to one output ulp), so those two use the criterion
    for long sums, with the RMS taken per example and head (the sums of an example run over its own queries)."""
    dt = wl.dtype
    q, k, v, d_o = to_dev(wl.q, dt), to_dev(wl.k, dt), to_dev(wl.v, dt), to_dev(wl.d_o, dt)
    kvo, qo = offsets_dev(wl.kv_offsets), offsets_dev(wl.q_offsets)
    max_q = wl.meta.get("max_q", wl.Nq)
    o, lse = kb.gdpa_fwd(q, k, v, kvo, wl.scale, act, q_offsets=qo, max_q=max_q, max_kv=max(wl.max_kv, 1),
                         head_act=head_act)
    dq, dk, dv = kb.gdpa_bwd(q, k, v, d_o, kvo, wl.scale, act, o=o, lse=lse, q_offsets=qo, max_q=max_q,
                             max_kv=max(wl.max_kv, 1), head_act=head_act)
    torch.cuda.synchronize()
    dq_ref, dk_ref, dv_ref = oracle.gdpa_bwd(wl.q, wl.k, wl.v, wl.d_o, wl.kv_offsets, wl.scale, act,
                                             q_offsets=wl.q_offsets, max_q=wl.Nq, head_act=head_act)
    tol = TOL[dt]
    assert_close(to_np(dq), dq_ref, tol, f"{wl.name} dQ act={act}")
    if long_sums:
        assert_close_sums(to_np(dk), dk_ref, tol, f"{wl.name} dK act={act}", offsets=wl.kv_offsets)
        assert_close_sums(to_np(dv), dv_ref, tol, f"{wl.name} dV act={act}", offsets=wl.kv_offsets)
    else:
        assert_close(to_np(dk), dk_ref, tol, f"{wl.name} dK act={act}")
        assert_close(to_np(dv), dv_ref, tol, f"{wl.name} dV act={act}")


@pytest.mark.parametrize("act", ["gelu", "softmax"])
def test_cfg5_backward(kb, oracle, act):
    wl = W.make("cfg5", 0, softmax=(act == "softmax"))
    check_gdpa_bwd(kb, oracle, wl, ACTS[act])


@pytest.mark.parametrize("act", list(ACTS))
@pytest.mark.parametrize("strength,lengths", [(1.0, ("uniform", 8, 96)), (1.5, ("uniform", 1, 24))])
def test_backward_all_activations_nonlinear_range(kb, oracle, act, strength, lengths):
    wl = W.make("cfg5", 1, B=24, lengths=lengths, scale=strength / math.sqrt(64))
    check_gdpa_bwd(kb, oracle, wl, ACTS[act])


@pytest.mark.parametrize("act", ["gelu_poly", "gelu"])
@pytest.mark.parametrize("d,Nq", [(64, 32), (128, 64), (128, 100)])
def test_scores_far_into_the_tails(kb, oracle, act, d, Nq):
    """Scores with a standard deviation of 2: one in twenty lies beyond the polynomial GELU's clamp at +-3.875,
    where its weight is exactly 0 or exactly the score and its slope exactly 0 or 1 (forward and backward).
    Weights of size 4..8 are rounded to bf16 with errors of 0.01..0.03 each, so every output is held to the
    criterion for sums of rounded products (RMS per example and head); a CPU emulation of that rounding (fp32
    polynomial, weights rounded to bf16) reproduces the GPU's forward output on this case element for element."""
    wl = W.make("cfg5", 5, B=40, H=2, d=d, Nq=Nq, lengths=("uniform", 1, 16), scale=8.0 / math.sqrt(d))
    a = ACTS[act]
    q, k, v, d_o = [to_dev(x, "bf16") for x in (wl.q, wl.k, wl.v, wl.d_o)]
    kvo = offsets_dev(wl.kv_offsets)
    o, _ = kb.gdpa_fwd(q, k, v, kvo, wl.scale, a, max_q=wl.Nq, max_kv=16)
    dq, dk, dv = kb.gdpa_bwd(q, k, v, d_o, kvo, wl.scale, a, max_q=wl.Nq, max_kv=16)
    torch.cuda.synchronize()
    o_ref, _ = oracle.gdpa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, wl.scale, a, max_q=wl.Nq)
    dq_ref, dk_ref, dv_ref = oracle.gdpa_bwd(wl.q, wl.k, wl.v, wl.d_o, wl.kv_offsets, wl.scale, a, max_q=wl.Nq)
    q_rows = np.arange(wl.B + 1) * wl.Nq
    tol = TOL["bf16"]
    assert_close_sums(to_np(o), o_ref, tol, f"O act={act}", offsets=q_rows)
    assert_close_sums(to_np(dq), dq_ref, tol, f"dQ act={act}", offsets=q_rows)
    assert_close_sums(to_np(dk), dk_ref, tol, f"dK act={act}", offsets=wl.kv_offsets)
    assert_close_sums(to_np(dv), dv_ref, tol, f"dV act={act}", offsets=wl.kv_offsets)
    if act == "gelu_poly":
        # the case does reach the tails: the same inputs through GELU give a different result at the size of the fit's error
        o_gelu, _ = oracle.gdpa_fwd(wl.q, wl.k, wl.v, wl.kv_offsets, wl.scale, ACTS["gelu"], max_q=wl.Nq)
        assert 1e-4 < np.abs(o_gelu - o_ref).max() < 5e-3


@pytest.mark.parametrize("d,Nq", [(64, 32), (64, 20), (128, 64), (128, 40), (64, 70), (32, 32), (32, 20), (32, 64), (32, 70)])
def test_backward_ragged(kb, oracle, d, Nq):
    wl = W.make("cfg5", 2, B=len(RAGGED), H=2, d=d, Nq=Nq, lengths=("list", RAGGED), scale=0.5 / math.sqrt(d))
    for act in (3, 0):
        check_gdpa_bwd(kb, oracle, wl, act)


@pytest.mark.parametrize("d", [32, 64, 128])
@pytest.mark.parametrize("act", list(ACTS))
def test_backward_long_jagged_queries_few_keys(kb, oracle, d, act):
    """Backward in the PFFN direction (sequence tokens are the queries): two-pass matrix-core path."""
    rng = np.random.default_rng(31)
    H = 2
    lens_q = np.array([300, 1, 0, 128, 129, 65, 257, 90])
    lens_kv = np.array([16, 32, 8, 0, 64, 33, 1, 100])
    B = len(lens_q)
    wl = W.make("cfg5", 32, B=B, H=H, d=d, Nq=1, lengths=("list", lens_kv), scale=0.5 / math.sqrt(d))
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.d_o = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32))
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = int(lens_q.max())
    check_gdpa_bwd(kb, oracle, wl, ACTS[act])


@pytest.mark.parametrize("d", [32, 64, 128])
@pytest.mark.parametrize("act", list(ACTS))
def test_backward_long_jagged_queries_at_most_32_keys(kb, oracle, d, act):
    """The PFFN direction proper (every example has at most 32 keys): the one-pass backward with
    per-tile partial sums of dK / dV.  Examples with no key, one key, a full tile, no query."""
    rng = np.random.default_rng(41)
    H = 3
    lens_q = np.array([300, 1, 0, 128, 129, 65, 257, 90, 640])
    lens_kv = np.array([16, 32, 8, 0, 31, 1, 32, 5, 24])
    B = len(lens_q)
    wl = W.make("cfg5", 42, B=B, H=H, d=d, Nq=1, lengths=("list", lens_kv), scale=0.5 / math.sqrt(d))
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.d_o = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32))
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = int(lens_q.max())
    check_gdpa_bwd(kb, oracle, wl, ACTS[act])
    if act == "gelu":
        check_gdpa_bwd(kb, oracle, wl, 0, head_act=[0, 5, 3])


@pytest.mark.parametrize("d,B,lo,hi,chunk", [(128, 24, 1500, 2500, 2), (64, 48, 1000, 2000, 4), (32, 48, 4000, 8000, 8)])
def test_backward_at_most_32_keys_chunked_workgroups(kb, oracle, d, B, lo, hi, chunk):
    """Enough query tiles that a workgroup of the one-pass backward walks `chunk` tiles (the chunk length
    grows with the tile count), with ragged ends, an example without queries and one with a single query."""
    rng = np.random.default_rng(50 + d)
    H = 8
    lens_q = rng.integers(lo, hi + 1, size=B)
    lens_q[3], lens_q[5] = 0, 1
    lens_kv = rng.integers(1, 33, size=B)
    lens_kv[0], lens_kv[1] = 32, 0
    tiles = int(sum((n + 127) // 128 for n in lens_q))
    total_q = int(lens_q.sum())
    tile_heads = (total_q // 128 + B) * H   # the library's own measure
    assert {8: tile_heads >= 16384, 4: 4096 <= tile_heads < 16384, 2: 2048 <= tile_heads < 4096}[chunk], (tiles, tile_heads)
    wl = W.make("cfg5", 52, B=B, H=H, d=d, Nq=1, lengths=("list", lens_kv), scale=0.5 / math.sqrt(d))
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.d_o = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32))
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = int(lens_q.max())
    check_gdpa_bwd(kb, oracle, wl, 0, head_act=[3, 0, 5, 2, 1, 4, 3, 0], long_sums=True)


def test_backward_dense_long_queries_per_head(kb, oracle):
    wl = W.make("cfg5", 33, B=4, H=6, d=128, Nq=150, lengths=("list", [40, 0, 64, 7]), scale=0.5 / math.sqrt(128))
    check_gdpa_bwd(kb, oracle, wl, 0, head_act=[3, 0, 5, 2, 1, 4])


def test_backward_d128_jagged_queries_up_to_64_all_activations(kb, oracle):
    """d = 128 with up to 64 queries per example (the wave-pair kernel): query counts 0..64 in one
    batch, histories with 0, 1 and 2 pairs' worth of tiles and ragged tails, one activation per head."""
    rng = np.random.default_rng(41)
    H, d = 6, 128
    lens_q = np.array([64, 33, 0, 1, 32, 63, 48, 64, 17, 40, 64, 5])
    lens_kv = np.array([0, 1, 31, 32, 33, 63, 64, 65, 96, 97, 129, 200])
    B = len(lens_q)
    wl = W.make("cfg5", 41, B=B, H=H, d=d, Nq=1, lengths=("list", lens_kv), scale=0.5 / math.sqrt(d))
    q_off = W.offsets_from_lengths(lens_q)
    wl.q = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32) * 0.5)
    wl.d_o = W.round_to_bf16(rng.standard_normal((q_off[-1], H, d), dtype=np.float32))
    wl.q_offsets, wl.Nq = q_off, None
    wl.meta["max_q"] = 64
    check_gdpa_bwd(kb, oracle, wl, 0, head_act=[3, 0, 5, 2, 1, 4])


def test_backward_per_head_activations(kb, oracle):
    wl = W.make("cfg5", 3, B=10, H=6, lengths=("uniform", 8, 96), scale=0.125)
    check_gdpa_bwd(kb, oracle, wl, 0, head_act=[3, 0, 5, 2, 1, 4])


# ---------------- SumKronLinear ----------------

def _sumkron_inputs(seed, B, S, T, D, k, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, S, D), dtype=np.float32)
    z = rng.standard_normal((k, S, T), dtype=np.float32) / math.sqrt(S)
    w = rng.standard_normal((k, D, D), dtype=np.float32) / math.sqrt(D)
    if dtype == "bf16":
        x, z, w = W.round_to_bf16(x), W.round_to_bf16(z), W.round_to_bf16(w)
    return x, z, w


@pytest.mark.parametrize("B,S,T,D,k", [(5, 256, 32, 384, 8),     # the paper's typical configuration
                                       (3, 64, 32, 128, 2),      # one tile in every direction
                                       (7, 96, 20, 256, 3),      # k*T = 60 and B*T = 140: ragged row tiles
                                       (2, 32, 1, 128, 1),       # a single output token, a single term
                                       (1, 160, 48, 512, 5)])
def test_sumkron_forward_tiled(kb, oracle, B, S, T, D, k):
    """bf16 matrix-core path (two tiled GEMMs).  The intermediate Z^T X (sums of S products of
    magnitude 1/sqrt(S), so O(1)) is rounded to bf16 once: relative 2^-9 per term of the second sum."""
    x, z, w = _sumkron_inputs(50 + B, B, S, T, D, k, "bf16")
    y = kb.sumkron_fwd(to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16"))
    torch.cuda.synchronize()
    assert_close(to_np(y), oracle.sumkron_fwd(x, z, w), TOL["bf16"], f"sumkron B={B} S={S} T={T} D={D} k={k}")


@pytest.mark.parametrize("B,S,T,D,k", [(5, 256, 32, 384, 8),     # the paper's typical configuration; a last group of one example
                                       (4, 256, 32, 384, 8),
                                       (7, 256, 32, 384, 7),     # three examples in the last group, an odd number of factors
                                       (1, 256, 32, 128, 1),     # one example, one factor, two channel blocks
                                       (3, 128, 32, 256, 3),     # the shorter X; waves without a factor
                                       (6, 128, 32, 256, 5),     # an odd number of factors: the two halves differ
                                       (1101, 128, 32, 128, 2)]) # more groups of four than compute units: several groups per workgroup
def test_sumkron_forward_fused(kb, oracle, B, S, T, D, k):
    """bf16, T = 32, S in {128, 256}, D in {128, 256, 384}, k <= 8: one kernel, Z^T X stays on the compute unit (rounded to
    bf16 once, as in the two-GEMM path).  Every output element against the oracle."""
    x, z, w = _sumkron_inputs(150 + B, B, S, T, D, k, "bf16")
    yd = torch.full((B, T, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    kb.sumkron_fwd(to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16"), out=yd)
    torch.cuda.synchronize()
    assert_close(to_np(yd), oracle.sumkron_fwd(x, z, w), TOL["bf16"], f"sumkron fused B={B} S={S} T={T} D={D} k={k}")


def test_sumkron_fused_paper_shape_large_batch(kb, oracle):
    """The paper's shape with more groups of four examples than compute units (a workgroup takes several groups, the X blocks
    of the next group are on their way during the last step of the current one): sampled examples against the oracle (examples
    are independent), every output row written."""
    B, S, T, D, k = 1100, 256, 32, 384, 8
    x, z, w = _sumkron_inputs(171, B, S, T, D, k, "bf16")
    yd = torch.full((B, T, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    kb.sumkron_fwd(to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16"), out=yd)
    torch.cuda.synchronize()
    y = to_np(yd)
    assert np.isfinite(y).all()
    pick = np.array([0, 1, 2, 3, 510, 511, 512, 513, 514, 1022, 1023, 1024, 1025, 1097, 1098, 1099])
    assert_close(y[pick], oracle.sumkron_fwd(x[pick], z, w), TOL["bf16"], "sumkron fused, paper shape, B = 1100 (sampled examples)")


def test_sumkron_fused_examples_are_isolated_and_repeatable(kb):
    x, z, w = _sumkron_inputs(161, 7, 256, 32, 384, 8, "bf16")
    xd, zd, wd = to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16")
    y1 = kb.sumkron_fwd(xd, zd, wd)
    y2 = kb.sumkron_fwd(xd, zd, wd)
    y3 = kb.sumkron_fwd(xd[3:6].contiguous(), zd, wd)   # other partners in the groups, same results
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    assert torch.equal(y1[3:6], y3)


@pytest.mark.parametrize("dtype,B,S,T,D,k", [("fp32", 3, 40, 6, 24, 3), ("bf16", 2, 24, 5, 40, 2), ("fp32", 2, 64, 32, 128, 2)])
def test_sumkron_forward_plain_kernels(kb, oracle, dtype, B, S, T, D, k):
    x, z, w = _sumkron_inputs(60, B, S, T, D, k, dtype)
    y = kb.sumkron_fwd(to_dev(x, dtype), to_dev(z, dtype), to_dev(w, dtype))
    torch.cuda.synchronize()
    assert_close(to_np(y), oracle.sumkron_fwd(x, z, w), TOL[dtype], f"sumkron plain {dtype}")


def test_sumkron_examples_are_isolated_and_repeatable(kb):
    x, z, w = _sumkron_inputs(61, 6, 64, 32, 128, 2, "bf16")
    xd, zd, wd = to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16")
    y1 = kb.sumkron_fwd(xd, zd, wd)
    y2 = kb.sumkron_fwd(xd, zd, wd)
    y3 = kb.sumkron_fwd(xd[2:5].contiguous(), zd, wd)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    assert torch.equal(y1[2:5], y3)


def _sumkron_dy(seed, B, T, D, dtype):
    dy = np.random.default_rng(seed).standard_normal((B, T, D), dtype=np.float32)
    return W.round_to_bf16(dy) if dtype == "bf16" else dy


def _check_sumkron_bwd(kb, oracle, B, S, T, D, k, dtype, tol, seed):
    x, z, w = _sumkron_inputs(seed, B, S, T, D, k, dtype)
    dy = _sumkron_dy(seed + 1, B, T, D, dtype)
    dx, dz, dw = kb.sumkron_bwd(to_dev(x, dtype), to_dev(z, dtype), to_dev(w, dtype), to_dev(dy, dtype))
    torch.cuda.synchronize()
    rx, rz, rw = oracle.sumkron_bwd(x, z, w, dy)
    tag = f"sumkron bwd {dtype} B={B} S={S} T={T} D={D} k={k}"
    assert_close(to_np(dx), rx, tol, tag + " dX")
    # bf16: sums over the batch of products with a bf16-rounded factor - error relative to the typical output;
    # fp32 (fp64 sums and intermediates inside the kernels): the standard criterion
    sums = assert_close if dtype == "fp32" else assert_close_sums
    sums(to_np(dz), rz, tol, tag + " dZ")
    sums(to_np(dw), rw, tol, tag + " dW")


@pytest.mark.parametrize("B,S,T,D,k", [(5, 256, 32, 384, 8),     # the paper's typical configuration
                                       (3, 128, 32, 128, 2),     # one tile in most directions
                                       (4, 128, 16, 256, 2),     # k*T = 32: a ragged row tile in the dZ contraction
                                       (2, 256, 48, 128, 2),     # T*k = 96, k*T = 96
                                       (3, 128, 32, 128, 3),     # k*D = 384: 128-row tiles in the dW contraction
                                       (2, 128, 16, 128, 6),
                                       (16, 128, 32, 128, 2)])   # enough rows for several split-K ranges
def test_sumkron_backward_tiled(kb, oracle, B, S, T, D, k):
    """bf16 matrix-core path (five tiled GEMMs, two of them split-K).  The intermediates Z^T X and
    dY W^T (O(1) values) are rounded to bf16 once; sums over the batch are accumulated in fp32."""
    _check_sumkron_bwd(kb, oracle, B, S, T, D, k, "bf16", TOL["bf16"], 70 + B)


@pytest.mark.parametrize("dtype,B,S,T,D,k", [("fp32", 3, 40, 6, 24, 3), ("bf16", 2, 24, 5, 40, 2), ("fp32", 2, 128, 32, 128, 2),
                                             ("bf16", 2, 64, 32, 128, 2)])   # the last: tiled forward shape, plain backward
def test_sumkron_backward_plain_kernels(kb, oracle, dtype, B, S, T, D, k):
    _check_sumkron_bwd(kb, oracle, B, S, T, D, k, dtype, TOL[dtype], 80)


def test_sumkron_backward_repeatable_and_empty_batch(kb):
    x, z, w = _sumkron_inputs(81, 16, 128, 32, 128, 2, "bf16")
    dy = _sumkron_dy(82, 16, 32, 128, "bf16")
    xd, zd, wd, dyd = to_dev(x, "bf16"), to_dev(z, "bf16"), to_dev(w, "bf16"), to_dev(dy, "bf16")
    a = kb.sumkron_bwd(xd, zd, wd, dyd)
    b = kb.sumkron_bwd(xd, zd, wd, dyd)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)   # partial sums are added in a fixed order
    # dX of an example depends on that example alone
    c = kb.sumkron_bwd(xd[4:8].contiguous(), zd, wd, dyd[4:8].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(a[0][4:8], c[0])
    # no example: zero weight gradients
    e = kb.sumkron_bwd(xd[:0].contiguous(), zd, wd, dyd[:0].contiguous())
    torch.cuda.synchronize()
    assert e[0].numel() == 0 and float(e[1].float().abs().max()) == 0.0 and float(e[2].float().abs().max()) == 0.0


# ---------------- autograd wrappers ----------------

def test_autograd_wrappers_route_to_the_library(kb):
    """The torch.autograd.Function wrappers return exactly what the forward / backward entry points return."""
    from paper_2602_10016_amd import autograd as ka
    wl = W.make("cfg5", 9, B=12, lengths=("uniform", 8, 96), scale=0.125)
    q, k, v, d_o = [to_dev(a, "bf16") for a in (wl.q, wl.k, wl.v, wl.d_o)]
    kvo = offsets_dev(wl.kv_offsets)
    acts = [0, 3, 5, 0][:wl.H] if wl.H <= 4 else None
    for t in (q, k, v):
        t.requires_grad_(True)
    o = ka.gdpa(q, k, v, kvo, wl.scale, 3, max_q=wl.Nq, max_kv=wl.max_kv, head_act=acts)
    o.backward(d_o)
    o_ref, lse = kb.gdpa_fwd(q.detach(), k.detach(), v.detach(), kvo, wl.scale, 3, max_q=wl.Nq, max_kv=wl.max_kv, head_act=acts)
    g_ref = kb.gdpa_bwd(q.detach(), k.detach(), v.detach(), d_o, kvo, wl.scale, 3, o=o_ref, lse=lse, max_q=wl.Nq,
                        max_kv=wl.max_kv, head_act=acts)
    torch.cuda.synchronize()
    assert torch.equal(o.detach(), o_ref)
    for t, g in zip((q, k, v), g_ref):
        assert torch.equal(t.grad, g)

    ws = W.make("cfg3", 9, B=4)
    q, k, v = [to_dev(a, "bf16").requires_grad_(True) for a in (ws.q, ws.k, ws.v)]
    off = offsets_dev(ws.kv_offsets)
    d_o = to_dev(W.round_to_bf16(np.random.default_rng(3).standard_normal(ws.q.shape, dtype=np.float32)), "bf16")
    o = ka.sliding_window_attention(q, k, v, off, 255, 0, ws.scale, max_len=ws.max_kv)
    o.backward(d_o)
    o_ref, lse = kb.swa_fwd(q.detach(), k.detach(), v.detach(), off, 255, 0, ws.scale, max_len=ws.max_kv)
    g_ref = kb.swa_bwd(q.detach(), k.detach(), v.detach(), o_ref, lse, d_o, off, 255, 0, ws.scale, max_len=ws.max_kv)
    torch.cuda.synchronize()
    assert torch.equal(o.detach(), o_ref)
    for t, g in zip((q, k, v), g_ref):
        assert torch.equal(t.grad, g)

    x, z, w = [to_dev(a, "bf16").requires_grad_(True) for a in _sumkron_inputs(90, 4, 128, 32, 128, 2, "bf16")]
    dy = to_dev(_sumkron_dy(91, 4, 32, 128, "bf16"), "bf16")
    y = ka.sumkron_linear(x, z, w)
    y.backward(dy)
    g_ref = kb.sumkron_bwd(x.detach(), z.detach(), w.detach(), dy)
    torch.cuda.synchronize()
    assert torch.equal(y.detach(), kb.sumkron_fwd(x.detach(), z.detach(), w.detach()))
    for t, g in zip((x, z, w), g_ref):
        assert torch.equal(t.grad, g)


# ---------------- HIP graph capture ----------------

def test_graph_capture_replays_match_eager(kb):
    """The calls enqueue kernels only (no allocation, no memset, no synchronisation), so a captured
    graph of forward + backward + window replays bit-identically to the eager calls."""
    wl = W.make("cfg5", 21, B=40, H=8, d=128, Nq=64, lengths=("uniform", 1, 300))
    ws3 = W.make("cfg3", 22, B=6)
    dt = "bf16"
    q, k, v, d_o = to_dev(wl.q, dt), to_dev(wl.k, dt), to_dev(wl.v, dt), to_dev(wl.d_o, dt)
    kvo = offsets_dev(wl.kv_offsets)
    qs, ks, vs, so = to_dev(ws3.q, dt), to_dev(ws3.k, dt), to_dev(ws3.v, dt), offsets_dev(ws3.kv_offsets)
    mk = wl.max_kv
    wsz = max(kb.workspace_bytes(op, 64, 8, 128, 2048, 2048, q.shape[0], k.shape[0]) for op in range(4))
    w1, w2, w3 = (torch.empty(wsz, dtype=torch.uint8, device="cuda") for _ in range(3))
    o, lse = torch.empty_like(q), torch.empty((8, q.shape[0]), dtype=torch.float32, device="cuda")
    o_s = torch.empty_like(qs)

    def run():
        kb.gdpa_fwd(q, k, v, kvo, 0.05, 0, max_q=64, max_kv=mk, out=o, lse=lse, workspace=w1)
        g = kb.gdpa_bwd(q, k, v, d_o, kvo, 0.05, 0, o=o, lse=lse, max_q=64, max_kv=mk, workspace=w2)
        kb.swa_fwd(qs, ks, vs, so, 255, 0, ws3.scale, max_len=ws3.max_kv, out=o_s, want_lse=False, workspace=w3)
        return g

    eager = [t.clone() for t in run()] + [o.clone(), o_s.clone()]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = run()
    for rep in range(3):
        o.zero_(); o_s.zero_()
        for t in captured:
            t.zero_()
        junk = torch.randn(1 << 20, device="cuda").sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(list(captured) + [o, o_s], eager):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager result"
        del junk


def test_graph_capture_of_the_later_entry_points(kb):
    """The same for the sliding-window backward, the long-query backward with few keys (one-pass kernel with
    partial sums in the workspace) and SumKronLinear forward / backward (split-K partial sums in the workspace)."""
    rng = np.random.default_rng(77)
    dt = "bf16"
    ws3 = W.make("cfg3", 23, B=5)
    qs, ks, vs, so = to_dev(ws3.q, dt), to_dev(ws3.k, dt), to_dev(ws3.v, dt), offsets_dev(ws3.kv_offsets)
    dos = to_dev(W.round_to_bf16(rng.standard_normal(ws3.q.shape, dtype=np.float32)), dt)
    o_s, lse_s = kb.swa_fwd(qs, ks, vs, so, 255, 0, ws3.scale, max_len=ws3.max_kv)
    lens_q, lens_kv = np.array([700, 130, 0, 64, 300]), np.array([32, 7, 16, 0, 20])
    H, d = 4, 128
    q_off, kv_off = W.offsets_from_lengths(lens_q), W.offsets_from_lengths(lens_kv)
    bf = lambda shape, s: to_dev(W.round_to_bf16((rng.standard_normal(shape) * s).astype(np.float32)), dt)
    q, d_o = bf((q_off[-1], H, d), 0.5), bf((q_off[-1], H, d), 1.0)
    k, v = bf((kv_off[-1], H, d), 0.5), bf((kv_off[-1], H, d), 0.5)
    qo, kvo = offsets_dev(q_off), offsets_dev(kv_off)
    x, z, w = [to_dev(a, dt) for a in _sumkron_inputs(92, 8, 128, 32, 128, 2, dt)]
    dy = to_dev(_sumkron_dy(93, 8, 32, 128, dt), dt)
    w1 = torch.empty(kb.workspace_bytes(kb.OP_SWA_BWD, 5, ws3.H, ws3.d, ws3.max_kv, ws3.max_kv, qs.shape[0], qs.shape[0]), dtype=torch.uint8, device="cuda")
    w2 = torch.empty(kb.workspace_bytes(kb.OP_GDPA_BWD, 5, H, d, 700, 32, q.shape[0], k.shape[0]), dtype=torch.uint8, device="cuda")
    w3 = torch.empty(kb.sumkron_workspace_bytes(8, 128, 32, 128, 2), dtype=torch.uint8, device="cuda")
    w4 = torch.empty(kb.sumkron_bwd_workspace_bytes(8, 128, 32, 128, 2), dtype=torch.uint8, device="cuda")

    def run():
        a = kb.swa_bwd(qs, ks, vs, o_s, lse_s, dos, so, 255, 0, ws3.scale, max_len=ws3.max_kv, workspace=w1)
        b = kb.gdpa_bwd(q, k, v, d_o, kvo, 0.04, 3, q_offsets=qo, max_q=700, max_kv=32, workspace=w2)
        y = kb.sumkron_fwd(x, z, w, workspace=w3)
        c = kb.sumkron_bwd(x, z, w, dy, workspace=w4)
        return list(a) + list(b) + [y] + list(c)

    eager = [t.clone() for t in run()]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = run()
    for rep in range(3):
        for t in captured:
            t.zero_()
        junk = torch.randn(1 << 20, device="cuda").sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(captured, eager)):
            assert torch.equal(got, ref), f"replay {rep}: output {i} differs from the eager result"
        del junk


def test_check_offsets_counts_contract_violations(kb):
    good = np.array([0, 5, 5, 40, 100], dtype=np.int32)
    assert kb.check_offsets(offsets_dev(good), 100, 64) == 0
    assert kb.check_offsets(offsets_dev(good), 100, 50) == 1          # one example longer than max_len
    assert kb.check_offsets(offsets_dev(good), 99, 64) == 1           # last offset is not the total
    bad = np.array([1, 5, 3, 40, 100], dtype=np.int32)                # first offset not 0, one negative length
    assert kb.check_offsets(offsets_dev(bad), 100, 64) == 2
    big = W.offsets_from_lengths(np.full(5000, 7))
    assert kb.check_offsets(offsets_dev(big), 35000, 7) == 0          # more examples than threads


# ---------------- degenerate calls ----------------

def test_empty_batch_and_all_empty_histories(kb):
    z = torch.zeros((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    off = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, _ = kb.gdpa_fwd(z, z, z, off, 1.0, 3, max_q=4, max_kv=1)
    assert o.numel() == 0
    B, Nq = 3, 4
    q = torch.randn((B * Nq, 2, 64), device="cuda").to(torch.bfloat16)
    off = torch.zeros(B + 1, dtype=torch.int32, device="cuda")
    for act in (3, 0):
        o, lse = kb.gdpa_fwd(q, z, z, off, 1.0, act, max_q=Nq, max_kv=1)
        torch.cuda.synchronize()
        assert torch.all(o == 0)
        if act == 0:
            assert torch.all(torch.isneginf(lse))


def test_smoke_entry_point():
    import __graft_entry__
    __graft_entry__.smoke()
