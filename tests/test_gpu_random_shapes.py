"""GPU parity on seeded random shapes: every entry point against the CPU oracle with batch size,
head count, head dimension, query counts (dense or jagged), history lengths (zero included),
score functions and windows drawn per case, so that rarely used template paths and tile-boundary
combinations are exercised.  Scores are kept in the regime where the bf16 rounding of the
weights stays inside the tolerance (small scale, short histories)."""
import math
import os

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


# number of drawn cases (KUNLUN_RANDOM_CASES raises it for a longer hunt)
N_CASES = int(os.environ.get("KUNLUN_RANDOM_CASES", "24"))


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 7))
    H = int(rng.choice([1, 2, 3, 8]))
    d = int(rng.choice([32, 64, 128]))
    max_q = int(rng.choice([1, 7, 32, 33, 64, 65, 130, 300]))
    max_kv = int(rng.choice([1, 31, 33, 64, 100, 260]))
    jagged_q = bool(rng.integers(2))
    lens_q = rng.integers(0, max_q + 1, size=B) if jagged_q else np.full(B, max_q)
    lens_q[rng.integers(B)] = max_q
    lens_kv = rng.integers(0, max_kv + 1, size=B)
    lens_kv[rng.integers(B)] = max_kv
    acts = [int(a) for a in rng.integers(0, 7, size=H)]
    q_off, kv_off = W.offsets_from_lengths(lens_q), W.offsets_from_lengths(lens_kv)
    bf = lambda shape, s: W.round_to_bf16((rng.standard_normal(shape) * s).astype(np.float32))
    return dict(B=B, H=H, d=d, max_q=max_q, max_kv=max_kv, jagged_q=jagged_q, q_off=q_off, kv_off=kv_off, acts=acts,
                q=bf((q_off[-1], H, d), 0.5), k=bf((kv_off[-1], H, d), 0.5), v=bf((kv_off[-1], H, d), 0.5),
                d_o=bf((q_off[-1], H, d), 1.0), scale=0.4 / math.sqrt(d), rng=rng)


@pytest.mark.parametrize("seed", range(N_CASES))
def test_gdpa_forward_backward_random_shapes(kb, oracle, seed):
    c = _draw(seed)
    what = f"seed {seed}: B={c['B']} H={c['H']} d={c['d']} max_q={c['max_q']} max_kv={c['max_kv']} jagged_q={c['jagged_q']} acts={c['acts']}"
    q, k, v, d_o = [to_dev(c[n], "bf16") for n in ("q", "k", "v", "d_o")]
    qo = offsets_dev(c["q_off"]) if c["jagged_q"] else None
    kvo = offsets_dev(c["kv_off"])
    o, lse = kb.gdpa_fwd(q, k, v, kvo, c["scale"], 0, q_offsets=qo, max_q=c["max_q"], max_kv=c["max_kv"], head_act=c["acts"])
    dq, dk, dv = kb.gdpa_bwd(q, k, v, d_o, kvo, c["scale"], 0, o=o, lse=lse, q_offsets=qo, max_q=c["max_q"],
                             max_kv=c["max_kv"], head_act=c["acts"])
    torch.cuda.synchronize()
    kw = dict(q_offsets=c["q_off"], max_q=None, head_act=c["acts"])
    o_ref, lse_ref = oracle.gdpa_fwd(c["q"], c["k"], c["v"], c["kv_off"], c["scale"], 0, **kw)
    assert_close(to_np(o), o_ref, TOL["bf16"], what + " O")
    for h, a in enumerate(c["acts"]):
        if a == 0:
            assert_lse_close(to_np(lse)[h], lse_ref[h], 1e-2, what + f" lse h={h}")
    dq_ref, dk_ref, dv_ref = oracle.gdpa_bwd(c["q"], c["k"], c["v"], c["d_o"], c["kv_off"], c["scale"], 0, **kw)
    assert_close(to_np(dq), dq_ref, TOL["bf16"], what + " dQ")
    # dK / dV sum over up to 300 queries whose weights were rounded to bf16 (softmax over one or two keys:
    # weights of order one): error relative to the typical output of the same example and head
    assert_close_sums(to_np(dk), dk_ref, TOL["bf16"], what + " dK", offsets=c["kv_off"])
    assert_close_sums(to_np(dv), dv_ref, TOL["bf16"], what + " dV", offsets=c["kv_off"])


@pytest.mark.parametrize("seed", range(max(1, 2 * N_CASES // 3)))
def test_sliding_window_forward_backward_random_shapes(kb, oracle, seed):
    rng = np.random.default_rng(2000 + seed)
    B = int(rng.integers(1, 6))
    H = int(rng.choice([1, 2, 4]))
    d = int(rng.choice([32, 64, 128]))
    max_len = int(rng.choice([1, 30, 129, 260, 400]))
    lens = rng.integers(0, max_len + 1, size=B)
    lens[rng.integers(B)] = max_len
    left = int(rng.choice([-1, 0, 5, 31, 32, 100, 255, 1000]))
    right = int(rng.choice([-1, 0, 0, 3, 40, 128]))
    off = W.offsets_from_lengths(lens)
    bf = lambda s: W.round_to_bf16((rng.standard_normal((off[-1], H, d)) * s).astype(np.float32))
    qn, kn, vn, don = bf(0.5), bf(0.5), bf(0.5), bf(1.0)
    scale = 0.5 / math.sqrt(d)
    what = f"seed {seed}: B={B} H={H} d={d} lens={list(lens)} window=({left},{right})"
    q, k, v, d_o = [to_dev(a, "bf16") for a in (qn, kn, vn, don)]
    offd = offsets_dev(off)
    o, lse = kb.swa_fwd(q, k, v, offd, left, right, scale, max_len=max_len)
    dq, dk, dv = kb.swa_bwd(q, k, v, o, lse, d_o, offd, left, right, scale, max_len=max_len)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.swa_fwd(qn, kn, vn, off, left, right, scale)
    assert_close(to_np(o), o_ref, TOL["bf16"], what + " O")
    assert_lse_close(to_np(lse), lse_ref, 1e-2, what + " lse")
    dq_ref, dk_ref, dv_ref = oracle.swa_bwd(qn, kn, vn, don, off, left, right, scale)
    assert_close(to_np(dq), dq_ref, TOL["bf16"], what + " dQ")
    assert_close(to_np(dk), dk_ref, TOL["bf16"], what + " dK")
    assert_close(to_np(dv), dv_ref, TOL["bf16"], what + " dV")


@pytest.mark.parametrize("seed", range(max(1, N_CASES // 2)))
def test_sumkron_forward_backward_random_shapes(kb, oracle, seed):
    """Shapes on both sides of the conditions of the matrix-core path (D a multiple of 128, S of 32 for
    the forward; S of 128, T*k and B*T of 32 in addition for the backward) and fp32."""
    rng = np.random.default_rng(3000 + seed)
    dtype = "fp32" if rng.integers(5) == 0 else "bf16"
    B = int(rng.integers(1, 7))
    S = int(rng.choice([32, 64, 128, 160, 256, 24]))
    T = int(rng.choice([1, 5, 16, 32, 48]))
    D = int(rng.choice([128, 256, 384, 40, 24]))
    k = int(rng.integers(1, 9))
    draw = lambda shape, s: (rng.standard_normal(shape) * s).astype(np.float32)
    x, z, w, dy = draw((B, S, D), 1.0), draw((k, S, T), 1 / math.sqrt(S)), draw((k, D, D), 1 / math.sqrt(D)), draw((B, T, D), 1.0)
    if dtype == "bf16":
        x, z, w, dy = [W.round_to_bf16(a) for a in (x, z, w, dy)]
    tol = TOL[dtype]
    what = f"seed {seed}: {dtype} B={B} S={S} T={T} D={D} k={k}"
    xd, zd, wd, dyd = [to_dev(a, dtype) for a in (x, z, w, dy)]
    y = kb.sumkron_fwd(xd, zd, wd)
    dx, dz, dw = kb.sumkron_bwd(xd, zd, wd, dyd)
    torch.cuda.synchronize()
    assert_close(to_np(y), oracle.sumkron_fwd(x, z, w), tol, what + " Y")
    rx, rz, rw = oracle.sumkron_bwd(x, z, w, dy)
    assert_close(to_np(dx), rx, tol, what + " dX")
    # bf16: sums over the batch of products with a bf16-rounded factor - error relative to the typical output;
    # fp32 (fp64 sums and intermediates inside the kernels): the standard criterion
    sums = assert_close if dtype == "fp32" else assert_close_sums
    sums(to_np(dz), rz, tol, what + " dZ")
    sums(to_np(dw), rw, tol, what + " dW")
