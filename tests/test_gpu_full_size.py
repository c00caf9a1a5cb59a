"""Config 4 at full size (B = 1024, H = 8, d = 128, Nq = 64, log-normal histories of 32..4096: the workload
bench.py times), in the launch configuration bench.py uses, against the CPU oracle.

Values are drawn on the device with a seeded torch generator (N(0,1) * sigma, rounded to bf16): 2.3 GB
per tensor, which numpy would take minutes to draw.  The oracle gets the same bf16 values, copied back.

Every output tensor is filled with NaN before the call, so "all finite" afterwards means that every row of
every example was written.  Compared against the oracle:
  forward            every (example, head) item, GELU and softmax
  backward           a seeded quarter of the examples + the 32 longest + the 32 shortest, all heads
  sliding window     such a sample as well, forward and backward
The oracle runs one call per group of examples (OpenMP over examples and heads)."""
import math

import numpy as np
import pytest
import torch

from paper_2602_10016_amd import workloads as W
from tests.helpers import TOL, assert_close, assert_lse_close, offsets_dev, to_np

pytestmark = pytest.mark.gpu

ACTS = {"softmax": 0, "gelu": 3}


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


def device_normal(shape, sigma, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    rows = shape[0]
    step = max(1, (1 << 27) // (shape[1] * shape[2]))
    for s in range(0, rows, step):
        e = min(rows, s + step)
        out[s:e] = (torch.randn((e - s,) + tuple(shape[1:]), generator=g, device="cuda", dtype=torch.float32)
                    * sigma).to(torch.bfloat16)
    return out


class Cfg4:
    """Inputs of the bench step on the device, shared by the tests of this module."""

    def __init__(self):
        r = W.CONFIGS["cfg4"]
        self.B, self.H, self.d, self.Nq, self.tau = r["B"], r["H"], r["d"], r["Nq"], r["tau"]
        self.lengths = W.make_lengths("cfg4", 0)
        self.off = W.offsets_from_lengths(self.lengths)
        self.T = int(self.off[-1])
        self.offd = offsets_dev(self.off)
        self.q = device_normal((self.B * self.Nq, self.H, self.d), 0.5, 1)
        self.k = device_normal((self.T, self.H, self.d), 0.5, 2)
        self.v = device_normal((self.T, self.H, self.d), 0.5, 3)
        self.d_o = device_normal((self.B * self.Nq, self.H, self.d), 1.0, 4)

    def sample(self, fraction, seed):
        """Sorted example indices: a seeded fraction of the batch, the 32 longest and the 32 shortest."""
        rng = np.random.default_rng(seed)
        order = np.argsort(self.lengths, kind="stable")
        picks = set(order[:32].tolist()) | set(order[-32:].tolist())
        picks |= set(rng.choice(self.B, size=int(round(self.B * fraction)), replace=False).tolist())
        return np.array(sorted(picks), dtype=np.int64)

    def groups(self, picks, max_rows=160_000):
        """Cuts a sorted pick list into groups of at most max_rows history rows (bounds the fp64 copies)."""
        out, cur, rows = [], [], 0
        for b in picks:
            if cur and rows + self.lengths[b] > max_rows:
                out.append(np.array(cur)); cur, rows = [], 0
            cur.append(int(b)); rows += int(self.lengths[b])
        if cur:
            out.append(np.array(cur))
        return out

    def kv_rows(self, ex):
        return torch.cat([torch.arange(int(self.off[b]), int(self.off[b + 1])) for b in ex]).cuda()

    def q_rows(self, ex):
        return torch.cat([torch.arange(b * self.Nq, (b + 1) * self.Nq) for b in ex]).cuda()


@pytest.fixture(scope="module")
def cfg4():
    return Cfg4()


def nan_like(t):
    return torch.full_like(t, float("nan"))


def all_written(*tensors):
    for t in tensors:
        assert bool(torch.isfinite(t).all()), "an output row was left unwritten (NaN prefill survives)"


@pytest.mark.parametrize("act,fraction", [("gelu", 1.0), ("softmax", 1.0)])
def test_cfg4_forward(kb, oracle, cfg4, act, fraction):
    c = cfg4
    scale = 1 / math.sqrt(c.d) if act == "softmax" else 1.0 / c.tau
    o = nan_like(c.q)
    lse = torch.full((c.H, c.q.shape[0]), float("nan"), dtype=torch.float32, device="cuda")
    kb.gdpa_fwd(c.q, c.k, c.v, c.offd, scale, ACTS[act], max_q=c.Nq, max_kv=4096, out=o, lse=lse)
    torch.cuda.synchronize()
    all_written(o)
    if act == "softmax":
        all_written(lse)   # no example is empty, so no -inf either
    picks = np.arange(c.B) if fraction >= 1.0 else c.sample(fraction, 0)
    n_items = 0
    for ex in c.groups(picks):
        kr, qr = c.kv_rows(ex), c.q_rows(ex)
        sub_off = W.offsets_from_lengths(c.lengths[ex])
        o_ref, lse_ref = oracle.gdpa_fwd(to_np(c.q[qr]), to_np(c.k[kr]), to_np(c.v[kr]), sub_off, scale, ACTS[act], max_q=c.Nq)
        got = to_np(o[qr])
        # per (example, head) item, so that the relative clause is taken over the item's own outputs
        for i, b in enumerate(ex):
            rows = slice(i * c.Nq, (i + 1) * c.Nq)
            for h in range(c.H):
                assert_close(got[rows, h], o_ref[rows, h], TOL["bf16"], f"cfg4 fwd {act} b={b} h={h} L={c.lengths[b]}")
                n_items += 1
        if act == "softmax":
            assert_lse_close(to_np(lse[:, qr]), lse_ref, 1e-2)
    assert n_items >= int(c.B * c.H * min(fraction, 1.0))


@pytest.mark.parametrize("act,fraction", [("gelu", 0.25), ("softmax", 0.25)])
def test_cfg4_backward(kb, oracle, cfg4, act, fraction):
    c = cfg4
    scale = 1 / math.sqrt(c.d) if act == "softmax" else 1.0 / c.tau
    o, lse = kb.gdpa_fwd(c.q, c.k, c.v, c.offd, scale, ACTS[act], max_q=c.Nq, max_kv=4096)
    grads = (nan_like(c.q), nan_like(c.k), nan_like(c.v))
    dq, dk, dv = kb.gdpa_bwd(c.q, c.k, c.v, c.d_o, c.offd, scale, ACTS[act], o=o, lse=lse, max_q=c.Nq, max_kv=4096, out=grads)
    torch.cuda.synchronize()
    all_written(dq, dk, dv)
    picks = c.sample(fraction, 1)
    assert len(picks) >= 0.1 * c.B + 32
    for ex in c.groups(picks):
        kr, qr = c.kv_rows(ex), c.q_rows(ex)
        sub_off = W.offsets_from_lengths(c.lengths[ex])
        refs = oracle.gdpa_bwd(to_np(c.q[qr]), to_np(c.k[kr]), to_np(c.v[kr]), to_np(c.d_o[qr]), sub_off, scale, ACTS[act], max_q=c.Nq)
        gq, gk, gv = to_np(dq[qr]), to_np(dk[kr]), to_np(dv[kr])
        for i, b in enumerate(ex):
            qs, ks = slice(i * c.Nq, (i + 1) * c.Nq), slice(int(sub_off[i]), int(sub_off[i + 1]))
            for h in range(c.H):
                what = f"cfg4 bwd {act} b={b} h={h} L={c.lengths[b]}"
                assert_close(gq[qs, h], refs[0][qs, h], TOL["bf16"], what + " dQ")
                assert_close(gk[ks, h], refs[1][ks, h], TOL["bf16"], what + " dK")
                assert_close(gv[ks, h], refs[2][ks, h], TOL["bf16"], what + " dV")


def test_cfg4_sliding_window_forward_and_backward(kb, oracle, cfg4):
    """The sliding-window call of the bench step (256 causal keys over the cfg4 batch) and its backward."""
    c = cfg4
    q = device_normal((c.T, c.H, c.d), 0.5, 5)
    d_o = device_normal((c.T, c.H, c.d), 1.0, 6)
    scale = 1 / math.sqrt(c.d)
    o = nan_like(q)
    lse = torch.full((c.H, c.T), float("nan"), dtype=torch.float32, device="cuda")
    kb.swa_fwd(q, c.k, c.v, c.offd, 255, 0, scale, max_len=4096, out=o, lse=lse)
    grads = (nan_like(q), nan_like(q), nan_like(q))
    dq, dk, dv = kb.swa_bwd(q, c.k, c.v, o, lse, d_o, c.offd, 255, 0, scale, max_len=4096, out=grads)
    torch.cuda.synchronize()
    all_written(o, lse, dq, dk, dv)
    picks = c.sample(0.25, 2)
    for ex in c.groups(picks, max_rows=100_000):
        rows = c.kv_rows(ex)
        sub_off = W.offsets_from_lengths(c.lengths[ex])
        hq, hk, hv, hdo = to_np(q[rows]), to_np(c.k[rows]), to_np(c.v[rows]), to_np(d_o[rows])
        o_ref, lse_ref = oracle.swa_fwd(hq, hk, hv, sub_off, 255, 0, scale)
        refs = oracle.swa_bwd(hq, hk, hv, hdo, sub_off, 255, 0, scale)
        got_o, got = to_np(o[rows]), [to_np(t[rows]) for t in (dq, dk, dv)]
        assert_lse_close(to_np(lse[:, rows]), lse_ref, 1e-2)
        for i, b in enumerate(ex):
            rs = slice(int(sub_off[i]), int(sub_off[i + 1]))
            for h in range(c.H):
                what = f"cfg4 swa b={b} h={h} L={c.lengths[b]}"
                assert_close(got_o[rs, h], o_ref[rs, h], TOL["bf16"], what + " O")
                for g, r, name in zip(got, refs, ("dQ", "dK", "dV")):
                    assert_close(g[rs, h], r[rs, h], TOL["bf16"], what + " " + name)
