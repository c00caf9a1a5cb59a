"""Seeded synthetic workloads: jagged lengths, offsets and N(0, sigma^2) tensors.

This module serves both the tests of the CPU oracle and the GPU library, so it holds
none of the operators' arithmetic: only random draws, offsets bookkeeping and
round-to-nearest-even casting to bf16.  It imports neither the oracle nor the binding.

The five named workloads stand in for the paper's production inputs (large batches of
jagged user histories of hundreds to thousands of events, few context/seed tokens,
small head dimensions; Sec. "Experiment Setup" and App. "GDPA and Fused PFFN Kernel"),
which are not public.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

# name -> recipe.  tau is the temperature of the GDPA equation (max history length of
# the workload); softmax uses 1/sqrt(d).  window = (left, right) keys around a query.
CONFIGS = {
    "cfg1": dict(op="gdpa_fwd", dtype="fp32", B=2, H=2, d=32, Nq=8, lengths=("const", 64), sigma=1.0, tau=64),
    "cfg2": dict(op="gdpa_fwd", dtype="bf16", B=256, H=4, d=64, Nq=32, lengths=("uniform", 64, 1024), sigma=0.5,
                 tau=1024),
    "cfg3": dict(op="swa_fwd", dtype="bf16", B=128, H=4, d=128, Nq=None, lengths=("uniform", 256, 2048),
                 sigma=0.5, window=(255, 0)),
    "cfg4": dict(op="gdpa_fwd", dtype="bf16", B=1024, H=8, d=128, Nq=64,
                 lengths=("lognormal", 800.0, 1.0, 32, 4096), sigma=0.5, tau=4096),
    "cfg5": dict(op="gdpa_bwd", dtype="bf16", B=256, H=4, d=64, Nq=32, lengths=("uniform", 64, 1024), sigma=0.5,
                 tau=1024),
}


def draw_lengths(spec, B: int, rng: np.random.Generator) -> np.ndarray:
    kind = spec[0]
    if kind == "const":
        return np.full(B, int(spec[1]), dtype=np.int64)
    if kind == "uniform":
        return rng.integers(int(spec[1]), int(spec[2]) + 1, size=B).astype(np.int64)
    if kind == "lognormal":
        median, sigma, lo, hi = spec[1:]
        x = rng.lognormal(mean=np.log(median), sigma=sigma, size=B)
        return np.clip(np.rint(x), lo, hi).astype(np.int64)
    if kind == "list":
        return np.asarray(spec[1], dtype=np.int64)
    raise ValueError(f"unknown length recipe {kind!r}")


def offsets_from_lengths(lengths) -> np.ndarray:
    off = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=off[1:])
    assert off[-1] < 2**31, "offsets are int32"
    return off.astype(np.int32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already exactly representable in bf16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


@dataclass
class Workload:
    name: str
    op: str
    dtype: str                       # "bf16" or "fp32": storage type on the GPU side
    B: int
    H: int
    d: int
    Nq: Optional[int]                # queries per example (dense Q); None for self-attention
    lengths: np.ndarray              # [B] history lengths
    kv_offsets: np.ndarray           # int32 [B+1]
    q_offsets: Optional[np.ndarray]  # int32 [B+1] or None (dense Q)
    q: np.ndarray                    # fp32 [total_q, H, d], exactly representable in `dtype`
    k: np.ndarray
    v: np.ndarray
    d_o: Optional[np.ndarray]
    scale: float
    window: Optional[Tuple[int, int]] = None
    meta: dict = field(default_factory=dict)

    @property
    def total_q(self) -> int:
        return int(self.q.shape[0])

    @property
    def total_kv(self) -> int:
        return int(self.k.shape[0])

    @property
    def max_kv(self) -> int:
        return int(self.lengths.max()) if self.lengths.size else 0


def _normal(rng, shape, sigma, dtype):
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)
    return round_to_bf16(x) if dtype == "bf16" else x


def make(name: str, seed: int = 0, *, softmax: bool = False, scale: Optional[float] = None, **override) -> Workload:
    """Build a named workload (or a variation of it through keyword overrides of the recipe).

    Draw order is fixed: lengths, Q, K, V, dO.  `softmax=True` selects 1/sqrt(d) instead of
    1/tau as the default scale.
    """
    r = dict(CONFIGS[name])
    r.update(override)
    rng = np.random.default_rng(seed)
    B, H, d = r["B"], r["H"], r["d"]
    lengths = draw_lengths(r["lengths"], B, rng)
    assert lengths.shape == (B,)
    kv_off = offsets_from_lengths(lengths)
    T = int(kv_off[-1])
    self_attn = r["op"].startswith("swa")
    if self_attn:
        nq_total, q_off, Nq = T, kv_off.copy(), None
    else:
        Nq = r["Nq"]
        nq_total, q_off = B * Nq, None
    q = _normal(rng, (nq_total, H, d), r["sigma"], r["dtype"])
    k = _normal(rng, (T, H, d), r["sigma"], r["dtype"])
    v = _normal(rng, (T, H, d), r["sigma"], r["dtype"])
    d_o = _normal(rng, (nq_total, H, d), 1.0, r["dtype"])
    if scale is None:
        scale = 1.0 / np.sqrt(d) if (self_attn or softmax) else 1.0 / float(r["tau"])
    return Workload(name=name, op=r["op"], dtype=r["dtype"], B=B, H=H, d=d, Nq=Nq, lengths=lengths,
                    kv_offsets=kv_off, q_offsets=q_off, q=q, k=k, v=v, d_o=d_o, scale=float(scale),
                    window=r.get("window"), meta=r)


def make_lengths(name: str, seed: int = 0, **override) -> np.ndarray:
    """Only the length draw of make() (same stream position), for sizing without the tensors."""
    r = dict(CONFIGS[name])
    r.update(override)
    return draw_lengths(r["lengths"], r["B"], np.random.default_rng(seed))


# ---- algorithmic work of one call: flops and compulsory HBM bytes ----

def gdpa_flops(H: int, d: int, Nq: int, T: int, backward: bool = False) -> float:
    """Two contractions forward (4*d flops per query-key pair per head), five backward."""
    return (10.0 if backward else 4.0) * d * H * Nq * T


def gdpa_bytes(H: int, d: int, total_q: int, T: int, elt: int = 2, backward: bool = False,
               softmax: bool = False) -> float:
    """Forward: K, V read once, Q read, O written.  Backward: K, V, Q, dO read; dK, dV, dQ written
    (softmax heads also read O, and LSE which is not counted)."""
    if backward:
        return float(elt) * (4.0 * T * H * d + (4.0 if softmax else 3.0) * total_q * H * d)
    return float(elt) * (2.0 * T * H * d + 2.0 * total_q * H * d)


def swa_pairs(lengths, left: int, right: int) -> int:
    """Number of (query, key) pairs inside the window, per head."""
    total = 0
    for L in np.asarray(lengths, dtype=np.int64):
        t = np.arange(L)
        lo = np.maximum(0, t - left) if left >= 0 else np.zeros_like(t)
        hi = np.minimum(L - 1, t + right) if right >= 0 else np.full_like(t, L - 1)
        total += int((hi - lo + 1).sum())
    return total


def swa_flops(H: int, d: int, pairs: int) -> float:
    return 4.0 * d * H * pairs


def swa_bytes(H: int, d: int, T: int, elt: int = 2) -> float:
    return float(elt) * 4.0 * T * H * d
