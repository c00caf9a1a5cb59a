"""Shared helpers of the GPU parity tests: upload a workload, call the C ABI through the
binding, compare with the CPU oracle."""
import numpy as np
import torch

TOL = {"bf16": 2e-2, "fp32": 1e-5}
TORCH_DTYPE = {"bf16": torch.bfloat16, "fp32": torch.float32}


def to_dev(x, dtype):
    """fp32 numpy values (exactly representable in dtype) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(TORCH_DTYPE[dtype]).cuda()


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def offsets_dev(off):
    return None if off is None else torch.from_numpy(np.ascontiguousarray(off, dtype=np.int32)).cuda()


def assert_close(got, ref, tol, what=""):
    """max-abs/rel criterion: |x - r| <= tol (1 + |r|) for every element, and the largest
    error relative to the largest reference magnitude is below tol as well (the second clause
    keeps the test meaningful when all values are far below 1)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    bad = err > tol * (1.0 + np.abs(ref))
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond tol, worst {err.max():.3e}"
    scale = np.abs(ref).max()
    if scale > 0:
        assert err.max() / scale <= tol, f"{what}: max err {err.max():.3e} vs max |ref| {scale:.3e} (tol {tol})"


def assert_close_sums(got, ref, tol, what="", offsets=None):
    """Criterion for outputs that are sums of many products whose factors were rounded on the way
    (weight gradients: sums over the batch; dK / dV over thousands of queries; the factor is a bf16 or
    fp32 intermediate).  The rounding errors of the terms add up like a random walk: their total is
    about the unit roundoff (2^-9 for bf16) / sqrt(3) times the root of the sum of the squared terms,
    which is the typical magnitude (RMS) of the outputs that sum the same kind of terms, whatever the
    value of the one output at hand.  So: |x - r| <= tol (rms + |r|) for every element, where rms is
    taken over the whole tensor, or - with `offsets` (rows grouped by example, shape [rows, H, d]) - over
    the rows of the same example and head, whose sums run over the same queries.  A misplaced or missing
    operand changes outputs by the order of that RMS and fails."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    if offsets is None:
        rms = np.full_like(ref, np.sqrt(np.mean(ref * ref)))
    else:
        rms = np.zeros_like(ref)
        for b in range(len(offsets) - 1):
            lo, hi = int(offsets[b]), int(offsets[b + 1])
            if hi > lo:
                rms[lo:hi] = np.sqrt(np.mean(ref[lo:hi] ** 2, axis=(0, 2), keepdims=True))
        # blocks whose exact result is (nearly) zero - one key under softmax: dK = 0 - still carry the
        # noise of the terms that cancel; a hundredth of the tensor's RMS is the floor
        rms = np.maximum(rms, 1e-2 * np.sqrt(np.mean(ref * ref)))
    # 1e-3: absolute floor for tensors that are zero altogether (inputs are of order one)
    bound = tol * (rms + np.abs(ref) + 1e-3)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond tol, worst excess {(err - bound).max():.3e}"


def assert_lse_close(got, ref, tol, what="lse"):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{what}: -inf pattern differs"
    assert np.all(np.abs(got[~inf] - ref[~inf]) <= tol * (1.0 + np.abs(ref[~inf]))), what
