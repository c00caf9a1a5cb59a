"""Pins of the SumKronLinear oracle (CPU only): the oracle is the quadruple sum of Eq.
(SumKronLinear) written out; these tests hold it against things that are not itself - a
hand-worked example, the explicit Kronecker-product matrix that gives the layer its name,
single-entry probes that fix every index, special cases that reduce to a selection or to two
library matrix products, multilinearity, and for the gradient central finite differences and
library autograd."""
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "sumkron_hand_worked.txt")


def _golden():
    arrays = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, shape, vals = [p.strip() for p in line.split(":")]
        arrays[name] = np.array([float(t) for t in vals.split()]).reshape([int(t) for t in shape.split()])
    return arrays


def _rand(seed, B=3, S=5, T=2, D=4, k=3):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, S, D)), rng.standard_normal((k, S, T)), rng.standard_normal((k, D, D))


def test_sumkron_hand_worked(oracle):
    g = _golden()
    np.testing.assert_allclose(oracle.sumkron_fwd(g["x"], g["z"], g["w"]), g["y"], rtol=0, atol=1e-12)


def test_sumkron_equals_explicit_kronecker_matrix(oracle):
    """vec(Z^T X W) = (Z^T kron W^T) vec(X) for row-major vec: the layer is the sum of k Kronecker
    products applied to the flattened input."""
    x, z, w = _rand(1)
    B, S, D = x.shape
    k, _, T = z.shape
    M = sum(np.kron(z[i].T, w[i].T) for i in range(k))  # [T*D, S*D]
    ref = (x.reshape(B, S * D) @ M.T).reshape(B, T, D)
    np.testing.assert_allclose(oracle.sumkron_fwd(x, z, w), ref, rtol=1e-12, atol=1e-12)


def test_sumkron_single_entry_probes(oracle):
    """Z_i = e_s e_t^T and W_i = e_c e_e^T pick out one input entry: Y[b, t, e] = X[b, s, c], all
    other outputs zero.  Fixes which index of Z is the sequence and which side of W is the input."""
    rng = np.random.default_rng(2)
    B, S, T, D, k = 2, 4, 3, 5, 2
    x = rng.standard_normal((B, S, D))
    for (i, s, t, c, e) in [(0, 1, 2, 3, 4), (1, 3, 0, 0, 2), (1, 0, 1, 4, 4)]:
        z = np.zeros((k, S, T)); w = np.zeros((k, D, D))
        z[i, s, t] = 1.0
        w[i, c, e] = 1.0
        w[1 - i] = rng.standard_normal((D, D))  # the other term has Z = 0: must not contribute
        y = oracle.sumkron_fwd(x, z, w)
        ref = np.zeros((B, T, D))
        ref[:, t, e] = x[:, s, c]
        np.testing.assert_allclose(y, ref, rtol=0, atol=1e-15)


def test_sumkron_selection_and_separable_cases(oracle):
    rng = np.random.default_rng(3)
    B, S, T, D = 2, 6, 3, 4
    x = rng.standard_normal((B, S, D))
    # k = 1, Z = first T columns of the identity, W = identity: the first T rows of X
    y = oracle.sumkron_fwd(x, np.eye(S)[None, :, :T], np.eye(D)[None])
    np.testing.assert_allclose(y, x[:, :T, :], rtol=0, atol=1e-15)
    # k = 1 is the separable factorisation P_seq^T X P_emb: two library matrix products
    z, w = rng.standard_normal((1, S, T)), rng.standard_normal((1, D, D))
    np.testing.assert_allclose(oracle.sumkron_fwd(x, z, w), np.matmul(np.matmul(z[0].T, x), w[0]), rtol=1e-12, atol=1e-12)
    # identical terms add up: k copies of (Z, W) give k times the single term
    np.testing.assert_allclose(oracle.sumkron_fwd(x, np.repeat(z, 3, 0), np.repeat(w, 3, 0)),
                               3 * oracle.sumkron_fwd(x, z, w), rtol=1e-12, atol=1e-12)


def test_sumkron_multilinear(oracle):
    x, z, w = _rand(4)
    x2, z2, w2 = _rand(5)
    f = oracle.sumkron_fwd
    np.testing.assert_allclose(f(x + 2 * x2, z, w), f(x, z, w) + 2 * f(x2, z, w), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(f(x, z - 3 * z2, w), f(x, z, w) - 3 * f(x, z2, w), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(f(x, z, w + 0.5 * w2), f(x, z, w) + 0.5 * f(x, z, w2), rtol=1e-11, atol=1e-11)
    # examples are independent
    np.testing.assert_array_equal(f(x[1:2], z, w), f(x, z, w)[1:2])


def test_sumkron_backward_finite_differences(oracle):
    x, z, w = _rand(6, B=2, S=3, T=2, D=3, k=2)
    dy = np.random.default_rng(7).standard_normal((2, 2, 3))
    dx, dz, dw = oracle.sumkron_bwd(x, z, w, dy)
    loss = lambda a, b, c: float((oracle.sumkron_fwd(a, b, c) * dy).sum())
    h = 1e-6
    for grad, which in ((dx, 0), (dz, 1), (dw, 2)):
        args = [x, z, w]
        num = np.zeros_like(args[which])
        it = np.nditer(args[which], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            plus = [a.copy() for a in args]; minus = [a.copy() for a in args]
            plus[which][idx] += h; minus[which][idx] -= h
            num[idx] = (loss(*plus) - loss(*minus)) / (2 * h)
        np.testing.assert_allclose(grad, num, rtol=1e-6, atol=1e-7)


def test_sumkron_backward_vs_autograd(oracle):
    x, z, w = _rand(8)
    dy = np.random.default_rng(9).standard_normal((x.shape[0], z.shape[2], x.shape[2]))
    tx, tz, tw = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, z, w)]
    y = sum(tz[i].T @ tx @ tw[i] for i in range(z.shape[0]))
    np.testing.assert_allclose(oracle.sumkron_fwd(x, z, w), y.detach().numpy(), rtol=1e-12, atol=1e-12)
    (y * torch.tensor(dy)).sum().backward()
    dx, dz, dw = oracle.sumkron_bwd(x, z, w, dy)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dz, tz.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_sumkron_paper_shape_sample(oracle):
    """The paper's typical configuration (S=256, T=32, D=384, k=8), one example: a few output
    entries against the separable-term form evaluated with library matrix products."""
    rng = np.random.default_rng(10)
    S, T, D, k = 256, 32, 384, 8
    x = rng.standard_normal((1, S, D)); z = rng.standard_normal((k, S, T)) / 16; w = rng.standard_normal((k, D, D)) / 20
    y = oracle.sumkron_fwd(x, z, w)
    ref = sum(z[i].T @ x[0] @ w[i] for i in range(k))
    np.testing.assert_allclose(y[0], ref, rtol=1e-10, atol=1e-10)
