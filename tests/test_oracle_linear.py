"""Pins for the linear-layer oracle (Section 2.1, Appendix B "FC layer").

The oracle is nested C loops; the pins are things it shares nothing with: a
hand-worked fixture, numpy's matmul, torch's autograd, finite differences and
the dense-layer identity W = U V^T.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_worked_fixture():
    # tests/golden/linear_hand.json: a 2x3 input through rank-2 factors, worked by hand.
    g = json.load(open(os.path.join(GOLDEN, "linear_hand.json")))
    X, V, U, b, dY = (np.array(g[k], dtype=np.float64) for k in ("X", "V", "U", "bias", "dY"))
    Y, T = oracle.lowrank_linear_fwd(X, V, U, b)
    assert np.array_equal(T, np.array(g["T"]))
    assert np.array_equal(Y, np.array(g["Y"]))
    dX, dU, dV, db = oracle.lowrank_linear_bwd(X, V, U, dY)
    assert np.array_equal(dX, np.array(g["dX"]))
    assert np.array_equal(dU, np.array(g["dU"]))
    assert np.array_equal(dV, np.array(g["dV"]))
    assert np.array_equal(db, np.array(g["db"]))


@pytest.mark.parametrize("M,n_in,n_out,r", [(1, 1, 1, 1), (5, 7, 4, 3), (9, 4, 11, 4), (33, 65, 17, 9)])
def test_fwd_equals_dense_layer_with_W_UVt(M, n_in, n_out, r):
    # Section 2.1: the factorized layer is the dense layer with W = U V^T.
    X, V, U, b = _rand((M, n_in), 1), _rand((n_in, r), 2), _rand((n_out, r), 3), _rand((n_out,), 4)
    Y, T = oracle.lowrank_linear_fwd(X, V, U, b)
    W = U @ V.T  # numpy's routine, independent of the oracle's loops
    np.testing.assert_allclose(Y, X @ W.T + b, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(T, X @ V, rtol=1e-12, atol=1e-12)
    # the oracle's own dense loop agrees as well
    np.testing.assert_allclose(oracle.dense_linear_fwd(X, W, b), Y, rtol=1e-12, atol=1e-12)
    # no bias
    Y0, _ = oracle.lowrank_linear_fwd(X, V, U, None)
    np.testing.assert_allclose(Y0, X @ W.T, rtol=1e-12, atol=1e-12)


def test_factor_roles_are_not_interchangeable():
    # U is the output-side factor [out x r], V the input-side factor [in x r]:
    # with in != out a transposed operand cannot even produce the right shape, and with
    # in == out swapping the two gives W^T, which the dense identity rejects.
    n = 6
    X, V, U = _rand((4, n), 5), _rand((n, 2), 6), _rand((n, 2), 7)
    Y, _ = oracle.lowrank_linear_fwd(X, V, U, None)
    assert np.abs(Y - X @ (U @ V.T).T).max() < 1e-12
    assert np.abs(Y - X @ (V @ U.T).T).max() > 1e-3


@pytest.mark.parametrize("M,n_in,n_out,r", [(3, 5, 4, 2), (8, 6, 7, 5), (17, 33, 9, 4)])
def test_bwd_matches_torch_autograd(M, n_in, n_out, r):
    X, V, U, b, dY = (_rand(s, i) for i, s in enumerate([(M, n_in), (n_in, r), (n_out, r), (n_out,), (M, n_out)]))
    tX, tV, tU, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (X, V, U, b))
    Y = (tX @ tV) @ tU.T + tb
    Y.backward(torch.tensor(dY))
    dX, dU, dV, db = oracle.lowrank_linear_bwd(X, V, U, dY)
    np.testing.assert_allclose(dX, tX.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dU, tU.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dV, tV.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_bwd_finite_differences():
    M, n_in, n_out, r = 3, 4, 5, 2
    X, V, U, b, G = (_rand(s, 10 + i) for i, s in enumerate([(M, n_in), (n_in, r), (n_out, r), (n_out,), (M, n_out)]))

    def loss(X_, V_, U_, b_):
        return float((oracle.lowrank_linear_fwd(X_, V_, U_, b_)[0] * G).sum())

    dX, dU, dV, db = oracle.lowrank_linear_bwd(X, V, U, G)
    eps = 1e-6
    for name, arr, grad in (("X", X, dX), ("V", V, dV), ("U", U, dU), ("b", b, db)):
        for idx in np.ndindex(arr.shape):
            args = dict(X=X.copy(), V=V.copy(), U=U.copy(), b=b.copy())
            args[name][idx] += eps
            up = loss(args["X"], args["V"], args["U"], args["b"])
            args[name][idx] -= 2 * eps
            dn = loss(args["X"], args["V"], args["U"], args["b"])
            assert abs((up - dn) / (2 * eps) - grad[idx]) < 1e-6, (name, idx)


def test_bwd_consistent_with_dense_gradient():
    # dW = dY^T X is the dense layer's weight gradient; with W = U V^T the chain rule
    # gives dU = dW V and dV = dW^T U.
    M, n_in, n_out, r = 12, 9, 7, 3
    X, V, U, dY = _rand((M, n_in), 20), _rand((n_in, r), 21), _rand((n_out, r), 22), _rand((M, n_out), 23)
    dX, dU, dV, db = oracle.lowrank_linear_bwd(X, V, U, dY)
    dW = dY.T @ X
    np.testing.assert_allclose(dU, dW @ V, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dV, dW.T @ U, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dX, dY @ (U @ V.T), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, dY.sum(0), rtol=1e-12, atol=1e-12)


def test_parameter_counts_table1():
    # Table 1: vanilla FC m*n, factorized r(m+n); VGG-19's fc17/fc18 at 512 -> 128 -> 512.
    m = n = 512
    r = 128
    assert r * (m + n) == 131072 and m * n == 262144


@pytest.mark.parametrize("M,n_in,n_out,r,G", [(3, 5, 4, 2, 3), (9, 6, 7, 5, 2), (4, 3, 3, 3, 1)])
def test_shared_input_projections_match_torch_autograd(M, n_in, n_out, r, G):
    """Q, K, V style projections of one input (Section 2.4) against autograd of the block written as ONE layer:
    the factors V_g side by side, the factors U_g on a block diagonal.  A dropped term in the sum over the
    projections, or gradients filed under the wrong projection, fail here."""
    X, V, U, b, dY = (_rand(s, 20 + i) for i, s in enumerate(
        [(M, n_in), (G, n_in, r), (G, n_out, r), (G, n_out), (G, M, n_out)]))
    tX, tV, tU, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (X, V, U, b))
    Vcat = torch.cat([tV[g] for g in range(G)], dim=1)                      # [in, G r]
    Ublk = torch.block_diag(*[tU[g] for g in range(G)])                     # [G out, G r]
    Ycat = (tX @ Vcat) @ Ublk.T + tb.reshape(-1)                            # [M, G out]
    Ycat.backward(torch.tensor(np.concatenate([dY[g] for g in range(G)], axis=1)))
    Y, T = oracle.lowrank_linear_shared_fwd(X, V, U, b)
    assert Y.shape == (G, M, n_out) and T.shape == (G, M, r)
    np.testing.assert_allclose(np.concatenate([Y[g] for g in range(G)], axis=1), Ycat.detach().numpy(),
                               rtol=1e-11, atol=1e-11)
    dX, dU, dV, db = oracle.lowrank_linear_shared_bwd(X, V, U, dY)
    np.testing.assert_allclose(dX, tX.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dU, tU.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dV, tV.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)
