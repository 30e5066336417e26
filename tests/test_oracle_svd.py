"""Pins for the SVD split of Algorithm 1 (U = Ut S^(1/2), V^T = S^(1/2) Vt^T).

The oracle's one-sided Jacobi routine is pinned against numpy.linalg.svd
(singular values), exact reconstruction at full rank, the Eckart-Young
residual, and the balanced-factor invariant U^T U = V^T V = diag(sigma_r).
The factors themselves are unique only up to signs/rotations, so they are
never compared element-wise.
"""
import numpy as np
import pytest

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("m,n", [(1, 1), (6, 4), (4, 6), (9, 9), (20, 7), (18, 32)])
def test_full_rank_reconstructs_W(m, n):
    W = _rand((m, n), m * 100 + n)
    r = min(m, n)
    U, V, sigma = oracle.svd_split(W, r)
    np.testing.assert_allclose(U @ V.T, W, rtol=0, atol=1e-12 * max(1.0, np.abs(W).max()) * 10)
    np.testing.assert_allclose(sigma, np.linalg.svd(W, compute_uv=False), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("m,n,r", [(8, 5, 2), (5, 8, 3), (16, 16, 4), (30, 12, 1)])
def test_truncation_is_eckart_young_optimal_and_balanced(m, n, r):
    W = _rand((m, n), 7 * m + n)
    U, V, sigma = oracle.svd_split(W, r)
    s_ref = np.linalg.svd(W, compute_uv=False)
    np.testing.assert_allclose(sigma, s_ref, rtol=1e-12, atol=1e-12)
    resid = np.linalg.norm(W - U @ V.T, "fro") ** 2
    np.testing.assert_allclose(resid, (s_ref[r:] ** 2).sum(), rtol=1e-10)
    np.testing.assert_allclose(U.T @ U, np.diag(s_ref[:r]), rtol=0, atol=1e-11)
    np.testing.assert_allclose(V.T @ V, np.diag(s_ref[:r]), rtol=0, atol=1e-11)


def test_known_singular_values():
    # W = diag(3, 2, 1) padded: singular values are known in closed form
    W = np.zeros((4, 3))
    W[0, 0], W[1, 1], W[2, 2] = 3.0, 2.0, 1.0
    U, V, sigma = oracle.svd_split(W, 2)
    np.testing.assert_allclose(sigma, [3.0, 2.0, 1.0], atol=1e-14)
    expect = np.zeros((4, 3))
    expect[0, 0], expect[1, 1] = 3.0, 2.0
    np.testing.assert_allclose(U @ V.T, expect, atol=1e-14)


def test_conv_unroll_and_full_rank_layer_equivalence():
    # Section 2.2 / Section 3: SVD of the unrolled [C k^2 x Cout] matrix; at full rank the
    # factorized convolution reproduces the dense one.
    Cout, C, k = 5, 3, 3
    Wd = _rand((Cout, C, k, k), 11)
    r = min(C * k * k, Cout)
    Uk, Vp, sigma = oracle.svd_split_conv(Wd, r)
    assert Uk.shape == (r, C, k, k) and Vp.shape == (Cout, r)
    np.testing.assert_allclose(np.einsum("oq,qcij->ocij", Vp, Uk), Wd, atol=1e-12)
    X = _rand((2, C, 5, 5), 12)
    Y, _ = oracle.lowrank_conv_fwd(X, Uk, Vp, 1, 1)
    np.testing.assert_allclose(Y, oracle.dense_conv_fwd(X, Wd, 1, 1), atol=1e-11)


def test_full_rank_linear_layer_equivalence():
    W = _rand((7, 10), 13)  # [out x in]
    U, V, _ = oracle.svd_split(W, 7)
    X = _rand((4, 10), 14)
    Y, _ = oracle.lowrank_linear_fwd(X, V, U, None)
    np.testing.assert_allclose(Y, X @ W.T, atol=1e-12)
