"""Pins for the convolution oracle (Section 2.2, Appendix B "Convolution layer").

Pinned against torch's conv2d and autograd (library routines the oracle does
not use), the dense layer with W_unrolled = U V^T, the k = 1 reduction to the
linear layer, a hand-worked fixture and finite differences.
"""
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

SHAPES = [
    # N, C, H, W, Cout, r, k, stride, pad
    (1, 1, 3, 3, 1, 1, 3, 1, 1),
    (2, 3, 5, 4, 4, 2, 3, 1, 1),
    (2, 4, 6, 7, 5, 3, 3, 2, 1),
    (3, 5, 4, 4, 6, 2, 1, 1, 0),
    (1, 2, 7, 5, 3, 2, 5, 1, 2),
    (2, 3, 6, 6, 2, 4, 3, 1, 0),
]


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _inputs(shape):
    N, C, H, W, Cout, r, k, s, p = shape
    Ho, Wo = oracle.conv_out_dim(H, k, s, p), oracle.conv_out_dim(W, k, s, p)
    return (_rand((N, C, H, W), 1), _rand((r, C, k, k), 2), _rand((Cout, r), 3), _rand((N, Cout, Ho, Wo), 4))


def test_hand_worked_fixture():
    g = json.load(open(os.path.join(GOLDEN, "conv_hand.json")))
    X, Uk, Vp, dY = (np.array(g[k], dtype=np.float64) for k in ("X", "Uk", "Vp", "dY"))
    Y, T = oracle.lowrank_conv_fwd(X, Uk, Vp, stride=1, pad=1)
    assert np.array_equal(T, np.array(g["T"]))
    assert np.array_equal(Y, np.array(g["Y"]))
    dX, dUk, dVp = oracle.lowrank_conv_bwd(X, Uk, Vp, dY, stride=1, pad=1)
    assert np.array_equal(dVp, np.array(g["dVp"]))
    assert np.array_equal(dUk, np.array(g["dUk"]))
    assert np.array_equal(dX, np.array(g["dX"]))


@pytest.mark.parametrize("shape", SHAPES)
def test_fwd_matches_torch_two_stage(shape):
    N, C, H, W, Cout, r, k, s, p = shape
    X, Uk, Vp, _ = _inputs(shape)
    Y, T = oracle.lowrank_conv_fwd(X, Uk, Vp, s, p)
    tT = F.conv2d(torch.tensor(X), torch.tensor(Uk), stride=s, padding=p)
    tY = F.conv2d(tT, torch.tensor(Vp).reshape(Cout, r, 1, 1))
    np.testing.assert_allclose(T, tT.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(Y, tY.numpy(), rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("shape", SHAPES)
def test_fwd_equals_dense_conv_with_composed_filters(shape):
    # Section 2.2: the filter bank is a linear combination of r basis filters,
    # W[o,c,i,j] = sum_q Vp[o,q] Uk[q,c,i,j]  (W_unrolled = U V^T).
    N, C, H, W, Cout, r, k, s, p = shape
    X, Uk, Vp, _ = _inputs(shape)
    Y, _ = oracle.lowrank_conv_fwd(X, Uk, Vp, s, p)
    Wd = np.einsum("oq,qcij->ocij", Vp, Uk)
    tY = F.conv2d(torch.tensor(X), torch.tensor(Wd), stride=s, padding=p).numpy()
    np.testing.assert_allclose(Y, tY, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(oracle.dense_conv_fwd(X, Wd, s, p), tY, rtol=1e-10, atol=1e-10)
    # unrolled view: column o of W_unrolled [C k^2 x Cout] is filter o vectorised
    U2 = Uk.reshape(r, C * k * k).T
    np.testing.assert_allclose(Wd.reshape(Cout, -1).T, U2 @ Vp.T, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
def test_bwd_matches_torch_autograd(shape):
    N, C, H, W, Cout, r, k, s, p = shape
    X, Uk, Vp, dY = _inputs(shape)
    tX, tU, tV = (torch.tensor(a, requires_grad=True) for a in (X, Uk, Vp))
    tY = F.conv2d(F.conv2d(tX, tU, stride=s, padding=p), tV.reshape(Cout, r, 1, 1))
    tY.backward(torch.tensor(dY))
    dX, dUk, dVp = oracle.lowrank_conv_bwd(X, Uk, Vp, dY, s, p)
    np.testing.assert_allclose(dX, tX.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dUk, tU.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dVp, tV.grad.numpy(), rtol=1e-10, atol=1e-10)


def test_k1_reduces_to_linear_layer():
    # a 1x1 "thin" stage makes the layer a factorized linear map over channels at each pixel
    N, C, H, W, Cout, r = 2, 5, 3, 4, 6, 3
    X, Uk, Vp = _rand((N, C, H, W), 1), _rand((r, C, 1, 1), 2), _rand((Cout, r), 3)
    dY = _rand((N, Cout, H, W), 4)
    Y, T = oracle.lowrank_conv_fwd(X, Uk, Vp, 1, 0)
    Xm = X.transpose(0, 2, 3, 1).reshape(-1, C)
    V = Uk.reshape(r, C).T
    Ym, Tm = oracle.lowrank_linear_fwd(Xm, V, Vp, None)
    np.testing.assert_allclose(Y.transpose(0, 2, 3, 1).reshape(-1, Cout), Ym, rtol=1e-12, atol=1e-12)
    dX, dUk, dVp = oracle.lowrank_conv_bwd(X, Uk, Vp, dY, 1, 0)
    dXm, dU, dV, _ = oracle.lowrank_linear_bwd(Xm, V, Vp, dY.transpose(0, 2, 3, 1).reshape(-1, Cout))
    np.testing.assert_allclose(dX.transpose(0, 2, 3, 1).reshape(-1, C), dXm, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dVp, dU, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dUk.reshape(r, C).T, dV, rtol=1e-12, atol=1e-12)


def test_cross_correlation_not_flipped_and_stride_on_first_stage_only():
    # one 3x3 basis filter with a single 1 at tap (0, 2): output pixel (y, x) must read
    # input pixel (y - 1, x + 1) (no kernel flip), and with stride 2 the 1x1 stage keeps
    # the thin stage's output grid.
    X = np.arange(36, dtype=np.float64).reshape(1, 1, 6, 6)
    Uk = np.zeros((1, 1, 3, 3))
    Uk[0, 0, 0, 2] = 1.0
    Vp = np.array([[2.0]])
    Y, T = oracle.lowrank_conv_fwd(X, Uk, Vp, stride=1, pad=1)
    assert T[0, 0, 2, 3] == X[0, 0, 1, 4] and T[0, 0, 0, 0] == 0.0 and T[0, 0, 1, 5] == 0.0
    assert np.array_equal(Y, 2.0 * T)
    Y2, T2 = oracle.lowrank_conv_fwd(X, Uk, Vp, stride=2, pad=1)
    assert T2.shape == (1, 1, 3, 3) and Y2.shape == (1, 1, 3, 3)
    assert T2[0, 0, 1, 1] == X[0, 0, 1, 3]


def test_bwd_finite_differences():
    shape = (1, 2, 4, 3, 2, 2, 3, 1, 1)
    X, Uk, Vp, G = _inputs(shape)
    s, p = shape[7], shape[8]

    def loss(X_, Uk_, Vp_):
        return float((oracle.lowrank_conv_fwd(X_, Uk_, Vp_, s, p)[0] * G).sum())

    dX, dUk, dVp = oracle.lowrank_conv_bwd(X, Uk, Vp, G, s, p)
    eps = 1e-6
    for name, arr, grad in (("X", X, dX), ("Uk", Uk, dUk), ("Vp", Vp, dVp)):
        for idx in np.ndindex(arr.shape):
            args = dict(X=X.copy(), Uk=Uk.copy(), Vp=Vp.copy())
            args[name][idx] += eps
            up = loss(**{k + "_": v for k, v in args.items()})
            args[name][idx] -= 2 * eps
            dn = loss(**{k + "_": v for k, v in args.items()})
            assert abs((up - dn) / (2 * eps) - grad[idx]) < 1e-6, (name, idx)


def test_parameter_and_mac_counts():
    # Table 1: factorized conv has c_in r k^2 + r c_out parameters; ResNet-18 conv4_x
    # (256 -> 64 -> 256) and conv5_x (512 -> 128 -> 512) from the ResNet-18 table.
    assert 256 * 64 * 9 + 64 * 256 == 163840 and 256 * 256 * 9 == 589824
    assert 512 * 128 * 9 + 128 * 512 == 655360
    # The printed ResNet-50 totals (25,557,032 -> 15,202,344) are reproduced with
    # conv5_x ranks 128 (three bottleneck blocks) and a rank-256 downsample.
    dense = 3 * (512 * 512 * 9) + (1024 * 512 + 2 * 2048 * 512) + 3 * (512 * 2048) + 1024 * 2048
    low = (3 * (512 * 128 * 9 + 128 * 512) + (1024 * 128 + 128 * 512) + 2 * (2048 * 128 + 128 * 512)
           + 3 * (512 * 128 + 128 * 2048) + (1024 * 256 + 256 * 2048))
    assert dense - low == 25557032 - 15202344
