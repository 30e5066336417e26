"""Pins of the oracle's layer epilogues (bias / fixed-statistics batch norm, residual input, ReLU, and their
backward) against torch.nn.functional on the CPU in float64: a Transformer feed-forward block (Section 2.4,
FFN(x) = max(0, x W1 + b1) W2 + b2 with its residual connection) and a ResNet basic block (Appendix D: batch
norm after every convolution, ReLU, identity shortcut), each with W = (output-side factor)(input-side factor)^T."""
import numpy as np
import torch
import torch.nn.functional as F

import oracle

RTOL = 1e-10


def _close(got, want, name):
    want = want.detach().numpy() if isinstance(want, torch.Tensor) else np.asarray(want)
    err = np.abs(np.asarray(got) - want).max() / max(np.abs(want).max(), 1e-300)
    assert err <= RTOL, f"{name}: {err:.2e}"


def _t(a, grad=True):
    return torch.tensor(a, dtype=torch.float64, requires_grad=grad)


def test_feed_forward_block_against_torch():
    rng = np.random.default_rng(7)
    M, d, dff, r = 9, 12, 20, 5
    x = rng.standard_normal((M, d))
    V1, U1, b1 = rng.standard_normal((d, r)) * .4, rng.standard_normal((dff, r)) * .4, rng.standard_normal(dff) * .3
    V2, U2, b2 = rng.standard_normal((dff, r)) * .4, rng.standard_normal((d, r)) * .4, rng.standard_normal(d) * .3
    dY = rng.standard_normal((M, d))
    # torch: y = x + FFN(x), factors as leaves
    tx, tV1, tU1, tb1, tV2, tU2, tb2 = map(_t, (x, V1, U1, b1, V2, U2, b2))
    H = F.relu(F.linear(tx, tU1 @ tV1.t(), tb1))
    y = F.linear(H, tU2 @ tV2.t(), tb2) + tx
    y.backward(torch.tensor(dY))
    # oracle: two calls forward, two backward, the gradient of max(0, .) applied where dH is formed
    Ho, T1 = oracle.lowrank_linear_fwd_ep(x, V1, U1, b1, act="relu")
    yo, T2 = oracle.lowrank_linear_fwd_ep(Ho, V2, U2, b2, residual=x)
    _close(Ho, H, "H")
    _close(yo, y, "y")
    assert (Ho == 0).any() and (Ho > 0).any()  # the mask is exercised
    dZ1, dU2, dV2, db2 = oracle.lowrank_linear_bwd_ep(Ho, V2, U2, dY, x_is_relu=True)
    dx, dU1, dV1, db1 = oracle.lowrank_linear_bwd_ep(x, V1, U1, dZ1, dX_add=dY)
    for name, got, want in (("dx", dx, tx.grad), ("dU1", dU1, tU1.grad), ("dV1", dV1, tV1.grad), ("db1", db1, tb1.grad),
                            ("dU2", dU2, tU2.grad), ("dV2", dV2, tV2.grad), ("db2", db2, tb2.grad)):
        _close(got, want, name)


def test_epilogue_order_and_hand_values():
    # Z = P + b + R, then max(0, .): worked by hand for a 1 x 1 layer with X = 2, V = 3, U = -1 (P = -6)
    X, V, U = np.array([[2.0]]), np.array([[3.0]]), np.array([[-1.0]])
    Y, T = oracle.lowrank_linear_fwd_ep(X, V, U, np.array([1.0]), residual=np.array([[7.0]]), act="relu")
    assert T[0, 0] == 6.0 and Y[0, 0] == 2.0         # -6 + 1 + 7
    Y, _ = oracle.lowrank_linear_fwd_ep(X, V, U, np.array([1.0]), residual=np.array([[4.0]]), act="relu")
    assert Y[0, 0] == 0.0                             # -6 + 1 + 4 < 0: clipped after the residual is added
    Y, _ = oracle.lowrank_linear_fwd_ep(X, V, U, np.array([1.0]), residual=np.array([[4.0]]))
    assert Y[0, 0] == -1.0
    # backward: dX = (dZ U V^T + dX_add) [X > 0]
    dX, dU, dV, db = oracle.lowrank_linear_bwd_ep(X, V, U, np.array([[5.0]]), dX_add=np.array([[0.5]]), x_is_relu=True)
    assert dX[0, 0] == -14.5 and dU[0, 0] == 30.0 and dV[0, 0] == -10.0 and db[0] == 5.0
    dX, _, _, _ = oracle.lowrank_linear_bwd_ep(np.array([[0.0]]), V, U, np.array([[5.0]]), x_is_relu=True)
    assert dX[0, 0] == 0.0                            # an input at exactly zero passes no gradient (torch's convention)
    # convolution: per-channel scale before shift, residual before the activation
    Xc, Uk, Vp = np.full((1, 1, 1, 1), 2.0), np.full((1, 1, 1, 1), 3.0), np.array([[1.0], [-1.0]])
    Y, _ = oracle.lowrank_conv_fwd_ep(Xc, Uk, Vp, scale=[0.5, 2.0], shift=[1.0, 1.0],
                                      residual=np.array([0.0, 12.0]).reshape(1, 2, 1, 1), act="relu")
    assert Y.ravel().tolist() == [4.0, 1.0]           # 0.5*6+1 ; 2*(-6)+1+12
    dX, dUk, dVp, dsh = oracle.lowrank_conv_bwd_ep(Xc, Uk, Vp, [0.5, 2.0], np.array([1.0, 3.0]).reshape(1, 2, 1, 1))
    assert dsh.tolist() == [1.0, 3.0] and dVp.ravel().tolist() == [3.0, 36.0]  # scale * dZ * T, T = 6
    assert dX.ravel().tolist() == [(0.5 * 1.0 * 1.0 + 2.0 * 3.0 * -1.0) * 3.0]


def _bn_affine(rng, C, eps=1e-5):
    gamma, beta = rng.uniform(.5, 1.5, C), rng.standard_normal(C) * .2
    mean, var = rng.standard_normal(C) * .3, rng.uniform(.5, 2.0, C)
    scale = gamma / np.sqrt(var + eps)
    return (gamma, beta, mean, var, eps), scale, beta - mean * scale


def test_resnet_basic_block_against_torch():
    rng = np.random.default_rng(11)
    N, C, Hh, Ww, r = 3, 6, 5, 4, 2
    x = np.maximum(rng.standard_normal((N, C, Hh, Ww)), 0.0)   # the block's input is a ReLU output of the block below
    Uk1, Vp1 = rng.standard_normal((r, C, 3, 3)) * .3, rng.standard_normal((C, r)) * .5
    Uk2, Vp2 = rng.standard_normal((r, C, 3, 3)) * .3, rng.standard_normal((C, r)) * .5
    bn1, s1, h1 = _bn_affine(rng, C)
    bn2, s2, h2 = _bn_affine(rng, C)
    dY = rng.standard_normal((N, C, Hh, Ww))

    def bn(t, p, beta):
        gamma, _, mean, var, eps = p
        return F.batch_norm(t, torch.tensor(mean), torch.tensor(var), torch.tensor(gamma), beta, training=False, eps=eps)

    tx, tU1, tV1, tU2, tV2 = map(_t, (x, Uk1, Vp1, Uk2, Vp2))
    tb1, tb2 = _t(bn1[1]), _t(bn2[1])
    conv = lambda t, U, V: F.conv2d(F.conv2d(t, U, padding=1), V[:, :, None, None])
    y1 = F.relu(bn(conv(tx, tU1, tV1), bn1, tb1))
    y2 = F.relu(bn(conv(y1, tU2, tV2), bn2, tb2) + tx)
    y2.backward(torch.tensor(dY))

    y1o, _ = oracle.lowrank_conv_fwd_ep(x, Uk1, Vp1, s1, h1, act="relu", stride=1, pad=1)
    y2o, _ = oracle.lowrank_conv_fwd_ep(y1o, Uk2, Vp2, s2, h2, residual=x, act="relu", stride=1, pad=1)
    _close(y1o, y1, "y1")
    _close(y2o, y2, "y2")
    dZ2 = dY * (y2o > 0)   # the block above would have applied this mask where it formed the gradient of its input
    dZ1, dUk2, dVp2, dsh2 = oracle.lowrank_conv_bwd_ep(y1o, Uk2, Vp2, s2, dZ2, 1, 1, x_is_relu=True)
    dx, dUk1, dVp1, dsh1 = oracle.lowrank_conv_bwd_ep(x, Uk1, Vp1, s1, dZ1, 1, 1, dX_add=dZ2)
    for name, got, want in (("dx", dx, tx.grad), ("dUk1", dUk1, tU1.grad), ("dVp1", dVp1, tV1.grad),
                            ("dUk2", dUk2, tU2.grad), ("dVp2", dVp2, tV2.grad), ("dshift1", dsh1, tb1.grad),
                            ("dshift2", dsh2, tb2.grad)):
        _close(got, want, name)
    # with the mask on the block's own input (the gradient handed to the block below)
    dxm, _, _, _ = oracle.lowrank_conv_bwd_ep(x, Uk1, Vp1, s1, dZ1, 1, 1, dX_add=dZ2, x_is_relu=True)
    _close(dxm, tx.grad.numpy() * (x > 0), "masked dx")


def test_strided_epilogue_and_no_scale():
    """Stride 2 on the k x k stage, no scale, no activation: the epilogue reduces to a bias and a residual add."""
    rng = np.random.default_rng(13)
    x = rng.standard_normal((2, 4, 7, 6))
    Uk, Vp, sh = rng.standard_normal((3, 4, 3, 3)) * .3, rng.standard_normal((5, 3)) * .5, rng.standard_normal(5)
    R = rng.standard_normal((2, 5, 4, 3))
    tx, tU, tV, tb = map(_t, (x, Uk, Vp, sh))
    y = F.conv2d(F.conv2d(tx, tU, stride=2, padding=1), tV[:, :, None, None], bias=tb) + torch.tensor(R)
    dY = rng.standard_normal(y.shape)
    y.backward(torch.tensor(dY))
    yo, _ = oracle.lowrank_conv_fwd_ep(x, Uk, Vp, None, sh, residual=R, stride=2, pad=1)
    _close(yo, y, "y")
    dx, dUk, dVp, dsh = oracle.lowrank_conv_bwd_ep(x, Uk, Vp, None, dY, 2, 1)
    for name, got, want in (("dx", dx, tx.grad), ("dUk", dUk, tU.grad), ("dVp", dVp, tV.grad), ("dshift", dsh, tb.grad)):
        _close(got, want, name)
