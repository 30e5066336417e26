"""GPU parity of the layer epilogues (pf_lowrank_linear_fwd_ep/bwd_ep, pf_lowrank_conv_fwd_ep/bwd_ep, through the C
ABI) against the CPU oracle: the feed-forward block of a Transformer layer (Section 2.4) and a ResNet basic block
(Appendix D), chained the way a training step chains them, on the fused kernels' shapes and on odd ones."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu


def _round(a, dtype):
    """Values as the GPU holds them (bf16-exact for bf16 runs), as float64."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy().astype(np.float64)


def _ffn_block(M, d, dff, r, dtype, seed):
    """y = x + FFN(x): forward through two *_fwd_ep calls, backward through two *_bwd_ep calls; every call is
    compared with the oracle given the same (GPU-produced, hence dtype-exact) inputs."""
    import paper_2103_03936_amd as pf
    a1 = workloads.linear_inputs(M, d, dff, r, dtype=dtype, seed=seed, bias=True)
    a2 = workloads.linear_inputs(M, dff, d, r, dtype=dtype, seed=seed + 1, bias=True)
    x, dY = a1["X"], a2["dY"]
    g1 = {k: to_gpu(v, dtype) for k, v in a1.items()}
    g2 = {k: to_gpu(v, dtype) for k, v in a2.items()}
    tag = f"ffn({M},{d},{dff},{r})[{dtype}]"
    # forward
    H, T1 = pf.pf_lowrank_linear_fwd_ep(g1["X"], g1["V"], g1["U"], g1["bias"], act="relu")
    Ho, T1o = oracle.lowrank_linear_fwd_ep(x, a1["V"], a1["U"], a1["bias"], act="relu")
    assert_close(H, Ho, dtype, tag + " H")
    assert float((H == 0).float().mean()) > 0.2 and float((H > 0).float().mean()) > 0.2
    Hn = H.float().cpu().numpy().astype(np.float64)   # the second layer sees what the first one stored
    Y, T2 = pf.pf_lowrank_linear_fwd_ep(H, g2["V"], g2["U"], g2["bias"], residual=g1["X"])
    Yo, _ = oracle.lowrank_linear_fwd_ep(Hn, a2["V"], a2["U"], a2["bias"], residual=x)
    assert_close(Y, Yo, dtype, tag + " Y")
    # backward: the mask of max(0, .) where dH is formed, the skip gradient where dx is formed
    dZ1, dU2, dV2, db2 = pf.pf_lowrank_linear_bwd_ep(H, g2["V"], g2["U"], g2["dY"], T_saved=T2, x_is_relu=True,
                                                      has_bias=True)
    dZ1o, dU2o, dV2o, db2o = oracle.lowrank_linear_bwd_ep(Hn, a2["V"], a2["U"], dY, x_is_relu=True)
    for name, got, ref in (("dZ1", dZ1, dZ1o), ("dU2", dU2, dU2o), ("dV2", dV2, dV2o), ("db2", db2, db2o)):
        assert_close(got, ref, dtype, f"{tag} {name}")
    assert bool(((dZ1 == 0) | (H > 0)).all()), "gradient passed where the activation is zero"
    dZ1n = dZ1.float().cpu().numpy().astype(np.float64)
    dx, dU1, dV1, db1 = pf.pf_lowrank_linear_bwd_ep(g1["X"], g1["V"], g1["U"], dZ1, T_saved=T1, dX_add=g2["dY"],
                                                    has_bias=True)
    dxo, dU1o, dV1o, db1o = oracle.lowrank_linear_bwd_ep(x, a1["V"], a1["U"], dZ1n, dX_add=dY)
    for name, got, ref in (("dx", dx, dxo), ("dU1", dU1, dU1o), ("dV1", dV1, dV1o), ("db1", db1, db1o)):
        assert_close(got, ref, dtype, f"{tag} {name}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(5, 7, 9, 3), (64, 512, 512, 128), (300, 96, 200, 24), (1, 4, 4, 4)])
def test_feed_forward_block(shape, dtype):
    _ffn_block(*shape, dtype, seed=60)


def test_feed_forward_block_transformer_size():
    # Appendix D: d_model 512, d_ff 2048, rank 128, 8192 tokens, bf16: the fused kernels
    _ffn_block(8192, 512, 2048, 128, "bf16", seed=3)


def _bn(rng, C):
    gamma, beta = rng.uniform(.5, 1.5, C), rng.standard_normal(C) * .2
    mean, var = rng.standard_normal(C) * .3, rng.uniform(.5, 2.0, C)
    scale = gamma / np.sqrt(var + 1e-5)
    return scale.astype(np.float32), (beta - mean * scale).astype(np.float32)


def _basic_block(N, C, H, W, r, k, dtype, seed):
    """y1 = relu(bn1(conv1(x))), y2 = relu(bn2(conv2(y1)) + x) and the matching backward, call by call."""
    import paper_2103_03936_amd as pf
    p = k // 2
    rng = np.random.default_rng(seed)
    a1 = workloads.conv_inputs(N, C, H, W, C, r, k, 1, p, dtype=dtype, seed=seed)
    a2 = workloads.conv_inputs(N, C, H, W, C, r, k, 1, p, dtype=dtype, seed=seed + 1)
    x = _round(np.maximum(a1["X"], 0.0), dtype)   # the block's input is the block below's ReLU output
    (s1, h1), (s2, h2) = _bn(rng, C), _bn(rng, C)
    dY = a2["dY"]
    gx = to_gpu(x.astype(np.float32), dtype)
    g1 = {k_: to_gpu(v, dtype) for k_, v in a1.items()}
    g2 = {k_: to_gpu(v, dtype) for k_, v in a2.items()}
    f32 = lambda v: torch.from_numpy(v).cuda()
    tag = f"block({N},{C},{H},{W},{r},{k})[{dtype}]"
    y1, T1, W1 = pf.pf_lowrank_conv_fwd_ep(gx, g1["Uk"], g1["Vp"], f32(s1), f32(h1), act="relu", stride=1, pad=p, save_W=True)
    y1o, _ = oracle.lowrank_conv_fwd_ep(x, a1["Uk"], a1["Vp"], s1, h1, act="relu", stride=1, pad=p)
    assert_close(y1, y1o, dtype, tag + " y1")
    y1n = y1.float().cpu().numpy().astype(np.float64)
    y2, T2, W2 = pf.pf_lowrank_conv_fwd_ep(y1, g2["Uk"], g2["Vp"], f32(s2), f32(h2), residual=gx, act="relu", stride=1,
                                           pad=p, save_W=True)
    y2o, _ = oracle.lowrank_conv_fwd_ep(y1n, a2["Uk"], a2["Vp"], s2, h2, residual=x, act="relu", stride=1, pad=p)
    assert_close(y2, y2o, dtype, tag + " y2")
    assert float((y2 == 0).float().mean()) > 0.1
    # what the block above hands down: dL/dZ2, already masked by y2 > 0
    dZ2 = _round(dY * (y2.float().cpu().numpy() > 0), dtype)
    gdZ2 = to_gpu(dZ2.astype(np.float32), dtype)
    dZ1, dUk2, dVp2, dsh2 = pf.pf_lowrank_conv_bwd_ep(y1, g2["Uk"], g2["Vp"], f32(s2), gdZ2, T_saved=T2, stride=1, pad=p,
                                                      x_is_relu=True, W_saved=W2)
    dZ1o, dUk2o, dVp2o, dsh2o = oracle.lowrank_conv_bwd_ep(y1n, a2["Uk"], a2["Vp"], s2, dZ2, 1, p, x_is_relu=True)
    for name, got, ref in (("dZ1", dZ1, dZ1o), ("dUk2", dUk2, dUk2o), ("dVp2", dVp2, dVp2o), ("dshift2", dsh2, dsh2o)):
        assert_close(got, ref, dtype, f"{tag} {name}")
    assert bool(((dZ1 == 0) | (y1 > 0)).all())
    dZ1n = dZ1.float().cpu().numpy().astype(np.float64)
    dx, dUk1, dVp1, dsh1 = pf.pf_lowrank_conv_bwd_ep(gx, g1["Uk"], g1["Vp"], f32(s1), dZ1, T_saved=T1, stride=1, pad=p,
                                                     dX_add=gdZ2, x_is_relu=True, W_saved=W1)
    dxo, dUk1o, dVp1o, dsh1o = oracle.lowrank_conv_bwd_ep(x, a1["Uk"], a1["Vp"], s1, dZ1n, 1, p, dX_add=dZ2, x_is_relu=True)
    for name, got, ref in (("dx", dx, dxo), ("dUk1", dUk1, dUk1o), ("dVp1", dVp1, dVp1o), ("dshift1", dsh1, dsh1o)):
        assert_close(got, ref, dtype, f"{tag} {name}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 6, 5, 4, 2, 3), (3, 16, 8, 8, 4, 3), (2, 10, 7, 7, 3, 1)])
def test_basic_block(shape, dtype):
    _basic_block(*shape, dtype, seed=70)


@pytest.mark.parametrize("shape", [(9, 256, 8, 8, 64, 3), (5, 512, 7, 7, 128, 3), (6, 256, 7, 7, 128, 1)])
def test_basic_block_fused_shapes(shape):
    _basic_block(*shape, "bf16", seed=80)


def test_basic_block_resnet18_conv4_size():
    c = workloads.CONFIGS["resnet18_conv4_bf16"]
    _basic_block(c["N"], c["C"], c["H"], c["W"], c["r"], c["k"], "bf16", seed=c["seed"])


def test_epilogue_options_one_at_a_time():
    """No scale, no shift, no residual, no activation reduce to the plain calls bit for bit; accumulation works."""
    import paper_2103_03936_amd as pf
    a = workloads.conv_inputs(3, 8, 6, 6, 10, 4, 3, 1, 1, dtype="f32", seed=90)
    g = {k_: to_gpu(v) for k_, v in a.items()}
    Y0, T0 = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], 1, 1)
    Y1, T1 = pf.pf_lowrank_conv_fwd_ep(g["X"], g["Uk"], g["Vp"], stride=1, pad=1)
    assert torch.equal(Y0, Y1) and torch.equal(T0, T1)
    sc = torch.from_numpy(np.linspace(.5, 2, 10).astype(np.float32)).cuda()
    dX0, dUk0, dVp0 = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], T_saved=T0, stride=1, pad=1)
    dX1, dUk1, dVp1, dsh = pf.pf_lowrank_conv_bwd_ep(g["X"], g["Uk"], g["Vp"], None, g["dY"], T_saved=T0, stride=1, pad=1)
    assert torch.equal(dX0, dX1) and torch.equal(dUk0, dUk1) and torch.equal(dVp0, dVp1)
    assert_close(dsh, a["dY"].astype(np.float64).sum(axis=(0, 2, 3)), "f32", "dshift")
    grads = (dUk1.clone(), dVp1.clone(), dsh.clone())
    pf.pf_lowrank_conv_bwd_ep(g["X"], g["Uk"], g["Vp"], sc, g["dY"], T_saved=T0, stride=1, pad=1, grads=grads)
    _, dUo, dVo, dso = oracle.lowrank_conv_bwd_ep(a["X"], a["Uk"], a["Vp"], sc.cpu().numpy(), a["dY"], 1, 1)
    _, dUp, dVpp, _ = oracle.lowrank_conv_bwd_ep(a["X"], a["Uk"], a["Vp"], None, a["dY"], 1, 1)
    assert_close(grads[0], dUo + dUp, "f32", "accumulated dUk")
    assert_close(grads[1], dVo + dVpp, "f32", "accumulated dVp")
    assert_close(grads[2], 2 * dso, "f32", "accumulated dshift")
    b = workloads.linear_inputs(40, 24, 16, 4, dtype="f32", seed=91, bias=True)
    gb = {k_: to_gpu(v) for k_, v in b.items()}
    Ya, Ta = pf.pf_lowrank_linear_fwd(gb["X"], gb["V"], gb["U"], gb["bias"])
    Yb, Tb = pf.pf_lowrank_linear_fwd_ep(gb["X"], gb["V"], gb["U"], gb["bias"])
    assert torch.equal(Ya, Yb) and torch.equal(Ta, Tb)


def test_epilogue_validation():
    import ctypes
    import paper_2103_03936_amd as pf
    fake, z = ctypes.c_void_p(256), ctypes.c_size_t(1 << 30)
    d = pf.pf_linear_desc(4, 8, 8, 2, 0, 0, 0)
    assert pf.lib.pf_lowrank_linear_fwd_ep(ctypes.byref(d), fake, fake, fake, None, None, 7, fake, None, fake, z, None) == 3
    assert pf.lib.pf_lowrank_linear_fwd_ep(ctypes.byref(d), fake, fake, fake, None, ctypes.c_void_p(260), 1, fake, None,
                                           fake, z, None) == 3
    c = pf.pf_conv_desc(2, 3, 5, 5, 4, 2, 3, 1, 1, 0, 0, 0)
    assert pf.lib.pf_lowrank_conv_fwd_ep(ctypes.byref(c), fake, fake, fake, None, None, None, 2, fake, None, None, fake, z,
                                         None) == 3
    need = pf.lib.pf_lowrank_conv_bwd_ep_workspace_bytes(ctypes.byref(c))
    assert need > pf.lib.pf_lowrank_conv_bwd_workspace_bytes(ctypes.byref(c))
    assert pf.lib.pf_lowrank_conv_bwd_ep(ctypes.byref(c), fake, fake, fake, fake, fake, None, None, None, 0, fake, fake, fake,
                                         None, 0, fake, ctypes.c_size_t(need - 1), None) == 4
