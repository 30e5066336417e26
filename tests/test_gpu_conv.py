"""GPU parity of pf_lowrank_conv_fwd/bwd (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

SHAPES = [
    # N, C, H, W, Cout, r, k, stride, pad
    (1, 1, 3, 3, 1, 1, 3, 1, 1),
    (2, 3, 5, 4, 4, 2, 3, 1, 1),
    (2, 4, 6, 7, 5, 3, 3, 2, 1),
    (3, 5, 4, 4, 6, 2, 1, 1, 0),
    (1, 2, 7, 5, 3, 2, 5, 1, 2),
    (3, 20, 9, 7, 70, 33, 3, 1, 1),
    (5, 64, 8, 8, 64, 16, 3, 1, 1),     # ResNet-18 conv2_x at a small batch
    (4, 48, 16, 16, 40, 12, 3, 2, 1),   # strided stage
    (6, 96, 7, 7, 160, 32, 1, 1, 0),    # 1x1 bottleneck convolution
]


def _run(shape, dtype, saved_T=True, seed=0, saved_W=False):
    import paper_2103_03936_amd as pf
    N, C, H, W, Cout, r, k, s, p = shape
    a = workloads.conv_inputs(N, C, H, W, Cout, r, k, s, p, dtype=dtype, seed=seed)
    Yo, To = oracle.lowrank_conv_fwd(a["X"], a["Uk"], a["Vp"], s, p)
    dXo, dUo, dVo = oracle.lowrank_conv_bwd(a["X"], a["Uk"], a["Vp"], a["dY"], s, p)
    g = {k_: to_gpu(v, dtype) for k_, v in a.items()}
    Wsv = None
    if saved_W:
        Y, T, Wsv = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], s, p, save_T=True, save_W=True)
    else:
        Y, T = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], s, p, save_T=True)
    dX, dUk, dVp = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], T_saved=T if saved_T else None,
                                          stride=s, pad=p, W_saved=Wsv)
    torch.cuda.synchronize()
    tag = f"conv{shape}[{dtype}]"
    assert_close(Y, Yo, dtype, tag + " Y")
    assert_close(T, To, dtype, tag + " T")
    assert_close(dX, dXo, dtype, tag + " dX")
    assert_close(dUk, dUo, dtype, tag + " dUk")
    assert_close(dVp, dVo, dtype, tag + " dVp")
    assert dUk.dtype == torch.float32 and dVp.dtype == torch.float32
    return g, (Y, T, dX, dUk, dVp)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_parity(shape, dtype):
    _run(shape, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_parity_with_weights_saved_by_forward(shape, dtype):
    """The forward call also re-orders the factors for the backward kernels (W_save); where the backward pass
    reads them in place the buffer is empty and nothing changes."""
    _run(shape, dtype, saved_W=True, seed=3)


# shapes the fused small-image kernels take in bfloat16 (channels a multiple of 256, rank 64 or 128, images of at
# most 8 x 8): 8 x 8 and 7 x 7 have their own instantiations, every other height and width shares one
FUSED_SHAPES = [
    (9, 256, 8, 8, 256, 64, 3, 1, 1),
    (5, 512, 7, 7, 256, 128, 3, 1, 1),
    (6, 256, 7, 7, 512, 128, 1, 1, 0),
    (3, 256, 5, 6, 256, 64, 3, 1, 1),
    (4, 256, 3, 8, 256, 128, 3, 1, 1),
    (2, 256, 4, 4, 512, 128, 1, 1, 0),
    (7, 512, 2, 3, 256, 64, 1, 1, 0),
    (1, 256, 1, 1, 256, 64, 3, 1, 1),
    (37, 256, 8, 8, 256, 64, 3, 1, 1),   # image groups of unequal length
    (29, 512, 7, 7, 512, 128, 3, 1, 1),
    (45, 1024, 7, 7, 256, 128, 1, 1, 0),
    (11, 768, 7, 7, 256, 64, 1, 1, 0),   # 7 x 7 planes copied flat, rank 64, three rounds of 256 channels
    (3, 256, 8, 8, 768, 64, 1, 1, 0),
]


@pytest.mark.parametrize("saved_W", [False, True])
@pytest.mark.parametrize("shape", FUSED_SHAPES)
def test_parity_fused_shapes(shape, saved_W):
    _run(shape, "bf16", saved_W=saved_W, seed=11)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_parity_recomputed_T(dtype):
    _run((3, 20, 9, 7, 70, 33, 3, 1, 1), dtype, saved_T=False, seed=4)


def test_accumulate_and_skip_dX():
    import paper_2103_03936_amd as pf
    shape = (2, 12, 6, 6, 10, 4, 3, 1, 1)
    N, C, H, W, Cout, r, k, s, p = shape
    a = workloads.conv_inputs(*shape, dtype="f32", seed=8)
    g = {k_: to_gpu(v) for k_, v in a.items()}
    dX, dUk, dVp = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], stride=s, pad=p)
    grads = (dUk.clone(), dVp.clone())
    dX2, _, _ = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], stride=s, pad=p, need_dX=False, grads=grads)
    _, dUo, dVo = oracle.lowrank_conv_bwd(a["X"], a["Uk"], a["Vp"], a["dY"], s, p)
    assert dX2 is None
    assert_close(grads[0], 2 * dUo, "f32", "accumulated dUk")
    assert_close(grads[1], 2 * dVo, "f32", "accumulated dVp")


def test_empty_batch():
    import paper_2103_03936_amd as pf
    a = workloads.conv_inputs(0, 4, 5, 5, 6, 2, 3, 1, 1, dtype="f32", seed=1)
    g = {k_: to_gpu(v) for k_, v in a.items()}
    Y, T = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], 1, 1)
    assert Y.shape == (0, 6, 5, 5)
    dX, dUk, dVp = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], T_saved=T, stride=1, pad=1)
    torch.cuda.synchronize()
    assert float(dUk.abs().max()) == 0.0 and float(dVp.abs().max()) == 0.0


def test_deterministic():
    _, out1 = _run((5, 64, 8, 8, 64, 16, 3, 1, 1), "bf16", seed=3)
    _, out2 = _run((5, 64, 8, 8, 64, 16, 3, 1, 1), "bf16", seed=3)
    for u, v in zip(out1, out2):
        assert torch.equal(u, v)


def test_dense_comparator_matches_oracle():
    import paper_2103_03936_amd as pf
    shape = (2, 12, 6, 6, 10, 4, 3, 1, 1)
    N, C, H, W, Cout, r, k, s, p = shape
    a = workloads.conv_inputs(*shape, dtype="f32", seed=6)
    Wd = np.einsum("oq,qcij->ocij", a["Vp"].astype(np.float64), a["Uk"].astype(np.float64)).astype(np.float32)
    g = {k_: to_gpu(v) for k_, v in a.items()}
    Y = pf.pf_dense_conv_fwd(g["X"], to_gpu(Wd), s, p)
    assert_close(Y, oracle.dense_conv_fwd(a["X"], Wd, s, p), "f32", "dense conv Y")
    dX, dW = pf.pf_dense_conv_bwd(g["X"], to_gpu(Wd), g["dY"], s, p)
    tX = torch.tensor(a["X"], dtype=torch.float64, requires_grad=True)
    tW = torch.tensor(Wd, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.conv2d(tX, tW, stride=s, padding=p).backward(torch.tensor(a["dY"], dtype=torch.float64))
    assert_close(dX, tX.grad.numpy(), "f32", "dense conv dX")
    assert_close(dW, tW.grad.numpy(), "f32", "dense conv dW")


def test_resnet18_conv4_full_size():
    # CIFAR ResNet-18 conv4_x, batch 128 (Appendix D): the benchmark workload, in the
    # configuration bench.py times
    c = workloads.CONFIGS["resnet18_conv4_bf16"]
    _run((c["N"], c["C"], c["H"], c["W"], c["Cout"], c["r"], c["k"], c["stride"], c["pad"]), c["dtype"], seed=c["seed"],
         saved_W=True)


@pytest.mark.parametrize("layer", ["conv1", "conv2", "conv3"])
def test_resnet50_conv5_full_size(layer):
    # ResNet-50 conv5_x bottleneck (Appendix D) at its full batch of 256, the launch plan bench.py times
    # (the image groups of the filter-gradient kernel depend on the batch): every tensor against the oracle
    c = workloads.CONFIGS["resnet50_conv5_bf16"]
    Cin, Cout, r, k, p = c["layers"][layer]
    _run((c["N"], Cin, c["H"], c["W"], Cout, r, k, 1, p), c["dtype"], seed=c["seed"], saved_W=True)


@pytest.mark.parametrize("layer", ["conv1", "conv2", "conv3"])
def test_resnet50_conv5_small_batch(layer):
    # the same layers at batch 16: fewer, differently sized image groups, T recomputed by the backward call
    c = workloads.CONFIGS["resnet50_conv5_bf16"]
    Cin, Cout, r, k, p = c["layers"][layer]
    _run((16, Cin, c["H"], c["W"], Cout, r, k, 1, p), c["dtype"], seed=c["seed"] + 1, saved_T=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_geometries(dtype):
    """Sixteen seeded random geometries (generic path, and the fused path where a drawn shape qualifies)."""
    rng = np.random.default_rng(3936)
    for case in range(16):
        k = int(rng.choice([1, 3, 5]))
        s = int(rng.choice([1, 2]))
        p = int(rng.integers(0, k // 2 + 1))
        N, C, Cout, r = int(rng.integers(1, 6)), int(rng.integers(1, 40)), int(rng.integers(1, 48)), int(rng.integers(1, 20))
        H, W = int(rng.integers(k, 13)), int(rng.integers(k, 13))
        _run((N, C, H, W, Cout, r, k, s, p), dtype, saved_T=bool(rng.integers(0, 2)), seed=300 + case,
             saved_W=bool(rng.integers(0, 2)))
    # channel counts the fused kernels take (multiples of 64, rank 64 or 128, small images)
    for case in range(4):
        C, Cout = 64 * int(rng.integers(1, 4)), 64 * int(rng.integers(1, 4))
        r, k = int(rng.choice([64, 128])), int(rng.choice([1, 3]))
        H = int(rng.choice([7, 8]))
        _run((int(rng.integers(1, 9)), C, H, H, Cout, r, k, 1, k // 2), dtype, seed=400 + case, saved_W=True)
