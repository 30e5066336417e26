"""GPU parity of pf_lowrank_linear_fwd/bwd (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

SHAPES = [
    # M, in, out, r
    (1, 1, 1, 1),
    (3, 5, 4, 2),
    (64, 64, 64, 32),
    (150, 200, 130, 40),
    (257, 96, 192, 64),
    (64, 512, 512, 128),   # VGG-19 fc17/fc18
    (70, 33, 31, 33),      # rank above min(in, out)
    (100, 130, 260, 129),  # fp32: four row blocks on the streaming kernels, every extent ragged
    (150, 256, 512, 64),   # fused-kernel shapes with a ragged last row tile
    (257, 512, 256, 128),
    (1000, 256, 256, 128),
    (100, 768, 1024, 128),  # fused kernel: four output-block pairs per wavefront forward, three backward
    (65, 1280, 1280, 128),  # fused kernel: ten chunks of the contraction, five pairs (the loop for any count), ragged rows
]


def _run(M, n_in, n_out, r, dtype, bias, saved_T, seed=0):
    import paper_2103_03936_amd as pf
    a = workloads.linear_inputs(M, n_in, n_out, r, dtype=dtype, seed=seed, bias=bias)
    Yo, To = oracle.lowrank_linear_fwd(a["X"], a["V"], a["U"], a["bias"])
    dXo, dUo, dVo, dbo = oracle.lowrank_linear_bwd(a["X"], a["V"], a["U"], a["dY"])
    g = {k: to_gpu(v, dtype) for k, v in a.items()}
    Y, T = pf.pf_lowrank_linear_fwd(g["X"], g["V"], g["U"], g["bias"], save_T=True)
    dX, dU, dV, db = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T if saved_T else None,
                                              has_bias=bias)
    torch.cuda.synchronize()
    tag = f"linear[{M},{n_in},{n_out},{r},{dtype}]"
    assert_close(Y, Yo, dtype, tag + " Y")
    assert_close(T, To, dtype, tag + " T")
    assert_close(dX, dXo, dtype, tag + " dX")
    assert_close(dU, dUo, dtype, tag + " dU")
    assert_close(dV, dVo, dtype, tag + " dV")
    if bias:
        assert_close(db, dbo, dtype, tag + " db")
    assert dU.dtype == torch.float32 and dV.dtype == torch.float32
    return g, (Y, T, dX, dU, dV, db)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_parity(shape, dtype):
    _run(*shape, dtype=dtype, bias=True, saved_T=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_parity_recomputed_T_no_bias(dtype):
    _run(150, 200, 130, 40, dtype=dtype, bias=False, saved_T=False, seed=5)


def test_no_T_save_and_accumulate():
    import paper_2103_03936_amd as pf
    a = workloads.linear_inputs(90, 70, 50, 20, dtype="f32", seed=9, bias=True)
    g = {k: to_gpu(v) for k, v in a.items()}
    Y, T = pf.pf_lowrank_linear_fwd(g["X"], g["V"], g["U"], g["bias"], save_T=False)
    assert T is None
    Yo, _ = oracle.lowrank_linear_fwd(a["X"], a["V"], a["U"], a["bias"])
    assert_close(Y, Yo, "f32", "Y without T_save")
    dX, dU, dV, db = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], has_bias=True)
    grads = (dU.clone(), dV.clone(), db.clone())
    pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], has_bias=True, grads=grads)
    _, dUo, dVo, dbo = oracle.lowrank_linear_bwd(a["X"], a["V"], a["U"], a["dY"])
    assert_close(grads[0], 2 * dUo, "f32", "accumulated dU")
    assert_close(grads[1], 2 * dVo, "f32", "accumulated dV")
    assert_close(grads[2], 2 * dbo, "f32", "accumulated db")
    # skipping dX leaves the other gradients unchanged
    dX2, dU2, dV2, _ = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], need_dX=False, has_bias=True)
    assert dX2 is None and torch.equal(dU2, dU) and torch.equal(dV2, dV)


def test_empty_batch():
    import paper_2103_03936_amd as pf
    a = workloads.linear_inputs(0, 16, 8, 4, dtype="f32", seed=1)
    g = {k: to_gpu(v) for k, v in a.items()}
    Y, T = pf.pf_lowrank_linear_fwd(g["X"], g["V"], g["U"])
    assert Y.shape == (0, 8)
    dX, dU, dV, _ = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T)
    torch.cuda.synchronize()
    assert float(dU.abs().max()) == 0.0 and float(dV.abs().max()) == 0.0


def test_deterministic():
    g, out1 = _run(257, 96, 192, 64, "bf16", True, True, seed=3)
    _, out2 = _run(257, 96, 192, 64, "bf16", True, True, seed=3)
    for u, v in zip(out1, out2):
        assert torch.equal(u, v)


def test_dense_comparator_matches_oracle():
    import paper_2103_03936_amd as pf
    a = workloads.linear_inputs(100, 72, 40, 8, dtype="f32", seed=2, bias=True)
    W = (a["U"].astype(np.float64) @ a["V"].astype(np.float64).T).astype(np.float32)
    g = {k: to_gpu(v) for k, v in a.items()}
    Y = pf.pf_dense_linear_fwd(g["X"], to_gpu(W), g["bias"])
    assert_close(Y, oracle.dense_linear_fwd(a["X"], W, a["bias"]), "f32", "dense Y")
    dX, dW, db = pf.pf_dense_linear_bwd(g["X"], to_gpu(W), g["dY"], has_bias=True)
    X64, dY64 = a["X"].astype(np.float64), a["dY"].astype(np.float64)
    assert_close(dX, dY64 @ W.astype(np.float64), "f32", "dense dX")
    assert_close(dW, dY64.T @ X64, "f32", "dense dW")
    assert_close(db, dY64.sum(0), "f32", "dense db")


@pytest.mark.parametrize("layer", ["wq", "ffn1", "ffn2"])
def test_transformer_block_full_size(layer):
    # one low-rank Transformer encoder layer at M = 64 x 128 tokens (Section 2.4, Appendix D)
    cfg = workloads.CONFIGS["transformer_block_bf16"]
    n_in, n_out, r = cfg["layers"][layer]
    _run(cfg["M"], n_in, n_out, r, "bf16", True, True, seed=cfg["seed"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_geometries(dtype):
    """Sixteen seeded random geometries, with and without bias and saved T (few-row, generic and fused paths)."""
    rng = np.random.default_rng(2103)
    for case in range(16):
        M = int(rng.choice([1, 7, 33, 129, 300]))
        n_in, n_out, r = int(rng.integers(1, 200)), int(rng.integers(1, 200)), int(rng.integers(1, 64))
        if case >= 12:  # shapes of the fused bf16 kernel
            n_in, n_out, r = 256 * int(rng.integers(1, 4)), 256 * int(rng.integers(1, 4)), 128
        _run(M, n_in, n_out, r, dtype, bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), seed=500 + case)
