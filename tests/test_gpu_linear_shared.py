"""GPU parity of pf_lowrank_linear_shared_fwd/bwd (projections that share their input, e.g. Q, K, V) against the
CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

SHAPES = [
    # M, in, out, r, groups
    (1, 1, 1, 1, 1),
    (7, 5, 4, 3, 3),
    (70, 33, 31, 9, 2),
    (100, 130, 260, 129, 3),  # fp32: the streaming kernels, layer by layer
    (100, 512, 512, 128, 3),  # bf16: all three projections in one launch per direction, ragged last row tile
    (257, 256, 768, 128, 2),  # output wider than the input: separate outputs forward, one summed output backward
    (64, 1024, 256, 128, 4),  # input wider than 512: the backward pass sums layer by layer
    (33, 512, 256, 128, 8),
]


def _run(M, n_in, n_out, r, G, dtype, bias=True, saved_T=True, seed=0):
    import paper_2103_03936_amd as pf
    a = workloads.linear_shared_inputs(M, n_in, n_out, r, G, dtype=dtype, seed=seed, bias=bias)
    Yo, To = oracle.lowrank_linear_shared_fwd(a["X"], a["V"], a["U"], a["bias"])
    dXo, dUo, dVo, dbo = oracle.lowrank_linear_shared_bwd(a["X"], a["V"], a["U"], a["dY"])
    g = {k: to_gpu(v, dtype) for k, v in a.items()}
    Y, T = pf.pf_lowrank_linear_shared_fwd(g["X"], g["V"], g["U"], g["bias"], save_T=True)
    dX, dU, dV, db = pf.pf_lowrank_linear_shared_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T if saved_T else None,
                                                     has_bias=bias)
    torch.cuda.synchronize()
    tag = f"shared[{M},{n_in},{n_out},{r},G{G},{dtype}]"
    assert_close(Y, Yo, dtype, tag + " Y")
    assert_close(T, To, dtype, tag + " T")
    assert_close(dX, dXo, dtype, tag + " dX")
    assert_close(dU, dUo, dtype, tag + " dU")
    assert_close(dV, dVo, dtype, tag + " dV")
    if bias:
        assert_close(db, dbo, dtype, tag + " db")
    return g, (Y, T, dX, dU, dV, db)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_parity(shape, dtype):
    _run(*shape, dtype=dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_parity_recomputed_T_no_bias(dtype):
    _run(100, 512, 512, 128, 3, dtype=dtype, bias=False, saved_T=False, seed=5)


def test_equals_separate_layers_bit_for_bit_forward():
    """One launch for the three projections computes exactly what three single-layer calls compute."""
    import paper_2103_03936_amd as pf
    a = workloads.linear_shared_inputs(150, 512, 512, 128, 3, dtype="bf16", seed=2, bias=True)
    g = {k: to_gpu(v, "bf16") for k, v in a.items()}
    Y, T = pf.pf_lowrank_linear_shared_fwd(g["X"], g["V"], g["U"], g["bias"])
    for i in range(3):
        Yi, Ti = pf.pf_lowrank_linear_fwd(g["X"], g["V"][i].contiguous(), g["U"][i].contiguous(), g["bias"][i].contiguous())
        assert torch.equal(Y[i], Yi) and torch.equal(T[i], Ti)


def test_accumulate_and_empty_batch():
    import paper_2103_03936_amd as pf
    a = workloads.linear_shared_inputs(100, 512, 512, 128, 3, dtype="bf16", seed=4, bias=True)
    g = {k: to_gpu(v, "bf16") for k, v in a.items()}
    _, dU, dV, db = pf.pf_lowrank_linear_shared_bwd(g["X"], g["V"], g["U"], g["dY"], has_bias=True)
    grads = (dU.clone(), dV.clone(), db.clone())
    pf.pf_lowrank_linear_shared_bwd(g["X"], g["V"], g["U"], g["dY"], has_bias=True, grads=grads)
    torch.cuda.synchronize()
    _, dUo, dVo, dbo = oracle.lowrank_linear_shared_bwd(a["X"], a["V"], a["U"], a["dY"])
    assert_close(grads[0], 2 * dUo, "bf16", "accumulated dU")
    assert_close(grads[1], 2 * dVo, "bf16", "accumulated dV")
    assert_close(grads[2], 2 * dbo, "bf16", "accumulated db")
    e = workloads.linear_shared_inputs(0, 8, 6, 2, 2, dtype="f32", seed=1, bias=True)
    ge = {k: to_gpu(v) for k, v in e.items()}
    Y, T = pf.pf_lowrank_linear_shared_fwd(ge["X"], ge["V"], ge["U"], ge["bias"])
    dX, dU, dV, db = pf.pf_lowrank_linear_shared_bwd(ge["X"], ge["V"], ge["U"], ge["dY"], T_saved=T, has_bias=True)
    torch.cuda.synchronize()
    assert Y.shape == (2, 0, 6) and dX.shape == (0, 8)
    assert float(dU.abs().max()) == 0.0 and float(dV.abs().max()) == 0.0 and float(db.abs().max()) == 0.0


def test_transformer_qkv_full_size():
    """The query, key and value projections of the Transformer configuration (Appendix D: 512 -> 128 -> 512,
    8192 tokens), as bench.py times them; every output is compared."""
    c = workloads.CONFIGS["transformer_block_bf16"]
    n_in, n_out, r = c["layers"]["wq"]
    _run(c["M"], n_in, n_out, r, 3, dtype=c["dtype"], seed=c["seed"])
