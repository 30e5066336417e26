"""Parameter gradients written straight into one flat buffer (the paper's single all-reduce payload, Section 4
"implementation details"): every backward entry point gets slices of one float32 buffer with no padding between
them, so most slices start at addresses that are only 4-byte aligned; two micro-batches are accumulated.  The
buffer must equal the oracle's gradients laid out the same way, and the guard words around it must survive."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import TOL, to_gpu

pytestmark = pytest.mark.gpu

GUARD = 12345.0


def _oracle_layers(dtype, seed):
    """Oracle gradients of one micro-batch for three layers; returns (inputs, ordered (name, array) list)."""
    lin = workloads.linear_inputs(70, 33, 30, 9, dtype=dtype, seed=seed, bias=True)
    lin2 = workloads.linear_inputs(100, 256, 512, 128, dtype=dtype, seed=seed + 4, bias=True)  # fused / streaming kernels
    conv = workloads.conv_inputs(3, 5, 6, 7, 7, 3, 3, stride=1, pad=1, dtype=dtype, seed=seed + 1)
    big = workloads.conv_inputs(4, 256, 8, 8, 256, 64, 3, stride=1, pad=1, dtype=dtype, seed=seed + 2)
    lstm = workloads.lstm_cell_inputs(5, 13, 11, 7, groups=1, dtype="f32", seed=seed + 3)
    out = []
    for tag, l in (("lin", lin), ("lin2", lin2)):
        _, dU, dV, db = oracle.lowrank_linear_bwd(l["X"], l["V"], l["U"], l["dY"])
        out += [(tag + ".dU", dU), (tag + ".dV", dV), (tag + ".db", db)]
    for tag, c in (("conv", conv), ("big", big)):
        _, dUk, dVp = oracle.lowrank_conv_bwd(c["X"], c["Uk"], c["Vp"], c["dY"], stride=1, pad=1)
        out += [(tag + ".dUk", dUk), (tag + ".dVp", dVp)]
    _, c, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(lstm["x"], lstm["h_prev"], lstm["c_prev"], lstm["Vx"],
                                                       lstm["Ux"], lstm["Vh"], lstm["Uh"], lstm["bias"])
    f = dict(c=c, gates=gates, Tx=Tx, Th=Th)
    b = oracle.lowrank_lstm_cell_bwd(lstm["x"], lstm["h_prev"], lstm["c_prev"], c, gates, Tx, Th, lstm["Vx"],
                                     lstm["Ux"], lstm["Vh"], lstm["Uh"], lstm["dh"], lstm["dc"])[3]
    out += [("lstm." + k, b[k]) for k in ("dVx", "dUx", "dVh", "dUh", "dbias")]
    return dict(lin=lin, lin2=lin2, conv=conv, big=big, lstm=lstm, lstm_fwd=f), out


def _gpu_layers(pf, inp, dtype, views):
    lstm = inp["lstm"]
    for tag in ("lin", "lin2"):
        g = {k: to_gpu(v, dtype) for k, v in inp[tag].items()}
        pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], has_bias=True,
                                 grads=(views[tag + ".dU"], views[tag + ".dV"], views[tag + ".db"]))
    for tag in ("conv", "big"):
        g = {k: to_gpu(v, dtype) for k, v in inp[tag].items() if isinstance(v, np.ndarray)}
        pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], stride=1, pad=1,
                               grads=(views[tag + ".dUk"], views[tag + ".dVp"]))
    g = {k: to_gpu(v) for k, v in lstm.items() if isinstance(v, np.ndarray)}
    f = {k: to_gpu(np.asarray(v, dtype=np.float32)) for k, v in inp["lstm_fwd"].items()}
    pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], f["c"], f["gates"], f["Tx"], f["Th"], g["Vx"],
                                g["Ux"], g["Vh"], g["Uh"], g["dh"], g["dc"],
                                grads={k: views["lstm." + k] for k in ("dVx", "dUx", "dVh", "dUh", "dbias")})


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_flat_gradient_buffer_two_micro_batches(dtype):
    import paper_2103_03936_amd as pf
    inp0, ref0 = _oracle_layers(dtype, 0)
    inp1, ref1 = _oracle_layers(dtype, 10)
    entries = [("guard0", (1,))] + [(n, a.shape) for n, a in ref0] + [("guard1", (3,))]
    buf = pf.GradBuffer(entries).zero()
    buf.views["guard0"].fill_(GUARD)
    buf.views["guard1"].fill_(GUARD)
    assert any((o * 4) % 16 for o, _ in buf.offsets.values())  # slices that are not 16-byte aligned exist
    _gpu_layers(pf, inp0, dtype, buf.views)
    _gpu_layers(pf, inp1, dtype, buf.views)
    torch.cuda.synchronize()
    got = buf.flat.cpu().numpy().astype(np.float64)
    assert (got[:1] == GUARD).all() and (got[-3:] == GUARD).all()
    for (name, a0), (_, a1) in zip(ref0, ref1):
        o, sh = buf.offsets[name]
        ref = np.asarray(a0, dtype=np.float64) + np.asarray(a1, dtype=np.float64)
        seg = got[o:o + ref.size].reshape(sh)
        tol = TOL["f32" if name.startswith("lstm.") else dtype]
        err = np.abs(seg - ref).max() / np.abs(ref).max()
        assert err <= tol, f"{name}: rel err {err:.3e} > {tol:.1e}"
