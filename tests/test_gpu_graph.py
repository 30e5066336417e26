"""The hot path under HIP graph replay (how bench.py times it): a graph that holds forward + backward of a layer is
replayed several times with new inputs copied into its buffers and the library's own eager calls in between, and
every replay must reproduce the eager result bit for bit (the kernels are deterministic)."""
import pytest
import torch

import workloads
from parity import to_gpu

pytestmark = pytest.mark.gpu


def _replay_matches_eager(make_inputs, run, names):
    torch.cuda.synchronize()
    static = {k: v.clone() for k, v in make_inputs(0).items() if v is not None}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream, as torch asks for
        run(static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        outs = run(static)
    for rep in range(1, 4):
        fresh = make_inputs(rep)
        eager = run({k: v for k, v in fresh.items()})  # eager work of the same library between the replays
        torch.cuda.synchronize()
        for k in static:
            static[k].copy_(fresh[k])
        g.replay()
        torch.cuda.synchronize()
        for name, o, e in zip(names, outs, eager):
            assert torch.equal(o, e), f"replay {rep}: {name} differs from the eager result"


def test_conv_layer_graph_replay():
    import paper_2103_03936_amd as pf
    c = workloads.CONFIGS["resnet18_conv4_bf16"]

    def make(seed):
        a = workloads.conv_inputs(16, c["C"], c["H"], c["W"], c["Cout"], c["r"], c["k"], 1, 1, dtype="bf16", seed=seed)
        return {k: to_gpu(v, "bf16") for k, v in a.items()}

    def run(g):
        Y, T, Wsv = pf.pf_lowrank_conv_fwd(g["X"], g["Uk"], g["Vp"], 1, 1, save_T=True, save_W=True)
        dX, dUk, dVp = pf.pf_lowrank_conv_bwd(g["X"], g["Uk"], g["Vp"], g["dY"], T_saved=T, stride=1, pad=1, W_saved=Wsv)
        return Y, T, dX, dUk, dVp

    _replay_matches_eager(make, run, ("Y", "T", "dX", "dUk", "dVp"))


def test_linear_layers_graph_replay():
    import paper_2103_03936_amd as pf

    def make(seed):
        a = workloads.linear_shared_inputs(300, 512, 512, 128, 3, dtype="bf16", seed=seed, bias=True)
        return {k: to_gpu(v, "bf16") for k, v in a.items()}

    def run(g):
        Y, T = pf.pf_lowrank_linear_shared_fwd(g["X"], g["V"], g["U"], g["bias"])
        dX, dU, dV, db = pf.pf_lowrank_linear_shared_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T, has_bias=True)
        Y0, T0 = pf.pf_lowrank_linear_fwd(g["X"], g["V"][0], g["U"][0], g["bias"][0])
        dX0, dU0, dV0, db0 = pf.pf_lowrank_linear_bwd(g["X"], g["V"][0], g["U"][0], g["dY"][0], T_saved=T0, has_bias=True)
        return Y, T, dX, dU, dV, db, Y0, dX0, dU0, dV0, db0

    _replay_matches_eager(make, run, ("Y", "T", "dX", "dU", "dV", "db", "Y0", "dX0", "dU0", "dV0", "db0"))


def test_lstm_cell_graph_replay():
    import paper_2103_03936_amd as pf

    def make(seed):
        a = workloads.lstm_cell_inputs(20, 200, 160, 40, groups=1, seed=seed)
        return {k: to_gpu(v) for k, v in a.items()}

    def run(g):
        h, c, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(g["x"], g["h_prev"], g["c_prev"], g["Vx"], g["Ux"], g["Vh"],
                                                           g["Uh"], g["bias"])
        dx, dhp, dcp, gr = pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], c, gates, Tx, Th, g["Vx"],
                                                       g["Ux"], g["Vh"], g["Uh"], g["dh"], g["dc"])
        return h, c, dx, dhp, dcp, gr["dVx"], gr["dUx"], gr["dVh"], gr["dUh"], gr["dbias"]

    _replay_matches_eager(make, run, ("h", "c", "dx", "dh_prev", "dc_prev", "dVx", "dUx", "dVh", "dUh", "dbias"))


@pytest.mark.parametrize("T", [5, 9])
@pytest.mark.parametrize("groups", [1, 4])
def test_lstm_stack_graph_replay(groups, T):
    """Two stacked layers over a short sequence (groups = 1: the fused pre-activation + gate kernel and the packed
    factors; groups = 4: the unfused launches), forward and backward in one graph.  T = 9 gives 180 rows, from
    where the weight gradients are summed on the matrix unit."""
    import paper_2103_03936_amd as pf
    B, d, h, r, L = 20, 72, 80, 20, 2

    def make(seed):
        s = workloads.Stream(workloads.SEED_BASE + 700 + seed, "f32")
        out = {"x": to_gpu(s.normal((T, B, d))), "dh_top": to_gpu(s.normal((T, B, h)))}
        for l in range(L):
            a = workloads.lstm_cell_inputs(B, d if l == 0 else h, h, r, groups=groups, seed=10 * seed + l)
            for k in ("h_prev", "c_prev", "Vx", "Ux", "Vh", "Uh", "bias"):
                out[f"{k}{l}"] = to_gpu(a[k])
        return out

    def run(g):
        col = lambda k: [g[f"{k}{l}"] for l in range(L)]
        saved = pf.pf_lowrank_lstm_stack_fwd(g["x"], col("h_prev"), col("c_prev"), col("Vx"), col("Ux"), col("Vh"),
                                             col("Uh"), col("bias"), groups)
        dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], col("h_prev"), col("c_prev"), *saved, col("Vx"),
                                                        col("Ux"), col("Vh"), col("Uh"), g["dh_top"], None, None, groups)
        return (saved[0][L - 1], saved[1][0], dx, dh0[0], dc0[1], gr[0]["dVx"], gr[0]["dUh"], gr[1]["dUx"], gr[1]["dVh"],
                gr[1]["dbias"])

    _replay_matches_eager(make, run, ("h_top", "c_0", "dx", "dh0_0", "dc0_1", "dVx_0", "dUh_0", "dUx_1", "dVh_1", "dbias_1"))
