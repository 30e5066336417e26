"""GPU parity of pf_lowrank_lstm_cell_fwd/bwd (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

CELLS = [
    # B, d, h, r
    (1, 1, 1, 1),
    (3, 5, 4, 2),
    (20, 70, 50, 13),
    (32, 37, 29, 7),    # small-batch path: every extent ragged
    (7, 130, 260, 129),  # several column tiles and contraction slices, all with tails
    (33, 96, 128, 32),
    (20, 1500, 1500, 375),  # the language model's layer shape (Appendix D)
]


def _cell(B, d, h, r, groups, seed=0, bias=True):
    import paper_2103_03936_amd as pf
    a = workloads.lstm_cell_inputs(B, d, h, r, groups=groups, seed=seed, bias=bias)
    ho, co, gates_o, Txo, Tho = oracle.lowrank_lstm_cell_fwd(a["x"], a["h_prev"], a["c_prev"], a["Vx"], a["Ux"],
                                                             a["Vh"], a["Uh"], a["bias"], groups)
    dxo, dhpo, dcpo, go = oracle.lowrank_lstm_cell_bwd(a["x"], a["h_prev"], a["c_prev"], co, gates_o, Txo, Tho,
                                                       a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["dh"], a["dc"], groups)
    g = {k: to_gpu(v) for k, v in a.items()}
    h_out, c_out, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(g["x"], g["h_prev"], g["c_prev"], g["Vx"], g["Ux"],
                                                              g["Vh"], g["Uh"], g["bias"], groups)
    dx, dhp, dcp, gr = pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], c_out, gates, Tx, Th, g["Vx"],
                                                   g["Ux"], g["Vh"], g["Uh"], g["dh"], g["dc"], groups)
    torch.cuda.synchronize()
    tag = f"lstm[{B},{d},{h},{r},g{groups}]"
    assert_close(h_out, ho, "f32", tag + " h")
    assert_close(c_out, co, "f32", tag + " c")
    assert_close(gates, gates_o, "f32", tag + " gates")
    assert_close(Tx, Txo, "f32", tag + " Tx")
    assert_close(Th, Tho, "f32", tag + " Th")
    assert_close(dx, dxo, "f32", tag + " dx")
    assert_close(dhp, dhpo, "f32", tag + " dh_prev")
    assert_close(dcp, dcpo, "f32", tag + " dc_prev")
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert_close(gr[k], go[k], "f32", tag + " " + k)
    return a, g, (h_out, c_out, gates, Tx, Th), gr


@pytest.mark.parametrize("groups", [1, 4])
@pytest.mark.parametrize("shape", CELLS)
def test_cell_parity(shape, groups):
    _cell(*shape, groups=groups)


def test_cell_no_bias_no_dc_and_accumulate():
    import paper_2103_03936_amd as pf
    B, d, h, r, groups = 7, 19, 23, 5, 4
    a = workloads.lstm_cell_inputs(B, d, h, r, groups=groups, seed=11, bias=False)
    ho, co, gates_o, Txo, Tho = oracle.lowrank_lstm_cell_fwd(a["x"], a["h_prev"], a["c_prev"], a["Vx"], a["Ux"],
                                                             a["Vh"], a["Uh"], None, groups)
    _, _, _, go = oracle.lowrank_lstm_cell_bwd(a["x"], a["h_prev"], a["c_prev"], co, gates_o, Txo, Tho, a["Vx"],
                                               a["Ux"], a["Vh"], a["Uh"], a["dh"], None, groups)
    g = {k: to_gpu(v) for k, v in a.items()}
    h_out, c_out, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(g["x"], g["h_prev"], g["c_prev"], g["Vx"], g["Ux"],
                                                              g["Vh"], g["Uh"], None, groups)
    assert_close(h_out, ho, "f32", "h without bias")
    _, _, _, gr = pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], c_out, gates, Tx, Th, g["Vx"],
                                              g["Ux"], g["Vh"], g["Uh"], g["dh"], None, groups)
    _, _, _, gr = pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], c_out, gates, Tx, Th, g["Vx"],
                                              g["Ux"], g["Vh"], g["Uh"], g["dh"], None, groups, grads=gr)
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert_close(gr[k], 2 * go[k], "f32", "accumulated " + k)


def lm_oracle(inp, groups):
    """Forward and BPTT of the stacked LSTM on the CPU oracle; returns top-layer h and all gradients."""
    T, B = inp["tokens"].shape
    L = len(inp["layers"])
    h_dim = inp["layers"][0]["Uh"].shape[0] // 4
    xs = [inp["E"][inp["tokens"][t]].astype(np.float64) for t in range(T)]
    hs = [np.zeros((B, h_dim)) for _ in range(L)]
    cs = [np.zeros((B, h_dim)) for _ in range(L)]
    saved = [[None] * T for _ in range(L)]
    top = []
    for t in range(T):
        x = xs[t]
        for l, p in enumerate(inp["layers"]):
            ho, co, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(x, hs[l], cs[l], p["Vx"], p["Ux"], p["Vh"], p["Uh"],
                                                                 p["bias"], groups)
            saved[l][t] = (x, hs[l], cs[l], co, gates, Tx, Th)
            hs[l], cs[l] = ho, co
            x = ho
        top.append(x)
    grads = [None] * L
    dE_rows = [None] * T
    dh_next = [np.zeros((B, h_dim)) for _ in range(L)]
    dc_next = [np.zeros((B, h_dim)) for _ in range(L)]
    for t in reversed(range(T)):
        d_from_above = inp["dH_top"][t].astype(np.float64)
        for l in reversed(range(L)):
            p = inp["layers"][l]
            x, hp, cp, co, gates, Tx, Th = saved[l][t]
            dx, dhp, dcp, grads[l] = oracle.lowrank_lstm_cell_bwd(x, hp, cp, co, gates, Tx, Th, p["Vx"], p["Ux"],
                                                                  p["Vh"], p["Uh"], d_from_above + dh_next[l],
                                                                  dc_next[l], groups, grads=grads[l])
            dh_next[l], dc_next[l] = dhp, dcp
            d_from_above = dx
        dE_rows[t] = d_from_above
    return np.stack(top), grads, np.stack(dE_rows)


def lm_gpu(inp, groups):
    """The same sequence through the C ABI, one cell call per (step, layer)."""
    import paper_2103_03936_amd as pf
    T, B = inp["tokens"].shape
    L = len(inp["layers"])
    h_dim = inp["layers"][0]["Uh"].shape[0] // 4
    E = to_gpu(inp["E"])
    tok = torch.from_numpy(inp["tokens"]).cuda()
    P = [{k: to_gpu(v) for k, v in p.items()} for p in inp["layers"]]
    dH = to_gpu(inp["dH_top"])
    zeros = torch.zeros((B, h_dim), device="cuda")
    hs, cs = [zeros] * L, [zeros] * L
    saved = [[None] * T for _ in range(L)]
    top = []
    for t in range(T):
        x = E[tok[t]].contiguous()  # embedding lookup: a gather, not part of the factorized path
        for l, p in enumerate(P):
            ho, co, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(x, hs[l], cs[l], p["Vx"], p["Ux"], p["Vh"], p["Uh"],
                                                                p["bias"], groups)
            saved[l][t] = (x, hs[l], cs[l], co, gates, Tx, Th)
            hs[l], cs[l] = ho, co
            x = ho
        top.append(x)
    grads = [None] * L
    dE_rows = [None] * T
    dh_next, dc_next = [zeros] * L, [zeros] * L
    for t in reversed(range(T)):
        d_from_above = dH[t]
        for l in reversed(range(L)):
            p = P[l]
            x, hp, cp, co, gates, Tx, Th = saved[l][t]
            dh_total = (d_from_above + dh_next[l]).contiguous()  # gradient fan-in, outside the cell
            dx, dhp, dcp, grads[l] = pf.pf_lowrank_lstm_cell_bwd(x, hp, cp, co, gates, Tx, Th, p["Vx"], p["Ux"],
                                                                 p["Vh"], p["Uh"], dh_total, dc_next[l], groups,
                                                                 grads=grads[l])
            dh_next[l], dc_next[l] = dhp, dcp
            d_from_above = dx
        dE_rows[t] = d_from_above
    torch.cuda.synchronize()
    return torch.stack(top), grads, torch.stack(dE_rows)


@pytest.mark.parametrize("groups", [1, 4])
def test_stacked_sequence_small(groups):
    inp = workloads.lstm_lm_inputs(vocab=50, d=40, h=40, r=10, layers=2, T=6, B=5, groups=groups, seed=21, scale=0.3)
    top_o, grads_o, dE_o = lm_oracle(inp, groups)
    top, grads, dE = lm_gpu(inp, groups)
    assert_close(top, top_o, "f32", "top h")
    assert_close(dE, dE_o, "f32", "d embedding rows")
    for l in range(2):
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(grads[l][k], grads_o[l][k], "f32", f"layer {l} {k}")


def test_language_model_full_size():
    # the 2-layer LSTM language model of Appendix D: d = h = 1500, r = 375, sequence 35, batch 20;
    # one shared rank-375 pair per path (groups = 1), forward and back-propagation through time
    c = workloads.CONFIGS["lstm_lm_f32"]
    inp = workloads.lstm_lm_inputs(c["vocab"], c["d"], c["h"], c["r"], c["layers"], c["T"], c["B"], groups=1,
                                   seed=c["seed"])
    top_o, grads_o, dE_o = lm_oracle(inp, 1)
    top, grads, dE = lm_gpu(inp, 1)
    assert_close(top, top_o, "f32", "top h")
    assert_close(dE, dE_o, "f32", "d embedding rows")
    for l in range(2):
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(grads[l][k], grads_o[l][k], "f32", f"layer {l} {k}")


def test_empty_batch():
    """B = 0: nothing to compute forward; backward zeroes the parameter gradients it owns."""
    import paper_2103_03936_amd as pf
    a = workloads.lstm_cell_inputs(0, 6, 5, 3, groups=1, seed=2)
    g = {k: to_gpu(v) for k, v in a.items()}
    h_out, c_out, gates, Tx, Th = pf.pf_lowrank_lstm_cell_fwd(g["x"], g["h_prev"], g["c_prev"], g["Vx"], g["Ux"],
                                                              g["Vh"], g["Uh"], g["bias"], 1)
    assert h_out.shape == (0, 5) and gates.shape == (0, 20)
    dx, dhp, dcp, gr = pf.pf_lowrank_lstm_cell_bwd(g["x"], g["h_prev"], g["c_prev"], c_out, gates, Tx, Th, g["Vx"],
                                                   g["Ux"], g["Vh"], g["Uh"], g["dh"], g["dc"], 1)
    torch.cuda.synchronize()
    assert dx.shape == (0, 6)
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert float(gr[k].abs().max()) == 0.0


SEQS = [
    # T, B, d, h, r
    (1, 3, 8, 8, 4),
    (6, 5, 40, 36, 10),
    (4, 20, 70, 50, 13),
    (3, 32, 37, 29, 7),
]


def _seq_inputs(T, B, d, h, r, groups, seed):
    rng_cell = workloads.lstm_cell_inputs(B, d, h, r, groups=groups, seed=seed)  # factors, bias, h0 / c0
    s = workloads.Stream(workloads.SEED_BASE + 500 + seed, "f32")
    return dict(x=s.normal((T, B, d)), h0=rng_cell["h_prev"], c0=rng_cell["c_prev"], Vx=rng_cell["Vx"],
                Ux=rng_cell["Ux"], Vh=rng_cell["Vh"], Uh=rng_cell["Uh"], bias=rng_cell["bias"],
                dh_all=s.normal((T, B, h)), dhT=s.normal((B, h)), dcT=s.normal((B, h)))


@pytest.mark.parametrize("groups", [1, 4])
@pytest.mark.parametrize("shape", SEQS)
def test_sequence_layer(shape, groups):
    """pf_lowrank_lstm_seq_fwd/bwd against the sequence oracle (cells chained over time, BPTT)."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r = shape
    a = _seq_inputs(T, B, d, h, r, groups, seed=7)
    ho, co, go, Txo, Tho = oracle.lowrank_lstm_seq_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"],
                                                       a["bias"], groups)
    dxo, dh0o, dc0o, gro = oracle.lowrank_lstm_seq_bwd(a["x"], a["h0"], a["c0"], ho, co, go, Txo, Tho, a["Vx"], a["Ux"],
                                                      a["Vh"], a["Uh"], a["dh_all"], a["dhT"], a["dcT"], groups)
    g = {k: to_gpu(v) for k, v in a.items()}
    h_all, c_all, gates_all, Tx_all, Th_all = pf.pf_lowrank_lstm_seq_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"],
                                                                         g["Vh"], g["Uh"], g["bias"], groups)
    tag = f"seq {shape} groups={groups}"
    for name, got, want in (("h", h_all, ho), ("c", c_all, co), ("gates", gates_all, go), ("Tx", Tx_all, Txo),
                            ("Th", Th_all, Tho)):
        assert_close(got, want, "f32", f"{tag} {name}")
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_seq_bwd(g["x"], g["h0"], g["c0"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                  g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["dh_all"], g["dhT"], g["dcT"],
                                                  groups)
    assert_close(dx, dxo, "f32", tag + " dx")
    assert_close(dh0, dh0o, "f32", tag + " dh0")
    assert_close(dc0, dc0o, "f32", tag + " dc0")
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert_close(gr[k], gro[k], "f32", f"{tag} {k}")
    # a second call accumulates onto the first; without dx, final-state gradients or bias
    dx2, _, _, gr2 = pf.pf_lowrank_lstm_seq_bwd(g["x"], g["h0"], g["c0"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["dh_all"], g["dhT"], g["dcT"],
                                                groups, need_dx=False, grads=gr)
    assert dx2 is None
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert_close(gr2[k], 2 * gro[k], "f32", f"{tag} accumulated {k}")


def test_sequence_layer_matches_cells_full_size():
    """Language-model layer shape (Appendix D), 35 steps: the sequence entry points against the cell entry
    points chained by hand (both on the GPU; the cells are checked against the oracle above)."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r = 35, 20, 1500, 1500, 375
    a = _seq_inputs(T, B, d, h, r, 1, seed=9)
    g = {k: to_gpu(v) for k, v in a.items()}
    h_all, c_all, gates_all, Tx_all, Th_all = pf.pf_lowrank_lstm_seq_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"],
                                                                         g["Vh"], g["Uh"], g["bias"], 1)
    hp, cp = g["h0"], g["c0"]
    saved = []
    for t in range(T):
        ht, ct, gt, Txt, Tht = pf.pf_lowrank_lstm_cell_fwd(g["x"][t], hp, cp, g["Vx"], g["Ux"], g["Vh"], g["Uh"],
                                                          g["bias"], 1)
        saved.append((hp, cp, ct, gt, Txt, Tht))
        hp, cp = ht, ct
        if t in (0, 17, 34):
            assert_close(h_all[t], ht.double().cpu().numpy(), "f32", f"h_{t}")
            assert_close(c_all[t], ct.double().cpu().numpy(), "f32", f"c_{t}")
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_seq_bwd(g["x"], g["h0"], g["c0"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                  g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["dh_all"], g["dhT"], g["dcT"], 1)
    dh, dc, grc = g["dh_all"][T - 1] + g["dhT"], g["dcT"], None
    for t in range(T - 1, -1, -1):
        hp, cp, ct, gt, Txt, Tht = saved[t]
        dxt, dhp, dc, grc = pf.pf_lowrank_lstm_cell_bwd(g["x"][t], hp, cp, ct, gt, Txt, Tht, g["Vx"], g["Ux"], g["Vh"],
                                                        g["Uh"], dh, dc, 1, grads=grc)
        if t in (0, 17, 34):
            assert_close(dx[t], dxt.double().cpu().numpy(), "f32", f"dx_{t}")
        dh = dhp + (g["dh_all"][t - 1] if t > 0 else 0)
    assert_close(dh0, dh.double().cpu().numpy(), "f32", "dh0")
    assert_close(dc0, dc.double().cpu().numpy(), "f32", "dc0")
    for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
        assert_close(gr[k], grc[k].double().cpu().numpy(), "f32", "full size " + k)


def _stack_inputs(T, B, d, h, r, groups, L, seed):
    s = workloads.Stream(workloads.SEED_BASE + 900 + seed, "f32")
    layers = [workloads.lstm_cell_inputs(B, d if l == 0 else h, h, r, groups=groups, seed=seed + 10 * l) for l in range(L)]
    col = lambda k: [p[k] for p in layers]
    return dict(x=s.normal((T, B, d)), h0=col("h_prev"), c0=col("c_prev"), Vx=col("Vx"), Ux=col("Ux"), Vh=col("Vh"),
                Uh=col("Uh"), bias=col("bias"), dh_top=s.normal((T, B, h)), dhT=[s.normal((B, h)) for _ in range(L)],
                dcT=[s.normal((B, h)) for _ in range(L)])


def _gpu_lists(a):
    return {k: [to_gpu(t) for t in v] if isinstance(v, list) else to_gpu(v) for k, v in a.items()}


STACKS = [
    # T, B, d, h, r, layers
    (1, 3, 8, 8, 4, 2),
    (5, 4, 12, 20, 6, 1),
    (6, 5, 40, 36, 10, 2),
    (2, 7, 24, 16, 5, 4),     # more layers than time steps: the diagonals never hold every layer
    (4, 20, 70, 50, 13, 3),
    (3, 32, 37, 29, 7, 2),
    (3, 6, 130, 260, 129, 2),  # several column tiles and contraction slices, all with tails
    (2, 4, 16, 24, 516, 2),    # a rank beyond what the fused pre-activation + gate kernel stages on chip
    (9, 20, 70, 150, 37, 2),   # 180 rows: weight gradients on the matrix unit, ragged last chunk and tiles
    (5, 32, 200, 130, 140, 2), # 160 rows = whole chunks; more than one column tile
]


@pytest.mark.parametrize("groups", [1, 4])
@pytest.mark.parametrize("shape", STACKS)
def test_layer_stack(shape, groups):
    """pf_lowrank_lstm_stack_fwd/bwd (diagonal schedule) against the stacked oracle (layer after layer)."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r, L = shape
    a = _stack_inputs(T, B, d, h, r, groups, L, seed=3)
    ho, co, go, Txo, Tho = oracle.lowrank_lstm_stack_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"],
                                                         a["bias"], groups)
    dxo, dh0o, dc0o, gro = oracle.lowrank_lstm_stack_bwd(a["x"], a["h0"], a["c0"], ho, co, go, Txo, Tho, a["Vx"],
                                                        a["Ux"], a["Vh"], a["Uh"], a["dh_top"], a["dhT"], a["dcT"],
                                                        groups)
    g = _gpu_lists(a)
    h_all, c_all, gates_all, Tx_all, Th_all = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"],
                                                                           g["Vh"], g["Uh"], g["bias"], groups)
    tag = f"stack {shape} groups={groups}"
    for l in range(L):
        for name, got, want in (("h", h_all, ho), ("c", c_all, co), ("gates", gates_all, go), ("Tx", Tx_all, Txo),
                                ("Th", Th_all, Tho)):
            assert_close(got[l], want[l], "f32", f"{tag} {name}{l}")
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                    g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["dh_top"], g["dhT"], g["dcT"],
                                                    groups)
    assert_close(dx, dxo, "f32", tag + " dx")
    for l in range(L):
        assert_close(dh0[l], dh0o[l], "f32", f"{tag} dh0 {l}")
        assert_close(dc0[l], dc0o[l], "f32", f"{tag} dc0 {l}")
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(gr[l][k], gro[l][k], "f32", f"{tag} {k}{l}")
    # a second call accumulates onto the first; without dx
    dx2, _, _, gr2 = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], h_all, c_all, gates_all, Tx_all, Th_all,
                                                  g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["dh_top"], g["dhT"], g["dcT"],
                                                  groups, need_dx=False, grads=gr)
    assert dx2 is None
    for l in range(L):
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(gr2[l][k], 2 * gro[l][k], "f32", f"{tag} accumulated {k}{l}")


def test_layer_stack_without_bias_and_final_state_gradients():
    import paper_2103_03936_amd as pf
    T, B, d, h, r, L, groups = 4, 6, 20, 24, 8, 2, 1
    a = _stack_inputs(T, B, d, h, r, groups, L, seed=5)
    ho, co, go, Txo, Tho = oracle.lowrank_lstm_stack_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"],
                                                         None, groups)
    dhT = [None, a["dhT"][1]]
    dxo, dh0o, dc0o, gro = oracle.lowrank_lstm_stack_bwd(a["x"], a["h0"], a["c0"], ho, co, go, Txo, Tho, a["Vx"],
                                                        a["Ux"], a["Vh"], a["Uh"], a["dh_top"], dhT, None, groups)
    g = _gpu_lists(a)
    outs = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"], g["Vh"], g["Uh"], None, groups)
    for l in range(L):
        assert_close(outs[0][l], ho[l], "f32", f"no bias h{l}")
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"], g["Uh"],
                                                    g["dh_top"], [None, g["dhT"][1]], None, groups)
    assert_close(dx, dxo, "f32", "no bias dx")
    for l in range(L):
        assert_close(dh0[l], dh0o[l], "f32", f"no bias dh0 {l}")
        assert_close(dc0[l], dc0o[l], "f32", f"no bias dc0 {l}")
        for k in ("dVx", "dUx", "dVh", "dUh"):
            assert_close(gr[l][k], gro[l][k], "f32", f"no bias {k}{l}")


def test_layer_stack_matches_sequence_layers_full_size():
    """The language model's two layers (Appendix D), 35 steps at batch 20: the stack entry points against the
    sequence entry points run layer after layer (both on the GPU; those are checked against the oracle above)."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r, L = 35, 20, 1500, 1500, 375, 2
    a = _stack_inputs(T, B, d, h, r, 1, L, seed=11)
    g = _gpu_lists(a)
    outs = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["bias"], 1)
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"], g["Uh"],
                                                    g["dh_top"], g["dhT"], g["dcT"], 1)
    xin, saved = g["x"], []
    for l in range(L):
        o = pf.pf_lowrank_lstm_seq_fwd(xin, g["h0"][l], g["c0"][l], g["Vx"][l], g["Ux"][l], g["Vh"][l], g["Uh"][l],
                                       g["bias"][l], 1)
        saved.append((xin,) + o)
        for name, i in (("h", 0), ("c", 1), ("gates", 2), ("Tx", 3), ("Th", 4)):
            assert_close(outs[i][l], o[i].double().cpu().numpy(), "f32", f"full size {name}{l}")
        xin = o[0]
    above = g["dh_top"]
    for l in reversed(range(L)):
        xin, h_all, c_all, gates_all, Tx_all, Th_all = saved[l]
        above, dh0s, dc0s, grs = pf.pf_lowrank_lstm_seq_bwd(xin, g["h0"][l], g["c0"][l], h_all, c_all, gates_all, Tx_all,
                                                            Th_all, g["Vx"][l], g["Ux"][l], g["Vh"][l], g["Uh"][l], above,
                                                            g["dhT"][l], g["dcT"][l], 1)
        assert_close(dh0[l], dh0s.double().cpu().numpy(), "f32", f"full size dh0 {l}")
        assert_close(dc0[l], dc0s.double().cpu().numpy(), "f32", f"full size dc0 {l}")
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(gr[l][k], grs[k].double().cpu().numpy(), "f32", f"full size {k}{l}")
    assert_close(dx, above.double().cpu().numpy(), "f32", "full size dx")


@pytest.mark.parametrize("groups", [1, 4])
def test_layer_stack_full_size_against_oracle(groups):
    """The language model's two layers over all 35 steps at batch 20 (Appendix D), forward and back-propagation
    through time and depth, directly against the fp64 oracle: with one rank-375 factor pair per path (groups = 1,
    the fused schedule) and with one pair per gate and path (groups = 4, Appendix D's table, the general schedule)."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r, L = 35, 20, 1500, 1500, 375, 2
    a = _stack_inputs(T, B, d, h, r, groups, L, seed=21)
    ho, co, go, Txo, Tho = oracle.lowrank_lstm_stack_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"],
                                                         a["bias"], groups)
    dxo, dh0o, dc0o, gro = oracle.lowrank_lstm_stack_bwd(a["x"], a["h0"], a["c0"], ho, co, go, Txo, Tho, a["Vx"],
                                                        a["Ux"], a["Vh"], a["Uh"], a["dh_top"], a["dhT"], a["dcT"], groups)
    g = _gpu_lists(a)
    outs = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["bias"], groups)
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"], g["Uh"],
                                                    g["dh_top"], g["dhT"], g["dcT"], groups)
    for l in range(L):
        for name, got, want in (("h", outs[0], ho), ("c", outs[1], co), ("gates", outs[2], go), ("Tx", outs[3], Txo),
                                ("Th", outs[4], Tho)):
            assert_close(got[l], want[l], "f32", f"full size {name}{l}")
        assert_close(dh0[l], dh0o[l], "f32", f"full size dh0 {l}")
        assert_close(dc0[l], dc0o[l], "f32", f"full size dc0 {l}")
        for k in ("dVx", "dUx", "dVh", "dUh", "dbias"):
            assert_close(gr[l][k], gro[l][k], "f32", f"full size {k}{l}")
    assert_close(dx, dxo, "f32", "full size dx")


def test_layer_stack_random_shapes():
    """Twelve seeded random geometries (steps, batch, widths, rank, depth, factor layout, bias) against the oracle."""
    import paper_2103_03936_amd as pf
    rng = np.random.default_rng(2103)
    for case in range(12):
        T, B, L = int(rng.integers(1, 6)), int(rng.integers(1, 33)), int(rng.integers(1, 5))
        G, bias = int(rng.choice([1, 4])), bool(rng.integers(0, 2))
        d, h, r = int(rng.integers(4, 80)), int(rng.integers(4, 80)), int(rng.integers(4, 40))
        a = _stack_inputs(T, B, d, h, r, G, L, seed=100 + case)
        if not bias:
            a["bias"] = None
        tag = f"random stack {case}: T={T} B={B} d={d} h={h} r={r} L={L} groups={G} bias={bias}"
        o = oracle.lowrank_lstm_stack_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["bias"], G)
        ob = oracle.lowrank_lstm_stack_bwd(a["x"], a["h0"], a["c0"], *o, a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["dh_top"],
                                           a["dhT"], a["dcT"], G)
        g = {k: (None if v is None else _gpu_lists({k: v})[k]) for k, v in a.items()}
        outs = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["bias"], G)
        dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"],
                                                        g["Uh"], g["dh_top"], g["dhT"], g["dcT"], G)
        assert_close(dx, ob[0], "f32", tag + " dx")
        for l in range(L):
            for i, name in enumerate(("h", "c", "gates", "Tx", "Th")):
                assert_close(outs[i][l], o[i][l], "f32", f"{tag} {name}{l}")
            assert_close(dh0[l], ob[1][l], "f32", f"{tag} dh0 {l}")
            assert_close(dc0[l], ob[2][l], "f32", f"{tag} dc0 {l}")
            for k in ("dVx", "dUx", "dVh", "dUh") + (("dbias",) if bias else ()):
                assert_close(gr[l][k], ob[3][l][k], "f32", f"{tag} {k}{l}")


def _check_stack_case(pf, T, B, d, h, r, L, G, bias, seed, tag):
    a = _stack_inputs(T, B, d, h, r, G, L, seed=seed)
    if not bias:
        a["bias"] = None
    o = oracle.lowrank_lstm_stack_fwd(a["x"], a["h0"], a["c0"], a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["bias"], G)
    ob = oracle.lowrank_lstm_stack_bwd(a["x"], a["h0"], a["c0"], *o, a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["dh_top"],
                                       a["dhT"], a["dcT"], G)
    g = {k: (None if v is None else _gpu_lists({k: v})[k]) for k, v in a.items()}
    outs = pf.pf_lowrank_lstm_stack_fwd(g["x"], g["h0"], g["c0"], g["Vx"], g["Ux"], g["Vh"], g["Uh"], g["bias"], G)
    dx, dh0, dc0, gr = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"],
                                                    g["Uh"], g["dh_top"], g["dhT"], g["dcT"], G)
    assert_close(dx, ob[0], "f32", tag + " dx")
    for l in range(L):
        assert_close(dh0[l], ob[1][l], "f32", f"{tag} dh0 {l}")
        assert_close(dc0[l], ob[2][l], "f32", f"{tag} dc0 {l}")
        for k in ("dVx", "dUx", "dVh", "dUh") + (("dbias",) if bias else ()):
            assert_close(gr[l][k], ob[3][l][k], "f32", f"{tag} {k}{l}")
    # a second call accumulates onto the first
    _, _, _, gr2 = pf.pf_lowrank_lstm_stack_bwd(g["x"], g["h0"], g["c0"], *outs, g["Vx"], g["Ux"], g["Vh"], g["Uh"],
                                                g["dh_top"], g["dhT"], g["dcT"], G, grads=gr)
    for l in range(L):
        for k in ("dVx", "dUx", "dVh", "dUh") + (("dbias",) if bias else ()):
            assert_close(gr2[l][k], 2 * ob[3][l][k], "f32", f"{tag} accumulated {k}{l}")


def test_layer_stack_long_sequences_random_shapes():
    """Seeded random geometries with T B between 128 and 512, where the weight gradients are summed on the matrix
    unit: widths and ranks around its 64- and 128-wide tiles, both factor layouts, with and without bias, written
    and accumulated."""
    import paper_2103_03936_amd as pf
    rng = np.random.default_rng(3936)
    for case in range(10):
        T, B, L = int(rng.integers(8, 17)), int(rng.integers(16, 33)), int(rng.integers(1, 3))
        G, bias = int(rng.choice([1, 4])), bool(rng.integers(0, 2))
        d, h, r = int(rng.integers(4, 200)), int(rng.integers(4, 150)), int(rng.integers(4, 140))
        tag = f"long random stack {case}: T={T} B={B} d={d} h={h} r={r} L={L} groups={G} bias={bias}"
        _check_stack_case(pf, T, B, d, h, r, L, G, bias, 300 + case, tag)


@pytest.mark.parametrize("shape", [(4, 32, 64, 64, 128, 1, 1), (32, 4, 20, 12, 6, 2, 1), (16, 8, 4, 4, 4, 1, 4),
                                   (16, 8, 4, 4, 4, 2, 1), (5, 32, 7, 33, 129, 1, 1)])
def test_layer_stack_long_sequences_edges(shape):
    """T B >= 128 at the edges of the matrix-unit weight-gradient kernel: exactly one full tile and whole chunks,
    many short steps, the smallest extents the entry points take (rows of four floats), one column past a tile."""
    import paper_2103_03936_amd as pf
    T, B, d, h, r, L, G = shape
    _check_stack_case(pf, T, B, d, h, r, L, G, True, 77, f"long stack edge {shape}")
