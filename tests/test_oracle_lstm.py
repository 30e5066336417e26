"""Pins for the LSTM-cell oracle (Section 2.3, eq. (1) and eq. (2)).

Pinned against torch.nn.LSTMCell (a library routine with the same i, f, g, o
gate order), torch autograd, finite differences through three time steps, the
dense cell with W = U V^T, a hand-checkable special case, and the printed
parameter / MAC totals that fix the per-gate reading.
"""
import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _cell_inputs(B, d, h, r, groups, seed=0):
    gr = groups * r
    return dict(
        x=_rand((B, d), seed + 1), hprev=_rand((B, h), seed + 2), cprev=_rand((B, h), seed + 3),
        Vx=_rand((d, gr), seed + 4, 0.4), Ux=_rand((4 * h, r), seed + 5, 0.4),
        Vh=_rand((h, gr), seed + 6, 0.4), Uh=_rand((4 * h, r), seed + 7, 0.4),
        bias=_rand((4 * h,), seed + 8, 0.4),
    )


def _dense_weights(a, h, r, groups):
    """W_x = U_x V_x^T per gate block (eq. (2) -> eq. (1))."""
    Wx = np.zeros((4 * h, a["Vx"].shape[0]))
    Wh = np.zeros((4 * h, h))
    for g in range(4):
        cols = slice(g * r, (g + 1) * r) if groups == 4 else slice(0, r)
        Wx[g * h:(g + 1) * h] = a["Ux"][g * h:(g + 1) * h] @ a["Vx"][:, cols].T
        Wh[g * h:(g + 1) * h] = a["Uh"][g * h:(g + 1) * h] @ a["Vh"][:, cols].T
    return Wx, Wh


@pytest.mark.parametrize("groups", [1, 4])
@pytest.mark.parametrize("B,d,h,r", [(1, 1, 1, 1), (3, 5, 4, 2), (4, 7, 6, 3)])
def test_fwd_matches_torch_lstmcell(B, d, h, r, groups):
    a = _cell_inputs(B, d, h, r, groups)
    ho, co, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(
        a["x"], a["hprev"], a["cprev"], a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["bias"], groups)
    Wx, Wh = _dense_weights(a, h, r, groups)
    cell = torch.nn.LSTMCell(d, h, bias=True, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.tensor(Wx))
        cell.weight_hh.copy_(torch.tensor(Wh))
        cell.bias_ih.copy_(torch.tensor(0.25 * a["bias"]))  # eq. (1) has two bias vectors;
        cell.bias_hh.copy_(torch.tensor(0.75 * a["bias"]))  # only their sum matters
        th, tc = cell(torch.tensor(a["x"]), (torch.tensor(a["hprev"]), torch.tensor(a["cprev"])))
    np.testing.assert_allclose(ho, th.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(co, tc.numpy(), rtol=1e-11, atol=1e-11)
    # the oracle's own eq. (1) cell agrees
    dh, dc = oracle.dense_lstm_cell_fwd(a["x"], a["hprev"], a["cprev"], Wx, Wh, a["bias"])
    np.testing.assert_allclose(dh, th.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dc, tc.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(Tx, a["x"] @ a["Vx"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Th, a["hprev"] @ a["Vh"], rtol=1e-12, atol=1e-12)
    # gates are stored activated, i | f | g | o
    z = a["x"] @ Wx.T + a["hprev"] @ Wh.T + a["bias"]
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    np.testing.assert_allclose(gates[:, :h], sig(z[:, :h]), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(gates[:, h:2 * h], sig(z[:, h:2 * h]), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(gates[:, 2 * h:3 * h], np.tanh(z[:, 2 * h:3 * h]), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(gates[:, 3 * h:], sig(z[:, 3 * h:]), rtol=1e-11, atol=1e-11)


def test_hand_checkable_cell():
    # all pre-activations zero: i = f = o = 1/2, g = 0, so c = c_prev / 2, h = tanh(c) / 2
    B, d, h, r = 2, 3, 2, 1
    z = np.zeros
    cprev = np.array([[2.0, -4.0], [0.0, 1.0]])
    ho, co, gates, _, _ = oracle.lowrank_lstm_cell_fwd(
        z((B, d)), z((B, h)), cprev, z((d, r)), z((4 * h, r)), z((h, r)), z((4 * h, r)), None, 1)
    assert np.array_equal(co, cprev / 2)
    np.testing.assert_allclose(ho, np.tanh(cprev / 2) / 2, rtol=1e-15)
    # a large bias on one gate saturates it: forget gate -> 1, others -> 1/2
    bias = np.zeros(4 * h)
    bias[h:2 * h] = 50.0
    ho, co, gates, _, _ = oracle.lowrank_lstm_cell_fwd(
        z((B, d)), z((B, h)), cprev, z((d, r)), z((4 * h, r)), z((h, r)), z((4 * h, r)), bias, 1)
    np.testing.assert_allclose(co, cprev, rtol=1e-15)


def test_groups4_with_replicated_V_equals_groups1():
    B, d, h, r = 3, 5, 4, 2
    a = _cell_inputs(B, d, h, r, 1)
    ref = oracle.lowrank_lstm_cell_fwd(a["x"], a["hprev"], a["cprev"], a["Vx"], a["Ux"], a["Vh"], a["Uh"],
                                       a["bias"], 1)
    Vx4, Vh4 = np.tile(a["Vx"], (1, 4)), np.tile(a["Vh"], (1, 4))
    got = oracle.lowrank_lstm_cell_fwd(a["x"], a["hprev"], a["cprev"], Vx4, a["Ux"], Vh4, a["Uh"], a["bias"], 4)
    for u, v in zip(ref[:3], got[:3]):
        np.testing.assert_allclose(u, v, rtol=1e-12, atol=1e-12)


def _torch_cell(x, hp, cp, Vx, Ux, Vh, Uh, b, h, r, groups):
    zs = []
    for g in range(4):
        cols = slice(g * r, (g + 1) * r) if groups == 4 else slice(0, r)
        rows = slice(g * h, (g + 1) * h)
        zs.append((x @ Vx[:, cols]) @ Ux[rows].T + (hp @ Vh[:, cols]) @ Uh[rows].T + b[rows])
    i, f, g_, o = torch.sigmoid(zs[0]), torch.sigmoid(zs[1]), torch.tanh(zs[2]), torch.sigmoid(zs[3])
    c = f * cp + i * g_
    return o * torch.tanh(c), c


@pytest.mark.parametrize("groups", [1, 4])
def test_bwd_matches_torch_autograd(groups):
    B, d, h, r = 3, 5, 4, 2
    a = _cell_inputs(B, d, h, r, groups, seed=30)
    dh, dc = _rand((B, h), 50), _rand((B, h), 51)
    t = {k: torch.tensor(v, requires_grad=True) for k, v in a.items()}
    th, tc = _torch_cell(t["x"], t["hprev"], t["cprev"], t["Vx"], t["Ux"], t["Vh"], t["Uh"], t["bias"], h, r, groups)
    (th * torch.tensor(dh)).sum().add((tc * torch.tensor(dc)).sum()).backward()
    ho, co, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(
        a["x"], a["hprev"], a["cprev"], a["Vx"], a["Ux"], a["Vh"], a["Uh"], a["bias"], groups)
    dx, dhp, dcp, gr = oracle.lowrank_lstm_cell_bwd(
        a["x"], a["hprev"], a["cprev"], co, gates, Tx, Th, a["Vx"], a["Ux"], a["Vh"], a["Uh"], dh, dc, groups)
    np.testing.assert_allclose(dx, t["x"].grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dhp, t["hprev"].grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dcp, t["cprev"].grad.numpy(), rtol=1e-10, atol=1e-10)
    for name in ("Vx", "Ux", "Vh", "Uh"):
        np.testing.assert_allclose(gr["d" + name], t[name].grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(gr["dbias"], t["bias"].grad.numpy(), rtol=1e-10, atol=1e-10)
    # dc_next = None means zero; accumulate adds to what is there
    dx0, dhp0, dcp0, gr0 = oracle.lowrank_lstm_cell_bwd(
        a["x"], a["hprev"], a["cprev"], co, gates, Tx, Th, a["Vx"], a["Ux"], a["Vh"], a["Uh"], dh, None, groups)
    dx1, _, _, gr1 = oracle.lowrank_lstm_cell_bwd(
        a["x"], a["hprev"], a["cprev"], co, gates, Tx, Th, a["Vx"], a["Ux"], a["Vh"], a["Uh"], dh,
        np.zeros((B, h)), groups, grads={k: v.copy() for k, v in gr0.items()})
    np.testing.assert_allclose(dx0, dx1, rtol=1e-14)
    for k in gr0:
        np.testing.assert_allclose(gr1[k], 2 * gr0[k], rtol=1e-12, atol=1e-14)


def _run_sequence(p, xs, groups, h, r):
    """Three-step unroll; returns loss ingredients and per-step saved state."""
    B = xs[0].shape[0]
    hp, cp = np.zeros((B, h)), np.zeros((B, h))
    saved = []
    for x in xs:
        ho, co, gates, Tx, Th = oracle.lowrank_lstm_cell_fwd(x, hp, cp, p["Vx"], p["Ux"], p["Vh"], p["Uh"],
                                                             p["bias"], groups)
        saved.append((x, hp, cp, co, gates, Tx, Th, ho))
        hp, cp = ho, co
    return saved


@pytest.mark.parametrize("groups", [1, 4])
def test_bptt_finite_differences_three_steps(groups):
    B, d, h, r, T = 2, 3, 2, 2, 3
    a = _cell_inputs(B, d, h, r, groups, seed=70)
    p = {k: a[k] for k in ("Vx", "Ux", "Vh", "Uh", "bias")}
    xs = [_rand((B, d), 80 + t) for t in range(T)]
    G = [_rand((B, h), 90 + t) for t in range(T)]

    def loss(params):
        saved = _run_sequence(params, xs, groups, h, r)
        return sum(float((s[7] * g).sum()) for s, g in zip(saved, G))

    saved = _run_sequence(p, xs, groups, h, r)
    grads = None
    dh_next, dc_next = np.zeros((B, h)), np.zeros((B, h))
    for t in reversed(range(T)):
        x, hp, cp, co, gates, Tx, Th, _ = saved[t]
        dx, dh_prev, dc_prev, grads = oracle.lowrank_lstm_cell_bwd(
            x, hp, cp, co, gates, Tx, Th, p["Vx"], p["Ux"], p["Vh"], p["Uh"], G[t] + dh_next, dc_next,
            groups, grads=grads)
        dh_next, dc_next = dh_prev, dc_prev
    eps = 1e-6
    for name in ("Vx", "Ux", "Vh", "Uh", "bias"):
        g = grads["d" + name]
        for idx in np.ndindex(p[name].shape):
            q = {k: v.copy() for k, v in p.items()}
            q[name][idx] += eps
            up = loss(q)
            q[name][idx] -= 2 * eps
            dn = loss(q)
            assert abs((up - dn) / (2 * eps) - g[idx]) < 2e-6, (name, idx)


def test_printed_totals_fix_the_per_gate_reading():
    # The LSTM architecture table lists eight factor pairs per layer (1500x375 / 375x1500
    # per gate and per path).  Printed totals: 85,962,278 vanilla, 67,962,278 factorized.
    vocab, d, h, r, layers = 33278, 1500, 1500, 375, 2
    shared = vocab * d + vocab + layers * 4 * h  # tied embedding, decoder bias, one 4h bias per layer
    vanilla = shared + layers * 4 * (d * h + h * h)
    per_gate = shared + layers * (4 * (d * r + r * h) + 4 * (h * r + r * h))
    assert vanilla == 85962278 and per_gate == 67962278
    # Table 1's formula 4dr + 12hr is the same count
    assert 4 * (d * r + r * h) + 4 * (h * r + r * h) == 4 * d * r + 12 * h * r
    # MACs per token per layer: 18 M dense, 9 M factorized per gate
    assert 4 * (d * h + h * h) == 18_000_000 and 8 * (d * r + r * h) == 9_000_000


@pytest.mark.parametrize("groups", [1, 4])
def test_sequence_matches_torch_lstm_and_autograd(groups):
    """The sequence oracle (cells chained over time, BPTT with accumulated parameter gradients) against
    torch.nn.LSTM with W = U V^T and torch autograd through the factors (library routines)."""
    T, B, d, h, r = 5, 3, 4, 6, 2
    rng = np.random.default_rng(77 + groups)
    gr = groups * r
    x = rng.standard_normal((T, B, d))
    h0, c0 = rng.standard_normal((B, h)) * 0.5, rng.standard_normal((B, h)) * 0.5
    Vx, Ux = rng.standard_normal((d, gr)) * 0.4, rng.standard_normal((4 * h, r)) * 0.4
    Vh, Uh = rng.standard_normal((h, gr)) * 0.4, rng.standard_normal((4 * h, r)) * 0.4
    bias = rng.standard_normal((4 * h,)) * 0.3
    G, GhT, GcT = rng.standard_normal((T, B, h)), rng.standard_normal((B, h)), rng.standard_normal((B, h))

    h_all, c_all, gates_all, Tx_all, Th_all = oracle.lowrank_lstm_seq_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias, groups)
    dx_all, dh0, dc0, grads = oracle.lowrank_lstm_seq_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all,
                                                         Vx, Ux, Vh, Uh, G, GhT, GcT, groups)

    tt = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    tx, th0, tc0, tVx, tUx, tVh, tUh, tb = map(tt, (x, h0, c0, Vx, Ux, Vh, Uh, bias))

    def dense(U, V):  # gate block g of W is U_g V_g^T (per-gate V when groups == 4, shared otherwise)
        blocks = []
        for g in range(4):
            Vg = V[:, g * r:(g + 1) * r] if groups == 4 else V
            blocks.append(U[g * h:(g + 1) * h] @ Vg.T)
        return torch.cat(blocks, 0)

    lstm = torch.nn.LSTM(d, h, num_layers=1, bias=True, dtype=torch.float64)
    params = {"weight_ih_l0": dense(tUx, tVx), "weight_hh_l0": dense(tUh, tVh), "bias_ih_l0": tb,
              "bias_hh_l0": torch.zeros(4 * h, dtype=torch.float64)}
    out, (hT, cT) = torch.func.functional_call(lstm, params, (tx, (th0[None], tc0[None])))
    np.testing.assert_allclose(h_all, out.detach().numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(c_all[-1], cT[0].detach().numpy(), rtol=1e-10, atol=1e-10)
    loss = (out * torch.tensor(G)).sum() + (hT[0] * torch.tensor(GhT)).sum() + (cT[0] * torch.tensor(GcT)).sum()
    loss.backward()
    np.testing.assert_allclose(dx_all, tx.grad.numpy(), rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(dh0, th0.grad.numpy(), rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(dc0, tc0.grad.numpy(), rtol=1e-9, atol=1e-9)
    for name, tv in (("dVx", tVx), ("dUx", tUx), ("dVh", tVh), ("dUh", tUh), ("dbias", tb)):
        np.testing.assert_allclose(grads[name], tv.grad.numpy(), rtol=1e-9, atol=1e-9, err_msg=name)


@pytest.mark.parametrize("groups", [1, 4])
def test_stack_matches_two_layer_torch_lstm_and_autograd(groups):
    """The stacked oracle (layer after layer, backward from the last layer to the first) against a 2-layer
    torch.nn.LSTM with W = U V^T and torch autograd through the factors (library routines)."""
    T, B, d, h, r, L = 4, 3, 5, 6, 2, 2
    rng = np.random.default_rng(91 + groups)
    gr = groups * r
    x = rng.standard_normal((T, B, d))
    h0 = [rng.standard_normal((B, h)) * 0.5 for _ in range(L)]
    c0 = [rng.standard_normal((B, h)) * 0.5 for _ in range(L)]
    Vx = [rng.standard_normal((d if l == 0 else h, gr)) * 0.4 for l in range(L)]
    Ux = [rng.standard_normal((4 * h, r)) * 0.4 for _ in range(L)]
    Vh = [rng.standard_normal((h, gr)) * 0.4 for _ in range(L)]
    Uh = [rng.standard_normal((4 * h, r)) * 0.4 for _ in range(L)]
    bias = [rng.standard_normal((4 * h,)) * 0.3 for _ in range(L)]
    G = rng.standard_normal((T, B, h))
    GhT = [rng.standard_normal((B, h)) for _ in range(L)]
    GcT = [rng.standard_normal((B, h)) for _ in range(L)]

    h_all, c_all, gates_all, Tx_all, Th_all = oracle.lowrank_lstm_stack_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias, groups)
    dx_all, dh0, dc0, grads = oracle.lowrank_lstm_stack_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all, Vx, Ux,
                                                           Vh, Uh, G, GhT, GcT, groups)

    tt = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    tx = tt(x)
    th0, tc0, tVx, tUx, tVh, tUh, tb = ([tt(a) for a in lst] for lst in (h0, c0, Vx, Ux, Vh, Uh, bias))

    def dense(U, V):
        blocks = []
        for g in range(4):
            Vg = V[:, g * r:(g + 1) * r] if groups == 4 else V
            blocks.append(U[g * h:(g + 1) * h] @ Vg.T)
        return torch.cat(blocks, 0)

    lstm = torch.nn.LSTM(d, h, num_layers=L, bias=True, dtype=torch.float64)
    params = {}
    for l in range(L):
        params[f"weight_ih_l{l}"] = dense(tUx[l], tVx[l])
        params[f"weight_hh_l{l}"] = dense(tUh[l], tVh[l])
        params[f"bias_ih_l{l}"] = tb[l]
        params[f"bias_hh_l{l}"] = torch.zeros(4 * h, dtype=torch.float64)
    out, (hT, cT) = torch.func.functional_call(lstm, params, (tx, (torch.stack(th0), torch.stack(tc0))))
    np.testing.assert_allclose(h_all[L - 1], out.detach().numpy(), rtol=1e-10, atol=1e-10)
    for l in range(L):
        np.testing.assert_allclose(h_all[l][-1], hT[l].detach().numpy(), rtol=1e-10, atol=1e-10)
        np.testing.assert_allclose(c_all[l][-1], cT[l].detach().numpy(), rtol=1e-10, atol=1e-10)
    loss = (out * torch.tensor(G)).sum()
    for l in range(L):
        loss = loss + (hT[l] * torch.tensor(GhT[l])).sum() + (cT[l] * torch.tensor(GcT[l])).sum()
    loss.backward()
    np.testing.assert_allclose(dx_all, tx.grad.numpy(), rtol=1e-9, atol=1e-9)
    for l in range(L):
        np.testing.assert_allclose(dh0[l], th0[l].grad.numpy(), rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose(dc0[l], tc0[l].grad.numpy(), rtol=1e-9, atol=1e-9)
        for name, tv in (("dVx", tVx), ("dUx", tUx), ("dVh", tVh), ("dUh", tUh), ("dbias", tb)):
            np.testing.assert_allclose(grads[l][name], tv[l].grad.numpy(), rtol=1e-9, atol=1e-9, err_msg=f"{name}{l}")
