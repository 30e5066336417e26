"""CPU oracle for the factorized-layer forward/backward -- TEST INFRASTRUCTURE.

A thin ctypes wrapper over ``pf_oracle.c`` (plain double-precision nested
loops written from the paper's layer definitions).  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import this package; the
GPU library never does, and this package never imports the GPU library.

All arrays are C-contiguous ``float64`` numpy arrays.  Shapes follow the
paper's layers: Section 2.1 (fully connected), Section 2.2 (convolution),
Section 2.3 eq. (1)/(2) (LSTM), Algorithm 1 (SVD split).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pf_oracle.c")
_LIB = os.path.join(_HERE, "libpf_oracle.so")

_c_double_p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64


def build(force=False):
    """Compile pf_oracle.c with gcc -O2 (OpenMP on the outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.pfo_num_threads.restype = ctypes.c_int
        _lib.pfo_conv_out_dim.restype = _i64
        _lib.pfo_conv_out_dim.argtypes = [_i64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        _lib.pfo_svd_split.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(lib().pfo_num_threads())


def set_num_threads(n):
    lib().pfo_set_num_threads(ctypes.c_int(int(n)))


def _in(a, shape=None):
    """float64 C-contiguous view/copy of an input (None -> NULL)."""
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a, a.ctypes.data_as(_c_double_p)


def _out(shape):
    a = np.zeros(shape, dtype=np.float64)
    return a, a.ctypes.data_as(_c_double_p)


def conv_out_dim(H, k, s, p):
    return (H + 2 * p - k) // s + 1


# ---------------------------------------------------------------- linear

def dense_linear_fwd(X, W, bias=None):
    M, n_in = X.shape
    n_out = W.shape[0]
    X, pX = _in(X)
    W, pW = _in(W, (n_out, n_in))
    bias, pb = _in(bias, (n_out,)) if bias is not None else (None, None)
    Y, pY = _out((M, n_out))
    lib().pfo_dense_linear_fwd(_i64(M), _i64(n_in), _i64(n_out), pX, pW, pb, pY)
    return Y


def lowrank_linear_fwd(X, V, U, bias=None):
    """Y = (X V) U^T + b; returns (Y, T) with T = X V."""
    M, n_in = X.shape
    n_out, r = U.shape
    X, pX = _in(X)
    V, pV = _in(V, (n_in, r))
    U, pU = _in(U)
    bias, pb = _in(bias, (n_out,)) if bias is not None else (None, None)
    Y, pY = _out((M, n_out))
    T, pT = _out((M, r))
    lib().pfo_lowrank_linear_fwd(_i64(M), _i64(n_in), _i64(n_out), _i64(r), pX, pV, pU, pb, pY, pT)
    return Y, T


def lowrank_linear_bwd(X, V, U, dY):
    """Returns (dX, dU, dV, db)."""
    M, n_in = X.shape
    n_out, r = U.shape
    X, pX = _in(X)
    V, pV = _in(V, (n_in, r))
    U, pU = _in(U)
    dY, pdY = _in(dY, (M, n_out))
    dX, pdX = _out((M, n_in))
    dU, pdU = _out((n_out, r))
    dV, pdV = _out((n_in, r))
    db, pdb = _out((n_out,))
    lib().pfo_lowrank_linear_bwd(_i64(M), _i64(n_in), _i64(n_out), _i64(r), pX, pV, pU, pdY,
                                 pdX, pdU, pdV, pdb)
    return dX, dU, dV, db


def lowrank_linear_shared_fwd(X, V, U, bias=None):
    """Projections that read one input (Section 2.4: the query, key and value matrices, each the layer of
    Section 2.1): Y_g = (X V_g) U_g^T + b_g.  V[G,in,r], U[G,out,r], bias[G,out]; returns (Y[G,M,out], T[G,M,r])."""
    G = U.shape[0]
    Ys, Ts = [], []
    for g in range(G):
        Y, T = lowrank_linear_fwd(X, V[g], U[g], None if bias is None else bias[g])
        Ys.append(Y)
        Ts.append(T)
    return np.stack(Ys), np.stack(Ts)


def lowrank_linear_shared_bwd(X, V, U, dY):
    """The input is shared, so its gradient is the sum of the projections' input gradients; the parameter
    gradients are each projection's own.  Returns (dX[M,in], dU[G,out,r], dV[G,in,r], db[G,out])."""
    G = U.shape[0]
    dX = np.zeros(X.shape, dtype=np.float64)
    dUs, dVs, dbs = [], [], []
    for g in range(G):
        dXg, dU, dV, db = lowrank_linear_bwd(X, V[g], U[g], dY[g])
        dX += dXg
        dUs.append(dU)
        dVs.append(dV)
        dbs.append(db)
    return dX, np.stack(dUs), np.stack(dVs), np.stack(dbs)


def lowrank_linear_fwd_ep(X, V, U, bias=None, residual=None, act="none"):
    """The factorized layer of Section 2.1 with what follows it in a Transformer block (Section 2.4): the bias, an
    optional residual input R of Y's shape, and the feed-forward network's max(0, .):
        Z = (X V) U^T + b + R,   Y = max(0, Z) if act == "relu" else Z.
    FFN(x) = max(0, x W_1 + b_1) W_2 + b_2 is act="relu" on the first layer and act="none" on the second.
    Returns (Y, T)."""
    assert act in ("none", "relu")
    Z, T = lowrank_linear_fwd(X, V, U, bias)
    if residual is not None:
        Z = Z + np.asarray(residual, dtype=np.float64)
    return (np.maximum(Z, 0.0) if act == "relu" else Z), T


def lowrank_linear_bwd_ep(X, V, U, dZ, dX_add=None, x_is_relu=False):
    """Backward of lowrank_linear_fwd_ep from dZ = dL/dZ (the gradient of the pre-activation; for act == "none"
    that is dL/dY, and a residual input receives dZ unchanged).  The layer's own input may be the output of a
    max(0, .) and may also feed a skip connection:
        dX = (dZ U V^T + dX_add) * [X > 0]      (the mask only when x_is_relu; dX_add optional),
    i.e. dX is dL/d(pre-activation of the layer below).  dU, dV, db as in lowrank_linear_bwd with dY = dZ.
    Returns (dX, dU, dV, db)."""
    dX, dU, dV, db = lowrank_linear_bwd(X, V, U, dZ)
    if dX_add is not None:
        dX = dX + np.asarray(dX_add, dtype=np.float64)
    if x_is_relu:
        dX = dX * (np.asarray(X, dtype=np.float64) > 0.0)
    return dX, dU, dV, db


# ------------------------------------------------------------------ conv

def dense_conv_fwd(X, Wd, stride=1, pad=0):
    N, C, H, W = X.shape
    Cout, _, k, _ = Wd.shape
    Ho, Wo = conv_out_dim(H, k, stride, pad), conv_out_dim(W, k, stride, pad)
    X, pX = _in(X)
    Wd, pW = _in(Wd, (Cout, C, k, k))
    Y, pY = _out((N, Cout, Ho, Wo))
    lib().pfo_dense_conv_fwd(_i64(N), _i64(C), _i64(H), _i64(W), _i64(Cout), ctypes.c_int(k),
                             ctypes.c_int(stride), ctypes.c_int(pad), pX, pW, pY)
    return Y


def lowrank_conv_fwd(X, Uk, Vp, stride=1, pad=0):
    """Thin k x k conv (Uk[r,C,k,k]) then 1x1 conv (Vp[Cout,r]); returns (Y, T)."""
    N, C, H, W = X.shape
    r, _, k, _ = Uk.shape
    Cout = Vp.shape[0]
    Ho, Wo = conv_out_dim(H, k, stride, pad), conv_out_dim(W, k, stride, pad)
    X, pX = _in(X)
    Uk, pU = _in(Uk, (r, C, k, k))
    Vp, pV = _in(Vp, (Cout, r))
    Y, pY = _out((N, Cout, Ho, Wo))
    T, pT = _out((N, r, Ho, Wo))
    lib().pfo_lowrank_conv_fwd(_i64(N), _i64(C), _i64(H), _i64(W), _i64(Cout), _i64(r),
                               ctypes.c_int(k), ctypes.c_int(stride), ctypes.c_int(pad),
                               pX, pU, pV, pY, pT)
    return Y, T


def lowrank_conv_bwd(X, Uk, Vp, dY, stride=1, pad=0):
    """Returns (dX, dUk, dVp)."""
    N, C, H, W = X.shape
    r, _, k, _ = Uk.shape
    Cout = Vp.shape[0]
    Ho, Wo = conv_out_dim(H, k, stride, pad), conv_out_dim(W, k, stride, pad)
    X, pX = _in(X)
    Uk, pU = _in(Uk, (r, C, k, k))
    Vp, pV = _in(Vp, (Cout, r))
    dY, pdY = _in(dY, (N, Cout, Ho, Wo))
    dX, pdX = _out((N, C, H, W))
    dUk, pdU = _out((r, C, k, k))
    dVp, pdV = _out((Cout, r))
    lib().pfo_lowrank_conv_bwd(_i64(N), _i64(C), _i64(H), _i64(W), _i64(Cout), _i64(r),
                               ctypes.c_int(k), ctypes.c_int(stride), ctypes.c_int(pad),
                               pX, pU, pV, pdY, pdX, pdU, pdV)
    return dX, dUk, dVp


# ------------------------------------------------------------------ LSTM

def lowrank_conv_fwd_ep(X, Uk, Vp, scale=None, shift=None, residual=None, act="none", stride=1, pad=0):
    """The factorized convolution of Section 2.2 followed by what Appendix D puts after every convolution: batch
    normalisation (here with fixed statistics, i.e. a per-channel scale and shift: scale = gamma / sqrt(var + eps),
    shift = beta - mean * scale), the residual input of a ResNet block, and ReLU:
        P = Vp * (Uk * X),  Z[n,o,y,x] = scale[o] P[n,o,y,x] + shift[o] + R[n,o,y,x],  Y = max(0, Z) or Z.
    Returns (Y, T)."""
    assert act in ("none", "relu")
    P, T = lowrank_conv_fwd(X, Uk, Vp, stride, pad)
    Z = P
    if scale is not None:
        Z = Z * np.asarray(scale, dtype=np.float64)[None, :, None, None]
    if shift is not None:
        Z = Z + np.asarray(shift, dtype=np.float64)[None, :, None, None]
    if residual is not None:
        Z = Z + np.asarray(residual, dtype=np.float64)
    return (np.maximum(Z, 0.0) if act == "relu" else Z), T


def lowrank_conv_bwd_ep(X, Uk, Vp, scale, dZ, stride=1, pad=0, dX_add=None, x_is_relu=False):
    """Backward of lowrank_conv_fwd_ep from dZ = dL/dZ:  dP = scale * dZ (per output channel), dshift[o] = the sum
    of dZ over batch and pixels, dT, dVp, dUk from dP as in lowrank_conv_bwd, and
        dX = (transposed convolution of dT + dX_add) * [X > 0]   (mask only when x_is_relu; dX_add optional).
    The scale is a constant (fixed statistics), so it has no gradient.  Returns (dX, dUk, dVp, dshift)."""
    dZ = np.asarray(dZ, dtype=np.float64)
    dP = dZ if scale is None else dZ * np.asarray(scale, dtype=np.float64)[None, :, None, None]
    dX, dUk, dVp = lowrank_conv_bwd(X, Uk, Vp, dP, stride, pad)
    if dX_add is not None:
        dX = dX + np.asarray(dX_add, dtype=np.float64)
    if x_is_relu:
        dX = dX * (np.asarray(X, dtype=np.float64) > 0.0)
    return dX, dUk, dVp, dZ.sum(axis=(0, 2, 3))


def dense_lstm_cell_fwd(x, hprev, cprev, Wx, Wh, bias=None):
    """Eq. (1): returns (h, c)."""
    B, d = x.shape
    h = hprev.shape[1]
    x, px = _in(x)
    hprev, ph = _in(hprev, (B, h))
    cprev, pc = _in(cprev, (B, h))
    Wx, pWx = _in(Wx, (4 * h, d))
    Wh, pWh = _in(Wh, (4 * h, h))
    bias, pb = _in(bias, (4 * h,)) if bias is not None else (None, None)
    ho, pho = _out((B, h))
    co, pco = _out((B, h))
    lib().pfo_dense_lstm_cell_fwd(_i64(B), _i64(d), _i64(h), px, ph, pc, pWx, pWh, pb, pho, pco)
    return ho, co


def lowrank_lstm_cell_fwd(x, hprev, cprev, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """Eq. (2): returns (h, c, gates, Tx, Th)."""
    B, d = x.shape
    h = hprev.shape[1]
    r = Ux.shape[1]
    gr = groups * r
    x, px = _in(x)
    hprev, ph = _in(hprev, (B, h))
    cprev, pc = _in(cprev, (B, h))
    Vx, pVx = _in(Vx, (d, gr))
    Ux, pUx = _in(Ux, (4 * h, r))
    Vh, pVh = _in(Vh, (h, gr))
    Uh, pUh = _in(Uh, (4 * h, r))
    bias, pb = _in(bias, (4 * h,)) if bias is not None else (None, None)
    ho, pho = _out((B, h))
    co, pco = _out((B, h))
    gates, pg = _out((B, 4 * h))
    Tx, pTx = _out((B, gr))
    Th, pTh = _out((B, gr))
    lib().pfo_lowrank_lstm_cell_fwd(_i64(B), _i64(d), _i64(h), _i64(r), ctypes.c_int(groups),
                                    px, ph, pc, pVx, pUx, pVh, pUh, pb, pho, pco, pg, pTx, pTh)
    return ho, co, gates, Tx, Th


def lowrank_lstm_cell_bwd(x, hprev, cprev, c_out, gates, Tx, Th, Vx, Ux, Vh, Uh, dh,
                          dc_next=None, groups=1, grads=None):
    """Returns (dx, dh_prev, dc_prev, grads) with grads = dict(dVx, dUx, dVh, dUh, dbias).

    If ``grads`` is given the parameter gradients are accumulated into it.
    """
    B, d = x.shape
    h = hprev.shape[1]
    r = Ux.shape[1]
    gr = groups * r
    x, px = _in(x)
    hprev, ph = _in(hprev, (B, h))
    cprev, pc = _in(cprev, (B, h))
    c_out, pco = _in(c_out, (B, h))
    gates, pg = _in(gates, (B, 4 * h))
    Tx, pTx = _in(Tx, (B, gr))
    Th, pTh = _in(Th, (B, gr))
    Vx, pVx = _in(Vx, (d, gr))
    Ux, pUx = _in(Ux, (4 * h, r))
    Vh, pVh = _in(Vh, (h, gr))
    Uh, pUh = _in(Uh, (4 * h, r))
    dh, pdh = _in(dh, (B, h))
    dc_next, pdc = _in(dc_next, (B, h)) if dc_next is not None else (None, None)
    dx, pdx = _out((B, d))
    dhp, pdhp = _out((B, h))
    dcp, pdcp = _out((B, h))
    accumulate = grads is not None
    if grads is None:
        grads = dict(dVx=np.zeros((d, gr)), dUx=np.zeros((4 * h, r)), dVh=np.zeros((h, gr)),
                     dUh=np.zeros((4 * h, r)), dbias=np.zeros((4 * h,)))
    ptr = {k: v.ctypes.data_as(_c_double_p) for k, v in grads.items()}
    lib().pfo_lowrank_lstm_cell_bwd(_i64(B), _i64(d), _i64(h), _i64(r), ctypes.c_int(groups),
                                    px, ph, pc, pco, pg, pTx, pTh, pVx, pUx, pVh, pUh, pdh, pdc,
                                    pdx, pdhp, pdcp, ptr["dVx"], ptr["dUx"], ptr["dVh"],
                                    ptr["dUh"], ptr["dbias"], ctypes.c_int(1 if accumulate else 0))
    return dx, dhp, dcp, grads


def lowrank_lstm_seq_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """One factorized LSTM layer over T time steps: eq. (2) applied step by step, h_t and c_t fed to step
    t + 1.  x is [T, B, d].  Returns (h_all [T,B,h], c_all [T,B,h], gates_all [T,B,4h], Tx_all, Th_all)."""
    T, B, d = x.shape
    h = h0.shape[1]
    gr = groups * Ux.shape[1]
    h_all, c_all = np.zeros((T, B, h)), np.zeros((T, B, h))
    gates_all, Tx_all, Th_all = np.zeros((T, B, 4 * h)), np.zeros((T, B, gr)), np.zeros((T, B, gr))
    hp, cp = np.asarray(h0, dtype=np.float64), np.asarray(c0, dtype=np.float64)
    for t in range(T):
        h_all[t], c_all[t], gates_all[t], Tx_all[t], Th_all[t] = lowrank_lstm_cell_fwd(
            x[t], hp, cp, Vx, Ux, Vh, Uh, bias, groups)
        hp, cp = h_all[t], c_all[t]
    return h_all, c_all, gates_all, Tx_all, Th_all


def lowrank_lstm_seq_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all, Vx, Ux, Vh, Uh, dh_all,
                         dhT=None, dcT=None, groups=1, grads=None):
    """Back-propagation through time of lowrank_lstm_seq_fwd: dh_all[t] is the gradient arriving at h_t from
    above, dhT / dcT the gradients arriving at the final state.  Steps are taken in reverse with the cell's
    backward; parameter gradients add up over time (and onto ``grads`` if given).
    Returns (dx_all [T,B,d], dh0, dc0, grads)."""
    T, B, d = x.shape
    h = h0.shape[1]
    dx_all = np.zeros((T, B, d))
    dh = np.array(dh_all[T - 1], dtype=np.float64) + (0.0 if dhT is None else np.asarray(dhT, dtype=np.float64))
    dc = np.zeros((B, h)) if dcT is None else np.asarray(dcT, dtype=np.float64)
    for t in range(T - 1, -1, -1):
        hp = h_all[t - 1] if t > 0 else np.asarray(h0, dtype=np.float64)
        cp = c_all[t - 1] if t > 0 else np.asarray(c0, dtype=np.float64)
        if grads is None:  # first call creates the gradient buffers, later calls accumulate
            dx_all[t], dhp, dc, grads = lowrank_lstm_cell_bwd(x[t], hp, cp, c_all[t], gates_all[t], Tx_all[t], Th_all[t],
                                                            Vx, Ux, Vh, Uh, dh, dc, groups)
        else:
            dx_all[t], dhp, dc, grads = lowrank_lstm_cell_bwd(x[t], hp, cp, c_all[t], gates_all[t], Tx_all[t], Th_all[t],
                                                            Vx, Ux, Vh, Uh, dh, dc, groups, grads)
        dh = dhp + (dh_all[t - 1] if t > 0 else 0.0)
    return dx_all, dh, dc, grads


def lowrank_lstm_stack_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """Stacked factorized LSTM layers (the 2-layer language model of Appendix D): layer 0 reads x, layer l > 0
    reads the hidden states of layer l - 1; one layer after the other.  Per-layer arguments are lists.
    Returns lists (h_all, c_all, gates_all, Tx_all, Th_all)."""
    outs = ([], [], [], [], [])
    inp = x
    for l in range(len(Ux)):
        res = lowrank_lstm_seq_fwd(inp, h0[l], c0[l], Vx[l], Ux[l], Vh[l], Uh[l], None if bias is None else bias[l],
                                   groups)
        for lst, v in zip(outs, res):
            lst.append(v)
        inp = res[0]
    return outs


def lowrank_lstm_stack_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all, Vx, Ux, Vh, Uh, dh_top, dhT=None,
                           dcT=None, groups=1):
    """Backward of lowrank_lstm_stack_fwd, the layers taken from the last to the first: the dx_all of layer l
    is the gradient arriving from above at every step of layer l - 1.  dh_top[T,B,h] arrives at the last
    layer.  Returns (dx_all, dh0 list, dc0 list, grads list)."""
    L = len(Ux)
    dh0, dc0, grads = [None] * L, [None] * L, [None] * L
    d_above = dh_top
    for l in range(L - 1, -1, -1):
        inp = x if l == 0 else h_all[l - 1]
        d_above, dh0[l], dc0[l], grads[l] = lowrank_lstm_seq_bwd(
            inp, h0[l], c0[l], h_all[l], c_all[l], gates_all[l], Tx_all[l], Th_all[l], Vx[l], Ux[l], Vh[l], Uh[l],
            d_above, None if dhT is None else dhT[l], None if dcT is None else dcT[l], groups)
    return d_above, dh0, dc0, grads


# ------------------------------------------------------------------- SVD

def svd_split(W, r):
    """Algorithm 1's SVD step: returns (U[m x r], V[n x r], sigma[min(m,n)]),
    U = Ut_r S_r^(1/2), V = Vt_r S_r^(1/2), so U V^T is the rank-r truncation."""
    m, n = W.shape
    W, pW = _in(W)
    U, pU = _out((m, r))
    V, pV = _out((n, r))
    sigma, ps = _out((min(m, n),))
    sweeps = lib().pfo_svd_split(_i64(m), _i64(n), _i64(r), pW, pU, pV, ps)
    if sweeps < 0:
        raise RuntimeError("Jacobi SVD did not converge")
    return U, V, sigma


def svd_split_conv(Wd, r):
    """Section 2.2 / Section 3: unroll Wd[Cout,C,k,k] to [C k^2, Cout] (column =
    one vectorised filter, row index c k^2 + i k + j), split at rank r, reshape
    the factors back to Uk[r,C,k,k] and Vp[Cout,r]."""
    Cout, C, k, _ = Wd.shape
    unrolled = np.ascontiguousarray(Wd.reshape(Cout, C * k * k).T)
    U, V, sigma = svd_split(unrolled, r)
    Uk = np.ascontiguousarray(U.T).reshape(r, C, k, k)
    return Uk, V, sigma
