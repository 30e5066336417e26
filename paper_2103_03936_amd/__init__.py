"""Python binding of libpufferfish.so (HIP kernels for gfx950).

Argument marshalling only: every function takes torch tensors that live on the
GPU, passes their device pointers and torch's current HIP stream through the
C ABI declared in include/pufferfish.h, and returns the output tensors.  torch
is used for device memory and streams; nothing here computes.  There is no
CPU fallback: importing without the built library, or calling with CPU
tensors, raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpufferfish.so")

PF_F32, PF_BF16 = 0, 1
PF_NCHW, PF_NHWC = 0, 1
PF_ACT_NONE, PF_ACT_RELU = 0, 1
_ACT = {None: 0, "none": 0, "relu": 1}


class PfError(RuntimeError):
    pass


class pf_linear_desc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("n_in", ctypes.c_int64), ("n_out", ctypes.c_int64), ("r", ctypes.c_int64),
                ("dtype", ctypes.c_int), ("wgrad_dtype", ctypes.c_int), ("has_bias", ctypes.c_int)]


class pf_linear_shared_desc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("n_in", ctypes.c_int64), ("n_out", ctypes.c_int64), ("r", ctypes.c_int64),
                ("groups", ctypes.c_int), ("dtype", ctypes.c_int), ("has_bias", ctypes.c_int)]


class pf_conv_desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("Cin", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Cout", ctypes.c_int64), ("r", ctypes.c_int64), ("k", ctypes.c_int), ("stride", ctypes.c_int),
                ("pad", ctypes.c_int), ("layout", ctypes.c_int), ("dtype", ctypes.c_int), ("wgrad_dtype", ctypes.c_int)]


class pf_lstm_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("d_in", ctypes.c_int64), ("h", ctypes.c_int64), ("r", ctypes.c_int64),
                ("groups", ctypes.c_int), ("dtype", ctypes.c_int), ("has_bias", ctypes.c_int)]


class pf_lstm_seq_desc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("B", ctypes.c_int64), ("d_in", ctypes.c_int64), ("h", ctypes.c_int64),
                ("r", ctypes.c_int64), ("groups", ctypes.c_int), ("dtype", ctypes.c_int), ("has_bias", ctypes.c_int)]


class pf_lstm_stack_desc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("B", ctypes.c_int64), ("d_in", ctypes.c_int64), ("h", ctypes.c_int64),
                ("r", ctypes.c_int64), ("groups", ctypes.c_int), ("layers", ctypes.c_int), ("dtype", ctypes.c_int),
                ("has_bias", ctypes.c_int)]


class pf_svd_desc(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("r", ctypes.c_int64)]


EXPORTS = [
    "pf_status_string", "pf_last_hip_error", "pf_version",
    "pf_lowrank_linear_fwd_workspace_bytes", "pf_lowrank_linear_bwd_workspace_bytes",
    "pf_lowrank_linear_fwd", "pf_lowrank_linear_bwd", "pf_static_scratch_bytes", "pf_lowrank_linear_bwd_static",
    "pf_lowrank_linear_shared_fwd_workspace_bytes", "pf_lowrank_linear_shared_bwd_workspace_bytes",
    "pf_lowrank_linear_shared_fwd", "pf_lowrank_linear_shared_bwd",
    "pf_lowrank_conv_fwd_workspace_bytes", "pf_lowrank_conv_bwd_workspace_bytes",
    "pf_lowrank_conv_saved_weights_bytes", "pf_lowrank_conv_fwd", "pf_lowrank_conv_bwd",
    "pf_lowrank_linear_fwd_ep", "pf_lowrank_linear_bwd_ep", "pf_lowrank_conv_bwd_ep_workspace_bytes",
    "pf_lowrank_conv_fwd_ep", "pf_lowrank_conv_bwd_ep",
    "pf_lowrank_lstm_cell_fwd_workspace_bytes", "pf_lowrank_lstm_cell_bwd_workspace_bytes",
    "pf_lowrank_lstm_cell_fwd", "pf_lowrank_lstm_cell_bwd",
    "pf_lowrank_lstm_seq_fwd_workspace_bytes", "pf_lowrank_lstm_seq_bwd_workspace_bytes",
    "pf_lowrank_lstm_seq_fwd", "pf_lowrank_lstm_seq_bwd",
    "pf_lowrank_lstm_stack_fwd_workspace_bytes", "pf_lowrank_lstm_stack_bwd_workspace_bytes",
    "pf_lowrank_lstm_stack_fwd", "pf_lowrank_lstm_stack_bwd",
    "pf_svd_split_workspace_bytes", "pf_svd_split",
    "pf_dense_linear_workspace_bytes", "pf_dense_linear_fwd", "pf_dense_linear_bwd",
    "pf_dense_conv_workspace_bytes", "pf_dense_conv_fwd", "pf_dense_conv_bwd",
    "pf_timing_enable", "pf_timing_collect", "pf_timing_entry", "pf_timing_reset",
]

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'); "
        "there is no fallback path")

lib = ctypes.CDLL(LIB_PATH)
lib.pf_status_string.restype = ctypes.c_char_p
for _n in EXPORTS:
    if _n.endswith("_bytes"):  # (size_t results)
        getattr(lib, _n).restype = ctypes.c_size_t


def _check(status, what):
    if status != 0:
        msg = lib.pf_status_string(int(status)).decode()
        raise PfError(f"{what}: status {status} ({msg}), hip error {lib.pf_last_hip_error()}")


def _dtype_code(t):
    if t.dtype == torch.float32:
        return PF_F32
    if t.dtype == torch.bfloat16:
        return PF_BF16
    raise PfError(f"unsupported dtype {t.dtype}")


def _ptr(t, dtype=None, allow_none=True):
    if t is None:
        if not allow_none:
            raise PfError("required tensor is None")
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise PfError("tensors must live on the GPU; there is no CPU path")
    if not t.is_contiguous():
        raise PfError("tensors must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise PfError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_ws_cache = {}
_ws_retired = []  # outgrown buffers: a HIP graph captured earlier may still hold their addresses, so they stay allocated


def _workspace(nbytes, device):
    """A reusable byte buffer of at least nbytes for torch's current stream on `device` (grown, never shrunk).

    One buffer per (device, stream): calls enqueued on one stream are ordered, so they may share scratch memory;
    calls on different streams get different buffers.  A buffer that is outgrown is kept alive rather than freed,
    so graphs captured through these wrappers stay valid when a later call needs more."""
    key = (device.type, device.index, torch.cuda.current_stream(device).cuda_stream)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        if buf is not None:
            _ws_retired.append(buf)
        buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


# ------------------------------------------------------------------ linear

def _linear_desc(X, U, bias_flag):
    M, n_in = X.shape
    n_out, r = U.shape
    return pf_linear_desc(M, n_in, n_out, r, _dtype_code(X), PF_F32, 1 if bias_flag else 0)


def pf_lowrank_linear_fwd(X, V, U, bias=None, save_T=True):
    """Y = (X V) U^T + bias.  Returns (Y, T) with T = X V saved for backward (None if not saved)."""
    d = _linear_desc(X, U, bias is not None)
    dt = X.dtype
    Y = torch.empty((d.M, d.n_out), dtype=dt, device=X.device)
    T = torch.empty((d.M, d.r), dtype=dt, device=X.device) if save_T else None
    n = lib.pf_lowrank_linear_fwd_workspace_bytes(ctypes.byref(d))
    ws = _workspace(n, X.device)
    _check(lib.pf_lowrank_linear_fwd(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(bias, dt),
                                     _ptr(Y), _ptr(T), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "pf_lowrank_linear_fwd")
    return Y, T


def pf_lowrank_linear_bwd(X, V, U, dY, T_saved=None, need_dX=True, has_bias=False, grads=None):
    """Returns (dX, dU, dV, dbias); dU, dV, dbias are float32.  If `grads` = (dU, dV, dbias) is given the
    parameter gradients are accumulated into those tensors."""
    d = _linear_desc(X, U, has_bias)
    dt = X.dtype
    dX = torch.empty_like(X) if need_dX else None
    accumulate = grads is not None
    if grads is None:
        dU = torch.empty((d.n_out, d.r), dtype=torch.float32, device=X.device)
        dV = torch.empty((d.n_in, d.r), dtype=torch.float32, device=X.device)
        db = torch.empty((d.n_out,), dtype=torch.float32, device=X.device) if has_bias else None
    else:
        dU, dV, db = grads
    n = lib.pf_lowrank_linear_bwd_workspace_bytes(ctypes.byref(d))
    ws = _workspace(n, X.device)
    _check(lib.pf_lowrank_linear_bwd(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(dY, dt),
                                     _ptr(T_saved, dt), _ptr(dX), _ptr(dU, torch.float32), _ptr(dV, torch.float32),
                                     _ptr(db, torch.float32), ctypes.c_int(1 if accumulate else 0), _ptr(ws),
                                     ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_linear_bwd")
    return dX, dU, dV, db


def pf_lowrank_linear_bwd_static(X, V, U, dY, T_saved, dX, dU, dV, dbias=None, accumulate=False):
    """pf_lowrank_linear_bwd with the library's own scratch array: no workspace and no allocation, so every output
    tensor is the caller's (dX, dbias nullable).  Raises PfError (workspace status) when the layer needs more scratch
    memory than the library holds."""
    d = _linear_desc(X, U, dbias is not None)
    dt, f32 = X.dtype, torch.float32
    _check(lib.pf_lowrank_linear_bwd_static(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(dY, dt),
                                            _ptr(T_saved, dt), _ptr(dX, dt), _ptr(dU, f32), _ptr(dV, f32),
                                            _ptr(dbias, f32), ctypes.c_int(1 if accumulate else 0), _stream()),
           "pf_lowrank_linear_bwd_static")
    return dX, dU, dV, dbias


def pf_lowrank_linear_fwd_ep(X, V, U, bias=None, residual=None, act="none", save_T=True):
    """Y = act((X V) U^T + bias + residual); returns (Y, T)."""
    d = _linear_desc(X, U, bias is not None)
    dt = X.dtype
    Y = torch.empty((d.M, d.n_out), dtype=dt, device=X.device)
    T = torch.empty((d.M, d.r), dtype=dt, device=X.device) if save_T else None
    ws = _workspace(lib.pf_lowrank_linear_fwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_linear_fwd_ep(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(bias, dt),
                                        _ptr(residual, dt), ctypes.c_int(_ACT[act]), _ptr(Y), _ptr(T), _ptr(ws),
                                        ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_linear_fwd_ep")
    return Y, T


def pf_lowrank_linear_bwd_ep(X, V, U, dZ, T_saved=None, dX_add=None, x_is_relu=False, need_dX=True, has_bias=False,
                             grads=None):
    """From dZ = dL/d(pre-activation): (dX, dU, dV, dbias) with dX = (dZ U V^T + dX_add) * [X > 0 if x_is_relu]."""
    d = _linear_desc(X, U, has_bias)
    dt, f32 = X.dtype, torch.float32
    dX = torch.empty_like(X) if need_dX else None
    accumulate = grads is not None
    if grads is None:
        dU = torch.empty((d.n_out, d.r), dtype=f32, device=X.device)
        dV = torch.empty((d.n_in, d.r), dtype=f32, device=X.device)
        db = torch.empty((d.n_out,), dtype=f32, device=X.device) if has_bias else None
    else:
        dU, dV, db = grads
    ws = _workspace(lib.pf_lowrank_linear_bwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_linear_bwd_ep(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(dZ, dt),
                                        _ptr(T_saved, dt), _ptr(dX_add, dt), ctypes.c_int(1 if x_is_relu else 0),
                                        _ptr(dX), _ptr(dU, f32), _ptr(dV, f32), _ptr(db, f32),
                                        ctypes.c_int(1 if accumulate else 0), _ptr(ws), ctypes.c_size_t(ws.numel()),
                                        _stream()), "pf_lowrank_linear_bwd_ep")
    return dX, dU, dV, db


def _shared_desc(X, U, bias_flag):
    M, n_in = X.shape
    G, n_out, r = U.shape
    return pf_linear_shared_desc(M, n_in, n_out, r, G, _dtype_code(X), 1 if bias_flag else 0)


def pf_lowrank_linear_shared_fwd(X, V, U, bias=None, save_T=True):
    """G projections of one input (Q, K, V of attention): X[M,in], V[G,in,r], U[G,out,r], bias[G,out] -> (Y[G,M,out],
    T[G,M,r])."""
    d = _shared_desc(X, U, bias is not None)
    dt = X.dtype
    Y = torch.empty((d.groups, d.M, d.n_out), dtype=dt, device=X.device)
    T = torch.empty((d.groups, d.M, d.r), dtype=dt, device=X.device) if save_T else None
    ws = _workspace(lib.pf_lowrank_linear_shared_fwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_linear_shared_fwd(ctypes.byref(d), _ptr(X), _ptr(V, dt), _ptr(U, dt), _ptr(bias, dt), _ptr(Y),
                                            _ptr(T), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "pf_lowrank_linear_shared_fwd")
    return Y, T


def pf_lowrank_linear_shared_bwd(X, V, U, dY, T_saved=None, need_dX=True, has_bias=False, grads=None):
    """dY[G,M,out] -> (dX[M,in] summed over the projections, dU[G,out,r], dV[G,in,r], dbias[G,out]); the parameter
    gradients are float32 and accumulate into `grads` = (dU, dV, dbias) when given."""
    d = _shared_desc(X, U, has_bias)
    dt = X.dtype
    f32 = torch.float32
    dX = torch.empty_like(X) if need_dX else None
    accumulate = grads is not None
    if grads is None:
        dU = torch.empty(U.shape, dtype=f32, device=X.device)
        dV = torch.empty(V.shape, dtype=f32, device=X.device)
        db = torch.empty((d.groups, d.n_out), dtype=f32, device=X.device) if has_bias else None
    else:
        dU, dV, db = grads
    ws = _workspace(lib.pf_lowrank_linear_shared_bwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_linear_shared_bwd(ctypes.byref(d), _ptr(X, dt), _ptr(V, dt), _ptr(U, dt), _ptr(dY, dt),
                                            _ptr(T_saved, dt), _ptr(dX), _ptr(dU, f32), _ptr(dV, f32), _ptr(db, f32),
                                            ctypes.c_int(1 if accumulate else 0), _ptr(ws),
                                            ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_linear_shared_bwd")
    return dX, dU, dV, db


def pf_dense_linear_fwd(X, W, bias=None):
    M, n_in = X.shape
    n_out = W.shape[0]
    d = pf_linear_desc(M, n_in, n_out, 1, _dtype_code(X), PF_F32, 1 if bias is not None else 0)
    Y = torch.empty((M, n_out), dtype=X.dtype, device=X.device)
    ws = _workspace(256, X.device)
    _check(lib.pf_dense_linear_fwd(ctypes.byref(d), _ptr(X), _ptr(W, X.dtype), _ptr(bias, X.dtype), _ptr(Y),
                                   _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()), "pf_dense_linear_fwd")
    return Y


def pf_dense_linear_bwd(X, W, dY, has_bias=False):
    M, n_in = X.shape
    n_out = W.shape[0]
    d = pf_linear_desc(M, n_in, n_out, 1, _dtype_code(X), PF_F32, 1 if has_bias else 0)
    dX = torch.empty_like(X)
    dW = torch.empty((n_out, n_in), dtype=torch.float32, device=X.device)
    db = torch.empty((n_out,), dtype=torch.float32, device=X.device) if has_bias else None
    ws = _workspace(lib.pf_dense_linear_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_dense_linear_bwd(ctypes.byref(d), _ptr(X), _ptr(W, X.dtype), _ptr(dY, X.dtype), _ptr(dX),
                                   _ptr(dW), _ptr(db), ctypes.c_int(0), _ptr(ws), ctypes.c_size_t(ws.numel()),
                                   _stream()), "pf_dense_linear_bwd")
    return dX, dW, db


# -------------------------------------------------------------------- conv

def _conv_desc(X, Uk, Vp, stride, pad):
    N, C, H, W = X.shape
    r, _, k, _ = Uk.shape
    return pf_conv_desc(N, C, H, W, Vp.shape[0], r, k, stride, pad, PF_NCHW, _dtype_code(X), PF_F32)


def conv_out_hw(d):
    return (d.H + 2 * d.pad - d.k) // d.stride + 1, (d.W + 2 * d.pad - d.k) // d.stride + 1


def pf_lowrank_conv_fwd(X, Uk, Vp, stride=1, pad=0, save_T=True, save_W=False):
    """Thin k x k conv (Uk[r,C,k,k]) then 1x1 conv (Vp[Cout,r]).  Returns (Y, T), or (Y, T, W) with
    save_W: W holds the factors as the backward kernels read them (None when they read them in place)."""
    d = _conv_desc(X, Uk, Vp, stride, pad)
    Ho, Wo = conv_out_hw(d)
    dt = X.dtype
    Y = torch.empty((d.N, d.Cout, Ho, Wo), dtype=dt, device=X.device)
    T = torch.empty((d.N, d.r, Ho, Wo), dtype=dt, device=X.device) if save_T else None
    nW = lib.pf_lowrank_conv_saved_weights_bytes(ctypes.byref(d)) if save_W else 0
    Wsv = torch.empty((nW,), dtype=torch.uint8, device=X.device) if nW else None
    ws = _workspace(lib.pf_lowrank_conv_fwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_conv_fwd(ctypes.byref(d), _ptr(X), _ptr(Uk, dt), _ptr(Vp, dt), _ptr(Y), _ptr(T),
                                   _ptr(Wsv), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "pf_lowrank_conv_fwd")
    return (Y, T, Wsv) if save_W else (Y, T)


def pf_lowrank_conv_bwd(X, Uk, Vp, dY, T_saved=None, stride=1, pad=0, need_dX=True, grads=None, W_saved=None):
    """Returns (dX, dUk, dVp); dUk, dVp are float32 (accumulated into `grads` = (dUk, dVp) if given)."""
    d = _conv_desc(X, Uk, Vp, stride, pad)
    dt = X.dtype
    dX = torch.empty_like(X) if need_dX else None
    accumulate = grads is not None
    if grads is None:
        dUk = torch.empty(Uk.shape, dtype=torch.float32, device=X.device)
        dVp = torch.empty(Vp.shape, dtype=torch.float32, device=X.device)
    else:
        dUk, dVp = grads
    ws = _workspace(lib.pf_lowrank_conv_bwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_conv_bwd(ctypes.byref(d), _ptr(X), _ptr(Uk, dt), _ptr(Vp, dt), _ptr(dY, dt),
                                   _ptr(T_saved, dt), _ptr(W_saved), _ptr(dX), _ptr(dUk, torch.float32),
                                   _ptr(dVp, torch.float32), ctypes.c_int(1 if accumulate else 0), _ptr(ws),
                                   ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_conv_bwd")
    return dX, dUk, dVp


def pf_lowrank_conv_fwd_ep(X, Uk, Vp, scale=None, shift=None, residual=None, act="none", stride=1, pad=0, save_T=True,
                           save_W=False):
    """Y = act(scale[o] (Vp * (Uk * X)) + shift[o] + residual); scale, shift float32 [Cout].  Returns (Y, T) or
    (Y, T, W_save)."""
    d = _conv_desc(X, Uk, Vp, stride, pad)
    dt, f32 = X.dtype, torch.float32
    Ho, Wo = conv_out_hw(d)
    Y = torch.empty((d.N, d.Cout, Ho, Wo), dtype=dt, device=X.device)
    T = torch.empty((d.N, d.r, Ho, Wo), dtype=dt, device=X.device) if save_T else None
    nW = lib.pf_lowrank_conv_saved_weights_bytes(ctypes.byref(d)) if save_W else 0
    Wsv = torch.empty((nW,), dtype=torch.uint8, device=X.device) if nW else None
    ws = _workspace(lib.pf_lowrank_conv_fwd_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_conv_fwd_ep(ctypes.byref(d), _ptr(X), _ptr(Uk, dt), _ptr(Vp, dt), _ptr(scale, f32),
                                      _ptr(shift, f32), _ptr(residual, dt), ctypes.c_int(_ACT[act]), _ptr(Y), _ptr(T),
                                      _ptr(Wsv), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "pf_lowrank_conv_fwd_ep")
    return (Y, T, Wsv) if save_W else (Y, T)


def pf_lowrank_conv_bwd_ep(X, Uk, Vp, scale, dZ, T_saved=None, stride=1, pad=0, dX_add=None, x_is_relu=False,
                           need_dX=True, need_dshift=True, grads=None, W_saved=None):
    """From dZ = dL/d(pre-activation): (dX, dUk, dVp, dshift), dX = (conv^T(dT) + dX_add) * [X > 0 if x_is_relu];
    `grads` = (dUk, dVp, dshift) accumulates."""
    d = _conv_desc(X, Uk, Vp, stride, pad)
    dt, f32 = X.dtype, torch.float32
    dX = torch.empty_like(X) if need_dX else None
    accumulate = grads is not None
    if grads is None:
        dUk = torch.empty(Uk.shape, dtype=f32, device=X.device)
        dVp = torch.empty(Vp.shape, dtype=f32, device=X.device)
        dsh = torch.empty((d.Cout,), dtype=f32, device=X.device) if need_dshift else None
    else:
        dUk, dVp, dsh = grads
    ws = _workspace(lib.pf_lowrank_conv_bwd_ep_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_lowrank_conv_bwd_ep(ctypes.byref(d), _ptr(X), _ptr(Uk, dt), _ptr(Vp, dt), _ptr(scale, f32),
                                      _ptr(dZ, dt), _ptr(T_saved, dt), _ptr(W_saved), _ptr(dX_add, dt),
                                      ctypes.c_int(1 if x_is_relu else 0), _ptr(dX), _ptr(dUk, f32), _ptr(dVp, f32),
                                      _ptr(dsh, f32), ctypes.c_int(1 if accumulate else 0), _ptr(ws),
                                      ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_conv_bwd_ep")
    return dX, dUk, dVp, dsh


def pf_dense_conv_fwd(X, Wd, stride=1, pad=0):
    N, C, H, W = X.shape
    Cout, _, k, _ = Wd.shape
    d = pf_conv_desc(N, C, H, W, Cout, 1, k, stride, pad, PF_NCHW, _dtype_code(X), PF_F32)
    Ho, Wo = conv_out_hw(d)
    Y = torch.empty((N, Cout, Ho, Wo), dtype=X.dtype, device=X.device)
    ws = _workspace(lib.pf_dense_conv_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_dense_conv_fwd(ctypes.byref(d), _ptr(X), _ptr(Wd, X.dtype), _ptr(Y), _ptr(ws),
                                 ctypes.c_size_t(ws.numel()), _stream()), "pf_dense_conv_fwd")
    return Y


def pf_dense_conv_bwd(X, Wd, dY, stride=1, pad=0):
    N, C, H, W = X.shape
    Cout, _, k, _ = Wd.shape
    d = pf_conv_desc(N, C, H, W, Cout, 1, k, stride, pad, PF_NCHW, _dtype_code(X), PF_F32)
    dX = torch.empty_like(X)
    dW = torch.empty(Wd.shape, dtype=torch.float32, device=X.device)
    ws = _workspace(lib.pf_dense_conv_workspace_bytes(ctypes.byref(d)), X.device)
    _check(lib.pf_dense_conv_bwd(ctypes.byref(d), _ptr(X), _ptr(Wd, X.dtype), _ptr(dY, X.dtype), _ptr(dX), _ptr(dW),
                                 ctypes.c_int(0), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "pf_dense_conv_bwd")
    return dX, dW


# -------------------------------------------------------------------- LSTM

def _lstm_desc(x, h_prev, Ux, groups, has_bias):
    B, d_in = x.shape
    return pf_lstm_desc(B, d_in, h_prev.shape[1], Ux.shape[1], groups, _dtype_code(x), 1 if has_bias else 0)


def pf_lowrank_lstm_cell_fwd(x, h_prev, c_prev, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """One factorized LSTM step.  Returns (h, c, gates, Tx, Th); the last three are saved for backward."""
    d = _lstm_desc(x, h_prev, Ux, groups, bias is not None)
    f32 = torch.float32
    dev = x.device
    h_out = torch.empty((d.B, d.h), dtype=f32, device=dev)
    c_out = torch.empty((d.B, d.h), dtype=f32, device=dev)
    gates = torch.empty((d.B, 4 * d.h), dtype=f32, device=dev)
    Tx = torch.empty((d.B, groups * d.r), dtype=f32, device=dev)
    Th = torch.empty((d.B, groups * d.r), dtype=f32, device=dev)
    ws = _workspace(lib.pf_lowrank_lstm_cell_fwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_cell_fwd(ctypes.byref(d), _ptr(x, f32), _ptr(h_prev, f32), _ptr(c_prev, f32),
                                        _ptr(Vx, f32), _ptr(Ux, f32), _ptr(Vh, f32), _ptr(Uh, f32), _ptr(bias, f32),
                                        _ptr(h_out), _ptr(c_out), _ptr(gates), _ptr(Tx), _ptr(Th), _ptr(ws),
                                        ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_lstm_cell_fwd")
    return h_out, c_out, gates, Tx, Th


def pf_lowrank_lstm_cell_bwd(x, h_prev, c_prev, c_out, gates, Tx, Th, Vx, Ux, Vh, Uh, dh, dc_next=None, groups=1,
                             need_dx=True, grads=None):
    """One BPTT step.  Returns (dx, dh_prev, dc_prev, grads) with grads = dict(dVx, dUx, dVh, dUh, dbias) in
    float32; if `grads` is given the parameter gradients are accumulated into it."""
    d = _lstm_desc(x, h_prev, Ux, groups, True)
    f32 = torch.float32
    dev = x.device
    dx = torch.empty_like(x) if need_dx else None
    dh_prev = torch.empty_like(h_prev)
    dc_prev = torch.empty_like(c_prev)
    accumulate = grads is not None
    if grads is None:
        grads = dict(dVx=torch.empty_like(Vx), dUx=torch.empty_like(Ux), dVh=torch.empty_like(Vh),
                     dUh=torch.empty_like(Uh), dbias=torch.empty((4 * d.h,), dtype=f32, device=dev))
    ws = _workspace(lib.pf_lowrank_lstm_cell_bwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_cell_bwd(
        ctypes.byref(d), _ptr(x, f32), _ptr(h_prev, f32), _ptr(c_prev, f32), _ptr(c_out, f32), _ptr(gates, f32),
        _ptr(Tx, f32), _ptr(Th, f32), _ptr(Vx, f32), _ptr(Ux, f32), _ptr(Vh, f32), _ptr(Uh, f32), _ptr(dh, f32),
        _ptr(dc_next, f32), _ptr(dx), _ptr(dh_prev), _ptr(dc_prev), _ptr(grads["dVx"], f32), _ptr(grads["dUx"], f32),
        _ptr(grads["dVh"], f32), _ptr(grads["dUh"], f32), _ptr(grads["dbias"], f32),
        ctypes.c_int(1 if accumulate else 0), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()),
        "pf_lowrank_lstm_cell_bwd")
    return dx, dh_prev, dc_prev, grads


def _lstm_seq_desc(x, h0, Ux, groups, has_bias):
    T, B, d_in = x.shape
    return pf_lstm_seq_desc(T, B, d_in, h0.shape[1], Ux.shape[1], groups, _dtype_code(x), 1 if has_bias else 0)


def pf_lowrank_lstm_seq_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """One factorized LSTM layer over a sequence x[T,B,d].  Returns (h_all, c_all, gates_all, Tx_all, Th_all)."""
    d = _lstm_seq_desc(x, h0, Ux, groups, bias is not None)
    f32 = torch.float32
    dev = x.device
    h_all = torch.empty((d.T, d.B, d.h), dtype=f32, device=dev)
    c_all = torch.empty((d.T, d.B, d.h), dtype=f32, device=dev)
    gates_all = torch.empty((d.T, d.B, 4 * d.h), dtype=f32, device=dev)
    Tx_all = torch.empty((d.T, d.B, groups * d.r), dtype=f32, device=dev)
    Th_all = torch.empty((d.T, d.B, groups * d.r), dtype=f32, device=dev)
    ws = _workspace(lib.pf_lowrank_lstm_seq_fwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_seq_fwd(ctypes.byref(d), _ptr(x, f32), _ptr(h0, f32), _ptr(c0, f32), _ptr(Vx, f32),
                                       _ptr(Ux, f32), _ptr(Vh, f32), _ptr(Uh, f32), _ptr(bias, f32), _ptr(h_all),
                                       _ptr(c_all), _ptr(gates_all), _ptr(Tx_all), _ptr(Th_all), _ptr(ws),
                                       ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_lstm_seq_fwd")
    return h_all, c_all, gates_all, Tx_all, Th_all


def pf_lowrank_lstm_seq_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all, Vx, Ux, Vh, Uh, dh_all, dhT=None,
                            dcT=None, groups=1, need_dx=True, grads=None):
    """Back-propagation through time.  Returns (dx_all, dh0, dc0, grads); if `grads` is given the parameter
    gradients are accumulated into it."""
    d = _lstm_seq_desc(x, h0, Ux, groups, True)
    f32 = torch.float32
    dev = x.device
    dx_all = torch.empty_like(x) if need_dx else None
    dh0 = torch.empty_like(h0)
    dc0 = torch.empty_like(c0)
    accumulate = grads is not None
    if grads is None:
        grads = dict(dVx=torch.empty_like(Vx), dUx=torch.empty_like(Ux), dVh=torch.empty_like(Vh),
                     dUh=torch.empty_like(Uh), dbias=torch.empty((4 * d.h,), dtype=f32, device=dev))
    ws = _workspace(lib.pf_lowrank_lstm_seq_bwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_seq_bwd(
        ctypes.byref(d), _ptr(x, f32), _ptr(h0, f32), _ptr(c0, f32), _ptr(h_all, f32), _ptr(c_all, f32),
        _ptr(gates_all, f32), _ptr(Tx_all, f32), _ptr(Th_all, f32), _ptr(Vx, f32), _ptr(Ux, f32), _ptr(Vh, f32),
        _ptr(Uh, f32), _ptr(dh_all, f32), _ptr(dhT, f32), _ptr(dcT, f32), _ptr(dx_all), _ptr(dh0), _ptr(dc0),
        _ptr(grads["dVx"], f32), _ptr(grads["dUx"], f32), _ptr(grads["dVh"], f32), _ptr(grads["dUh"], f32),
        _ptr(grads["dbias"], f32), ctypes.c_int(1 if accumulate else 0), _ptr(ws), ctypes.c_size_t(ws.numel()),
        _stream()), "pf_lowrank_lstm_seq_bwd")
    return dx_all, dh0, dc0, grads


def _ptr_array(ts, dtype=None):
    """A host array of device pointers, one per layer (None: a NULL array)."""
    if ts is None:
        return None
    return (ctypes.c_void_p * len(ts))(*[_ptr(t, dtype).value for t in ts])


def _lstm_stack_desc(x, h0, Ux, groups, has_bias):
    T, B, d_in = x.shape
    return pf_lstm_stack_desc(T, B, d_in, h0[0].shape[1], Ux[0].shape[1], groups, len(Ux), _dtype_code(x),
                              1 if has_bias else 0)


def pf_lowrank_lstm_stack_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bias=None, groups=1):
    """A stack of factorized LSTM layers over a sequence x[T,B,d]; h0, c0, Vx, Ux, Vh, Uh, bias are lists with one
    tensor per layer.  Returns lists (h_all, c_all, gates_all, Tx_all, Th_all), one tensor per layer."""
    d = _lstm_stack_desc(x, h0, Ux, groups, bias is not None)
    f32 = torch.float32
    dev = x.device
    L = d.layers
    new = lambda n: [torch.empty((d.T, d.B, n), dtype=f32, device=dev) for _ in range(L)]
    h_all, c_all, gates_all = new(d.h), new(d.h), new(4 * d.h)
    Tx_all, Th_all = new(groups * d.r), new(groups * d.r)
    ws = _workspace(lib.pf_lowrank_lstm_stack_fwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_stack_fwd(
        ctypes.byref(d), _ptr(x, f32), _ptr_array(h0, f32), _ptr_array(c0, f32), _ptr_array(Vx, f32),
        _ptr_array(Ux, f32), _ptr_array(Vh, f32), _ptr_array(Uh, f32), _ptr_array(bias, f32), _ptr_array(h_all),
        _ptr_array(c_all), _ptr_array(gates_all), _ptr_array(Tx_all), _ptr_array(Th_all), _ptr(ws),
        ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_lstm_stack_fwd")
    return h_all, c_all, gates_all, Tx_all, Th_all


def pf_lowrank_lstm_stack_bwd(x, h0, c0, h_all, c_all, gates_all, Tx_all, Th_all, Vx, Ux, Vh, Uh, dh_top, dhT=None,
                              dcT=None, groups=1, need_dx=True, grads=None):
    """Back-propagation through time and depth.  dh_top[T,B,h] arrives at the last layer; dhT, dcT: optional
    lists (entries may be None).  Returns (dx_all, dh0, dc0, grads) with dh0, dc0 lists and grads a list of dicts
    per layer; if `grads` is given the parameter gradients are accumulated into it."""
    d = _lstm_stack_desc(x, h0, Ux, groups, True)
    f32 = torch.float32
    dev = x.device
    L = d.layers
    dx_all = torch.empty_like(x) if need_dx else None
    dh0 = [torch.empty_like(t) for t in h0]
    dc0 = [torch.empty_like(t) for t in c0]
    accumulate = grads is not None
    if grads is None:
        grads = [dict(dVx=torch.empty_like(Vx[l]), dUx=torch.empty_like(Ux[l]), dVh=torch.empty_like(Vh[l]),
                      dUh=torch.empty_like(Uh[l]), dbias=torch.empty((4 * d.h,), dtype=f32, device=dev))
                 for l in range(L)]
    col = lambda k: _ptr_array([g[k] for g in grads], f32)
    ws = _workspace(lib.pf_lowrank_lstm_stack_bwd_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_lowrank_lstm_stack_bwd(
        ctypes.byref(d), _ptr(x, f32), _ptr_array(h0, f32), _ptr_array(c0, f32), _ptr_array(h_all, f32),
        _ptr_array(c_all, f32), _ptr_array(gates_all, f32), _ptr_array(Tx_all, f32), _ptr_array(Th_all, f32),
        _ptr_array(Vx, f32), _ptr_array(Ux, f32), _ptr_array(Vh, f32), _ptr_array(Uh, f32), _ptr(dh_top, f32),
        _ptr_array(dhT, f32), _ptr_array(dcT, f32), _ptr(dx_all), _ptr_array(dh0), _ptr_array(dc0), col("dVx"),
        col("dUx"), col("dVh"), col("dUh"), col("dbias"), ctypes.c_int(1 if accumulate else 0), _ptr(ws),
        ctypes.c_size_t(ws.numel()), _stream()), "pf_lowrank_lstm_stack_bwd")
    return dx_all, dh0, dc0, grads


def pf_svd_split(W, r, return_info=False):
    """Algorithm 1's factor initialisation: W[m, n] float32 -> (U[m, r], V[n, r], sigma[min(m, n)]) with
    U V^T the best rank-r approximation of W and the singular values split evenly between the factors.
    With return_info also the int32 device tensor [sweeps run, rotations in the last sweep (0 = converged)]."""
    if W.dtype != torch.float32 or W.dim() != 2:
        raise PfError("pf_svd_split takes a 2-D float32 matrix")
    W = W.contiguous()
    m, n = W.shape
    d = pf_svd_desc(m, n, r)
    dev = W.device
    U = torch.empty((m, r), dtype=torch.float32, device=dev)
    V = torch.empty((n, r), dtype=torch.float32, device=dev)
    sigma = torch.empty((min(m, n),), dtype=torch.float32, device=dev)
    info = torch.empty((2,), dtype=torch.int32, device=dev) if return_info else None
    ws = _workspace(lib.pf_svd_split_workspace_bytes(ctypes.byref(d)), dev)
    _check(lib.pf_svd_split(ctypes.byref(d), _ptr(W), _ptr(U), _ptr(V), _ptr(sigma), _ptr(info), _ptr(ws),
                            ctypes.c_size_t(ws.numel()), _stream()), "pf_svd_split")
    return (U, V, sigma, info) if return_info else (U, V, sigma)


def pf_svd_split_conv(Wd, r):
    """A dense filter bank Wd[c_out, c_in, k, k] -> (Uk[r, c_in, k, k], Vp[c_out, r]) (Section 2.2: unroll to
    [c_in k^2, c_out], factor, fold the left factor back into r thin filters)."""
    co, ci, k, _ = Wd.shape
    Wu = Wd.reshape(co, ci * k * k).t().contiguous()  # [c_in k^2, c_out], row index c k^2 + i k + j
    U, V, sigma = pf_svd_split(Wu, r)
    return U.t().contiguous().reshape(r, ci, k, k), V.contiguous(), sigma


# ------------------------------------------------------------------ timing

class GradBuffer:
    """One flat float32 device buffer that holds every parameter gradient of a model back to back, in the order
    the entries are given (paper Section 4, implementation details: all gradient tensors are packed into one
    flat buffer so that a single all-reduce sums them).  Nothing is copied: `views[name]` are slices of `flat`
    to pass as `grads=` to the backward calls, which then write (after `zero()`: accumulate) in place.  Gradient
    outputs need only 4-byte alignment, so no padding goes between the entries."""

    def __init__(self, entries, device="cuda"):
        self.offsets = {}
        n = 0
        for name, shape in entries:
            self.offsets[name] = (n, tuple(shape))
            n += int(torch.Size(shape).numel())
        self.flat = torch.empty((n,), dtype=torch.float32, device=device)
        self.views = {name: self.flat[o:o + int(torch.Size(sh).numel())].view(sh)
                      for name, (o, sh) in self.offsets.items()}

    def zero(self):
        self.flat.zero_()
        return self


def timing_enable(on=True):
    lib.pf_timing_enable(ctypes.c_int(1 if on else 0))


def timing_reset():
    lib.pf_timing_reset()


def timing_collect():
    """{kernel name: (launches, total_ms)} of everything recorded while timing was enabled."""
    n = lib.pf_timing_collect()
    out = {}
    for i in range(n):
        name = ctypes.c_char_p()
        launches = ctypes.c_int64()
        ms = ctypes.c_double()
        lib.pf_timing_entry(ctypes.c_int(i), ctypes.byref(name), ctypes.byref(launches), ctypes.byref(ms))
        out[name.value.decode()] = (int(launches.value), float(ms.value))
    return out
