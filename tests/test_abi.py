"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import paper_2103_03936_amd as pf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = ctypes.c_void_p
FAKE = P(256)  # never dereferenced: validation fails before any launch in these calls


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pufferfish.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pf_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert len(names) >= 25
    for n in names:
        assert hasattr(pf.lib, n), n
    assert set(names) == set(pf.EXPORTS)


def test_status_strings():
    assert pf.lib.pf_status_string(0) == b"ok"
    for s in range(1, 6):
        assert len(pf.lib.pf_status_string(s)) > 3
    assert pf.lib.pf_version() >= 1


def _lin(M=4, n_in=5, n_out=3, r=2, dtype=0, bias=0, wgrad_dtype=0):
    return pf.pf_linear_desc(M, n_in, n_out, r, dtype, wgrad_dtype, bias)


def test_linear_validation():
    f = pf.lib.pf_lowrank_linear_fwd
    z = ctypes.c_size_t(0)
    assert f(None, FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 1
    assert f(ctypes.byref(_lin(n_in=0)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(ctypes.byref(_lin(r=-1)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(ctypes.byref(_lin(M=-1)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(ctypes.byref(_lin(dtype=7)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 3
    # parameter gradients come as float only
    assert f(ctypes.byref(_lin(wgrad_dtype=1)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 3
    assert pf.lib.pf_lowrank_linear_bwd(ctypes.byref(_lin(dtype=1, wgrad_dtype=1)), FAKE, FAKE, FAKE, FAKE, None, FAKE,
                                        FAKE, FAKE, None, 0, FAKE, ctypes.c_size_t(1 << 30), None) == 3
    assert f(ctypes.byref(_lin()), None, FAKE, FAKE, None, FAKE, None, None, z, None) == 1
    assert f(ctypes.byref(_lin(bias=1)), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 1
    # workspace too small / missing
    d = _lin()
    need = pf.lib.pf_lowrank_linear_fwd_workspace_bytes(ctypes.byref(d))
    if need:
        assert f(ctypes.byref(d), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 4
        assert f(ctypes.byref(d), FAKE, FAKE, FAKE, None, FAKE, None, FAKE, ctypes.c_size_t(need - 1), None) == 4
    # an empty batch is legal and launches nothing
    assert f(ctypes.byref(_lin(M=0)), None, FAKE, FAKE, None, None, None, None, z, None) == 0
    b = pf.lib.pf_lowrank_linear_bwd
    assert b(ctypes.byref(_lin()), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, None, 0, None, z, None) == 1
    assert b(ctypes.byref(_lin()), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, 0, None, z, None) == 4
    # activations and factors 16-byte aligned, parameter gradients 4-byte aligned
    odd, odd2 = P(256 + 4), P(256 + 2)
    assert f(ctypes.byref(_lin()), odd, FAKE, FAKE, None, FAKE, None, None, z, None) == 3
    assert b(ctypes.byref(_lin()), FAKE, FAKE, odd, FAKE, None, FAKE, FAKE, FAKE, None, 0, None, z, None) == 3
    assert b(ctypes.byref(_lin()), FAKE, FAKE, FAKE, FAKE, None, FAKE, odd2, FAKE, None, 0, None, z, None) == 3
    assert b(ctypes.byref(_lin()), FAKE, FAKE, FAKE, FAKE, None, FAKE, odd, odd, None, 0, None, z, None) == 4
    assert b(ctypes.byref(_lin()), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, 0, P(256 + 16),
             ctypes.c_size_t(1 << 30), None) == 3  # workspace not 256-byte aligned
    # full rank and beyond is legal
    assert pf.lib.pf_lowrank_linear_fwd_workspace_bytes(ctypes.byref(_lin(r=64))) >= 0


def test_linear_shared_validation():
    f = pf.lib.pf_lowrank_linear_shared_fwd
    b = pf.lib.pf_lowrank_linear_shared_bwd
    z = ctypes.c_size_t(0)

    def d(M=4, n_in=5, n_out=3, r=2, G=3, dtype=0, bias=0):
        return ctypes.byref(pf.pf_linear_shared_desc(M, n_in, n_out, r, G, dtype, bias))

    assert f(None, FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 1
    assert f(d(G=0), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(d(G=65), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(d(n_out=0), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 2
    assert f(d(dtype=4), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 3
    assert f(d(bias=1), FAKE, FAKE, FAKE, None, FAKE, None, None, z, None) == 1
    assert f(d(), P(260), FAKE, FAKE, None, FAKE, None, None, z, None) == 3
    assert f(d(M=0), None, FAKE, FAKE, None, None, None, None, z, None) == 0
    assert b(d(), FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, None, 0, FAKE, z, None) == 1
    assert b(d(), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, 0, None, z, None) == 4
    need = pf.lib.pf_lowrank_linear_shared_bwd_workspace_bytes(d())
    assert need > pf.lib.pf_lowrank_linear_bwd_workspace_bytes(ctypes.byref(_lin()))
    assert b(d(), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, 0, FAKE, ctypes.c_size_t(need - 1), None) == 4


def _conv(N=2, C=3, H=5, W=5, Cout=4, r=2, k=3, s=1, p=1, dtype=0, layout=0, wgrad_dtype=0):
    return pf.pf_conv_desc(N, C, H, W, Cout, r, k, s, p, layout, dtype, wgrad_dtype)


def test_conv_validation():
    f = pf.lib.pf_lowrank_conv_fwd
    z = ctypes.c_size_t(0)
    assert f(None, FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 1
    assert f(ctypes.byref(_conv(C=0)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 2
    assert f(ctypes.byref(_conv(s=0)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 2
    assert f(ctypes.byref(_conv(H=2, W=2, k=5, p=0)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 2
    assert f(ctypes.byref(_conv(dtype=9)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 3
    # NCHW activations and float filter gradients are what is built
    assert f(ctypes.byref(_conv(layout=pf.PF_NHWC)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 3
    assert f(ctypes.byref(_conv(wgrad_dtype=pf.PF_BF16)), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 3
    assert pf.lib.pf_lowrank_conv_bwd(ctypes.byref(_conv(layout=1)), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE,
                                      0, FAKE, ctypes.c_size_t(1 << 30), None) == 3
    assert f(ctypes.byref(_conv()), FAKE, None, FAKE, FAKE, None, None, None, z, None) == 1
    d = _conv()
    need = pf.lib.pf_lowrank_conv_fwd_workspace_bytes(ctypes.byref(d))
    if need:
        assert f(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, None, None, None, z, None) == 4
    assert f(ctypes.byref(_conv(N=0)), None, FAKE, FAKE, None, None, None, None, z, None) == 0
    b = pf.lib.pf_lowrank_conv_bwd
    assert b(ctypes.byref(_conv()), FAKE, FAKE, FAKE, None, None, None, FAKE, FAKE, FAKE, 0, None, z, None) == 1
    assert b(ctypes.byref(_conv()), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, 0, None, z, None) == 4
    # the saved-weights buffer exists for the fused bf16 path only
    assert pf.lib.pf_lowrank_conv_saved_weights_bytes(ctypes.byref(_conv())) == 0
    fused = _conv(N=4, C=256, H=8, W=8, Cout=256, r=64, dtype=1)
    assert pf.lib.pf_lowrank_conv_saved_weights_bytes(ctypes.byref(fused)) == 2 * (256 * 64 + 9 * 256 * 64)
    assert f(ctypes.byref(fused), FAKE, FAKE, FAKE, FAKE, None, P(256 + 8), None, z, None) == 3


def _lstm(B=2, d=3, h=4, r=2, groups=1, dtype=0, bias=1):
    return pf.pf_lstm_desc(B, d, h, r, groups, dtype, bias)


def test_lstm_validation():
    f = pf.lib.pf_lowrank_lstm_cell_fwd
    z = ctypes.c_size_t(0)
    args = [FAKE] * 13
    assert f(None, *args, None, z, None) == 1
    assert f(ctypes.byref(_lstm(groups=2)), *args, None, z, None) == 3
    assert f(ctypes.byref(_lstm(dtype=1)), *args, None, z, None) == 3
    assert f(ctypes.byref(_lstm(h=0)), *args, None, z, None) == 2
    bad = list(args)
    bad[3] = None  # Vx
    assert f(ctypes.byref(_lstm()), *bad, None, z, None) == 1
    assert f(ctypes.byref(_lstm()), *args, None, z, None) == 4
    assert f(ctypes.byref(_lstm(B=0)), *args, None, z, None) == 0


def test_lstm_seq_validation():
    f = pf.lib.pf_lowrank_lstm_seq_fwd
    z = ctypes.c_size_t(0)
    args = [FAKE] * 13
    mk = lambda T=3, B=2, d=8, h=8, r=4, groups=1, dtype=0, bias=1: pf.pf_lstm_seq_desc(T, B, d, h, r, groups, dtype, bias)
    assert f(None, *args, None, z, None) == 1
    assert f(ctypes.byref(mk(groups=3)), *args, None, z, None) == 3
    assert f(ctypes.byref(mk(T=-1)), *args, None, z, None) == 2
    assert f(ctypes.byref(mk(B=40)), *args, None, z, None) == 3  # built for small batches
    assert f(ctypes.byref(mk()), *args, None, z, None) == 4      # workspace missing
    assert f(ctypes.byref(mk(T=0)), *args, None, z, None) == 0
    ws = pf.lib.pf_lowrank_lstm_seq_bwd_workspace_bytes(ctypes.byref(mk()))
    assert ws > 0


def test_lstm_stack_validation():
    f = pf.lib.pf_lowrank_lstm_stack_fwd
    z = ctypes.c_size_t(0)
    mk = lambda T=3, B=2, d=8, h=8, r=4, groups=1, layers=2, dtype=0, bias=1: pf.pf_lstm_stack_desc(
        T, B, d, h, r, groups, layers, dtype, bias)
    arr = lambda n=2, v=256: (ctypes.c_void_p * n)(*([v] * n))  # host arrays of never-dereferenced device pointers
    per_layer = lambda: [arr() for _ in range(12)]
    assert f(None, FAKE, *per_layer(), None, z, None) == 1
    assert f(ctypes.byref(mk(layers=0)), FAKE, *per_layer(), None, z, None) == 2
    assert f(ctypes.byref(mk(layers=5)), FAKE, *per_layer(), None, z, None) == 2
    assert f(ctypes.byref(mk(groups=2)), FAKE, *per_layer(), None, z, None) == 3
    assert f(ctypes.byref(mk(dtype=1)), FAKE, *per_layer(), None, z, None) == 3
    assert f(ctypes.byref(mk(B=33)), FAKE, *per_layer(), None, z, None) == 3      # built for small batches
    assert f(ctypes.byref(mk(r=2)), FAKE, *per_layer(), None, z, None) == 3       # every extent at least 4
    args = per_layer()
    args[2] = None                                                                  # the Vx array itself
    assert f(ctypes.byref(mk()), FAKE, *args, None, z, None) == 1
    args = per_layer()
    args[4] = arr(v=None)                                                           # a layer's Vh pointer
    assert f(ctypes.byref(mk()), FAKE, *args, None, z, None) == 1
    args = per_layer()
    args[7] = arr(v=260)                                                            # h_all not 16-byte aligned
    assert f(ctypes.byref(mk()), FAKE, *args, None, z, None) == 3
    assert f(ctypes.byref(mk()), None, *per_layer(), None, z, None) == 1            # x
    assert f(ctypes.byref(mk()), FAKE, *per_layer(), None, z, None) == 4            # workspace missing
    assert f(ctypes.byref(mk()), FAKE, *per_layer(), P(256 + 128), ctypes.c_size_t(1 << 30), None) == 3   # misaligned
    assert f(ctypes.byref(mk(T=0)), FAKE, *per_layer(), None, z, None) == 0
    assert f(ctypes.byref(mk(B=0)), FAKE, *per_layer(), None, z, None) == 0
    for q in (pf.lib.pf_lowrank_lstm_stack_fwd_workspace_bytes, pf.lib.pf_lowrank_lstm_stack_bwd_workspace_bytes):
        assert q(ctypes.byref(mk())) > 0
        assert q(ctypes.byref(mk(groups=4, r=600, h=700, d=700, B=20, T=5))) > 0   # the unfused schedule
        assert q(ctypes.byref(mk(layers=9))) == 0
    # one factor pair per path takes the fused schedule, whose packed copies differ in size from the general one
    fused = pf.lib.pf_lowrank_lstm_stack_fwd_workspace_bytes(ctypes.byref(mk(B=20, d=64, h=64, r=16, T=4)))
    general = pf.lib.pf_lowrank_lstm_stack_fwd_workspace_bytes(ctypes.byref(mk(B=20, d=64, h=64, r=16, T=4, groups=4)))
    assert fused > 0 and general > 0 and fused != general


def test_svd_validation():
    f = pf.lib.pf_svd_split
    z = ctypes.c_size_t(0)
    mk = lambda m=8, n=6, r=3: pf.pf_svd_desc(m, n, r)
    assert f(None, FAKE, FAKE, FAKE, None, None, None, z, None) == 1
    assert f(ctypes.byref(mk(r=7)), FAKE, FAKE, FAKE, None, None, None, z, None) == 2   # r > min(m, n)
    assert f(ctypes.byref(mk(m=0)), FAKE, FAKE, FAKE, None, None, None, z, None) == 2
    assert f(ctypes.byref(mk(m=20000, n=20000, r=4)), FAKE, FAKE, FAKE, None, None, None, z, None) == 3
    assert f(ctypes.byref(mk()), None, FAKE, FAKE, None, None, None, z, None) == 1
    assert f(ctypes.byref(mk()), FAKE, FAKE, FAKE, None, None, None, z, None) == 4      # workspace missing
    assert f(ctypes.byref(mk()), FAKE, FAKE, FAKE, None, P(258), FAKE, ctypes.c_size_t(1 << 30), None) == 3  # info
    # a workspace that is not 256-byte aligned is refused by every entry point that takes one
    assert f(ctypes.byref(mk()), FAKE, FAKE, FAKE, None, None, P(256 + 64), ctypes.c_size_t(1 << 30), None) == 3
    assert pf.lib.pf_svd_split_workspace_bytes(ctypes.byref(mk())) > 0
