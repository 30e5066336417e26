"""Host logic of the stacked-LSTM entry points without a GPU.

tests/emulation/lstm_stack_emulation.cpp compiles the library's own host code (pf_lstm_stack.hip, pf_skinny.hip) with
the launch macro redirected: every kernel launch becomes a CPU loop that does the kernel's arithmetic from its
argument block and checks every operand range against the buffers registered here.  What is tested is the diagonal
schedule, the slice and workspace layout and the packed addressing that the copy kernels and their consumers must agree
on - against the fp64 oracle, for the general and the fused schedule, all extents ragged."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


class _Desc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("B", ctypes.c_int64), ("d_in", ctypes.c_int64), ("h", ctypes.c_int64),
                ("r", ctypes.c_int64), ("groups", ctypes.c_int), ("layers", ctypes.c_int), ("dtype", ctypes.c_int),
                ("has_bias", ctypes.c_int)]


@pytest.fixture(scope="module")
def emu(tmp_path_factory):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not found")
    out = str(tmp_path_factory.mktemp("emu") / "liblstm_stack_emulation.so")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "paper_2103_03936_amd", "csrc"),
           os.path.join(ROOT, "tests", "emulation", "lstm_stack_emulation.cpp"), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    lib = ctypes.CDLL(out)
    lib.emu_error.restype = ctypes.c_char_p
    lib.pf_lowrank_lstm_stack_fwd_workspace_bytes.restype = ctypes.c_size_t
    lib.pf_lowrank_lstm_stack_bwd_workspace_bytes.restype = ctypes.c_size_t
    return lib


class _Buffers:
    """float32 arrays of exactly the stated size, 16-byte aligned, registered with the emulation's range checker."""

    def __init__(self, lib):
        self.lib, self.keep = lib, []
        lib.emu_clear()

    def _aligned(self, n):
        raw = np.zeros(n + 4, dtype=np.float32)
        off = (-raw.ctypes.data // 4) % 4
        return raw[off:off + n]

    def reg(self, a):
        self.keep.append(a)
        self.lib.emu_register(ctypes.c_void_p(a.ctypes.data), ctypes.c_size_t(a.nbytes))
        return a

    def workspace(self, nbytes):
        """nbytes of zeroed scratch memory, 256-byte aligned as the entry points require."""
        raw = np.zeros(nbytes + 256, dtype=np.uint8)
        off = (-raw.ctypes.data) % 256
        return self.reg(raw[off:off + nbytes])

    def copy(self, a):
        out = self._aligned(a.size).reshape(a.shape)
        out[...] = a
        return self.reg(out)

    def new(self, *shape):
        out = self._aligned(int(np.prod(shape))).reshape(shape)
        out[...] = np.nan
        return self.reg(out)


def _p(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _pa(lst):
    if lst is None:
        return None
    return (ctypes.c_void_p * len(lst))(*[None if a is None else a.ctypes.data for a in lst])


CASES = [
    # T, B, d, h, r, layers, groups, bias
    (1, 3, 8, 8, 4, 2, 1, True),
    (5, 4, 12, 20, 6, 1, 1, True),
    (6, 5, 40, 36, 10, 2, 1, True),
    (2, 7, 24, 16, 5, 4, 1, True),      # more layers than steps
    (4, 20, 70, 50, 13, 3, 1, False),
    (3, 32, 37, 29, 7, 2, 1, True),     # a full MFMA tile of rows
    (3, 6, 130, 260, 129, 2, 1, True),  # several column tiles and contraction slices
    (2, 4, 16, 24, 516, 2, 1, True),    # rank beyond the fused kernels: general schedule
    (9, 32, 70, 50, 13, 2, 1, True),    # 288 rows summed in the weight gradients
    (1, 3, 8, 8, 4, 2, 4, True),
    (6, 5, 40, 36, 10, 2, 4, False),
    (4, 20, 70, 50, 13, 3, 4, True),
    (3, 6, 130, 260, 129, 2, 4, True),
    (7, 20, 40, 36, 10, 2, 4, False),   # 140 rows, one factor pair per gate
]


@pytest.mark.parametrize("case", CASES)
def test_stack_host_logic_against_oracle(emu, case):
    T, B, d, h, r, L, G, bias = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    gr = G * r
    x = rng.standard_normal((T, B, d))
    h0 = [rng.standard_normal((B, h)) * .5 for _ in range(L)]
    c0 = [rng.standard_normal((B, h)) * .5 for _ in range(L)]
    Vx = [rng.uniform(-.3, .3, (d if l == 0 else h, gr)) for l in range(L)]
    Ux = [rng.uniform(-.3, .3, (4 * h, r)) for _ in range(L)]
    Vh = [rng.uniform(-.3, .3, (h, gr)) for _ in range(L)]
    Uh = [rng.uniform(-.3, .3, (4 * h, r)) for _ in range(L)]
    bs = [rng.uniform(-.3, .3, (4 * h,)) for _ in range(L)] if bias else None
    dtop = rng.standard_normal((T, B, h))
    dhT = [rng.standard_normal((B, h)) for _ in range(L)]
    dcT = [rng.standard_normal((B, h)) for _ in range(L)]
    o = oracle.lowrank_lstm_stack_fwd(x, h0, c0, Vx, Ux, Vh, Uh, bs, G)
    ob = oracle.lowrank_lstm_stack_bwd(x, h0, c0, *o, Vx, Ux, Vh, Uh, dtop, dhT, dcT, G)

    m = _Buffers(emu)
    desc = _Desc(T, B, d, h, r, G, L, 0, 1 if bias else 0)
    fx = m.copy(x)
    copies = lambda lst: [m.copy(a) for a in lst]
    fh0, fc0, fVx, fUx, fVh, fUh = map(copies, (h0, c0, Vx, Ux, Vh, Uh))
    fb = copies(bs) if bias else None
    outs = [[m.new(T, B, n) for _ in range(L)] for n in (h, h, 4 * h, gr, gr)]
    nbytes = emu.pf_lowrank_lstm_stack_fwd_workspace_bytes(ctypes.byref(desc))
    ws = m.workspace(max(nbytes, 16))
    st = emu.pf_lowrank_lstm_stack_fwd(ctypes.byref(desc), _p(fx), _pa(fh0), _pa(fc0), _pa(fVx), _pa(fUx), _pa(fVh),
                                       _pa(fUh), _pa(fb), *[_pa(v) for v in outs], _p(ws), ctypes.c_size_t(nbytes), None)
    assert st == 0, (st, emu.emu_error())
    rel = lambda got, want: np.abs(got - want).max() / max(np.abs(want).max(), 1e-30)
    for got, want, name in zip(outs, o, ("h", "c", "gates", "Tx", "Th")):
        for l in range(L):
            assert rel(got[l], want[l]) < 1e-5, (name, l)

    fdtop, fdhT, fdcT = m.copy(dtop), copies(dhT), copies(dcT)
    dx = m.new(T, B, d)
    dh0, dc0 = [m.new(B, h) for _ in range(L)], [m.new(B, h) for _ in range(L)]
    grads = {k: [m.new(*v[l].shape) for l in range(L)] for k, v in (("dVx", Vx), ("dUx", Ux), ("dVh", Vh), ("dUh", Uh))}
    grads["dbias"] = [m.new(4 * h) for _ in range(L)]
    nbytes = emu.pf_lowrank_lstm_stack_bwd_workspace_bytes(ctypes.byref(desc))
    ws2 = m.workspace(max(nbytes, 16))
    st = emu.pf_lowrank_lstm_stack_bwd(
        ctypes.byref(desc), _p(fx), _pa(fh0), _pa(fc0), *[_pa(v) for v in outs], _pa(fVx), _pa(fUx), _pa(fVh), _pa(fUh),
        _p(fdtop), _pa(fdhT), _pa(fdcT), _p(dx), _pa(dh0), _pa(dc0), _pa(grads["dVx"]), _pa(grads["dUx"]),
        _pa(grads["dVh"]), _pa(grads["dUh"]), _pa(grads["dbias"]), 0, _p(ws2), ctypes.c_size_t(nbytes), None)
    assert st == 0, (st, emu.emu_error())
    assert rel(dx, ob[0]) < 1e-5
    for l in range(L):
        assert rel(dh0[l], ob[1][l]) < 1e-5 and rel(dc0[l], ob[2][l]) < 1e-5, l
        for k in grads:
            assert rel(grads[k][l], ob[3][l][k]) < 1e-5, (k, l)


def test_a_workspace_one_byte_short_is_refused(emu):
    desc = _Desc(3, 4, 8, 8, 4, 1, 2, 0, 1)
    m = _Buffers(emu)
    need = emu.pf_lowrank_lstm_stack_fwd_workspace_bytes(ctypes.byref(desc))
    a = lambda n=2: (ctypes.c_void_p * n)(*([256] * n))
    args = [a() for _ in range(12)]
    ws = m.workspace(need)
    st = emu.pf_lowrank_lstm_stack_fwd(ctypes.byref(desc), ctypes.c_void_p(256), *args, _p(ws), ctypes.c_size_t(need - 1),
                                       None)
    assert st == 4
