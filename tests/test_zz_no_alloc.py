"""The backward call that allocates nothing (pf_lowrank_linear_bwd_static: scratch memory in a device array owned
by the library) against pf_lowrank_linear_bwd with a caller's workspace, through the C ABI: same kernels in the
same order, so the results must be bit-identical; they are also held to the oracle's tolerance.  Two calls in a
row, the second with a smaller input, so that what the first left in the shared array is seen not to matter."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

CASES = [
    # (M, in, out, r, dtype): first call, then a smaller one on the same array
    [(8192, 512, 2048, 128, "bf16"), (2048, 512, 512, 128, "bf16")],    # the fused kernels (Transformer shapes)
    [(300, 200, 100, 30, "f32"), (64, 512, 512, 128, "f32")],           # any-shape path, then the small-batch path
    [(777, 130, 260, 33, "bf16"), (5, 7, 3, 2, "bf16")],
]


def _both(shape, seed, T_from_fwd):
    import paper_2103_03936_amd as pf
    M, n_in, n_out, r, dtype = shape
    a = workloads.linear_inputs(M, n_in, n_out, r, dtype=dtype, seed=seed, bias=True)
    g = {k: to_gpu(v, dtype) for k, v in a.items()}
    T = pf.pf_lowrank_linear_fwd(g["X"], g["V"], g["U"], g["bias"])[1] if T_from_fwd else None
    want = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"], T_saved=T, has_bias=True)
    f32 = dict(dtype=torch.float32, device="cuda")
    out = (torch.empty_like(g["X"]), torch.empty((n_out, r), **f32), torch.empty((n_in, r), **f32),
           torch.empty((n_out,), **f32))
    before = torch.cuda.memory_allocated()
    # straight through the C ABI: no workspace argument exists, and torch hands out nothing during the call
    d = pf.pf_linear_desc(M, n_in, n_out, r, pf.PF_BF16 if dtype == "bf16" else pf.PF_F32, pf.PF_F32, 1)
    P = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)
    st = pf.lib.pf_lowrank_linear_bwd_static(ctypes.byref(d), P(g["X"]), P(g["V"]), P(g["U"]), P(g["dY"]), P(T), P(out[0]),
                                             P(out[1]), P(out[2]), P(out[3]), ctypes.c_int(0),
                                             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, pf.lib.pf_status_string(st)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name, got, ref in zip(("dX", "dU", "dV", "dbias"), out, want):
        assert torch.equal(got, ref), f"{shape} {name}: differs from pf_lowrank_linear_bwd"
    dXo, dUo, dVo, dbo = oracle.lowrank_linear_bwd(a["X"], a["V"], a["U"], a["dY"])
    for name, got, ref in zip(("dX", "dU", "dV", "dbias"), out, (dXo, dUo, dVo, dbo)):
        assert_close(got, ref, dtype, f"{shape} {name} vs oracle")


@pytest.mark.parametrize("case", range(len(CASES)))
def test_static_scratch_backward_two_calls_in_a_row(case):
    first, second = CASES[case]
    _both(first, seed=40 + case, T_from_fwd=True)
    _both(second, seed=50 + case, T_from_fwd=False)   # T recomputed into the shared array


def test_static_scratch_limit_and_accumulate():
    import paper_2103_03936_amd as pf
    assert pf.lib.pf_static_scratch_bytes() == 40 << 20
    # a layer whose partial sums exceed the array is refused before anything is launched
    big = pf.pf_linear_desc(1 << 16, 4096, 4096, 128, pf.PF_BF16, pf.PF_F32, 0)
    assert pf.lib.pf_lowrank_linear_bwd_workspace_bytes(ctypes.byref(big)) > 40 << 20
    fake = ctypes.c_void_p(256)
    assert pf.lib.pf_lowrank_linear_bwd_static(ctypes.byref(big), fake, fake, fake, fake, None, fake, fake, fake, None, 0,
                                               None) == 4
    # accumulate adds to what the gradient buffers hold, as in the workspace version
    a = workloads.linear_inputs(96, 64, 48, 8, dtype="f32", seed=77)
    g = {k: to_gpu(v) for k, v in a.items() if v is not None}
    dX, dU, dV, _ = pf.pf_lowrank_linear_bwd(g["X"], g["V"], g["U"], g["dY"])
    dU2, dV2 = dU.clone(), dV.clone()
    pf.pf_lowrank_linear_bwd_static(g["X"], g["V"], g["U"], g["dY"], None, None, dU2, dV2, accumulate=True)
    _, dUo, dVo, _ = oracle.lowrank_linear_bwd(a["X"], a["V"], a["U"], a["dY"])
    assert_close(dU2, 2 * dUo, "f32", "accumulated dU")
    assert_close(dV2, 2 * dVo, "f32", "accumulated dV")
