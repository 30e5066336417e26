"""Helpers shared by the GPU parity tests: move seeded inputs to the GPU and compare with the oracle.

Tolerances (error = max|gpu - oracle| / max|oracle| per tensor): 1e-5 for float32; 2e-2 for
bfloat16 inputs with float32 accumulation.
"""
import numpy as np
import torch

TOL = {"f32": 1e-5, "bf16": 2e-2}
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_gpu(a, dtype="f32"):
    """numpy float32 (already bf16-exact when dtype == 'bf16') -> contiguous GPU tensor of that dtype."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32:
        t = t.to(TORCH_DTYPE[dtype])
    return t.cuda().contiguous()


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    got = to_np(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    scale = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (scale if scale > 0 else 1.0))


def assert_close(got, ref, dtype, name, factor=1.0):
    e = rel_err(got, ref)
    assert e <= TOL[dtype] * factor, f"{name}: rel err {e:.3e} > {TOL[dtype] * factor:.1e}"
    return e
