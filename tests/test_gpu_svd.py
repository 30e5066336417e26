"""GPU truncated-SVD factor initialisation (Algorithm 1) against the oracle's Jacobi SVD.

The factors are unique only up to the sign of each column pair (and rotations inside repeated singular values),
so what is compared is what is unique: the singular values, the rank-r product U V^T, and the balanced-split
invariant U^T U = V^T V = diag(sigma_r).  Tolerance: the outputs are float32, the iteration runs in double.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity import assert_close, to_gpu

pytestmark = pytest.mark.gpu

SHAPES = [
    # m, n, r
    (1, 1, 1),
    (6, 4, 2),
    (5, 9, 3),       # more columns than rows: works on the transpose
    (33, 7, 7),      # odd number of columns (one player sits out each round), full rank kept
    (64, 64, 64),
    (200, 130, 40),
    (512, 512, 128),  # VGG-19 fc17/fc18 (Appendix D)
]


def _matrix(m, n, seed):
    return workloads.Stream(workloads.SEED_BASE + 900 + seed, "f32").normal((m, n)).astype(np.float32)


def _check(W, r, tag):
    import paper_2103_03936_amd as pf
    Uo, Vo, so = oracle.svd_split(W.astype(np.float64), r)
    U, V, sigma = pf.pf_svd_split(to_gpu(W), r)
    torch.cuda.synchronize()
    smax = float(so[0]) if so[0] > 0 else 1.0
    got = sigma.double().cpu().numpy()
    assert np.max(np.abs(got - so)) <= 1e-5 * smax, f"{tag}: singular values off by {np.max(np.abs(got - so)) / smax:.2e}"
    assert np.all(np.diff(got) <= 1e-6 * smax), f"{tag}: singular values not in descending order"
    assert_close(U.double() @ V.double().t(), Uo @ Vo.T, "f32", tag + " U V^T")
    Ud, Vd = U.double().cpu().numpy(), V.double().cpu().numpy()
    for name, F in (("U", Ud), ("V", Vd)):
        gram = F.T @ F
        assert np.max(np.abs(gram - np.diag(so[:r]))) <= 2e-5 * smax, f"{tag}: {name}^T {name} is not diag(sigma_r)"


@pytest.mark.parametrize("shape", SHAPES)
def test_svd_split(shape):
    m, n, r = shape
    _check(_matrix(m, n, seed=m + 3 * n), r, f"svd {shape}")


def test_rank_deficient_matrix():
    """Rank 3 matrix, r = 5 kept: two singular values are zero and their factor columns vanish."""
    a, b = _matrix(40, 3, 1).astype(np.float64), _matrix(3, 24, 2).astype(np.float64)
    W = (a @ b).astype(np.float32)
    import paper_2103_03936_amd as pf
    U, V, sigma = pf.pf_svd_split(to_gpu(W), 5)
    s = sigma.double().cpu().numpy()
    assert np.all(s[3:] <= 1e-5 * s[0])
    assert_close(U.double() @ V.double().t(), W.astype(np.float64), "f32", "rank-deficient reconstruction")


def test_convergence_is_reported_and_sweeps_stop():
    """The rounding-level threshold lets a converged sweep end the launches (info[0] well below the 24-sweep cap,
    info[1] == 0), also for an ill-conditioned matrix (singular values over nine decades) and a rank-deficient one."""
    import paper_2103_03936_amd as pf
    q1, _ = np.linalg.qr(_matrix(300, 60, 7).astype(np.float64))
    q2, _ = np.linalg.qr(_matrix(60, 60, 8).astype(np.float64))
    ill = ((q1 * np.logspace(0, -9, 60)) @ q2.T).astype(np.float32)
    deficient = (_matrix(200, 4, 9).astype(np.float64) @ _matrix(4, 90, 10).astype(np.float64)).astype(np.float32)
    # (a graded matrix needs more sweeps of an unpivoted one-sided Jacobi than a well-conditioned one)
    for tag, W, r, cap in (("well conditioned", _matrix(2000, 200, 11), 50, 12), ("ill conditioned", ill, 20, 23),
                           ("rank deficient", deficient, 6, 23)):
        U, V, sigma, info = pf.pf_svd_split(to_gpu(W), r, return_info=True)
        sweeps, last = (int(v) for v in info.cpu())
        assert last == 0, f"{tag}: {last} rotations in the last of {sweeps} sweeps"
        assert 1 <= sweeps <= cap, f"{tag}: {sweeps} sweeps"
        Uo, Vo, so = oracle.svd_split(W.astype(np.float64), r)
        assert np.max(np.abs(sigma.double().cpu().numpy() - so)) <= 1e-5 * so[0], tag
        assert_close(U.double() @ V.double().t(), Uo @ Vo.T, "f32", tag + " U V^T")


def test_conv_filter_bank():
    """ResNet-18 conv4_x filter bank 256 x 256 x 3 x 3 at rank 64 (Section 2.2 unrolling): the factorized layer's
    composed dense filters equal the oracle's rank-64 truncation."""
    import paper_2103_03936_amd as pf
    Wd = workloads.Stream(workloads.SEED_BASE + 950, "f32").normal((256, 256, 3, 3)).astype(np.float32) * 0.05
    Uko, Vpo, so = oracle.svd_split_conv(Wd.astype(np.float64), 64)
    Uk, Vp, sigma = pf.pf_svd_split_conv(to_gpu(Wd), 64)
    assert Uk.shape == (64, 256, 3, 3) and Vp.shape == (256, 64)
    got = torch.einsum("or,rcij->ocij", Vp.double(), Uk.double())
    want = np.einsum("or,rcij->ocij", Vpo, Uko)
    assert_close(got, want, "f32", "composed filters")
    assert np.max(np.abs(sigma.double().cpu().numpy() - so)) <= 1e-5 * so[0]


def test_deterministic():
    import paper_2103_03936_amd as pf
    W = to_gpu(_matrix(96, 48, 5))
    a = pf.pf_svd_split(W, 12)
    b = pf.pf_svd_split(W, 12)
    for u, v in zip(a, b):
        assert torch.equal(u, v)
