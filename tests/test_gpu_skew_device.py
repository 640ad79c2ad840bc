"""GPU parity of the offline skewing on the device (ig_skew_device) against the oracle's skew
(Section 4.2, Eq. 2 and Eq. 3).  A is only unique up to the spectrum's gaps, so the comparison goes
through what the paper fixes: A_h orthogonal, Q_h A_h has orthogonal columns of norms sigma
(descending, equal to the oracle's), Q~ K~^T = Q K^T; and element-wise where the singular values
are well separated."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def skew_on_gpu(ctx, Qcal, H):
    n, D = Qcal.shape
    d = D // H
    A = torch.zeros((H, d, d), device="cuda")
    sigma = torch.zeros((H, d), device="cuda")
    ctx.ig_skew_device(D, H, n, torch.from_numpy(np.ascontiguousarray(Qcal, dtype=np.float32)).cuda(), A, sigma)
    torch.cuda.synchronize()
    return A.cpu().numpy().astype(np.float64), sigma.cpu().numpy().astype(np.float64), ctx.ig_check_status()


def check_invariants(Qcal, H, A, sigma, ref_sigma):
    n, D = Qcal.shape
    d = D // H
    rng = np.random.default_rng(0)
    K = rng.standard_normal((64, D))
    for h in range(H):
        Ah = A[h]
        assert np.abs(Ah.T @ Ah - np.eye(d)).max() <= 2e-6
        Qh = Qcal[:, h * d:(h + 1) * d].astype(np.float64)
        gram = (Qh @ Ah).T @ (Qh @ Ah)
        scale = max(1.0, gram.max())
        assert np.abs(gram - np.diag(np.diag(gram))).max() <= 2e-5 * scale       # columns orthogonal
        assert np.all(np.diff(sigma[h]) <= 1e-6 * sigma[h, 0])                   # descending
        assert np.abs(sigma[h] - ref_sigma[h]).max() <= 1e-4 * ref_sigma[h, 0]
        Kh = K[:, h * d:(h + 1) * d]
        full = Qh @ Kh.T
        assert np.abs((Qh @ Ah) @ (Kh @ Ah).T - full).max() <= 1e-5 * np.abs(full).max()
        assert np.all(np.abs(Ah).argmax(0) == (Ah * np.sign(Ah[np.abs(Ah).argmax(0), np.arange(d)])).argmax(0))


@pytest.mark.parametrize("cfg,H,d", [(1, 4, 64), (2, 4, 128), (2, 3, 32)])
def test_matches_the_oracle_on_workload_calibration_queries(ctx, cfg, H, d):
    w = wl.shrink(wl.WORKLOADS[cfg], H=H, d=d)
    print(f"case {w.name} H{H} d{d} n_cal {w.n_cal}", flush=True)
    Qcal = (wl.calibration_input(w) @ wl.projection_weight(w, "Wq")).astype(np.float32)
    ref = o.skew(None, None, Qcal, H)
    A, sigma, status = skew_on_gpu(ctx, Qcal, H)
    assert status == 0
    check_invariants(Qcal, H, A, sigma, ref["sigma"].astype(np.float64))
    # element-wise on the columns whose singular value is separated from its neighbours
    for h in range(H):
        s = ref["sigma"][h].astype(np.float64)
        gap = np.minimum(np.abs(np.diff(s, prepend=np.inf)), np.abs(np.diff(s, append=-np.inf))) / s[0]
        cols = gap > 1e-3
        assert cols.sum() >= d // 4
        assert np.abs(A[h][:, cols] - ref["A"][h][:, cols]).max() <= 2e-3


def test_fewer_rows_than_columns_still_gives_an_orthogonal_basis(ctx):
    rng = np.random.default_rng(5)
    H, d, n = 2, 64, 20                       # rank 20 < d: the null space is completed arbitrarily
    Qcal = rng.standard_normal((n, H * d)).astype(np.float32)
    ref = o.skew(None, None, Qcal, H)
    A, sigma, status = skew_on_gpu(ctx, Qcal, H)
    assert status == 0
    for h in range(H):
        assert np.abs(A[h].T @ A[h] - np.eye(d)).max() <= 2e-6
        assert np.abs(sigma[h][:n] - ref["sigma"][h][:n]).max() <= 1e-4 * ref["sigma"][h][0]
        assert np.all(sigma[h][n:] <= 1e-3 * sigma[h][0])
        Qh = Qcal[:, h * d:(h + 1) * d].astype(np.float64)
        assert np.abs((Qh @ A[h]) @ (Qh @ A[h]).T - Qh @ Qh.T).max() <= 1e-5 * np.abs(Qh @ Qh.T).max()


def test_error_paths(ctx):
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    assert ctx.call("ig_skew_device", 66, 2, 8, p, p, None, 0) == ig.IG_ESHAPE      # odd d
    assert ctx.call("ig_skew_device", 64, 3, 8, p, p, None, 0) == ig.IG_ESHAPE      # D % H
    assert ctx.call("ig_skew_device", 1024, 2, 8, p, p, None, 0) == ig.IG_ESHAPE    # d > 256
    assert ctx.call("ig_skew_device", 64, 2, 8, None, p, None, 0) == ig.IG_EINVAL
