"""Pins for the oracle's offline skewing (Section 4.2, Eq. 2 and Eq. 3; Section 2.4)."""
import numpy as np
import pytest

import ig_workloads as wl
from oracle import ig_oracle as o


@pytest.fixture(scope="module")
def cfg1():
    w = wl.WORKLOADS[1]
    Wq = wl.projection_weight(w, "Wq")
    Wk = wl.projection_weight(w, "Wk")
    Xcal = wl.calibration_input(w)
    Qcal = (Xcal.astype(np.float64) @ Wq.astype(np.float64)).astype(np.float32)
    sk = o.skew(Wq, Wk, Qcal, w.H)
    return w, Wq, Wk, Xcal, Qcal, sk


def test_shapes_unchanged(cfg1):
    # Section 4.3 "Prefetching Scheme": the weight dimensions stay the same after skewing.
    w, Wq, Wk, _, _, sk = cfg1
    assert sk["Wq_s"].shape == Wq.shape and sk["Wk_s"].shape == Wk.shape
    assert sk["A"].shape == (w.H, w.d, w.d)
    assert sk["rc"] == o.OK


def test_A_is_orthogonal(cfg1):
    w, *_, sk = cfg1
    for h in range(w.H):
        A = sk["A"][h].astype(np.float64)
        assert np.abs(A.T @ A - np.eye(w.d)).max() <= 1e-6
        assert np.abs(A @ A.T - np.eye(w.d)).max() <= 1e-6


def test_skew_leaves_full_scores_unchanged(cfg1):
    # Eq. 2: Q~ K~^T = Q K^T per head, for any attention input; bound 1e-5 relative.
    w, Wq, Wk, _, _, sk = cfg1
    rng = np.random.default_rng(7)
    X = rng.standard_normal((40, w.D))
    Q, K = X @ Wq.astype(np.float64), X @ Wk.astype(np.float64)
    Qs, Ks = X @ sk["Wq_s"].astype(np.float64), X @ sk["Wk_s"].astype(np.float64)
    for h in range(w.H):
        sl = slice(h * w.d, (h + 1) * w.d)
        ref = Q[:, sl] @ K[:, sl].T
        got = Qs[:, sl] @ Ks[:, sl].T
        assert np.abs(got - ref).max() / np.abs(ref).max() <= 1e-5


def test_weights_are_right_multiplied_per_head(cfg1):
    # Eq. 2: W~ = W A (A on the right, block h acting on head h's columns only).
    w, Wq, Wk, _, _, sk = cfg1
    for name, W in (("Wq_s", Wq), ("Wk_s", Wk)):
        ref = np.einsum("ihk,hkj->ihj", W.reshape(w.D, w.H, w.d).astype(np.float64),
                        sk["A"].astype(np.float64)).reshape(w.D, w.D)
        assert np.abs(sk[name] - ref).max() <= 1e-6
        wrong = np.einsum("ihk,hjk->ihj", W.reshape(w.D, w.H, w.d).astype(np.float64),
                          sk["A"].astype(np.float64)).reshape(w.D, w.D)
        assert np.abs(sk[name] - wrong).max() > 1e-3   # A^T would be a different matrix


def test_skewed_calibration_queries_are_U_sigma(cfg1):
    # Eq. 3: Q A = U S V^T V = U S: columns mutually orthogonal, norms = singular values, descending.
    w, _, _, _, Qcal, sk = cfg1
    for h in range(w.H):
        Qh = Qcal[:, h * w.d:(h + 1) * w.d].astype(np.float64)
        G = (Qh @ sk["A"][h].astype(np.float64))
        gram = G.T @ G
        sig = np.sqrt(np.diag(gram))
        off = gram - np.diag(np.diag(gram))
        assert np.abs(off).max() <= 1e-5 * gram.max()
        assert np.all(np.diff(sig) <= 1e-9 * sig[0])
        ref = np.linalg.svd(Qh, compute_uv=False)          # LAPACK
        assert np.allclose(sig, ref, rtol=1e-5, atol=1e-6 * ref[0])
        assert np.allclose(sk["sigma"][h], ref, rtol=1e-5, atol=1e-6 * ref[0])


def test_A_matches_lapack_V_up_to_sign(cfg1):
    w, _, _, _, Qcal, sk = cfg1
    for h in range(w.H):
        Qh = Qcal[:, h * w.d:(h + 1) * w.d].astype(np.float64)
        _, s, Vt = np.linalg.svd(Qh, full_matrices=False)
        V = Vt.T
        arg = np.abs(V).argmax(axis=0)
        V = V * np.sign(V[arg, np.arange(w.d)])[None, :]
        gap = np.minimum(np.abs(np.diff(s, prepend=np.inf)), np.abs(np.diff(s, append=0)))
        ok = gap > 1e-3 * s[0]                             # well-separated singular values only
        assert ok.sum() >= w.d // 2
        assert np.abs(sk["A"][h][:, ok] - V[:, ok]).max() <= 1e-4


def test_two_by_two_worked_case():
    # Section 2.4, Fig. 1: Q = S R(theta) stretches along rotated axes; A undoes the rotation
    # so that Q A has one large and one small column (semi-axes 3 and 1).
    th = 0.6
    R = np.array([[np.cos(th), -np.sin(th)], [np.sin(th), np.cos(th)]])
    Q = (np.diag([3.0, 1.0]) @ R).astype(np.float32)
    sk = o.skew(None, None, Q, 1)
    A = sk["A"][0].astype(np.float64)
    QA = Q.astype(np.float64) @ A
    assert np.allclose(np.abs(QA), np.diag([3.0, 1.0]), atol=1e-6)
    assert np.allclose(np.abs(A), np.abs(R.T), atol=1e-6)
    assert np.allclose(sk["sigma"][0], [3.0, 1.0], atol=1e-6)


def test_bias_is_skewed_like_a_row(cfg1):
    w, Wq, Wk, _, Qcal, _ = cfg1
    bq = wl.query_bias(w)
    sk = o.skew(Wq, Wk, Qcal, w.H, bq=bq, bk=bq)
    ref = np.einsum("hk,hkj->hj", bq.reshape(w.H, w.d).astype(np.float64),
                    sk["A"].astype(np.float64)).reshape(-1)
    assert np.abs(sk["bq_s"] - ref).max() <= 1e-6
    assert np.abs(sk["bk_s"] - ref).max() <= 1e-6


def test_rank_deficient_calibration_still_orthogonal():
    rng = np.random.default_rng(3)
    Q = np.zeros((16, 8), np.float32)
    Q[:, :3] = rng.standard_normal((16, 3))
    sk = o.skew(None, None, Q, 1)
    A = sk["A"][0].astype(np.float64)
    assert np.abs(A.T @ A - np.eye(8)).max() <= 1e-6
    assert np.allclose(sk["sigma"][0][3:], 0, atol=1e-6)
    Z = o.skew(None, None, np.zeros((4, 8), np.float32), 1)
    assert np.allclose(Z["A"][0], np.eye(8))


def test_apply_skew_matches_weight_skew(cfg1):
    # X (W A) = (X W) A
    w, Wq, _, Xcal, Qcal, sk = cfg1
    lhs = Xcal[:8].astype(np.float64) @ sk["Wq_s"].astype(np.float64)
    rhs = o.apply_skew(Qcal[:8], sk["A"])
    assert np.abs(lhs - rhs).max() <= 1e-4
