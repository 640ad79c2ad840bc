"""Pins for the oracle's partial weight index generation (Section 4.3 "Prefill Stage")."""
import numpy as np
import pytest

import ig_workloads as wl
from oracle import ig_oracle as o


def brute_rank(Qs, Ks, H, r):
    n, D = Qs.shape
    d = D // H
    out = []
    for h in range(H):
        c = np.abs(Qs[:, h * d:(h + 1) * d].astype(np.float64)).sum(0)
        if Ks is not None:
            c = c + np.abs(Ks[:, h * d:(h + 1) * d].astype(np.float64)).sum(0)
        order = sorted(range(d), key=lambda j: (-c[j], j))   # full sort, ties to the lower column
        out.append(sorted(order[:r]))
    return np.array(out, np.int32)


@pytest.mark.parametrize("seed", range(6))
def test_matches_full_sort_on_small_heads(seed):
    rng = np.random.default_rng(seed)
    H, d, n = 3, 10, 7
    Qs = rng.standard_normal((n, H * d)).astype(np.float32)
    Ks = rng.standard_normal((n, H * d)).astype(np.float32)
    for ratio, ks in ((0.3, Ks), (0.5, Ks), (0.3, None), (1.0, Ks)):
        r = int(np.floor(ratio * d))
        assert np.array_equal(o.partial_index(Qs, ks, H, ratio), brute_rank(Qs, ks, H, r))


def test_ties_go_to_lower_column():
    Qs = np.ones((2, 8), np.float32)
    assert o.partial_index(Qs, None, 1, 0.5).tolist() == [[0, 1, 2, 3]]


def test_key_term_is_counted():
    # a column that is large only in K~ must be picked (|Q~| + |K~|, not |Q~| alone)
    rng = np.random.default_rng(0)
    Qs = rng.standard_normal((16, 10)).astype(np.float32)
    Qs[:, 9] *= 1e-3
    Ks = rng.standard_normal((16, 10)).astype(np.float32)
    Ks[:, 9] *= 100
    assert 9 in o.partial_index(Qs, Ks, 1, 0.3)[0]
    assert 9 not in o.partial_index(Qs, None, 1, 0.3)[0]


def test_signs_do_not_cancel():
    # absolute values are taken element-wise before summing: a column of +5/-5 outranks 0.1s
    Qs = np.full((4, 4), 0.1, np.float32)
    Qs[:, 2] = [5, -5, 5, -5]
    assert o.partial_index(Qs, None, 1, 0.25).tolist() == [[2]]


def test_svd_skewed_queries_pick_leading_columns():
    # With A = V the skewed calibration queries are U S: column abs-sums track sigma_j, which
    # decays quickly for the cfg-1 spectrum, so the query-only rule keeps columns 0..r-1.
    w = wl.WORKLOADS[1]
    Wq = wl.projection_weight(w, "Wq")
    Qcal = wl.calibration_input(w) @ Wq
    sk = o.skew(Wq, None, Qcal, w.H)
    Qs = o.apply_skew(Qcal, sk["A"])
    c = np.abs(Qs).reshape(w.n_cal, w.H, w.d).sum(0)
    idx = o.partial_index(Qs, None, w.H, w.ratio)
    r = idx.shape[1]
    for h in range(w.H):
        if np.all(np.diff(c[h][:r + 1]) < 0) and c[h][r:].max() < c[h][r - 1]:
            assert idx[h].tolist() == list(range(r))
    assert r == 19


def test_kept_fraction_matches_paper_memory_figures(golden):
    # Section 6.2: ratio 0.3 -> partial W_Q = 2.5 % of parameters (12 D^2 per block), partial K = 15 % of KV.
    ratio = golden["partial_ratio"][0]
    d, H = 128, 40
    D = H * d
    Qs = np.random.default_rng(0).standard_normal((4, D)).astype(np.float32)
    r = o.partial_index(Qs, None, H, ratio).shape[1]
    assert r == 38
    wq_frac = (D * H * r) / (12 * D * D)
    k_frac = (H * r) / (2 * H * d)
    assert abs(wq_frac - golden["partial_wq_fraction_of_params"][0]) < 5e-4
    assert abs(k_frac - golden["partial_k_fraction_of_kv"][0]) < 2e-3


def test_truncating_budget_rule(golden):
    # Section 5.3 prints 409 tokens for 20 % of 2048: budgets truncate; r = floor(ratio * d) likewise.
    assert int(np.floor(golden["h2o_budget_ratio"][0] * golden["h2o_budget_seq"][0])) == \
        int(golden["h2o_budget_tokens"][0])
    for ratio, d, r in ((0.3, 64, 19), (0.3, 128, 38), (0.2, 128, 25)):
        Qs = np.ones((1, d), np.float32)
        assert o.partial_index(Qs, None, 1, ratio).shape[1] == r
