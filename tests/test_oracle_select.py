"""Pins for the oracle's projection, speculated score scan and threshold selection
(Section 4.3 "Decoding Stage")."""
import itertools

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import ig_workloads as wl
from oracle import ig_oracle as o


def test_project_equals_sliced_matmul():
    rng = np.random.default_rng(1)
    B, H, d, r = 3, 4, 8, 3
    D = H * d
    x = rng.standard_normal((B, D)).astype(np.float32)
    W = rng.standard_normal((D, D)).astype(np.float32)
    b = rng.standard_normal(D).astype(np.float32)
    idx = np.stack([np.sort(rng.choice(d, r, replace=False)) for _ in range(H)]).astype(np.int32)
    cols = (np.arange(H)[:, None] * d + idx).reshape(-1)
    ref = (x.astype(np.float64) @ W.astype(np.float64)[:, cols]).reshape(B, H, r)
    assert np.abs(o.project(x, W, idx) - ref).max() <= 1e-5
    refb = ref + b[cols].reshape(1, H, r)
    assert np.abs(o.project(x, W, idx, bq_s=b) - refb).max() <= 1e-5


def rope_complex(X, pos, theta=10000.0):
    """Independent formulation: pairs (j, j+d/2) as complex numbers times exp(i pos theta_j)."""
    rows, H, d = X.shape
    half = d // 2
    z = X[..., :half].astype(np.float64) + 1j * X[..., half:].astype(np.float64)
    ang = np.asarray(pos, np.float64)[:, None] * theta ** (-2.0 * np.arange(half) / d)[None, :]
    z = z * np.exp(1j * ang)[:, None, :]
    return np.concatenate([z.real, z.imag], -1)


def test_rope_matches_complex_rotation_and_is_relative():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((5, 2, 16)).astype(np.float32)
    pos = np.array([0, 1, 7, 100, 4095], np.int32)
    Y = o.rope(X, pos)
    assert np.abs(Y - rope_complex(X, pos)).max() <= 1e-6
    assert np.array_equal(Y[0], X[0])                                    # position 0 is the identity
    assert np.allclose(np.linalg.norm(Y, axis=-1), np.linalg.norm(X, axis=-1), rtol=1e-6)
    q = rng.standard_normal((1, 1, 16)).astype(np.float32)
    k = rng.standard_normal((1, 1, 16)).astype(np.float32)
    dots = [float((o.rope(q, np.array([m], np.int32)) * o.rope(k, np.array([n], np.int32))).sum())
            for m, n in ((10, 3), (107, 100), (2007, 2000))]
    assert np.allclose(dots, dots[0], atol=1e-4)                         # depends on m - n only


def test_project_rope_is_projection_rotation_then_partial_skew():
    rng = np.random.default_rng(3)
    B, H, d, r = 2, 3, 8, 3
    D = H * d
    x = rng.standard_normal((B, D)).astype(np.float32)
    W = rng.standard_normal((D, D)).astype(np.float32)
    A = np.stack([np.linalg.qr(rng.standard_normal((d, d)))[0] for _ in range(H)]).astype(np.float32)
    idx = np.stack([np.sort(rng.choice(d, r, replace=False)) for _ in range(H)]).astype(np.int32)
    pos = np.array([5, 900], np.int32)
    q = (x.astype(np.float64) @ W.astype(np.float64)).reshape(B, H, d)
    qr = rope_complex(q, pos)
    ref = np.stack([[qr[b, h] @ A[h].astype(np.float64)[:, idx[h]] for h in range(H)] for b in range(B)])
    got = o.project_rope(x, W, pos, A, idx)
    assert np.abs(got - ref).max() <= 1e-4


def test_scan_with_all_columns_is_the_exact_logit():
    # idx = all columns and x = the layer's own input: speculated score == scale * q . k.
    rng = np.random.default_rng(4)
    B, H, N, d = 2, 3, 37, 8
    q = rng.standard_normal((B, H, d)).astype(np.float32)
    K = rng.standard_normal((B, H, N, d)).astype(np.float32)
    idx = np.tile(np.arange(d, dtype=np.int32), (H, 1))
    ref = 0.25 * np.einsum("bhd,bhnd->bhn", q.astype(np.float64), K.astype(np.float64))
    assert np.abs(o.scan(q, K, idx, 0.25) - ref).max() <= 1e-5


def test_scan_uses_the_same_columns_of_q_and_k():
    # Section 4.3: the same column indices must be used on both sides.
    rng = np.random.default_rng(5)
    H, N, d, r = 2, 9, 6, 2
    K = rng.standard_normal((1, H, N, d)).astype(np.float32)
    idx = np.array([[1, 4], [0, 5]], np.int32)
    qp = rng.standard_normal((1, H, r)).astype(np.float32)
    s = o.scan(qp, K, idx, 1.0)
    for h in range(H):
        ref = K[0, h][:, idx[h]].astype(np.float64) @ qp[0, h].astype(np.float64)
        assert np.abs(s[0, h] - ref).max() <= 1e-5
    # linear in q_p
    s2 = o.scan(2 * qp, K, idx, 1.0)
    assert np.allclose(s2, 2 * s, atol=1e-5)
    # N < N_cap reads only the first N rows
    s3 = o.scan(qp, K, idx, 1.0, N=5)
    assert s3.shape == (1, H, 5) and np.array_equal(s3, s[:, :, :5])


def sets_of(sel_idx, sel_cnt):
    return [sel_idx[i, :sel_cnt[i]].tolist() for i in range(len(sel_cnt))]


@pytest.mark.parametrize("seed", range(8))
def test_selection_by_enumeration_of_subsets(seed):
    # Brute force on tiny inputs, stated through softmax weights (Section 4.3): the kept set is the
    # only subset S such that every member's weight is at least (top weight / e^alpha) and every
    # non-member's is below it.  Scores are drawn away from the boundary.
    rng = np.random.default_rng(seed)
    N, alpha = 8, float(rng.choice([0.5, 1.0, 2.0, 4.0]))
    while True:
        s = (rng.standard_normal(N) * 2.5).astype(np.float32)
        if np.abs(np.abs(s - (s.max() - alpha))).min() > 1e-3:
            break
    p = np.exp(s.astype(np.float64) - s.max())
    p /= p.sum()
    bound = p.max() / np.exp(alpha)
    good = []
    for mask in itertools.product([0, 1], repeat=N):
        S = [t for t in range(N) if mask[t]]
        if all(p[t] >= bound for t in S) and all(p[t] < bound for t in range(N) if not mask[t]):
            good.append(S)
    assert len(good) == 1
    idx, cnt = o.select(s.reshape(1, 1, N), alpha)
    assert sets_of(idx, cnt) == [good[0]]


def test_paper_weight_example(golden):
    # Section 4.3: a token at (max - 5) has the top weight divided by e^5 ~ 148.4, under 1 %.
    a = golden["alpha_example"][0]
    assert abs(np.exp(a) - golden["exp_alpha5"][0]) < 0.05
    s = np.array([[[10.0, 10.0 - a, 10.0 - a - 0.01, 3.0]]], np.float32)
    idx, cnt = o.select(s, a)
    assert sets_of(idx, cnt) == [[0, 1]]                 # the token exactly at max - alpha is kept (>=)
    p = np.exp(s[0, 0].astype(np.float64)); p /= p.sum()
    assert abs(p[0] / p[1] - golden["exp_alpha5"][0]) < 0.05
    assert p[1] / p[0] < 0.01


scores = st.lists(st.integers(-64, 64), min_size=1, max_size=40)


@settings(max_examples=150, deadline=None)
@given(scores, st.sampled_from([0.0, 0.5, 1.0, 3.0, 8.0]), st.sampled_from([0.25, 2.0]))
def test_selection_invariants(vals, a1, da):
    s = (np.array(vals, np.float32) / 8.0).reshape(1, 1, -1)      # exactly representable eighths
    N = s.shape[-1]
    S1 = set(sets_of(*o.select(s, a1))[0])
    S2 = set(sets_of(*o.select(s, a1 + da))[0])
    assert int(np.argmax(s)) in S1                                 # the argmax is always kept
    assert S1 <= S2                                                # monotone in alpha
    assert S1 == {t for t in range(N) if s[0, 0, t] >= s.max() - a1}
    shifted = set(sets_of(*o.select(s + 16.0, a1))[0])             # constant shifts cancel
    assert shifted == S1
    perm = np.random.default_rng(N).permutation(N)
    Sp = set(sets_of(*o.select(s[:, :, perm], a1))[0])
    assert Sp == {int(np.where(perm == t)[0][0]) for t in S1}      # permutation equivariant
    assert sets_of(*o.select(s, np.inf))[0] == list(range(N))      # alpha = inf keeps everything
    lst = sets_of(*o.select(s, a1))[0]
    assert lst == sorted(lst)                                      # ascending token order


def test_dropped_tokens_weigh_less_than_exp_minus_alpha():
    # With exact scores every dropped token's weight is below e^-alpha times the top weight.
    rng = np.random.default_rng(11)
    s = (3 * rng.standard_normal((2, 3, 200))).astype(np.float32)
    for alpha in (2.0, 4.0, 5.0):
        idx, cnt = o.select(s, alpha)
        p = np.exp(s.astype(np.float64) - s.max(-1, keepdims=True)).reshape(6, 200)
        for i, S in enumerate(sets_of(idx, cnt)):
            dropped = np.setdiff1d(np.arange(200), S)
            assert np.all(p[i, dropped] < np.exp(-alpha) * p[i].max())
            assert np.all(p[i, S] >= np.exp(-alpha) * p[i].max() * (1 - 1e-6))


def test_select_is_per_head_and_rejects_bad_alpha():
    s = np.array([[[0, 1, 2, 3], [3, 3, 3, -9]]], np.float32)
    idx, cnt = o.select(s, 1.0)
    assert sets_of(idx, cnt) == [[2, 3], [0, 1, 2]]
    with pytest.raises(RuntimeError):
        o.select(s, -1.0)
    with pytest.raises(RuntimeError):
        o.select(s, float("nan"))


def test_cfg1_heavy_hitters_are_found():
    # cfg 1 end to end on the speculation side: heavy-hitter keys (4x norm) dominate the kept set
    # when the logit gain makes alpha bite; recall is reported, not asserted (parity unpinned).
    w = wl.WORKLOADS[1]
    Wq = wl.projection_weight(w, "Wq")
    Xcal = wl.calibration_input(w)
    Qcal = Xcal @ Wq
    sk = o.skew(Wq, None, Qcal, w.H)
    idx = o.partial_index(o.apply_skew(Qcal, sk["A"]), None, w.H, w.ratio)
    K, _ = wl.kv_cache(w)
    Kt = o.apply_skew(K.transpose(0, 2, 1, 3).reshape(w.B * w.N, w.D), sk["A"]) \
        .reshape(w.B, w.N, w.H, w.d).transpose(0, 2, 1, 3)
    x = wl.attention_input(w)
    qp = o.project(x, sk["Wq_s"], idx)
    s = o.scan(qp, Kt, idx, 1.0)
    sel_idx, sel_cnt = o.select(s, w.alpha)
    assert np.all(sel_cnt >= 1) and np.all(sel_cnt <= w.N)
    full = np.einsum("bhd,bhnd->bhn", (x @ sk["Wq_s"]).reshape(w.B, w.H, w.d), Kt)
    for i, S in enumerate(sets_of(sel_idx, sel_cnt)):
        assert int(np.argmax(s.reshape(-1, w.N)[i])) in S
