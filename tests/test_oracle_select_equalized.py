"""Pins for the oracle's head-equalised selection (Section 4.3 "Decoding Stage": every head of a
layer fetches the same number of tokens, the average over heads of the tokens above the threshold;
Section 5.1 "Key Metric": at most 20 % of the cache per layer)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import ig_oracle as o


def rank_count_reference(s, alpha, max_frac):
    """Independent formulation without any sort: a token is kept iff fewer than n tokens beat it,
    where u beats t when s[u] > s[t], or s[u] == s[t] and u < t."""
    B, H, N = s.shape
    cap = max(1, int(np.floor(max_frac * N)))
    lists, n_eq = [], []
    for b in range(B):
        c = [(s[b, h] >= s[b, h].max() - np.float32(alpha)).sum() for h in range(H)]
        n = max(1, min(int(sum(c)) // H, cap))
        n_eq.append(n)
        for h in range(H):
            v = s[b, h]
            keep = []
            for t in range(N):
                beats = int((v > v[t]).sum()) + int((v[:t] == v[t]).sum())
                if beats < n:
                    keep.append(t)
            lists.append(keep)
    return lists, n_eq


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 3), st.integers(1, 4), st.integers(1, 24), st.integers(0, 2 ** 31 - 1),
       st.sampled_from([0.0, 0.5, 2.0, float("inf")]), st.sampled_from([0.2, 0.5, 1.0]),
       st.booleans())
def test_matches_rank_counting_on_small_inputs(B, H, N, seed, alpha, max_frac, ties):
    rng = np.random.default_rng(seed)
    s = rng.standard_normal((B, H, N)).astype(np.float32)
    if ties:
        s = np.round(s * 2) / 2              # many equal scores
    idx, cnt, n_eq = o.select_equalized(s, alpha, max_frac)
    ref_lists, ref_n = rank_count_reference(s, alpha, max_frac)
    assert list(n_eq) == ref_n
    for bh in range(B * H):
        assert cnt[bh] == ref_n[bh // H]
        assert list(idx[bh, :cnt[bh]]) == ref_lists[bh]


def test_matches_a_library_sort():
    rng = np.random.default_rng(7)
    B, H, N = 3, 5, 700
    s = (rng.standard_normal((B, H, N)) * 3).astype(np.float32)
    s[:, :, ::7] = np.round(s[:, :, ::7])     # some ties
    idx, cnt, n_eq = o.select_equalized(s, 4.0, 0.2)
    for b in range(B):
        for h in range(H):
            order = np.lexsort((np.arange(N), -s[b, h].astype(np.float64)))   # score desc, then t asc
            want = np.sort(order[:n_eq[b]])
            bh = b * H + h
            assert np.array_equal(idx[bh, :cnt[bh]], want)


def test_reduces_to_threshold_lists_when_all_heads_keep_the_same_number():
    # every head gets exactly c tokens at score 10 and the rest below 10 - alpha: the average is c,
    # nothing has to be added or dropped, and the result is the plain threshold selection
    rng = np.random.default_rng(3)
    B, H, N, c, alpha = 2, 4, 200, 9, 4.0
    s = rng.uniform(-3.0, 5.0, (B, H, N)).astype(np.float32)
    for b in range(B):
        for h in range(H):
            top = rng.choice(N, c, replace=False)
            s[b, h, top] = 10.0 - rng.uniform(0.0, 3.0, c).astype(np.float32)
            s[b, h, top[0]] = 10.0
    t_idx, t_cnt = o.select(s, alpha)
    assert np.all(t_cnt == c)
    e_idx, e_cnt, n_eq = o.select_equalized(s, alpha, 0.2)
    assert np.all(n_eq == c) and np.array_equal(e_cnt, t_cnt)
    assert np.array_equal(e_idx[:, :c], t_idx[:, :c])


def test_count_is_the_truncated_mean_of_the_threshold_counts():
    rng = np.random.default_rng(11)
    B, H, N = 4, 6, 300
    s = (rng.standard_normal((B, H, N)) * rng.uniform(0.5, 4.0, (B, H, 1))).astype(np.float32)
    _, t_cnt = o.select(s, 3.0)
    _, e_cnt, n_eq = o.select_equalized(s, 3.0, 1.0)
    want = t_cnt.reshape(B, H).sum(1) // H
    assert np.array_equal(n_eq, np.maximum(want, 1))
    assert np.array_equal(e_cnt.reshape(B, H), np.repeat(n_eq[:, None], H, 1))


def test_cap_is_the_truncated_fraction_the_paper_prints(golden):
    # Section 5.3: a 20 % budget at sequence length 2048 is 409 tokens
    N = int(golden["h2o_budget_seq"][0])
    frac = golden["h2o_budget_ratio"][0]
    s = np.zeros((1, 2, N), np.float32)       # all scores equal: every token is above the threshold
    idx, cnt, n_eq = o.select_equalized(s, 4.0, frac)
    assert n_eq[0] == int(golden["h2o_budget_tokens"][0]) == 409
    # equal scores: the earliest tokens win
    assert np.array_equal(idx[0, :409], np.arange(409))


def test_kept_scores_dominate_dropped_scores_and_lists_ascend():
    rng = np.random.default_rng(5)
    B, H, N = 2, 3, 500
    s = rng.standard_normal((B, H, N)).astype(np.float32) * 2
    idx, cnt, n_eq = o.select_equalized(s, 2.0, 0.2)
    for bh in range(B * H):
        lst = idx[bh, :cnt[bh]]
        assert np.all(np.diff(lst) > 0)
        v = s.reshape(B * H, N)[bh]
        dropped = np.setdiff1d(np.arange(N), lst)
        assert v[lst].min() >= v[dropped].max()
        assert np.argmax(v) in lst            # the arg-max is always kept


def test_bad_arguments():
    s = np.zeros((1, 1, 4), np.float32)
    with pytest.raises(RuntimeError):
        o.select_equalized(s, -1.0, 0.2)
    with pytest.raises(RuntimeError):
        o.select_equalized(s, 1.0, 0.0)
    with pytest.raises(RuntimeError):
        o.select_equalized(s, 1.0, 1.5)
