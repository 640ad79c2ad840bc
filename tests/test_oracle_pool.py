"""Pins for the oracle's KV cache pool counters (Section 4.4: a counter per prefetched entry, the
victim is the smallest count, all counters are halved when one saturates)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import ig_oracle as o


def lists(rows, stride):
    idx = np.full((len(rows), stride), -1, np.int32)
    cnt = np.zeros(len(rows), np.int32)
    for i, r in enumerate(rows):
        idx[i, :len(r)] = r
        cnt[i] = len(r)
    return idx, cnt


def test_hand_worked_counts_and_victims():
    c = np.zeros((2, 6), np.int32)
    idx, cnt = lists([[0, 2, 5], [1]], 6)
    o.pool_touch(c, idx, cnt, 6)
    assert c.tolist() == [[1, 0, 1, 0, 0, 1], [0, 1, 0, 0, 0, 0]]
    idx, cnt = lists([[2], [1, 0]], 6)
    o.pool_touch(c, idx, cnt, 6)
    assert c.tolist() == [[1, 0, 2, 0, 0, 1], [1, 2, 0, 0, 0, 0]]
    # smallest count, lowest slot on ties; only the first N slots are candidates
    assert o.pool_victim(c, 6).tolist() == [1, 2]
    assert o.pool_victim(np.array([[3, 1, 2], [5, 5, 5]], np.int32), 3).tolist() == [1, 0]
    assert o.pool_victim(np.array([[3, 2, 0]], np.int32), 2).tolist() == [1]


def test_saturation_halves_only_that_pool_after_the_increments():
    c = np.array([[3, 1, 2, 0], [3, 3, 0, 0]], np.int32)
    idx, cnt = lists([[0, 3], [2]], 4)
    o.pool_touch(c, idx, cnt, 4, counter_max=4)
    # pool 0: slot 0 reaches 4 (saturated), slot 3 becomes 1, then everything halves
    assert c[0].tolist() == [2, 0, 1, 0]
    assert c[1].tolist() == [3, 3, 1, 0]            # pool 1 is untouched by pool 0's halving
    # a counter never exceeds the saturation value
    c = np.array([[4, 4]], np.int32)
    idx, cnt = lists([[0, 1]], 2)
    o.pool_touch(c, idx, cnt, 2, counter_max=4)
    assert c.tolist() == [[2, 2]]


@settings(max_examples=50, deadline=None)
@given(st.integers(1, 4), st.integers(1, 40), st.integers(0, 2 ** 31 - 1), st.integers(2, 9))
def test_matches_array_formulation(BH, N, seed, cmax):
    rng = np.random.default_rng(seed)
    N_cap = N + int(rng.integers(0, 4))
    c = rng.integers(0, cmax, (BH, N_cap)).astype(np.int32)
    rows = [np.sort(rng.choice(N, int(rng.integers(0, N + 1)), replace=False)) for _ in range(BH)]
    idx, cnt = lists(rows, N_cap)
    want = c.copy()
    for i, r in enumerate(rows):
        want[i, r] = np.minimum(want[i, r] + 1, cmax)
        if len(r) and want[i, r].max() >= cmax:
            want[i, :N] //= 2
    got = o.pool_touch(c.copy(), idx, cnt, N, counter_max=cmax)
    assert np.array_equal(got, want)
    assert np.array_equal(o.pool_victim(got, N), np.argmin(got[:, :N], axis=1))


def test_bad_arguments():
    c = np.zeros((1, 4), np.int32)
    idx, cnt = lists([[7]], 4)
    with pytest.raises(RuntimeError):
        o.pool_touch(c, idx, cnt, 4)                 # slot outside the pool
    with pytest.raises(RuntimeError):
        o.pool_touch(c, *lists([[0]], 4), 4, counter_max=0)
