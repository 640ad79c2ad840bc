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


# ---- the comparison policies of Section 4.4 / Table 2: FIFO and LRU --------------------------------
# Pinned against the textbook structures the paper names: a queue for FIFO, an access-ordered list
# for LRU (collections.OrderedDict.move_to_end is the "promote to the head" of the doubly linked
# list), driven by the same random trace of prefetches and replacements.

def test_fifo_and_lru_hand_worked():
    # one pool of 4 entries written at steps 0..3 (prefill: token positions)
    fifo = np.array([[0, 1, 2, 3]], np.int32)
    lru = fifo.copy()
    idx, cnt = lists([[0, 2]], 4)
    o.pool_touch_lru(lru, idx, cnt, 4, now=4)              # step 4 prefetches entries 0 and 2
    assert lru.tolist() == [[4, 1, 4, 3]]
    assert o.pool_victim_oldest(fifo, 4).tolist() == [0]   # FIFO: the oldest resident, used or not
    assert o.pool_victim_oldest(lru, 4).tolist() == [1]    # LRU: entry 1 was never used again
    fifo[0, 0] = 4                                          # FIFO overwrote slot 0 at step 4
    assert o.pool_victim_oldest(fifo, 4).tolist() == [1]
    # equal stamps: the lowest slot; only the first N slots are candidates
    assert o.pool_victim_oldest(np.array([[5, 5, 5], [7, 2, 2]], np.int32), 3).tolist() == [0, 1]
    assert o.pool_victim_oldest(np.array([[5, 4, 0]], np.int32), 2).tolist() == [1]


@settings(max_examples=40, deadline=None)
@given(st.integers(2, 24), st.integers(0, 2 ** 31 - 1))
def test_fifo_and_lru_match_queue_and_access_ordered_list(N, seed):
    from collections import OrderedDict, deque
    rng = np.random.default_rng(seed)
    fifo = np.arange(N, dtype=np.int32)[None].copy()       # prefill: entry t written at time t (all before 2 N)
    lru = fifo.copy()
    queue = deque(range(N))                                 # oldest resident on the left
    order = OrderedDict((t, None) for t in range(N))        # least recently used first
    for step in range(N, N + 30):
        used = np.sort(rng.choice(N, int(rng.integers(0, N)), replace=False))
        idx, cnt = lists([used], N)
        o.pool_touch_lru(lru, idx, cnt, N, now=2 * step)   # the step's prefetches come before its insertion
        for t in used:                                      # ascending slot order within a step
            order.move_to_end(int(t))
        v_fifo, v_lru = int(o.pool_victim_oldest(fifo, N)[0]), int(o.pool_victim_oldest(lru, N)[0])
        assert v_fifo == queue[0]
        assert v_lru == next(iter(order))
        # the new token replaces the victim of each policy in its own pool
        queue.popleft()
        queue.append(v_fifo)
        fifo[0, v_fifo] = 2 * step + 1
        order.move_to_end(v_lru)
        lru[0, v_lru] = 2 * step + 1


def test_lru_bad_slot_is_refused():
    s = np.zeros((1, 4), np.int32)
    with pytest.raises(RuntimeError):
        o.pool_touch_lru(s, *lists([[9]], 4), 4, now=1)
