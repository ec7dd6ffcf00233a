"""Pins for the oracle's Algorithm 3 (Section V-D) and shuffle pairing: brute force on tiny inputs,
hand-worked cases, the FIFO special case, and the window at offset 0 that the listing as printed never scores."""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as orc
import flover_synth as synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def brute_force(arr):
    """Definition: among all windows of size (#valid), the lowest offset leaving the fewest valid slots outside."""
    n1 = int(sum(1 for a in arr if a))
    if n1 == 0:
        return 0, 0
    best = None
    for off in range(len(arr) - n1 + 1):
        cost = n1 - sum(1 for a in arr[off:off + n1] if a)
        if best is None or cost < best[1]:
            best = (off, cost)
    return best


def test_all_binary_arrays_up_to_14():
    for n in range(1, 15):
        for bits in itertools.product((0, 1), repeat=n):
            off, cost, nz = orc.find_window(bits)
            assert nz == sum(bits)
            assert (off, cost) == brute_force(bits), bits


def test_hand_cases():
    for line in open(os.path.join(GOLD, "alg3_hand_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, off, cost = line.split("|")
        arr = [int(x) for x in a.split()]
        got = orc.find_window(arr)
        assert got[:2] == (int(off), int(cost)), arr


def test_fifo_needs_no_move():
    # Section V-D: when requests finish in arrival order the live region stays contiguous.
    for n in range(1, 20):
        for k in range(0, n + 1):
            for arr in ([0] * k + [1] * (n - k), [1] * (n - k) + [0] * k):
                off, cost, nz = orc.find_window(arr)
                assert cost == 0
                assert orc.plan_moves(arr, off, nz) == []


def test_first_window_is_scored():
    # Reading R1.  Worked by hand from the listing of Algorithm 3 for the occupancy [1, 1, 0]: two valid slots, so the
    # windows are [1,1] at offset 0 (nothing outside: no move) and [1,0] at offset 1 (one valid slot outside: one
    # move).  The listing starts its running sum at zero and its loop at the first index behind the offset-0 window,
    # so the only window it ever scores is offset 1, which it returns -- one move where none is needed, against
    # Section V-D's claim of minimal movement.  The oracle scores every window.
    assert orc.find_window([1, 1, 0])[:2] == (0, 0)
    # the mirrored case is where the listing happens to be right: the offset-1 window is the good one
    assert orc.find_window([0, 1, 1])[:2] == (1, 0)
    # a prefix of valid slots followed by holes of any length never needs a move
    for k in range(1, 8):
        for z in range(1, 8):
            assert orc.find_window([1] * k + [0] * z)[:2] == (0, 0)


def test_moves_are_a_valid_minimal_compaction():
    for arr in synth.occupancy_arrays(7, 300, 64):
        arr = arr.tolist()
        off, cost, nz = orc.find_window(arr)
        moves = orc.plan_moves(arr, off, nz)
        assert len(moves) == cost
        srcs = [s for s, _ in moves]
        dsts = [d for _, d in moves]
        assert srcs == sorted(srcs) and dsts == sorted(dsts)
        assert all(arr[s] == 1 and not (off <= s < off + nz) for s in srcs)
        assert all(arr[d] == 0 and (off <= d < off + nz) for d in dsts)
        after = list(arr)
        for s, d in moves:
            after[d], after[s] = 1, 0
        assert after == [0] * off + [1] * nz + [0] * (len(arr) - off - nz)


def test_weighted_entries_follow_the_listing():
    # The listing sums arr[i] itself, so non-0/1 weights minimise the weight left outside the window.
    rng = np.random.default_rng(3)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        arr = (rng.integers(0, 5, size=n) * (rng.random(n) < 0.6)).astype(int).tolist()
        nz = sum(1 for a in arr if a)
        off, cost, _ = orc.find_window(arr)
        if nz == 0:
            continue
        costs = [sum(arr) - sum(arr[o:o + nz]) for o in range(n - nz + 1)]
        assert cost == min(costs) and off == costs.index(min(costs))


def brute_force_weighted(arr):
    """Definition of the length-weighted variant: among all windows of size (#valid), the lowest offset leaving the
    least total weight outside (weights = the non-zero entries of arr, which Algorithm 3 sums as they are)."""
    n1 = sum(1 for a in arr if a)
    if n1 == 0:
        return 0, 0
    total = sum(arr)
    best = None
    for off in range(len(arr) - n1 + 1):
        cost = total - sum(arr[off:off + n1])
        if best is None or cost < best[1]:
            best = (off, cost)
    return best


def test_weighted_arrays_against_brute_force():
    # every array over {0,1,2,5} up to length 7, then random longer ones with length-like weights
    for n in range(1, 8):
        for a in itertools.product((0, 1, 2, 5), repeat=n):
            off, cost, nz = orc.find_window(a)
            assert nz == sum(1 for x in a if x)
            assert (off, cost) == brute_force_weighted(a), a
    rng = np.random.default_rng(3)
    for _ in range(2000):
        n = int(rng.integers(1, 60))
        a = [int(x) for x in rng.integers(1, 2049, size=n) * (rng.random(n) < 0.6)]
        off, cost, nz = orc.find_window(a)
        assert (off, cost) == brute_force_weighted(a), a


def test_weighted_window_never_moves_more_weight_than_the_unweighted_one():
    rng = np.random.default_rng(4)
    strictly_better = 0
    for _ in range(500):
        n = int(rng.integers(2, 40))
        w = [int(x) for x in rng.integers(1, 1000, size=n) * (rng.random(n) < 0.7)]
        b = [1 if x else 0 for x in w]
        off_b, _, nz = orc.find_window(b)
        off_w, cost_w, _ = orc.find_window(w)
        outside_b = sum(w) - sum(w[off_b:off_b + nz])
        assert cost_w <= outside_b
        strictly_better += cost_w < outside_b
    assert strictly_better > 0
