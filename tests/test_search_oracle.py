"""Pins for oracle/search_oracle.py: the neighbourhood moves against explicit Python lists, and invariants."""
from __future__ import annotations

import numpy as np

from oracle import search_oracle as SO
from paper_2503_09357_amd import workloads as W

import checkers as K


def _lists(P, pl, rk):
    lists = K.device_lists(P, pl, rk)
    assert lists is not None, "ranks are not dense"
    return lists


def _from_lists(n, lists):
    pl = np.zeros(n, dtype=np.int32)
    rk = np.zeros(n, dtype=np.int32)
    for j, lst in enumerate(lists):
        for r, v in enumerate(lst):
            pl[v], rk[v] = j, r
    return pl, rk


def _apply_on_lists(P, pl0, rk0, words, orders_only=False):
    """The move of the oracle's docstring, carried out with list.pop / list.insert."""
    n = len(pl0)
    lists = [list(l) for l in _lists(P, pl0, rk0)]
    r0, r1, r2, r3 = (int(x) for x in words)
    v = r1 % n
    m, r = int(pl0[v]), int(rk0[v])
    if r0 % 2 == 0:
        if r + 1 < len(lists[m]):
            lists[m][r], lists[m][r + 1] = lists[m][r + 1], lists[m][r]
    else:
        m2 = m if orders_only else r2 % P
        if m2 == m:
            pos = r3 % len(lists[m])
            lists[m].pop(r)
            lists[m].insert(pos, v)
        else:
            pos = r3 % (len(lists[m2]) + 1)
            lists[m].pop(r)
            lists[m2].insert(pos, v)
    return _from_lists(n, lists)


def test_moves_match_list_surgery():
    rng = np.random.default_rng(4401)
    for _ in range(8):
        n, P = int(rng.integers(3, 40)), int(rng.integers(1, 6))
        rp, ci = W.random_dag(rng, n, 2)
        pl, rk = W.list_schedules(rp, ci, P, 1, int(rng.integers(1, 1 << 30)))
        rnd = rng.integers(0, 1 << 32, size=4 * 200, dtype=np.uint64).astype(np.uint32)
        out_pl, out_rk = SO.propose(pl[0], rk[0], rnd, P)
        assert (out_pl[0] == pl[0]).all() and (out_rk[0] == rk[0]).all()      # candidate 0 is the base
        for c in range(1, 200):
            want_pl, want_rk = _apply_on_lists(P, pl[0], rk[0], rnd[4 * c:4 * c + 4])
            assert (out_pl[c] == want_pl).all() and (out_rk[c] == want_rk).all(), (c, rnd[4 * c:4 * c + 4])


def test_orders_only_moves_match_list_surgery_and_keep_the_placement():
    rng = np.random.default_rng(4402)
    for _ in range(6):
        n, P = int(rng.integers(3, 40)), int(rng.integers(1, 6))
        rp, ci = W.random_dag(rng, n, 2)
        pl, rk = W.list_schedules(rp, ci, P, 1, int(rng.integers(1, 1 << 30)))
        rnd = rng.integers(0, 1 << 32, size=4 * 150, dtype=np.uint64).astype(np.uint32)
        out_pl, out_rk = SO.propose(pl[0], rk[0], rnd, P, orders_only=True)
        assert (out_pl == pl[0]).all()                                         # x of the base in every candidate
        moved = 0
        for c in range(1, 150):
            want_pl, want_rk = _apply_on_lists(P, pl[0], rk[0], rnd[4 * c:4 * c + 4], orders_only=True)
            assert (out_pl[c] == want_pl).all() and (out_rk[c] == want_rk).all(), c
            moved += int((out_rk[c] != rk[0]).any())
        assert moved > 30 or n < 6


def test_candidates_stay_dense_and_move_one_operation():
    rng = np.random.default_rng(4402)
    rp, ci = W.random_dag(rng, 60, 3)
    pl, rk = W.list_schedules(rp, ci, 5, 1, 99)
    rnd = rng.integers(0, 1 << 32, size=4 * 500, dtype=np.uint64).astype(np.uint32)
    out_pl, out_rk = SO.propose(pl[0], rk[0], rnd, 5)
    kinds = set()
    for c in range(500):
        assert K.device_lists(5, out_pl[c], out_rk[c]) is not None
        moved = np.flatnonzero(out_pl[c] != pl[0])
        assert moved.size <= 1
        changed = np.flatnonzero((out_pl[c] != pl[0]) | (out_rk[c] != rk[0]))
        kinds.add("same" if changed.size == 0 else ("across" if moved.size else "within"))
    assert kinds == {"same", "across", "within"}


def test_single_machine_and_single_operation():
    out_pl, out_rk = SO.propose([0], [0], np.arange(40, dtype=np.uint32), 1)
    assert (out_pl == 0).all() and (out_rk == 0).all()
    out_pl, out_rk = SO.propose([0, 0, 0], [2, 0, 1], np.array([0, 0, 0, 0, 0, 1, 0, 0, 1, 2, 0, 0], dtype=np.uint32), 1)
    # base order on the machine: 1, 2, 0
    assert out_rk[1].tolist() == [2, 1, 0]        # swap: node 1 (rank 0) trades places with node 2 -> 2, 1, 0
    assert out_rk[2].tolist() == [2, 1, 0]        # move: node 2 (rank 1) re-inserted at position 0 -> 2, 1, 0


def test_select():
    assert SO.select([5, 3, 3, 9], [0, 0, 0, 0]) == (1, 3)
    assert SO.select([5, 3, 2, 9], [0, 1, 4, 0]) == (0, 5)
    assert SO.select([-1, -1], [1, 2]) == (-1, -1)
    assert SO.select([7], [0]) == (0, 7)
