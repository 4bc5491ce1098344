"""Independent, deliberately different evaluators used to pin the CPU oracle.

None of these share code with ``oracle/`` or with the HIP library:

* ``tick_simulate``      - unit-time-step simulation of non-preemptive machines (Sec. III assumptions)
* ``linear_extensions``  - brute-force enumeration of all topological orders of a tiny DAG
* ``check_constraints``  - the MIP rows (eqs. (2),(3),(7),(11)-(13),(17)-(19)) with the binaries fixed
* ``critical_path``      - textbook longest path by memoised recursion
"""
from __future__ import annotations

import itertools
from functools import lru_cache
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


def pred_lists(row_ptr, col_idx) -> List[List[int]]:
    n = len(row_ptr) - 1
    preds: List[List[int]] = [[] for _ in range(n)]
    for u in range(n):
        for k in range(row_ptr[u], row_ptr[u + 1]):
            preds[int(col_idx[k])].append(u)
    return preds


def device_lists(P: int, placement, rank) -> Optional[List[List[int]]]:
    """Per-machine operation lists, or None when ranks are not dense / placement is out of range."""
    n = len(placement)
    cnt = [0] * P
    for v in range(n):
        if not (0 <= placement[v] < P):
            return None
        cnt[placement[v]] += 1
    lists = [[-1] * cnt[j] for j in range(P)]
    for v in range(n):
        j, r = int(placement[v]), int(rank[v])
        if not (0 <= r < cnt[j]) or lists[j][r] != -1:
            return None
        lists[j][r] = v
    return lists


def tick_simulate(P, row_ptr, col_idx, dur, comm, mem_delta, placement, rank):
    """Advance a clock one unit at a time; at each tick every idle machine starts the next
    operation of its list iff every input has arrived (producer finished, plus the channel delay
    when the producer ran on another machine).  Returns None when the simulation stalls (no
    machine can ever start its next operation: the fixed orders contradict the DAG), else
    (makespan, bubble, peak_mem list, start, end).
    """
    n = len(dur)
    comm = np.asarray(comm).reshape(P, P)
    preds = pred_lists(row_ptr, col_idx)
    lists = device_lists(P, placement, rank)
    assert lists is not None
    ptr = [0] * P
    busy_until = [0] * P
    start: Dict[int, int] = {}
    end: Dict[int, int] = {}
    horizon = int(np.sum(dur)) + n * (int(comm.max()) + 1) + 2
    t = 0
    while len(start) < n:
        if t > horizon:
            return None
        changed = True
        while changed:                      # zero-duration operations may cascade inside one tick
            changed = False
            for j in range(P):
                if ptr[j] >= len(lists[j]) or busy_until[j] > t:
                    continue
                v = lists[j][ptr[j]]
                ok = True
                for u in preds[v]:
                    if u not in end:
                        ok = False
                        break
                    delay = int(comm[placement[u], j]) if placement[u] != j else 0
                    if end[u] + delay > t:
                        ok = False
                        break
                if ok:
                    start[v] = t
                    end[v] = t + int(dur[v])
                    busy_until[j] = end[v]
                    ptr[j] += 1
                    changed = True
        t += 1
    z = max(end.values()) if end else 0
    bubble = P * z - int(np.sum(dur))
    peaks = []
    for j in range(P):
        level, top = 0, 0
        for v in lists[j]:
            level += int(mem_delta[v])
            top = max(top, level)
        peaks.append(top)
    s = np.array([start[v] for v in range(n)], dtype=np.int64)
    e = np.array([end[v] for v in range(n)], dtype=np.int64)
    return z, bubble, peaks, s, e


def linear_extensions(row_ptr, col_idx):
    """All topological orders of a tiny DAG (n <= 9 or so)."""
    n = len(row_ptr) - 1
    preds = pred_lists(row_ptr, col_idx)
    order: List[int] = []
    used = [False] * n

    def rec():
        if len(order) == n:
            yield tuple(order)
            return
        for v in range(n):
            if not used[v] and all(used[u] for u in preds[v]):
                used[v] = True
                order.append(v)
                yield from rec()
                order.pop()
                used[v] = False

    yield from rec()


def all_order_tuples(P: int, placement):
    """Every tuple of per-machine permutations for a fixed placement, as rank arrays."""
    n = len(placement)
    groups = [[v for v in range(n) if placement[v] == j] for j in range(P)]
    for perms in itertools.product(*[itertools.permutations(g) for g in groups]):
        rank = np.zeros(n, dtype=np.int32)
        for lst in perms:
            for r, v in enumerate(lst):
                rank[v] = r
        yield tuple(tuple(p) for p in perms), rank


def project_extension(P: int, placement, ext: Sequence[int]):
    return tuple(tuple(v for v in ext if placement[v] == j) for j in range(P))


def critical_path(row_ptr, col_idx, dur, edge_delay=None) -> int:
    """Longest path (sum of node durations plus optional per-edge delays), memoised recursion."""
    n = len(dur)
    preds = pred_lists(row_ptr, col_idx)

    @lru_cache(maxsize=None)
    def finish(v: int) -> int:
        best = 0
        for u in preds[v]:
            d = 0 if edge_delay is None else edge_delay(u, v)
            best = max(best, finish(u) + d)
        return best + int(dur[v])

    import sys
    sys.setrecursionlimit(max(10000, 4 * n))
    return max(finish(v) for v in range(n)) if n else 0


def check_constraints(P, row_ptr, col_idx, dur, comm, mem_delta, placement, rank, start, end, m_minus, m_plus,
                      makespan, weight=None) -> None:
    """Assert the rows of the MIP with x, y, u fixed by (placement, rank), plus minimality."""
    n = len(dur)
    comm = np.asarray(comm).reshape(P, P)
    preds = pred_lists(row_ptr, col_idx)
    lists = device_lists(P, placement, rank)
    assert lists is not None
    # eq. (2): z >= e_i, and z is attained
    assert all(makespan >= end[v] for v in range(n))
    assert makespan == max(int(end[v]) for v in range(n))
    # eq. (3): e_i - s_i = D^o_i ; all machines available at the beginning: s >= 0
    for v in range(n):
        assert end[v] - start[v] == dur[v]
        assert start[v] >= 0
    # eq. (7) with y fixed: every earlier operation of the machine ends before a later one starts
    for lst in lists:
        for a in range(len(lst)):
            for b in range(a + 1, len(lst)):
                assert end[lst[a]] <= start[lst[b]]
    # eqs. (11)-(13): c >= e_u, d - c >= D^c, s_v >= d   =>   s_v >= e_u + D^c when machines differ
    for v in range(n):
        for u in preds[v]:
            delay = int(comm[placement[u], placement[v]]) if placement[u] != placement[v] else 0
            assert start[v] >= end[u] + delay
    # tightness (earliest-start schedule): s_v is 0 or equals one of its lower bounds
    pos = {}
    for lst in lists:
        for r, v in enumerate(lst):
            pos[v] = (lst, r)
    for v in range(n):
        bounds = [0]
        lst, r = pos[v]
        if r > 0:
            bounds.append(int(end[lst[r - 1]]))
        for u in preds[v]:
            delay = int(comm[placement[u], placement[v]]) if placement[u] != placement[v] else 0
            bounds.append(int(end[u]) + delay)
        assert start[v] == max(bounds)
    # eq. (16): m-_i >= sum of the static memory W of everything on i's machine, tight for the machine's first
    # operation (base level 0 without weights); eqs. (17)-(19): m+_i - m-_i = A_i ; m-_next = m+_prev
    for j, lst in enumerate(lists):
        base = 0 if weight is None else sum(int(weight[v]) for v in range(n) if placement[v] == j)
        for r, v in enumerate(lst):
            assert m_plus[v] - m_minus[v] == mem_delta[v]
            if r == 0:
                assert m_minus[v] == base
            else:
                assert m_minus[v] == m_plus[lst[r - 1]]


def tick_simulate_channels(P, row_ptr, col_idx, dur, comm, placement, rank, edge_order):
    """Unit-step simulation of the model WITH channel contention (Sec. III, eqs. (11)-(15)), written from the
    definition and independent of any graph rewriting: an edge (u, v) across machines is a transfer that occupies the
    channel (pi(u), pi(v)) for comm[pi(u)][pi(v)] time units, cannot start before u has ended, and must have ended
    before v starts; the transfers of a channel run one at a time in the order `edge_order[channel]` (a list of
    edge indices k into col_idx).  Edges inside a machine need no transfer.  Returns None when the simulation
    stalls, else (makespan, start [N], end [N], transfer_end {k: time}).
    """
    n = len(dur)
    comm = np.asarray(comm).reshape(P, P)
    src = np.repeat(np.arange(n), np.diff(row_ptr))
    in_edges: List[List[int]] = [[] for _ in range(n)]
    for k in range(len(col_idx)):
        in_edges[int(col_idx[k])].append(k)
    lists = device_lists(P, placement, rank)
    assert lists is not None
    ptr = [0] * P
    busy_until = [0] * P
    cptr = {ch: 0 for ch in edge_order}
    cbusy = {ch: 0 for ch in edge_order}
    start: Dict[int, int] = {}
    end: Dict[int, int] = {}
    t_end: Dict[int, int] = {}
    horizon = int(np.sum(dur)) + (len(col_idx) + n) * (int(comm.max()) + 1) + 2
    t = 0
    while len(start) < n:
        if t > horizon:
            return None
        changed = True
        while changed:                      # zero durations may cascade inside one tick
            changed = False
            for ch, order in edge_order.items():
                if cptr[ch] >= len(order) or cbusy[ch] > t:
                    continue
                k = order[cptr[ch]]
                u = int(src[k])
                if u in end and end[u] <= t:
                    t_end[k] = t + int(comm[ch[0], ch[1]])
                    cbusy[ch] = t_end[k]
                    cptr[ch] += 1
                    changed = True
            for j in range(P):
                if ptr[j] >= len(lists[j]) or busy_until[j] > t:
                    continue
                v = lists[j][ptr[j]]
                ok = True
                for k in in_edges[v]:
                    u = int(src[k])
                    if placement[u] == j:
                        ok = u in end and end[u] <= t
                    else:
                        ok = k in t_end and t_end[k] <= t
                    if not ok:
                        break
                if ok:
                    start[v] = t
                    end[v] = t + int(dur[v])
                    busy_until[j] = end[v]
                    ptr[j] += 1
                    changed = True
        t += 1
    z = max(end.values()) if end else 0
    s = np.array([start[v] for v in range(n)], dtype=np.int64)
    e = np.array([end[v] for v in range(n)], dtype=np.int64)
    return z, s, e, t_end
