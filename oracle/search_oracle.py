"""CPU oracle for the local-search helpers around the evaluator.  TEST INFRASTRUCTURE ONLY.

The paper hands the search over the binaries x, y to a MIP solver (Sec. IV-V); a planner that scores
candidates with the batched evaluator needs something that produces candidates.  The helpers here
define, in plain numpy, the neighbourhood used for that: every candidate is the base schedule with
ONE local move applied, the move being fixed by four random words that the caller passes in (so the
GPU path and this oracle see the same draws):

    candidate 0            the base schedule itself
    candidate c >= 1       r0..r3 = rnd[4c .. 4c+3];  v = r1 mod N is the operation that moves;
                           m = placement[v], r = rank[v], n_j = operations on machine j in the base
      r0 even  "swap"      v trades places with the operation right after it on its machine
                           (nothing happens when v is the last one there)
      r0 odd   "move"      m2 = r2 mod P.  m2 == m: v is re-inserted at position r3 mod n_m of its own
                           machine;  m2 != m: v is inserted at position r3 mod (n_m2 + 1) of machine m2.
                           Every other operation keeps its relative order.
    orders only            the same with m2 = m whatever r2 is: the allocation x of the base is kept and only the
                           orders are searched, as in the pipeline experiments of Sec. V, where the stage ->
                           machine map is given.

A dense base gives dense candidates (each machine's ranks stay 0..n_j-1); a move may well make the
combined graph cyclic, which the evaluator then flags.  `select` picks the feasible candidate of least
makespan, the lowest index among equals.

Pinned in tests/test_search_oracle.py against explicit Python lists (pop / insert) and by invariants.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def propose(base_placement, base_rank, rnd, n_devices: int, orders_only: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """-> (placement int32 [C, N], rank int32 [C, N]) with C = len(rnd) // 4."""
    pl0 = np.ascontiguousarray(base_placement, dtype=np.int32).reshape(-1)
    rk0 = np.ascontiguousarray(base_rank, dtype=np.int32).reshape(-1)
    rnd = np.ascontiguousarray(rnd).astype(np.uint32).reshape(-1, 4)
    n, c_total = pl0.shape[0], rnd.shape[0]
    cnt = np.bincount(pl0, minlength=n_devices)
    out_pl = np.tile(pl0, (c_total, 1))
    out_rk = np.tile(rk0, (c_total, 1))
    for c in range(1, c_total):
        r0, r1, r2, r3 = (int(x) for x in rnd[c])
        v = r1 % n
        m, r = int(pl0[v]), int(rk0[v])
        pl, rk = out_pl[c], out_rk[c]
        if r0 % 2 == 0:
            if r + 1 < cnt[m]:
                other = (pl0 == m) & (rk0 == r + 1)
                rk[other] = r
                rk[v] = r + 1
        else:
            m2 = m if orders_only else r2 % n_devices
            if m2 == m:
                r_new = r3 % int(cnt[m])
                same = pl0 == m
                if r_new > r:
                    rk[same & (rk0 > r) & (rk0 <= r_new)] -= 1
                elif r_new < r:
                    rk[same & (rk0 >= r_new) & (rk0 < r)] += 1
                rk[v] = r_new
            else:
                r_new = r3 % (int(cnt[m2]) + 1)
                rk[(pl0 == m) & (rk0 > r)] -= 1
                rk[(pl0 == m2) & (rk0 >= r_new)] += 1
                pl[v] = m2
                rk[v] = r_new
    return out_pl, out_rk


def select(makespan, flags) -> Tuple[int, int]:
    """-> (index, makespan) of the feasible candidate with the least makespan, lowest index among
    equals; (-1, -1) when no candidate is feasible."""
    makespan = np.asarray(makespan)
    flags = np.asarray(flags)
    ok = np.flatnonzero(flags == 0)
    if ok.size == 0:
        return -1, -1
    best = ok[int(np.argmin(makespan[ok]))]            # argmin returns the first of equal minima
    return int(best), int(makespan[best])
