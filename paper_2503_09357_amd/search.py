"""A small local search around the batched evaluator, all of it on the GPU.

The paper leaves the search over placements and orders to a MIP solver (Sec. IV-V).  This driver is
the plainest stand-in: hill climbing over the one-move neighbourhood of ``dagsched_propose``.  Every
iteration draws the random words with torch's device generator, builds the neighbours, scores them
with ``dagsched_evaluate``, picks the best feasible one with ``dagsched_select`` and makes it the
next base; candidate 0 of every batch is the base itself, so the makespan never gets worse.  Nothing
is copied to the host inside the loop.  Marshalling only: each step runs in the library's kernels.
"""
from __future__ import annotations

import json
from typing import List, Optional, Tuple

CAND_MAJOR = 0


def local_search(ev, base_placement, base_rank, iterations: int, n_cand: int, seed: int = 0,
                 orders_only: bool = False) -> Tuple["torch.Tensor", "torch.Tensor", List[int]]:
    """Hill-climb from a valid base schedule (device int32 [N] tensors).  orders_only: keep the base's placement and
    search the orders alone (an evaluator made with that placement as ``shared_placement`` then stays on its
    fast kernel for the whole search).

    Returns (placement [N], rank [N], makespan after every iteration, fetched once at the end)."""
    import torch
    dev = base_placement.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    pl, rk = base_placement.clone(), base_rank.clone()
    out = ev.alloc_outputs(n_cand)
    cand = None
    best = torch.empty((iterations, 2), dtype=torch.int32, device=dev)
    for it in range(iterations):
        rnd = torch.randint(0, 2 ** 31 - 1, (4 * n_cand,), dtype=torch.int32, device=dev, generator=gen)
        cand = ev.propose(pl, rk, rnd, out=cand, orders_only=orders_only)
        z, _, _, f = ev.evaluate(cand[0], cand[1], out)
        ev.select(z, f, out=best[it])
        idx = best[it, 0:1].clamp(min=0).to(torch.int64)      # no feasible candidate cannot happen: candidate 0 is the base
        if ev.layout == CAND_MAJOR:
            pl = cand[0].index_select(0, idx).reshape(-1).clone()
            rk = cand[1].index_select(0, idx).reshape(-1).clone()
        else:
            pl = cand[0].index_select(1, idx).reshape(-1).clone()
            rk = cand[1].index_select(1, idx).reshape(-1).clone()
    history = best[:, 1].cpu().tolist() if iterations else []
    return pl, rk, history


def chrome_trace(path: str, start, end, placement, names: Optional[List[str]] = None) -> None:
    """Write the schedule as a chrome://tracing / Perfetto JSON file: one row per machine, one slice per
    operation (times as microseconds)."""
    events = []
    for i, (s, e, m) in enumerate(zip(start, end, placement)):
        events.append({"name": names[i] if names else "op%d" % i, "ph": "X", "ts": int(s), "dur": int(e) - int(s),
                       "pid": 0, "tid": int(m)})
    with open(path, "w") as f:
        json.dump({"traceEvents": events, "displayTimeUnit": "ns"}, f)
