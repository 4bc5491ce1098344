"""Channel contention (Sec. III, eqs. (14)-(15)) for workloads whose candidates all share one placement.

The evaluator treats a channel delay as a pure latency: two transfers over the same channel may overlap.  The
paper's model lets them not: the transfers assigned to one channel are ordered and must not overlap.  When the
placement is the same for every candidate (a pipeline: stage -> machine), that model is expressed with what the
evaluator already has: every DAG edge (u, v) whose endpoints sit on different machines becomes a *transfer* node of
duration comm[pi(u)][pi(v)] on a channel-machine of its own pair (pi(u), pi(v)), with edges u -> transfer -> v and
zero delays; the order of the transfers of a channel is part of the candidate, like the order of the operations of
a machine.  Edges inside a machine stay as they are.  This module only rewrites inputs; it holds no evaluation.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

from .workloads import Workload, csr_from_edges


def with_channels(w: Workload, max_machines: int = 64) -> Tuple[Workload, np.ndarray, np.ndarray]:
    """Returns (expanded workload, cross_edges [Ec, 2], edge_rank [C, Ec]).

    The expanded workload has N + Ec nodes (the transfers last, in CSR order of the cross edges), P + (channels in
    use) machines and an all-zero delay matrix.  Transfers of a channel are ranked first-come-first-served: by the
    rank of their producer on its machine, ties (several edges out of one producer) by edge order - an order that
    can never contradict the DAG.  edge_rank is that rank, for callers that want to permute it.
    """
    pl0 = np.asarray(w.placement[0])
    if not (w.placement == pl0).all():
        raise ValueError("every candidate must use the same placement")
    n, p, c = w.n_nodes, w.n_devices, w.n_cand
    src = np.repeat(np.arange(n, dtype=np.int64), np.diff(w.row_ptr))
    dst = np.asarray(w.col_idx, dtype=np.int64)
    cross = np.nonzero(pl0[src] != pl0[dst])[0]
    pairs = sorted({(int(pl0[src[k]]), int(pl0[dst[k]])) for k in cross})
    chan = {ab: p + i for i, ab in enumerate(pairs)}
    p2 = p + len(pairs)
    if p2 > max_machines:
        raise ValueError("machines plus channels in use exceed %d" % max_machines)
    ec = len(cross)
    t_of = {int(k): n + i for i, k in enumerate(cross)}          # edge index -> transfer node
    e_src, e_dst = [], []
    for k in range(len(dst)):
        u, v = int(src[k]), int(dst[k])
        if k in t_of:
            e_src += [u, t_of[k]]
            e_dst += [t_of[k], v]
        else:
            e_src.append(u)
            e_dst.append(v)
    rp, ci = csr_from_edges(n + ec, e_src, e_dst)
    comm = np.asarray(w.comm).reshape(p, p)
    if any(comm[a, b] < 0 for a, b in pairs):
        raise ValueError("the shared placement sends a message over a machine pair without a channel (eq. (10))")
    dur = np.concatenate([w.dur, np.array([comm[pl0[src[k]], pl0[dst[k]]] for k in cross], dtype=np.int32)]).astype(np.int32)
    mem = np.concatenate([w.mem_delta, np.zeros(ec, dtype=np.int64)])
    t_machine = np.array([chan[(int(pl0[src[k]]), int(pl0[dst[k]]))] for k in cross], dtype=np.int32)
    placement = np.ascontiguousarray(
        np.concatenate([np.broadcast_to(pl0, (c, n)), np.broadcast_to(t_machine, (c, ec))], axis=1), dtype=np.int32)
    edge_rank = np.zeros((c, ec), dtype=np.int32)
    prod = src[cross]
    for ch in range(p, p2):
        idx = np.nonzero(t_machine == ch)[0]
        if len(idx) == 0:
            continue
        # first come, first served: producers of one channel share a machine, so their ranks order them
        key = w.rank[:, prod[idx]].astype(np.int64) * (len(dst) + 1) + cross[idx][None, :]
        order = np.argsort(key, axis=1, kind="stable")
        ranks = np.empty_like(order)
        np.put_along_axis(ranks, order, np.broadcast_to(np.arange(len(idx)), order.shape), axis=1)
        edge_rank[:, idx] = ranks
    rank = np.ascontiguousarray(np.concatenate([w.rank, edge_rank], axis=1), dtype=np.int32)
    weight = None if w.weight is None else np.concatenate([w.weight, np.zeros(ec, dtype=np.int64)])
    limit = None if w.mem_limit is None else np.concatenate([w.mem_limit, np.full(p2 - p, np.iinfo(np.int64).max // 4, dtype=np.int64)])
    out = Workload(w.name + " + channels", p2, rp, ci, dur, np.zeros((p2, p2), dtype=np.int32), mem, placement, rank,
                   dict(w.meta, n_compute_machines=p, n_operations=n), weight, limit)
    cross_edges = np.stack([src[cross], dst[cross]], axis=1).astype(np.int32) if ec else np.zeros((0, 2), np.int32)
    return out, cross_edges, edge_rank
