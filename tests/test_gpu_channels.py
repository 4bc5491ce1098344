"""Parity of dagsched_evaluate_contended (channel contention, Sec. III eqs. (11)-(15), a placement per candidate)
against the CPU oracle, element by element, through the C-ABI."""
from __future__ import annotations

import dataclasses
import os
import sys

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _say(msg):
    print("[gpu-channels] " + msg, flush=True)
    sys.stdout.flush()


def _parity(ds, w, er, layout=0, repeats=2):
    import torch
    dev = torch.device("cuda", 0)
    _say("%s | N=%d E=%d P=%d C=%d layout=%d" % (w.name, w.n_nodes, w.n_edges, w.n_devices, w.n_cand, layout))
    pl, rk, e = w.placement, w.rank, er
    if layout == 1:
        pl, rk, e = (np.ascontiguousarray(a.T) for a in (pl, rk, er))
    want = oracle.Problem.of(w).evaluate_contended(pl, rk, e, layout, threads=8)
    with ds.Evaluator.for_workload(w, layout=layout, contention=True) as ev:
        tp, tr, te = (torch.from_numpy(a).to(dev) for a in (pl, rk, e))
        for _ in range(repeats):
            got = [t.cpu().numpy() for t in ev.evaluate_contended(tp, tr, te)]
            for name, a, b in zip(("flags", "makespan", "bubble", "peak_mem"), (got[3], got[0], got[1], got[2]),
                                  (want[3], want[0], want[1], want[2])):
                bad = np.nonzero(np.asarray(a != b).reshape(len(a), -1).any(axis=1))[0] if a.shape == b.shape else [0]
                assert a.shape == b.shape and len(bad) == 0, "%s differs at %s: gpu %s oracle %s" % (
                    name, bad[:6], a[bad[:6]], b[bad[:6]])
        # the plain evaluation on the same handle is not disturbed by the other one
        plain = [t.cpu().numpy() for t in ev.evaluate(tp, tr)]
        want_plain = oracle.evaluate_workload(w, layout, threads=8)
        assert all((a == b).all() for a, b in zip(plain, want_plain))
    return got


def _shuffle_some_channels(rng, w, er, every=3):
    """A random order on every channel of every third candidate (may contradict the machines' orders: a cycle)."""
    p = w.n_devices
    src = np.repeat(np.arange(w.n_nodes), np.diff(w.row_ptr))
    for c in range(0, w.n_cand, every):
        pl = w.placement[c]
        if w.n_edges == 0 or (pl < 0).any() or (pl >= p).any():
            continue
        a, b = pl[src], pl[w.col_idx]
        ch = np.where(a != b, a * p + b, -1)
        for x in np.unique(ch[ch >= 0]):
            idx = np.nonzero(ch == x)[0]
            if len(idx) > 1:
                er[c, idx] = rng.permutation(len(idx))
    return er


def test_hand_worked_example(gpu_lib):
    vals = {}
    for line in open(os.path.join(GOLDEN, "hand_contention.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = [int(x) for x in v]
    n, P = vals["n_nodes"][0], vals["n_devices"][0]
    rp, ci = W.csr_from_edges(n, vals["edges"][0::2], vals["edges"][1::2])
    w = W.Workload("hand contention", P, rp, ci, np.array(vals["dur"], np.int32), np.array(vals["comm"], np.int32).reshape(P, P),
                   np.array(vals["mem_delta"], np.int64), np.array([vals["placement"]] * 2, np.int32),
                   np.array([vals["rank"]] * 2, np.int32))
    er = np.array([vals["edge_rank_a"], vals["edge_rank_b"]], np.int32)
    z, b, pk, f = _parity(gpu_lib, w, er)
    assert f.tolist() == [0, 0] and z.tolist() == [vals["makespan_a"][0], vals["makespan_b"][0]]
    assert b.tolist() == [vals["bubble_a"][0], vals["bubble_b"][0]] and pk[0].tolist() == vals["peak_mem"]


@pytest.mark.parametrize("seed", range(10))
def test_random_instances(gpu_lib, seed):
    """Placements per candidate; first-come-first-served and random channel orders; cyclic, malformed and
    out-of-range candidates; machine counts from 1 to 64 (4096 channels); no edges at all; both layouts."""
    rng = np.random.default_rng(8800 + seed)
    p = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64]))
    n = int(rng.choice([1, 2, 9, 64, 200, 257, 900]))
    w = W.random_instance(rng, n, p, int(rng.integers(1, 70)), max_fanin=int(rng.integers(0, 5)), max_comm=7,
                          frac_arbitrary=0.15, frac_bad=0.15)
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, p, w.placement, w.rank)
    er = _shuffle_some_channels(rng, w, er)
    if w.n_edges and w.n_cand > 4:                           # malformed channel orders
        er[1, int(rng.integers(0, w.n_edges))] += 1
        er[2, :] = 0
        er[4, int(rng.integers(0, w.n_edges))] = -1
    got = _parity(gpu_lib, w, er, layout=seed % 2)
    _say("flags seen: %s" % np.unique(got[3]).tolist())


def test_moe_workload_with_contention(gpu_lib):
    """Config 4 (a placement per candidate, 992 channels): contention delays most candidates."""
    w = W.gen_config(4, n_cand=96)
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, w.n_devices, w.placement, w.rank)
    z, b, pk, f = _parity(gpu_lib, w, er)
    z0 = oracle.evaluate_workload(w, threads=8)[0]
    assert (f == 0).all() and (z >= z0).all() and (z > z0).any()
    _say("MoE: makespan with contention / without, mean %.3f" % float((z / z0).mean()))
    w2 = dataclasses.replace(w, placement=w.placement[:33], rank=w.rank[:33])
    _parity(gpu_lib, w2, er[:33], layout=1)


@pytest.mark.parametrize("cfg,c", [(1, 300), (2, 200), (3, 40), (5, 6)])
def test_other_workloads_with_contention(gpu_lib, cfg, c):
    w = W.gen_config(cfg, n_cand=c)
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, w.n_devices, w.placement, w.rank)
    _parity(gpu_lib, w, er, repeats=1)


def test_missing_channels_static_memory_and_limits_on_top(gpu_lib):
    rng = np.random.default_rng(8900)
    w = W.random_instance(rng, 40, 16, 150, max_fanin=3, max_comm=6, frac_arbitrary=0.1, frac_bad=0.1)
    comm = w.comm.copy()
    comm[2, 4] = comm[0, 1] = comm[7, 3] = -1                # pairs without a channel (eq. (10))
    w = dataclasses.replace(w, comm=comm, weight=rng.integers(0, 20, 40).astype(np.int64),
                            mem_limit=np.array([45] + [10 ** 9] * 15, dtype=np.int64))
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, 16, w.placement, w.rank)
    z, b, pk, f = _parity(gpu_lib, w, er)
    assert {0, 16, 32} <= set(f.tolist()), np.unique(f)
    z, b, pk, f = _parity(gpu_lib, w, er, layout=1)


def test_handles_without_the_workspace_refuse_and_the_bound_counts_transfers(gpu_lib):
    import torch
    ds = gpu_lib
    dev = torch.device("cuda", 0)
    w = W.gen_config(1, n_cand=4)
    er = torch.zeros((4, w.n_edges), dtype=torch.int32, device=dev)
    with ds.Evaluator.for_workload(w) as ev:
        with pytest.raises(ds.DagschedError) as e:
            ev.evaluate_contended(torch.from_numpy(w.placement).to(dev), torch.from_numpy(w.rank).to(dev), er)
        assert e.value.code == ds.EINVAL
    rp, ci = W.csr_from_edges(3, [0, 0, 1], [1, 2, 2])
    big = (2 ** 31 - 1 - 3) // 3
    ds.Evaluator(2, rp, ci, [1, 1, 1], [[0, big], [big, 0]], [0, 0, 0], 4, contention=True).close()
    ds.Evaluator(2, rp, ci, [1, 1, 3], [[0, big], [big, 0]], [0, 0, 0], 4).close()        # fine without contention
    with pytest.raises(ds.DagschedError) as e:
        ds.Evaluator(2, rp, ci, [1, 1, 3], [[0, big], [big, 0]], [0, 0, 0], 4, contention=True)
    assert e.value.code == ds.EOVERFLOW
