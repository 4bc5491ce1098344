"""Parity of dagsched_coarsen (Sec. IV, Alg. 1 on the GPU) against the CPU oracle, through the C-ABI: the same
node map, coarse CSR, summed attributes and merge counts, bit for bit; at the size of the MoE operator graph, which
the oracle cannot finish, the invariants of MergeNodes instead."""
from __future__ import annotations

import sys

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[gpu-coarsen] " + msg, flush=True)
    sys.stdout.flush()


def _same(ds, rp, ci, dur, mem, req, **kw):
    n = len(rp) - 1
    _say("N=%d E=%d %s" % (n, len(ci), kw))
    got = ds.coarsen(rp, ci, dur, mem, req, **kw)
    want = oracle.coarsen(rp, ci, dur, mem, req, **kw)
    for key in ("n_coarse", "merges_edge", "merges_nonedge"):
        assert got[key] == want[key], (key, got[key], want[key])
    for key in ("node_map", "row_ptr", "col_idx", "dur", "mem_delta", "mem_req"):
        assert got[key].shape == want[key].shape and (got[key] == want[key]).all(), key
    return got


def _graph(n, edges):
    return W.csr_from_edges(n, [a for a, _ in edges], [b for _, b in edges])


def test_hand_worked_graphs(gpu_lib):
    ds = gpu_lib
    off = ds.NO_MERGES
    for n, edges in ((3, [(0, 1), (1, 2), (0, 2)]), (4, [(0, 1), (1, 2), (2, 3), (0, 3)]),
                     (4, [(0, 1), (0, 2), (1, 3), (2, 3)]), (4, [(0, 3), (1, 3), (2, 3)]), (1, []), (5, [])):
        rp, ci = _graph(n, edges)
        dur = np.arange(1, n + 1)
        for target in range(1, n + 1):
            _same(ds, rp, ci, dur, np.arange(n) - 1, None, target=target)
            _same(ds, rp, ci, dur, np.arange(n) - 1, None, target=target, nonedge_dur_max=off)
            _same(ds, rp, ci, dur, np.arange(n) - 1, np.arange(n), target=target, edge_dur_max=off, nonedge_mem_max=3)


def test_chains_under_a_threshold(gpu_lib):
    for n, T in ((10, 3), (64, 64), (65, 7), (130, 1), (200, 50)):
        rp, ci = _graph(n, [(i, i + 1) for i in range(n - 1)])
        got = _same(gpu_lib, rp, ci, np.ones(n), np.arange(n), None, target=1, edge_dur_max=T, nonedge_dur_max=gpu_lib.NO_MERGES)
        assert got["n_coarse"] == -(-n // T)


@pytest.mark.parametrize("seed", range(8))
def test_random_graphs(gpu_lib, seed):
    """Sizes around the 64-bit words of the adjacency rows, duplicate edges, zero durations, every mix of thresholds."""
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.choice([2, 17, 63, 64, 65, 128, 129, 300, 777]))
    rp, ci = W.random_dag(rng, n, int(rng.integers(1, 5)), window=int(rng.integers(3, 40)), dup_prob=0.1)
    dur = rng.integers(0, 12, n)
    mem = rng.integers(-9, 10, n)
    req = rng.integers(0, 8, n) if seed % 2 else None
    for _ in range(3):
        kw = dict(target=int(rng.integers(1, n + 1)),
                  edge_dur_max=int(rng.choice([-1, 10, 40, 2 ** 62])), edge_mem_max=int(rng.choice([5, 30, 2 ** 62])),
                  nonedge_dur_max=int(rng.choice([-1, 6, 25, 2 ** 62])), nonedge_mem_max=int(rng.choice([4, 20, 2 ** 62])))
        _same(gpu_lib, rp, ci, dur, mem, req, **kw)


def test_random_graph_of_section_5b_scale(gpu_lib):
    rng = np.random.default_rng(20250309)
    rp, ci = W.random_dag_bounded_degree(rng, 200, 3)
    got = _same(gpu_lib, rp, ci, rng.integers(1, 20, 200), rng.integers(-3, 4, 200), rng.integers(0, 10, 200), target=40,
                edge_dur_max=200, edge_mem_max=200, nonedge_dur_max=80, nonedge_mem_max=80)
    assert got["n_coarse"] == 40


@pytest.mark.parametrize("cfg,target", [(1, 8), (2, 100), (3, 5000)])
def test_operator_graphs_of_the_workloads(gpu_lib, cfg, target):
    """The pipeline graphs of configurations 1-3 (64, 768 and 6144 operations; for the last the oracle is given a
    target it reaches after few merges)."""
    w = W.gen_config(cfg, n_cand=1)
    if cfg == 3:
        n = 1200                                             # the first 1200 operations and the edges among them
        src, dst = W.edges_from_csr(w.row_ptr, w.col_idx)
        keep = (src < n) & (dst < n)
        rp, ci = W.csr_from_edges(n, src[keep], dst[keep])
        _same(gpu_lib, rp, ci, w.dur[:n], w.mem_delta[:n], None, target=1000, edge_dur_max=20, nonedge_dur_max=12)
        return
    _same(gpu_lib, w.row_ptr, w.col_idx, w.dur, w.mem_delta, None, target=target, edge_dur_max=30, nonedge_dur_max=15)


def test_moe_operator_graph_at_full_size(gpu_lib):
    """11712 operations, 25360 edges: beyond what the oracle finishes, so the properties that hold at any size: the
    sums per group, coarse edges = images of the original edges, acyclic, groups numbered by their smallest member,
    thresholds kept, and the counts add up."""
    w = W.gen_config(4, n_cand=1)
    n = w.n_nodes
    req = (np.arange(n) % 5).astype(np.int64)
    r = gpu_lib.coarsen(w.row_ptr, w.col_idx, w.dur, w.mem_delta, req, target=n - 700, edge_dur_max=40, edge_mem_max=9,
                        nonedge_dur_max=6, nonedge_mem_max=4)
    k, nm = r["n_coarse"], r["node_map"]
    _say("MoE graph: %d -> %d operations, %d edge merges, %d non-edge merges" % (n, k, r["merges_edge"], r["merges_nonedge"]))
    assert k == n - r["merges_edge"] - r["merges_nonedge"] and k >= n - 700 and r["merges_edge"] > 0
    assert sorted(set(nm.tolist())) == list(range(k))
    first = np.full(k, n)
    np.minimum.at(first, nm, np.arange(n))
    assert (np.diff(first) > 0).all()
    for src_attr, got in ((w.dur, r["dur"]), (w.mem_delta, r["mem_delta"]), (req, r["mem_req"])):
        want = np.zeros(k, np.int64)
        np.add.at(want, nm, src_attr.astype(np.int64))
        assert (want == got).all()
    src, dst = W.edges_from_csr(w.row_ptr, w.col_idx)
    want_edges = {(int(a), int(b)) for a, b in zip(nm[src], nm[dst]) if a != b}
    got_edges = {(u, int(v)) for u in range(k) for v in r["col_idx"][r["row_ptr"][u]:r["row_ptr"][u + 1]]}
    assert got_edges == want_edges and len(r["col_idx"]) == len(want_edges)
    size = np.bincount(nm, minlength=k)
    assert (r["dur"][size > 1] <= 40).all() and (r["mem_req"][size > 1] <= 9).all()
    # acyclic: peel sources
    indeg = np.bincount(r["col_idx"], minlength=k)
    stack = [v for v in range(k) if indeg[v] == 0]
    seen = 0
    while stack:
        u = stack.pop()
        seen += 1
        for v in r["col_idx"][r["row_ptr"][u]:r["row_ptr"][u + 1]]:
            indeg[v] -= 1
            if indeg[v] == 0:
                stack.append(int(v))
    assert seen == k


def test_refused_inputs(gpu_lib):
    ds = gpu_lib
    rp, ci = _graph(3, [(0, 1), (1, 2), (2, 0)])
    with pytest.raises(ds.DagschedError) as e:
        ds.coarsen(rp, ci, [1, 1, 1], [0, 0, 0])
    assert e.value.code == ds.ECYCLE
    rp, ci = _graph(2, [(0, 1)])
    for kw in (dict(dur=[1, -1]), dict(mem_req=[0, -2]), dict(target=0)):
        args = dict(dur=[1, 1], mem_req=None, target=1)
        args.update(kw)
        with pytest.raises(ds.DagschedError) as e:
            ds.coarsen(rp, ci, args["dur"], [0, 0], args["mem_req"], target=args["target"])
        assert e.value.code == ds.EINVAL
    with pytest.raises(ds.DagschedError) as e:
        ds.coarsen(rp, ci, [2 ** 31 - 1, 1], [0, 0])
    assert e.value.code == ds.EOVERFLOW
