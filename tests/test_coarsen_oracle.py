"""Pins of the coarsening oracle (oracle/coarsen_oracle.c; Sec. IV, Alg. 1) against what the section and the
mathematics fix: hand-worked graphs for the two-hop redundancy rule, the single-input / single-output rule and the
equal-depth rule, a closed form, invariants of MergeNodes, the scale of Sec. V-B, and a second evaluator written
with Python sets from the definitions.  No GPU."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W

OFF = oracle.NO_MERGES


def _graph(n, edges):
    return W.csr_from_edges(n, [a for a, _ in edges], [b for _, b in edges])


def _groups(node_map):
    g = {}
    for v, k in enumerate(node_map):
        g.setdefault(int(k), []).append(v)
    return [g[k] for k in sorted(g)]


def _coarse_edges(r):
    return {(u, int(v)) for u in range(r["n_coarse"]) for v in r["col_idx"][r["row_ptr"][u]:r["row_ptr"][u + 1]]}


def _critical_path(rp, ci, dur):
    """Longest path, durations summed over its operations (textbook DP in a topological order)."""
    n = len(rp) - 1
    indeg = np.zeros(n, int)
    for v in ci:
        indeg[v] += 1
    fin = np.array(dur, dtype=np.int64).copy()
    order = [v for v in range(n) if indeg[v] == 0]
    for u in order:
        for v in ci[rp[u]:rp[u + 1]]:
            fin[v] = max(fin[v], fin[u] + dur[v])
            indeg[v] -= 1
            if indeg[v] == 0:
                order.append(int(v))
    assert len(order) == n, "cyclic"
    return int(fin.max())


# --------------------------------------------------------------------------- hand-worked graphs

def test_two_hop_rule_makes_a_triangle_a_chain():
    """a->b->c with the shortcut a->c: the shortcut is redundant, so a has a single output and c a single input in
    the reduced graph and the lowest candidate edge is (a, b); then {a,b}->c.  With the shortcut counted, nothing
    would be a candidate (a has two outputs, c two inputs)."""
    rp, ci = _graph(3, [(0, 1), (1, 2), (0, 2)])
    r = oracle.coarsen(rp, ci, [1, 2, 4], [1, 1, 1], target=2, nonedge_dur_max=OFF)
    assert _groups(r["node_map"]) == [[0, 1], [2]] and r["dur"].tolist() == [3, 4] and r["merges_edge"] == 1
    assert _coarse_edges(r) == {(0, 1)}                       # the two edges into c collapse into one
    r = oracle.coarsen(rp, ci, [1, 2, 4], [1, 1, 1], target=1, nonedge_dur_max=OFF)
    assert r["n_coarse"] == 1 and r["dur"].tolist() == [7] and r["row_ptr"].tolist() == [0, 0]


def test_a_three_hop_shortcut_is_not_redundant():
    """a->b->c->d with a->d: only two-hop shortcuts are removed, so a keeps two outputs and d two inputs.  The only
    candidate is (b, c).  After that merge the shortcut a->d spans two hops, becomes redundant, and (a, {b,c}) is
    next: the sequence of merges is fixed by the rule."""
    rp, ci = _graph(4, [(0, 1), (1, 2), (2, 3), (0, 3)])
    r = oracle.coarsen(rp, ci, [1, 1, 1, 1], [0, 0, 0, 0], target=3, nonedge_dur_max=OFF)
    assert _groups(r["node_map"]) == [[0], [1, 2], [3]]
    assert _coarse_edges(r) == {(0, 1), (1, 2), (0, 2)}
    r = oracle.coarsen(rp, ci, [1, 1, 1, 1], [0, 0, 0, 0], target=2, nonedge_dur_max=OFF)
    assert _groups(r["node_map"]) == [[0, 1, 2], [3]]


def test_single_input_single_output_rule_on_a_diamond():
    """a->{b,c}->d: a has two outputs and d two inputs, so no edge is a candidate and without non-edge merges the
    graph stays as it is.  b and c have equal depth: the non-edge rule merges them, after which the graph is a
    chain and the edge rule finishes it."""
    rp, ci = _graph(4, [(0, 1), (0, 2), (1, 3), (2, 3)])
    r = oracle.coarsen(rp, ci, [5, 1, 2, 7], [1, -1, 2, -2], target=1, nonedge_dur_max=OFF)
    assert r["n_coarse"] == 4 and r["merges_edge"] == 0
    r = oracle.coarsen(rp, ci, [5, 1, 2, 7], [1, -1, 2, -2], target=3)
    assert _groups(r["node_map"]) == [[0], [1, 2], [3]] and (r["merges_edge"], r["merges_nonedge"]) == (0, 1)
    assert r["dur"].tolist() == [5, 3, 7] and r["mem_delta"].tolist() == [1, 1, -2]
    r = oracle.coarsen(rp, ci, [5, 1, 2, 7], [1, -1, 2, -2], target=1)
    assert r["n_coarse"] == 1 and (r["merges_edge"], r["merges_nonedge"]) == (2, 1) and r["dur"].tolist() == [15]


def test_non_edge_rule_takes_the_lightest_pair_of_equal_depth():
    """Three sources feeding one sink: the sources have depth 0, the sink depth 1.  The lightest pair of sources is
    merged first (durations 4 and 2: operations 1 and 2), never a source with the sink; a threshold below the
    lightest sum forbids every pair."""
    rp, ci = _graph(4, [(0, 3), (1, 3), (2, 3)])
    dur = [9, 4, 2, 1]
    r = oracle.coarsen(rp, ci, dur, [0] * 4, target=3, edge_dur_max=OFF)
    assert _groups(r["node_map"]) == [[0], [1, 2], [3]]
    r = oracle.coarsen(rp, ci, dur, [0] * 4, target=1, edge_dur_max=OFF)
    assert _groups(r["node_map"]) == [[0, 1, 2], [3]]        # the sink has no partner of its depth
    r = oracle.coarsen(rp, ci, dur, [0] * 4, target=1, edge_dur_max=OFF, nonedge_dur_max=5)
    assert r["n_coarse"] == 4
    # the memory requirement has a threshold of its own
    r = oracle.coarsen(rp, ci, dur, [0] * 4, mem_req=[1, 5, 5, 0], target=1, edge_dur_max=OFF, nonedge_mem_max=6)
    # summed durations: (0,1) 13, (0,2) 11, (1,2) 6; the lightest, (1,2), needs 10 > 6 and is forbidden; (0,2) needs
    # exactly 6 and is the lightest allowed pair; after it {0,2} needs 6 and no further pair fits
    assert _groups(r["node_map"]) == [[0, 2], [1], [3]] and r["mem_req"].tolist() == [6, 5, 0]


def test_chain_under_a_duration_threshold_has_a_closed_form():
    """A path of n unit operations, threshold T on a merged duration: the lowest edge is merged first, so the head
    group grows to T and the next group starts: ceil(n / T) groups, all of T operations but the last."""
    for n, T in ((10, 3), (17, 4), (64, 64), (9, 1), (33, 5)):
        rp, ci = _graph(n, [(i, i + 1) for i in range(n - 1)])
        r = oracle.coarsen(rp, ci, np.ones(n), np.arange(n), target=1, edge_dur_max=T, nonedge_dur_max=OFF)
        want = [list(range(s, min(n, s + T))) for s in range(0, n, T)]
        assert _groups(r["node_map"]) == want
        assert r["dur"].tolist() == [len(g) for g in want]
        assert r["mem_delta"].tolist() == [sum(g) for g in want]
        assert _coarse_edges(r) == {(k, k + 1) for k in range(len(want) - 1)}
        # the target stops the merging exactly when it is reached
        if n > 4 and T >= 2:
            r = oracle.coarsen(rp, ci, np.ones(n), np.arange(n), target=n - 1, edge_dur_max=T, nonedge_dur_max=OFF)
            assert r["n_coarse"] == n - 1 and _groups(r["node_map"])[0] == [0, 1]


# --------------------------------------------------------------------------- invariants

@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_random_graphs(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(20, 120))
    rp, ci = W.random_dag(rng, n, 3, window=15, dup_prob=0.1)
    dur = rng.integers(0, 9, n)
    mem = rng.integers(-5, 6, n)
    req = rng.integers(0, 7, n)
    target = int(rng.integers(1, n))
    r = oracle.coarsen(rp, ci, dur, mem, req, target=target, edge_dur_max=40, nonedge_dur_max=25, nonedge_mem_max=30)
    k, nm = r["n_coarse"], r["node_map"]
    assert k == n - r["merges_edge"] - r["merges_nonedge"] and k >= target
    assert sorted(set(nm.tolist())) == list(range(k))
    # groups are numbered by their smallest member
    firsts = [g[0] for g in _groups(nm)]
    assert firsts == sorted(firsts)
    # MergeNodes: sums of the attributes, group by group
    for name, src, got in (("dur", dur, r["dur"]), ("mem", mem, r["mem_delta"]), ("req", req, r["mem_req"])):
        assert np.bincount(nm, weights=src, minlength=k).astype(np.int64).tolist() == got.tolist(), name
    # ... and the original connectivity: coarse edges are exactly the images of the original edges between groups
    src_e, dst_e = W.edges_from_csr(rp, ci)
    want = {(int(nm[a]), int(nm[b])) for a, b in zip(src_e, dst_e) if nm[a] != nm[b]}
    assert _coarse_edges(r) == want
    for u in range(k):                                        # ascending, no duplicates
        row = r["col_idx"][r["row_ptr"][u]:r["row_ptr"][u + 1]].tolist()
        assert row == sorted(set(row))
    _critical_path(r["row_ptr"], r["col_idx"], r["dur"])      # asserts that the coarse graph is acyclic
    # thresholds hold for every group that was formed by a merge (a single operation may exceed them on its own)
    for g, d in zip(_groups(nm), r["dur"]):
        assert len(g) == 1 or d <= 40


@pytest.mark.parametrize("seed", range(5))
def test_edge_merges_keep_the_critical_path(seed):
    """Sec. IV: merging an edge whose head has a single input and whose tail has a single output does not lengthen
    the critical path.  With the non-edge merges switched off it is the same before and after, whatever the target."""
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(30, 150))
    rp, ci = W.random_dag(rng, n, 2, window=6)
    dur = rng.integers(1, 9, n)
    before = _critical_path(rp, ci, dur)
    r = oracle.coarsen(rp, ci, dur, np.zeros(n), target=1, nonedge_dur_max=OFF)
    assert r["merges_edge"] > 0 and r["merges_nonedge"] == 0
    assert _critical_path(r["row_ptr"], r["col_idx"], r["dur"]) == before
    assert int(r["dur"].sum()) == int(dur.sum())              # one machine: the makespan is the sum, merged or not


def test_random_graph_of_section_5b_scale():
    """Sec. V-B: a random graph of 200 operations with in- and out-degrees up to 3 is coarsened to 40 operations."""
    rng = np.random.default_rng(20250309)
    rp, ci = W.random_dag_bounded_degree(rng, 200, 3)
    src, dst = W.edges_from_csr(rp, ci)
    assert np.bincount(src, minlength=200).max() <= 3 and np.bincount(dst, minlength=200).max() <= 3
    dur = rng.integers(1, 20, 200)
    r = oracle.coarsen(rp, ci, dur, rng.integers(-3, 4, 200), rng.integers(0, 10, 200), target=40,
                       edge_dur_max=200, edge_mem_max=200, nonedge_dur_max=80, nonedge_mem_max=80)
    assert r["n_coarse"] == 40 and r["merges_edge"] > 0 and r["merges_nonedge"] > 0
    assert int(r["dur"].sum()) == int(dur.sum())
    _critical_path(r["row_ptr"], r["col_idx"], r["dur"])


# --------------------------------------------------------------------------- a second evaluator, from the definitions

def _coarsen_sets(n, edges, dur, target, e_max, n_max):
    """Alg. 1 with Python sets (durations only): names are frozensets of original operations."""
    succ = {v: set() for v in range(n)}
    for a, b in edges:
        succ[a].add(b)
    members = {v: {v} for v in range(n)}
    d = {v: int(dur[v]) for v in range(n)}

    def pred_of():
        p = {v: set() for v in succ}
        for a in succ:
            for b in succ[a]:
                p[b].add(a)
        return p

    def reduced():
        return {a: {b for b in succ[a] if not any(b in succ[w] for w in succ[a])} for a in succ}

    def cand_edge():
        red = reduced()
        indeg = {v: 0 for v in succ}
        for a in red:
            for b in red[a]:
                indeg[b] += 1
        ok = [(a, b) for a in red for b in red[a] if len(red[a]) == 1 and indeg[b] == 1 and d[a] + d[b] <= e_max]
        return min(ok) if ok else None

    def cand_nonedge():
        pred = pred_of()
        depth = {}

        def dep(v):
            if v not in depth:
                depth[v] = 1 + max((dep(u) for u in pred[v]), default=-1)
            return depth[v]
        ok = [(d[a] + d[b], a, b) for a in succ for b in succ if a < b and dep(a) == dep(b) and d[a] + d[b] <= n_max]
        return min(ok)[1:] if ok else None

    def merge(a, b):
        m, o = min(a, b), max(a, b)
        members[m] |= members.pop(o)
        d[m] += d.pop(o)
        succ[m] |= succ.pop(o)
        for x in succ:
            if o in succ[x]:
                succ[x].discard(o)
                succ[x].add(m)
        succ[m].discard(m)

    while len(succ) > target:
        merged = False
        while len(succ) > target and (c := cand_edge()):
            merge(*c); merged = True
        while len(succ) > target and (c := cand_nonedge()):
            merge(*c); merged = True
        if not merged:
            break
    names = sorted(succ)
    node_map = [0] * n
    for k, m in enumerate(names):
        for v in members[m]:
            node_map[v] = k
    return node_map, [d[m] for m in names]


@pytest.mark.parametrize("seed", range(12))
def test_against_a_set_based_evaluator_on_tiny_graphs(seed):
    rng = np.random.default_rng(900 + seed)
    n = int(rng.integers(2, 26))
    rp, ci = W.random_dag(rng, n, 3, window=8)
    src, dst = W.edges_from_csr(rp, ci)
    dur = rng.integers(0, 7, n)
    target = int(rng.integers(1, n + 1))
    e_max, n_max = int(rng.integers(3, 30)), int(rng.integers(0, 14))
    r = oracle.coarsen(rp, ci, dur, np.zeros(n), target=target, edge_dur_max=e_max, nonedge_dur_max=n_max)
    nm, d = _coarsen_sets(n, list(zip(src.tolist(), dst.tolist())), dur, target, e_max, n_max)
    assert r["node_map"].tolist() == nm and r["dur"].tolist() == d


# --------------------------------------------------------------------------- malformed problems

def test_malformed_problems_are_refused():
    rp, ci = _graph(3, [(0, 1), (1, 2), (2, 0)])
    with pytest.raises(oracle.OracleError) as e:
        oracle.coarsen(rp, ci, [1, 1, 1], [0, 0, 0])
    assert e.value.code == oracle.ECYCLE
    rp, ci = _graph(2, [(0, 1)])
    for bad in (dict(dur=[1, -1]), dict(mem_req=[0, -2]), dict(target=0)):
        kw = dict(dur=[1, 1], mem_delta=[0, 0], mem_req=None, target=1)
        kw.update(bad)
        with pytest.raises(oracle.OracleError) as e:
            oracle.coarsen(rp, ci, kw["dur"], kw["mem_delta"], kw["mem_req"], target=kw["target"])
        assert e.value.code == oracle.EINVAL
