"""Pins of the oracle's evaluation with channel contention (oracle/dagsched_oracle.c, eqs. (11)-(15)): a hand-worked
example, a unit-time-step simulation of the model written from its definition, the cases that reduce to the
evaluation without contention, and the same model expressed as extra nodes on channel-machines.  No GPU."""
from __future__ import annotations

import os

import numpy as np
import pytest

import oracle
from checkers import tick_simulate_channels
from paper_2503_09357_amd import channels
from paper_2503_09357_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden(name):
    vals = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = [int(x) for x in v]
    return vals


def _edge_order(P, row_ptr, col_idx, placement, edge_rank):
    """{channel: [edge indices in rank order]} for the step simulation."""
    src = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    chans = {}
    for k in range(len(col_idx)):
        a, b = int(placement[src[k]]), int(placement[col_idx[k]])
        if a != b:
            chans.setdefault((a, b), []).append(k)
    return {ch: sorted(ks, key=lambda k: edge_rank[k]) for ch, ks in chans.items()}


def test_hand_worked_example():
    g = _golden("hand_contention.txt")
    n, P = g["n_nodes"][0], g["n_devices"][0]
    rp, ci = W.csr_from_edges(n, g["edges"][0::2], g["edges"][1::2])
    prob = oracle.Problem(P, rp, ci, g["dur"], np.array(g["comm"]).reshape(P, P), g["mem_delta"])
    for tag in ("a", "b"):
        f, z, start, end, t_end = prob.schedule_contended(g["placement"], g["rank"], g["edge_rank_" + tag])
        assert f == 0 and z == g["makespan_" + tag][0]
        assert end.tolist() == g["end_" + tag] and t_end.tolist() == g["transfer_end_" + tag]
        zz, bb, pk, ff = prob.evaluate_contended([g["placement"]], [g["rank"]], [g["edge_rank_" + tag]])
        assert ff[0] == 0 and zz[0] == z and bb[0] == g["bubble_" + tag][0] and pk[0].tolist() == g["peak_mem"]
    # the delays-only evaluation of the same candidate: the second transfer does not wait for the first
    f, s, e, _, _ = prob.schedule(g["placement"], g["rank"])
    assert f == 0 and e.tolist() == g["end_no_contention"]


def _random_candidates(rng, n, p, n_cand, max_fanin=3, max_comm=6, zero_dur=True):
    w = W.random_instance(rng, n, p, n_cand, max_fanin=max_fanin, max_comm=max_comm, frac_arbitrary=0.15, frac_bad=0.1,
                          zero_dur=zero_dur)
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, p, w.placement, w.rank)
    return w, er


@pytest.mark.parametrize("seed", range(6))
def test_against_the_step_simulation(seed):
    """Random problems with a placement per candidate; channel orders first come first served, and for every third
    candidate a random permutation per channel (which may contradict the orders of the machines: then the simulation
    stalls and the oracle must say CYCLIC)."""
    rng = np.random.default_rng(3100 + seed)
    n, p = int(rng.integers(3, 14)), int(rng.integers(1, 5))
    w, er = _random_candidates(rng, n, p, 40, max_comm=4)
    src = np.repeat(np.arange(n), np.diff(w.row_ptr))
    for c in range(0, w.n_cand, 3):
        for ch in range(p * p):
            idx = np.nonzero((w.placement[c, src] * p + w.placement[c, w.col_idx] == ch) & (w.placement[c, src] != w.placement[c, w.col_idx]))[0] \
                if w.n_edges and (w.placement[c] >= 0).all() and (w.placement[c] < p).all() else []
            if len(idx) > 1:
                er[c, idx] = rng.permutation(len(idx))
    prob = oracle.Problem.of(w)
    z, b, pk, f = prob.evaluate_contended(w.placement, w.rank, er)
    z0, _, pk0, f0 = prob.evaluate(w.placement, w.rank)
    seen = set()
    for c in range(w.n_cand):
        seen.add(int(f[c]))
        if f0[c] in (oracle.FLAG_BAD_PLACEMENT, oracle.FLAG_BAD_RANK):
            assert f[c] == f0[c]
            continue
        sim = tick_simulate_channels(p, w.row_ptr, w.col_idx, w.dur, w.comm, w.placement[c], w.rank[c],
                                     _edge_order(p, w.row_ptr, w.col_idx, w.placement[c], er[c]))
        if sim is None:
            assert f[c] == oracle.FLAG_CYCLIC and z[c] == -1 and b[c] == -1 and (pk[c] == -1).all()
            continue
        zs, ss, es, ts = sim
        assert f[c] == 0 and z[c] == zs and b[c] == p * zs - int(w.dur.sum())
        ff, zz, start, end, t_end = prob.schedule_contended(w.placement[c], w.rank[c], er[c])
        assert (start == ss).all() and (end == es).all()
        assert all(t_end[k] == t for k, t in ts.items()) and int((t_end >= 0).sum()) == len(ts)
        # contention can only delay, and the memory peaks depend on the machines' orders alone
        if f0[c] == 0:
            assert z[c] >= z0[c] and (pk[c] == pk0[c]).all()
    assert 0 in seen


@pytest.mark.parametrize("seed", range(4))
def test_reduces_to_the_plain_evaluation(seed):
    rng = np.random.default_rng(3200 + seed)
    n, p = int(rng.integers(10, 60)), int(rng.integers(2, 9))
    w, er = _random_candidates(rng, n, p, 60)
    # (i) zero delays: a transfer of no duration occupies nothing
    w0 = W.Workload(w.name, p, w.row_ptr, w.col_idx, w.dur, np.zeros((p, p), np.int32), w.mem_delta, w.placement, w.rank)
    a = oracle.Problem.of(w0).evaluate_contended(w0.placement, w0.rank, er)
    b = oracle.Problem.of(w0).evaluate(w0.placement, w0.rank)
    assert all((x == y).all() for x, y in zip(a, b))
    # (ii) at most one transfer per channel: nothing to contend for.  A path over distinct machines has that.
    m = min(n, 12)
    rp, ci = W.csr_from_edges(m, list(range(m - 1)), list(range(1, m)))
    pl = np.stack([rng.permutation(64)[:m] for _ in range(20)]).astype(np.int32)
    rk = np.zeros_like(pl)
    comm = rng.integers(0, 9, (64, 64)).astype(np.int32)
    prob = oracle.Problem(64, rp, ci, rng.integers(0, 7, m), comm, rng.integers(-3, 4, m))
    a = prob.evaluate_contended(pl, rk, np.zeros((20, m - 1), np.int32))
    b = prob.evaluate(pl, rk)
    assert all((x == y).all() for x, y in zip(a, b)) and (a[3] == 0).all()


@pytest.mark.parametrize("cfg,n_cand", [(1, 60), (2, 12)])
def test_equals_the_model_with_transfers_as_nodes(cfg, n_cand):
    """Batches with one shared placement: every edge across machines becomes a node on a channel-machine of its
    pair, delays become zero, and the evaluation without any notion of a transfer gives the same schedule."""
    w = W.gen_config(cfg, n_cand=n_cand)
    wx, cross_edges, edge_rank_cross = channels.with_channels(w)
    zx, bx, pkx, fx = oracle.evaluate_workload(wx)
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, w.n_devices, w.placement, w.rank)
    z, b, pk, f = oracle.Problem.of(w).evaluate_contended(w.placement, w.rank, er)
    assert (f == fx).all() and (z == zx).all()
    assert (pk[f == 0] == pkx[f == 0][:, :w.n_devices]).all()
    # the bubble counts the P real machines here, all machines and channel-machines there
    assert (b[f == 0] == w.n_devices * z[f == 0].astype(np.int64) - int(w.dur.sum())).all()


def test_channel_ranks_are_validated_and_flags_keep_their_order():
    g = _golden("hand_contention.txt")
    n, P = g["n_nodes"][0], g["n_devices"][0]
    rp, ci = W.csr_from_edges(n, g["edges"][0::2], g["edges"][1::2])
    comm = np.array(g["comm"]).reshape(P, P)
    prob = oracle.Problem(P, rp, ci, g["dur"], comm, g["mem_delta"], mem_limit=[1, 100])
    pl, rk = np.array(g["placement"]), np.array(g["rank"])

    def flag(pl=pl, rk=rk, er=(0, 1, 0), prob=prob):
        return int(prob.evaluate_contended([pl], [rk], [er])[3][0])
    assert flag() == oracle.FLAG_OVER_MEMORY                 # feasible, but machine 0 peaks at 2 > 1
    assert flag(er=(0, 0, 0)) == oracle.FLAG_BAD_RANK        # two transfers of channel (0,1) with rank 0
    assert flag(er=(0, 2, 0)) == oracle.FLAG_BAD_RANK        # a gap
    assert flag(er=(-1, 0, 0)) == oracle.FLAG_BAD_RANK
    assert flag(er=(0, 1, 5)) == oracle.FLAG_BAD_RANK        # the only transfer of channel (1,0) must have rank 0
    one = np.zeros(n, int)
    assert flag(pl=one, rk=np.arange(n), er=(7, -3, 99)) == oracle.FLAG_OVER_MEMORY   # no transfers: ranks not looked at
    bad_pl = pl.copy(); bad_pl[3] = 2
    assert flag(pl=bad_pl, er=(0, 0, 0)) == oracle.FLAG_BAD_PLACEMENT
    bad_rk = rk.copy(); bad_rk[1] = 0
    assert flag(rk=bad_rk, er=(0, 0, 0)) == oracle.FLAG_BAD_RANK
    # a pair without a channel is found before a cycle is
    comm2 = comm.copy(); comm2[1, 0] = -1
    prob2 = oracle.Problem(P, rp, ci, g["dur"], comm2, g["mem_delta"])
    assert flag(prob=prob2) == oracle.FLAG_NO_CHANNEL
    # a cycle through a channel: k1 before k0 on the channel, but d (fed by k1) ... is after c (fed by k0) on machine
    # 1 only if the machines' orders say so; make c wait for k0 behind k1 while b, k1's producer, waits for e, which
    # waits for c: ranks on machine 0: a, e, b
    rk_cyc = np.array([0, 2, 0, 1, 1])
    assert flag(rk=rk_cyc, er=(1, 0, 0), prob=oracle.Problem(P, rp, ci, g["dur"], comm, g["mem_delta"])) == oracle.FLAG_CYCLIC
    assert flag(rk=rk_cyc, er=(0, 1, 0), prob=oracle.Problem(P, rp, ci, g["dur"], comm, g["mem_delta"])) == 0


def test_overflow_bound_counts_one_transfer_per_edge():
    rp, ci = W.csr_from_edges(3, [0, 0, 1], [1, 2, 2])
    big = (2 ** 31 - 1 - 3) // 3
    ok = oracle.Problem(2, rp, ci, [1, 1, 1], [[0, big], [big, 0]], [0, 0, 0])
    assert ok.evaluate_contended([[0, 1, 0]], [[0, 0, 1]], [[0, 0, 0]])[3][0] == 0
    too = oracle.Problem(2, rp, ci, [1, 1, 3], [[0, big], [big, 0]], [0, 0, 0])
    with pytest.raises(oracle.OracleError) as e:
        too.evaluate_contended([[0, 1, 0]], [[0, 0, 1]], [[0, 0, 0]])
    assert e.value.code == oracle.EOVERFLOW
