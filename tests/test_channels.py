"""Channel contention (Sec. III, eqs. (14)-(15)) expressed through transfer nodes on channel-machines, for workloads
whose candidates share one placement (paper_2503_09357_amd/channels.py).  The expansion is pinned against a
unit-step simulation of the model with contention written from the definition (tests/checkers.py), first on the
CPU oracle, then on the HIP path."""
import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import channels as CH
from paper_2503_09357_amd import workloads as W
from tests import checkers as K


def _fixed_placement_instance(rng, n, p, c, max_comm):
    rp, ci = W.random_dag(rng, n, 3, window=6)
    dur = rng.integers(0, 5, n).astype(np.int32)
    comm = rng.integers(0, max_comm + 1, (p, p)).astype(np.int32)
    mem = rng.integers(-3, 4, n).astype(np.int64)
    fixed = rng.integers(0, p, n).astype(np.int32)
    pl, rk = W.list_schedules(rp, ci, p, c, int(rng.integers(1, 1 << 30)), fixed_placement=fixed)
    return W.Workload("fixed placement n=%d p=%d" % (n, p), p, rp, ci, dur, comm, mem, pl, rk)


def _edge_order(w, cross_edges, edge_rank_c):
    """channel -> edge indices k (into col_idx) in the order of edge_rank, for the simulator."""
    src = np.repeat(np.arange(w.n_nodes), np.diff(w.row_ptr))
    pl = w.placement[0]
    cross_k = [k for k in range(w.n_edges) if pl[src[k]] != pl[w.col_idx[k]]]
    assert len(cross_k) == len(cross_edges)
    order = {}
    for i, k in enumerate(cross_k):
        ch = (int(pl[src[k]]), int(pl[w.col_idx[k]]))
        order.setdefault(ch, []).append((int(edge_rank_c[i]), k))
    return {ch: [k for _, k in sorted(v)] for ch, v in order.items()}


def test_two_transfers_on_one_channel_take_turns():
    # a -> c and b -> d, a and b on machine 0, c and d on machine 1, every duration 1, the channel takes 5:
    # without contention c and d start at 6 and 7; with it the second transfer waits for the first: d starts at 12
    rp, ci = W.csr_from_edges(4, [0, 1], [2, 3])
    w = W.Workload("two transfers", 2, rp, ci, np.ones(4, np.int32), np.array([[0, 5], [5, 0]], np.int32),
                   np.zeros(4, np.int64), np.array([[0, 0, 1, 1]], np.int32), np.array([[0, 1, 0, 1]], np.int32))
    assert oracle.evaluate_workload(w, 0, threads=1)[0][0] == 8          # latency only: b ends 2, +5, d runs 7..8
    w2, cross, er = CH.with_channels(w)
    assert (w2.n_nodes, w2.n_devices) == (6, 3) and er.tolist() == [[0, 1]]
    z2 = oracle.evaluate_workload(w2, 0, threads=1)[0][0]
    assert z2 == 12                                                       # transfers 1..6 and 6..11, d runs 11..12
    sim = K.tick_simulate_channels(2, rp, ci, w.dur, w.comm, w.placement[0], w.rank[0], {(0, 1): [0, 1]})
    assert sim[0] == 12
    # the other order of the two transfers: b's goes first although b ends later
    w2.rank[0, 4:] = [1, 0]
    # transfers 2..7 and 7..12; machine 1 runs c first (12..13), then d (13..14)
    assert oracle.evaluate_workload(w2, 0, threads=1)[0][0] == 14
    assert K.tick_simulate_channels(2, rp, ci, w.dur, w.comm, w.placement[0], w.rank[0], {(0, 1): [1, 0]})[0] == 14


def test_expansion_matches_the_simulation_with_contention():
    rng = np.random.default_rng(1415)
    contended = 0
    for _ in range(40):
        n, p = int(rng.integers(2, 14)), int(rng.integers(1, 4))
        w = _fixed_placement_instance(rng, n, p, 6, max_comm=int(rng.integers(0, 9)))
        w2, cross, er = CH.with_channels(w)
        z_lat = oracle.evaluate_workload(w, 0, threads=1)[0]
        z2, b2, pk2, f2 = oracle.evaluate_workload(w2, 0, threads=1)
        assert (f2 == 0).all()                                            # first come, first served never contradicts the DAG
        assert (z2 >= z_lat).all()                                        # contention can only delay
        for c in range(w.n_cand):
            sim = K.tick_simulate_channels(p, w.row_ptr, w.col_idx, w.dur, w.comm, w.placement[c], w.rank[c],
                                           _edge_order(w, cross, er[c]))
            assert sim is not None and sim[0] == z2[c], (n, p, c, sim[0] if sim else None, z2[c])
            contended += int(z2[c] > z_lat[c])
        assert (pk2[:, :p] == oracle.evaluate_workload(w, 0, threads=1)[2]).all()   # memory is about the operations only
    assert contended > 10                                                 # the instances do contend


def test_expansion_needs_one_placement():
    rng = np.random.default_rng(3)
    w = W.random_instance(rng, 20, 3, 5, frac_arbitrary=0.0, frac_bad=0.0)
    with pytest.raises(ValueError):
        CH.with_channels(w)


@pytest.mark.gpu
def test_gpu_evaluates_the_expanded_pipeline(gpu_lib):
    from tests.test_gpu_parity import assert_parity
    rng = np.random.default_rng(2718)
    # the 1F1B pipeline with slow channels (the transfers of a stage pair queue up), and a random instance
    w = W.gen_config(1, n_cand=200)
    w.comm[:] = np.where(np.eye(w.n_devices, dtype=bool), 0, 7)
    for base in (w, _fixed_placement_instance(rng, 300, 5, 64, max_comm=9)):
        w2, cross, er = CH.with_channels(base)
        (z2, b2, pk2, f2), info = assert_parity(gpu_lib, w2)
        z_lat = oracle.evaluate_workload(base, 0, threads=8)[0]
        assert (f2 == 0).all() and (z2 >= z_lat).all() and (z2 > z_lat).any()
