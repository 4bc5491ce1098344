"""GPU parity of the local-search helpers through the C-ABI (propose / select / schedule) and a short search run."""
from __future__ import annotations

import json
import os

import numpy as np
import pytest

import oracle
from oracle import search_oracle as SO
from paper_2503_09357_amd import workloads as W

pytestmark = pytest.mark.gpu


def _dev():
    import torch
    return torch.device("cuda", 0)


@pytest.mark.parametrize("layout", [0, 1])
def test_propose_matches_the_oracle(gpu_lib, layout):
    import torch
    ds = gpu_lib
    rng = np.random.default_rng(5501)
    for w in (W.gen_config(1, n_cand=2), W.gen_config(2, n_cand=2), W.gen_config(4, n_cand=1),
              W.random_instance(rng, 37, 3, 2, frac_bad=0.0, frac_arbitrary=0.0)):
        C = 700
        rnd = rng.integers(0, 1 << 32, size=4 * C, dtype=np.uint64).astype(np.uint32)
        with ds.Evaluator.for_workload(w, max_candidates=C, layout=layout) as ev:
            pl, rk = ev.propose(torch.from_numpy(w.placement[0]).to(_dev()), torch.from_numpy(w.rank[0]).to(_dev()),
                                torch.from_numpy(rnd.view(np.int32)).to(_dev()))
            torch.cuda.synchronize()
            got_pl, got_rk = pl.cpu().numpy(), rk.cpu().numpy()
            pl2, rk2 = ev.propose(torch.from_numpy(w.placement[0]).to(_dev()), torch.from_numpy(w.rank[0]).to(_dev()),
                                  torch.from_numpy(rnd.view(np.int32)).to(_dev()), orders_only=True)
            torch.cuda.synchronize()
            got_pl2, got_rk2 = pl2.cpu().numpy(), rk2.cpu().numpy()
        want_pl, want_rk = SO.propose(w.placement[0], w.rank[0], rnd, w.n_devices)
        want_pl2, want_rk2 = SO.propose(w.placement[0], w.rank[0], rnd, w.n_devices, orders_only=True)
        if layout == 1:
            got_pl, got_rk, got_pl2, got_rk2 = got_pl.T, got_rk.T, got_pl2.T, got_rk2.T
        assert (got_pl == want_pl).all() and (got_rk == want_rk).all(), w.name
        assert (got_pl2 == want_pl2).all() and (got_rk2 == want_rk2).all(), w.name
        assert (got_pl2 == w.placement[0]).all()


def test_select_matches_the_oracle(gpu_lib):
    import torch
    ds = gpu_lib
    rng = np.random.default_rng(5502)
    w = W.gen_config(1, n_cand=1)
    with ds.Evaluator.for_workload(w, max_candidates=1) as ev:
        for C, p_ok in ((1, 1.0), (5, 0.5), (4097, 0.3), (70000, 0.01), (300, 0.0)):
            z = rng.integers(0, 50, C).astype(np.int32)          # many ties
            f = np.where(rng.random(C) < p_ok, 0, rng.choice([1, 2, 4, 16], C)).astype(np.int32)
            z[f != 0] = -1
            best = ev.select(torch.from_numpy(z).to(_dev()), torch.from_numpy(f).to(_dev()))
            torch.cuda.synchronize()
            assert tuple(best.cpu().tolist()) == SO.select(z, f), (C, p_ok)


def _without_some_channels(w):
    """Three machine pairs lose their channel (eq. (10)): comm entry -1."""
    import dataclasses
    comm = w.comm.copy()
    comm[0, 1] = comm[4, 2] = comm[5, 3] = oracle.NO_CHANNEL
    return dataclasses.replace(w, name=w.name + " missing channels", comm=comm)


def test_schedule_matches_the_oracle(gpu_lib):
    import torch
    ds = gpu_lib
    rng = np.random.default_rng(5503)
    for w in (W.gen_config(1, n_cand=3), W.gen_config(3, n_cand=2), W.gen_config(5, n_cand=1),
              W.random_instance(rng, 90, 5, 12, frac_bad=0.3, frac_arbitrary=0.3),
              _without_some_channels(W.random_instance(rng, 70, 6, 16, frac_bad=0.2, frac_arbitrary=0.2))):
        prob = oracle.Problem.of(w)
        with ds.Evaluator.for_workload(w) as ev:
            for c in range(w.n_cand):
                s, e, f = ev.schedule(torch.from_numpy(w.placement[c]).to(_dev()), torch.from_numpy(w.rank[c]).to(_dev()))
                torch.cuda.synchronize()
                try:
                    flag, so, eo, _, _ = prob.schedule(w.placement[c], w.rank[c])
                except oracle.OracleError:
                    raise
                assert int(f.item()) == flag, (w.name, c)
                if flag == 0:
                    assert (s.cpu().numpy() == so).all() and (e.cpu().numpy() == eo).all(), (w.name, c)
                else:
                    assert (s.cpu().numpy() == -1).all() and (e.cpu().numpy() == -1).all()


@pytest.mark.parametrize("layout", [0, 1])
def test_local_search_never_gets_worse_and_ends_valid(gpu_lib, layout, tmp_path):
    import torch
    from paper_2503_09357_amd import search
    ds = gpu_lib
    w = W.gen_config(2, n_cand=1)
    prob = oracle.Problem.of(w)
    z0 = int(prob.evaluate(w.placement, w.rank)[0][0])
    with ds.Evaluator.for_workload(w, max_candidates=512, layout=layout) as ev:
        pl, rk, hist = search.local_search(ev, torch.from_numpy(w.placement[0]).to(_dev()),
                                           torch.from_numpy(w.rank[0]).to(_dev()), iterations=12, n_cand=512, seed=3)
        s, e, f = ev.schedule(pl, rk)
        torch.cuda.synchronize()
    assert len(hist) == 12 and hist[0] <= z0 and all(b <= a for a, b in zip(hist, hist[1:]))
    zo, _, _, fo = prob.evaluate(pl.cpu().numpy()[None, :], rk.cpu().numpy()[None, :])
    assert fo[0] == 0 and int(zo[0]) == hist[-1] and int(f.item()) == 0 and int(e.max().item()) == hist[-1]
    path = os.path.join(tmp_path, "trace.json")
    search.chrome_trace(path, s.cpu().tolist(), e.cpu().tolist(), pl.cpu().tolist())
    assert len(json.load(open(path))["traceEvents"]) == w.n_nodes


def test_search_over_the_orders_alone_stays_on_the_shared_placement_kernel(gpu_lib):
    """The pipeline search of Sec. V: the stage -> machine map is given, the orders are searched.  With the base's
    placement as the hint and moves that keep it, every batch is evaluated by the shared-placement kernel."""
    import torch
    from paper_2503_09357_amd import search
    from test_gpu_parity import _with_env
    ds = gpu_lib
    w = W.gen_config(2, n_cand=1)
    prob = oracle.Problem.of(w)
    z0 = int(prob.evaluate(w.placement, w.rank)[0][0])

    def go():
        with ds.Evaluator.for_workload(w, max_candidates=2048, shared_placement=w.placement[0]) as ev:
            assert ev.info()["variant"] == 6, ev.info()
            pl, rk, hist = search.local_search(ev, torch.from_numpy(w.placement[0]).to(_dev()),
                                               torch.from_numpy(w.rank[0]).to(_dev()), iterations=15, n_cand=2048, seed=5,
                                               orders_only=True)
            torch.cuda.synchronize()
            return pl.cpu().numpy(), rk.cpu().numpy(), hist

    pl, rk, hist = _with_env({"ignore_shared_placement": 0, "static_waves": 2}, go)
    assert (pl == w.placement[0]).all()
    assert hist[0] <= z0 and all(b <= a for a, b in zip(hist, hist[1:])) and hist[-1] < z0
    zo, _, _, fo = prob.evaluate(pl[None, :], rk[None, :])
    assert fo[0] == 0 and int(zo[0]) == hist[-1]


def test_cycles_and_range_stops_are_told_apart(gpu_lib):
    """In the optimistic 16-bit mode a deadlock is either a cycle (flagged at once) or an end time leaving the
    16-bit range (handed to the int32 kernel).  A neighbourhood of the MoE workload has plenty of cycles; the
    straddling instance has both kinds."""
    import dataclasses
    import test_gpu_parity as T
    rng = np.random.default_rng(5505)
    w = W.gen_config(4, n_cand=1)
    rnd = rng.integers(0, 1 << 32, size=4 * 300, dtype=np.uint64).astype(np.uint32)
    pl, rk = SO.propose(w.placement[0], w.rank[0], rnd, w.n_devices)
    (z, b, pk, f), info = T.assert_parity(gpu_lib, dataclasses.replace(w, name="cfg4 neighbourhood", placement=pl, rank=rk))
    assert info["variant"] == 4 and (f == 1).sum() >= 10 and (f == 0).sum() >= 10
    # long chain on few machines: makespans on both sides of 65535, plus cycles made by neighbourhood moves
    n, p = 600, 3
    rp, ci = W.random_dag(rng, n, 2, window=30)
    dur = rng.integers(60, 160, n).astype(np.int32)
    comm = rng.integers(1, 200, (p, p)).astype(np.int32)
    mem = rng.integers(-9, 10, n).astype(np.int64)
    pl0, rk0 = W.list_schedules(rp, ci, p, 40, 4242)
    pl1, rk1 = W.list_schedules(rp, ci, 1, 40, 99)
    rows_pl, rows_rk = [pl0, pl1], [rk0, rk1]
    for base_pl, base_rk in ((pl0[0], rk0[0]), (pl1[0], rk1[0])):
        rnd = rng.integers(0, 1 << 32, size=4 * 100, dtype=np.uint64).astype(np.uint32)
        a, c = SO.propose(base_pl, base_rk, rnd, p)
        rows_pl.append(a)
        rows_rk.append(c)
    w2 = W.Workload("straddles 16 bits, with cycles", p, rp, ci, dur, comm, mem, np.concatenate(rows_pl), np.concatenate(rows_rk))
    (z2, b2, pk2, f2), info2 = T._with_env({"state_bits": 16}, lambda: T.assert_parity(gpu_lib, w2))
    assert info2["variant"] == 4 and (f2 == 1).any() and (z2[f2 == 0] > 65535).any() and (z2[f2 == 0] < 65535).any()



@pytest.mark.parametrize("shared", [False, True])
def test_search_step_replays_from_a_hip_graph(gpu_lib, shared):
    """propose -> evaluate -> select enqueue kernels only (no allocation, no memset node), so one search step can
    be captured once and replayed; every replay must give what the eager calls give.  With the MoE workload the
    optimistic 16-bit kernel runs (counter reset + fallback kernel inside); with the pipeline and its placement as
    the hint the shared-placement kernel does, and the moves across machines are its strangers."""
    import torch
    import test_gpu_parity as T
    ds = gpu_lib
    rng = np.random.default_rng(5506)
    w = W.gen_config(2 if shared else 4, n_cand=1)
    C = 256
    dev = _dev()
    make = lambda: ds.Evaluator.for_workload(w, max_candidates=C, shared_placement=w.placement[0] if shared else None)
    with T._with_env({"ignore_shared_placement": 0, "static_waves": 2}, make) as ev:
        assert ev.info()["variant"] == (6 if shared else 4), ev.info()
        base_pl = torch.from_numpy(w.placement[0]).to(dev)
        base_rk = torch.from_numpy(w.rank[0]).to(dev)
        rnd = torch.zeros(4 * C, dtype=torch.int32, device=dev)
        cand = ev.propose(base_pl, base_rk, rnd)
        out = ev.alloc_outputs(C)
        best = torch.empty(2, dtype=torch.int32, device=dev)
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream(dev))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            ev.propose(base_pl, base_rk, rnd, out=cand)          # warm-up on the capture stream
            ev.evaluate(cand[0], cand[1], out)
            ev.select(out[0], out[3], out=best)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                ev.propose(base_pl, base_rk, rnd, out=cand)
                ev.evaluate(cand[0], cand[1], out)
                ev.select(out[0], out[3], out=best)
        torch.cuda.current_stream(dev).wait_stream(side)
        for rep in range(4):
            words = rng.integers(0, 1 << 31, size=4 * C).astype(np.int32)
            rnd.copy_(torch.from_numpy(words).to(dev))
            graph.replay()
            torch.cuda.synchronize()
            got = [t.clone() for t in out] + [best.clone()]
            eager_c = ev.propose(base_pl, base_rk, rnd)           # the program's own eager work between replays
            eager = ev.evaluate(eager_c[0], eager_c[1])
            eager_best = ev.select(eager[0], eager[3])
            torch.cuda.synchronize()
            for a, b in zip(got, list(eager) + [eager_best]):
                assert torch.equal(a, b), rep
            want_pl, want_rk = SO.propose(w.placement[0], w.rank[0], words.view(np.uint32), w.n_devices)
            zo, bo, pko, fo = oracle.Problem.of(w).evaluate(want_pl, want_rk, threads=8)
            assert (got[0].cpu().numpy() == zo).all() and (got[3].cpu().numpy() == fo).all()
            assert tuple(got[4].cpu().tolist()) == SO.select(zo, fo)
