"""Parity of the HIP path against the CPU oracle, element by element, through the C-ABI.

Every quantity is an integer, so the bar is bit-exact equality of makespan, bubble, peak_mem and flags.
"""
from __future__ import annotations

import os
import sys
from dataclasses import replace as dataclasses_replace

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _say(msg):
    print("[gpu-parity] " + msg, flush=True)
    sys.stdout.flush()


def gpu_evaluate(ds, w, layout=0, max_candidates=None, repeats=1):
    import torch
    dev = torch.device("cuda", 0)
    pl, rk = w.placement, w.rank
    if layout == 1:
        pl, rk = np.ascontiguousarray(pl.T), np.ascontiguousarray(rk.T)
    with ds.Evaluator.for_workload(w, max_candidates=max(1, w.n_cand) if max_candidates is None else max_candidates,
                                   layout=layout) as ev:
        tp = torch.from_numpy(pl).to(dev)
        tr = torch.from_numpy(rk).to(dev)
        outs = []
        for _ in range(repeats):
            out = ev.evaluate(tp, tr)
            torch.cuda.synchronize()
            outs.append(tuple(t.cpu().numpy() for t in out))
        info = ev.info()
    for o in outs[1:]:
        assert all((a == b).all() for a, b in zip(outs[0], o)), "evaluation is not deterministic"
    return outs[0], info


def assert_parity(ds, w, layout=0, **kw):
    _say("%s | N=%d E=%d P=%d C=%d layout=%d" % (w.name, w.n_nodes, w.n_edges, w.n_devices, w.n_cand, layout))
    (z, b, pk, f), info = gpu_evaluate(ds, w, layout, **kw)
    zo, bo, pko, fo = oracle.evaluate_workload(w, layout, threads=8)
    bad = np.nonzero(f != fo)[0]
    assert len(bad) == 0, "flags differ at candidates %s: gpu %s oracle %s (%s)" % (bad[:8], f[bad[:8]], fo[bad[:8]], info)
    bad = np.nonzero(z != zo)[0]
    assert len(bad) == 0, "makespan differs at %s: gpu %s oracle %s (%s)" % (bad[:8], z[bad[:8]], zo[bad[:8]], info)
    assert (b == bo).all(), "bubble differs"
    assert pk.shape == pko.shape and (pk == pko).all(), "peak_mem differs"
    return (z, b, pk, f), info


# --------------------------------------------------------------------------- anchors

def test_hand_worked_diamond(gpu_lib):
    vals = {}
    for line in open(os.path.join(GOLDEN, "hand_diamond.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = [int(x) for x in v]
    n, P = vals["n_nodes"][0], vals["n_devices"][0]
    rp, ci = W.csr_from_edges(n, vals["edges"][0::2], vals["edges"][1::2])
    w = W.Workload("hand diamond", P, rp, ci, np.array(vals["dur"], np.int32),
                   np.array(vals["comm"], np.int32).reshape(P, P), np.array(vals["mem_delta"], np.int64),
                   np.array([vals["placement"]], np.int32), np.array([vals["rank"]], np.int32))
    (z, b, pk, f), _ = gpu_evaluate(gpu_lib, w)
    assert f[0] == 0 and z[0] == vals["makespan"][0] and b[0] == vals["bubble"][0] and pk[0].tolist() == vals["peak_mem"]


@pytest.mark.parametrize("p,m,tf,tb", [(4, 8, 2, 4), (8, 8, 1, 2), (6, 13, 3, 7), (1, 5, 2, 3)])
def test_1f1b_closed_form(gpu_lib, p, m, tf, tb):
    w = W.uniform_pipeline(p, m, tf, tb, 0, "1f1b")
    (z, b, pk, f), _ = gpu_evaluate(gpu_lib, w)
    assert f[0] == 0 and z[0] == (m + p - 1) * (tf + tb) and b[0] == p * (p - 1) * (tf + tb)
    assert pk[0].tolist() == [min(m, p - s) for s in range(p)]


# --------------------------------------------------------------------------- fuzz (good, cyclic and malformed candidates)

@pytest.mark.parametrize("layout", [0, 1])
def test_random_instances(gpu_lib, layout):
    rng = np.random.default_rng(100 + layout)
    shapes = [(1, 1, 1), (2, 1, 3), (5, 2, 7), (17, 3, 33), (64, 4, 64), (65, 5, 70), (100, 7, 129), (257, 8, 100),
              (300, 13, 50), (129, 16, 65), (500, 31, 40), (700, 32, 37), (900, 33, 21), (1000, 64, 19), (63, 64, 10),
              (2000, 6, 30), (4097, 9, 12)]
    seen = set()
    for n, p, c in shapes:
        w = W.random_instance(rng, n, p, c, max_fanin=4, frac_arbitrary=0.25, frac_bad=0.25)
        (z, b, pk, f), _ = assert_parity(gpu_lib, w, layout)
        seen |= set(f.tolist())
    assert seen == {0, 1, 2, 4}


def test_wide_fan_in_and_large_values(gpu_lib):
    """In-degree well above any per-round batch; durations and delays near the int32 exactness bound."""
    rng = np.random.default_rng(7)
    n = 200
    src = list(range(n - 1)) + list(range(0, n - 1, 3))
    dst = [n - 1] * (n - 1) + list(range(1, n, 3))
    src, dst = zip(*[(a, b) for a, b in zip(src, dst) if a != b])
    rp, ci = W.csr_from_edges(n, src, dst)
    dur = rng.integers(0, 5_000_000, n).astype(np.int32)
    comm = rng.integers(0, 4_000_000, (5, 5)).astype(np.int32)
    mem = rng.integers(-2 ** 40, 2 ** 40, n).astype(np.int64)
    pl, rk = W.list_schedules(rp, ci, 5, 40, 99)
    w = W.Workload("wide fan-in, large values", 5, rp, ci, dur, comm, mem, pl, rk)
    assert oracle.Problem.of(w).check() == 0
    assert_parity(gpu_lib, w)


def test_edge_shapes(gpu_lib):
    import torch
    # a single node
    rp, ci = W.csr_from_edges(1, [], [])
    w = W.Workload("one node", 1, rp, ci, np.array([7], np.int32), np.zeros((1, 1), np.int32), np.array([-3], np.int64),
                   np.zeros((3, 1), np.int32), np.zeros((3, 1), np.int32))
    (z, b, pk, f), _ = assert_parity(gpu_lib, w)
    assert z.tolist() == [7, 7, 7] and pk.reshape(-1).tolist() == [0, 0, 0]
    # machines that receive no operation; every node alone on its machine
    rng = np.random.default_rng(5)
    rp, ci = W.random_dag(rng, 40, 3)
    dur = rng.integers(0, 9, 40).astype(np.int32)
    comm = rng.integers(0, 6, (64, 64)).astype(np.int32)
    mem = rng.integers(-4, 5, 40).astype(np.int64)
    pl = np.stack([rng.permutation(64)[:40] for _ in range(9)]).astype(np.int32)
    w = W.Workload("one machine per node", 64, rp, ci, dur, comm, mem, pl, np.zeros((9, 40), np.int32))
    assert_parity(gpu_lib, w)
    assert_parity(gpu_lib, w, layout=1)
    # an empty batch is legal and touches nothing
    with gpu_lib.Evaluator.for_workload(w, max_candidates=4) as ev:
        dev = torch.device("cuda", 0)
        empty = torch.empty((0, 40), dtype=torch.int32, device=dev)
        out = ev.evaluate(empty, empty)
        assert out[0].numel() == 0
        # more candidates than the workspace holds is an argument error
        too_many = torch.zeros((5, 40), dtype=torch.int32, device=dev)
        with pytest.raises(gpu_lib.DagschedError) as ei:
            ev.evaluate(too_many, too_many)
        assert ei.value.code == gpu_lib.EINVAL
    # a cyclic operator graph is rejected at create time
    rpc, cic = W.csr_from_edges(3, [0, 1, 2], [1, 2, 0])
    with pytest.raises(gpu_lib.DagschedError) as ei:
        gpu_lib.Evaluator(2, rpc, cic, [1, 1, 1], [[0, 1], [1, 0]], [0, 0, 0], 4)
    assert ei.value.code == gpu_lib.ECYCLE


def test_largest_supported_shape(gpu_lib):
    """N at the documented maximum, P = 64, a ragged candidate count."""
    rng = np.random.default_rng(11)
    n = 65535
    rp, ci = W.random_dag(rng, n, 2, window=400)
    dur = rng.integers(1, 20, n).astype(np.int32)
    comm = rng.integers(1, 9, (64, 64)).astype(np.int32)
    mem = rng.integers(-4, 5, n).astype(np.int64)
    pl, rk = W.list_schedules(rp, ci, 64, 3, 1234)
    rk[2, 0], rk[2, 1] = rk[2, 1], rk[2, 0]           # may or may not be feasible; the oracle decides
    w = W.Workload("N=65535 P=64", 64, rp, ci, dur, comm, mem, pl, rk)
    assert_parity(gpu_lib, w)


# --------------------------------------------------------------------------- the five configurations

@pytest.mark.parametrize("cfg,c", [(1, 1024), (2, 3000), (3, 300), (4, 130), (5, 33)])
def test_configs_reduced(gpu_lib, cfg, c):
    w = W.gen_config(cfg, n_cand=c)
    assert_parity(gpu_lib, w, repeats=2)


@pytest.mark.parametrize("cfg,c", [(1, 257), (2, 1000), (4, 65)])
def test_configs_candidate_minor_layout(gpu_lib, cfg, c):
    w = W.gen_config(cfg, n_cand=c)
    assert_parity(gpu_lib, w, layout=1)


@pytest.mark.parametrize("cfg,hint", [(1, 1), (2, 1), (3, 1), (4, 1), (5, 1), (1, 0), (2, 0), (3, 0)])
def test_configs_full_size(gpu_lib, cfg, hint):
    """Full candidate counts; the oracle evaluates every candidate (seconds per configuration), so the comparison is
    exhaustive.  hint = 1: the handle is made as bench.py makes it (Evaluator.for_workload passes the shared placement
    of the pipeline workloads as the hint, and the library dispatches by itself); hint = 0: the pipeline workloads
    without the hint, i.e. on the kernels that take a placement per candidate."""
    w = W.gen_config(cfg)
    (z, b, pk, f), info = _with_env({"ignore_shared_placement": 1 - hint}, lambda: assert_parity(gpu_lib, w))
    if cfg == 2:
        assert info["variant"] == (6 if hint else 3), info
    _say("cfg%d full ok, kernel info %s, flags %s" % (cfg, info, np.bincount(f).tolist()))
    if cfg == 2:
        marked = np.zeros(w.n_cand, bool)
        marked[w.meta["cyclic"]] = True
        assert ((f == 1) == marked).all()


# --------------------------------------------------------------------------- kernel variants and the 16-bit fallback

def _with_env(env, fn):
    """Run fn with the given dagsched_shape_t fields as the defaults of every evaluator it makes."""
    from paper_2503_09357_amd import dagsched as ds
    with ds.shape_defaults(**env):
        return fn()


@pytest.mark.parametrize("env", [
    {"kernel": 1},
    {"feeders": 1, "ring_slots": 4, "placement_mode": 1},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 1},
    {"feeders": 1, "ring_slots": 8, "placement_mode": 1, "cand_per_block": 1},
    {"feeders": 2, "ring_slots": 4, "placement_mode": 1},
    {"feeders": 3, "ring_slots": 8, "placement_mode": 1},
    {"feeders": 4, "ring_slots": 16, "placement_mode": 0},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 0},
    {"feeders": 2, "ring_slots": 16, "placement_mode": 0},
    {"feeders": 1, "ring_slots": 32, "placement_mode": 0},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 1, "preds_per_op": 4},
    {"feeders": 2, "ring_slots": 16, "placement_mode": 0, "preds_per_op": 4},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 1, "preds_per_op": 2},
    {"feeders": 3, "ring_slots": 16, "placement_mode": 0, "preds_per_op": 2},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 1, "state_bits": 32},
    {"feeders": 3, "ring_slots": 16, "placement_mode": 0, "state_bits": 32},
    {"feeders": 1, "ring_slots": 8, "placement_mode": 1, "state_bits": 32,
     "preds_per_op": 4},
])
def test_every_kernel_variant(gpu_lib, env):
    """The tuning knobs only pick among kernel instantiations; each one must give the same bits."""
    rng = np.random.default_rng(321)
    cases = [W.gen_config(1, n_cand=100), W.gen_config(2, n_cand=150), W.gen_config(4, n_cand=9),
             W.random_instance(rng, 333, 7, 41, max_fanin=6, frac_arbitrary=0.3, frac_bad=0.2),
             W.random_instance(rng, 210, 5, 37, max_fanin=4, frac_arbitrary=0.3, frac_bad=0.2, dup_prob=0.0)]   # single-part operations
    for w in cases:
        (z, b, pk, f), info = _with_env(env, lambda: assert_parity(gpu_lib, w))
        if "kernel" in env:
            assert info["state_bits"] == 32
        else:
            assert info["state_bits"] == env.get("state_bits", 16)
            assert info["variant"] == (5 if info["state_bits"] == 32 else info["variant"]) and info["variant"] in (3, 4, 5)
            assert info["feeders"] == env["feeders"] and info["ring_slots"] == env["ring_slots"]
            assert info["placement_bytes_in_lds"] == env["placement_mode"]
            if "cand_per_block" in env:
                assert info["cand_per_block"] == env["cand_per_block"]
            # the pipeline workloads keep a single DAG predecessor per operation once implied edges are dropped: the
            # one-predecessor kernels take them (where that shape is built; else, and with 32-bit cells, the
            # two-predecessor ones) unless the knob says otherwise
            pipe = w.name.startswith(("cfg1", "cfg2"))
            if env.get("preds_per_op", 0) == 4:
                assert info["kernel_kind"] == 0 and info["preds_per_op"] == 4
            elif pipe and env.get("preds_per_op", 0) == 2:
                assert info["kernel_kind"] == 2 and info["preds_per_op"] == 2, (w.name, info)
            elif pipe:
                assert info["kernel_kind"] in (2, 3) and info["preds_per_op"] in (1, 2), (w.name, info)
                if info["state_bits"] == 16 and (env["placement_mode"], env["ring_slots"], env["feeders"]) in (
                        (1, 8, 1), (1, 8, 2), (1, 8, 3), (1, 4, 1), (1, 4, 2), (0, 8, 2), (0, 16, 2)):
                    assert info["kernel_kind"] == 3, (w.name, info)
            elif w.name.startswith("random n=210"):
                assert info["kernel_kind"] in (1, 2), (w.name, info)


@pytest.mark.parametrize("env", [
    {"feeders": 2, "ring_slots": 8, "placement_mode": 2},
    {"feeders": 1, "ring_slots": 4, "placement_mode": 2},
    {"feeders": 2, "ring_slots": 4, "placement_mode": 2, "preds_per_op": 4},
    {"feeders": 2, "ring_slots": 8, "placement_mode": 2, "preds_per_op": 2},
    {"feeders": 1, "ring_slots": 8, "placement_mode": 2, "cand_per_block": 1},
])
def test_nibble_placement_kernels(gpu_lib, env):
    """Up to 16 machines: the placement can sit in LDS as four bits per node (and time then starts at 255
    inside the kernel).  Same bits as the oracle, on even and odd N, with bad inputs, with a machine count of
    exactly 16 and with end times around the 16-bit limit."""
    rng = np.random.default_rng(2024)
    cases = [W.gen_config(1, n_cand=100), W.gen_config(2, n_cand=150), W.gen_config(3, n_cand=10),
             W.random_instance(rng, 333, 16, 41, max_fanin=6, frac_arbitrary=0.3, frac_bad=0.2),
             W.random_instance(rng, 201, 7, 50, max_fanin=2, frac_arbitrary=0.2, frac_bad=0.2),
             W.random_instance(rng, 64, 16, 30, max_fanin=3)]
    for w in cases:
        (z, b, pk, f), info = _with_env(env, lambda: assert_parity(gpu_lib, w))
        assert info["state_bits"] == 16 and info["placement_bytes_in_lds"] == 2, (w.name, info)
    # end times around 65535: the origin of 255 must not turn an exact problem into a wrong one
    n, p = 600, 3
    rp, ci = W.random_dag(rng, n, 2, window=30)
    dur = rng.integers(60, 160, n).astype(np.int32)
    comm = rng.integers(1, 200, (p, p)).astype(np.int32)
    mem = rng.integers(-9, 10, n).astype(np.int64)
    pl, rk = W.list_schedules(rp, ci, p, 200, 4243)
    pl1, rk1 = W.list_schedules(rp, ci, 1, 67, 98)
    pl[::3], rk[::3] = pl1, rk1
    w = W.Workload("straddles 16 bits", p, rp, ci, dur, comm, mem, pl, rk)
    env16 = dict(env, state_bits=16)           # (left alone the library would take 32-bit end times here)
    (z, b, pk, f), info = _with_env(env16, lambda: assert_parity(gpu_lib, w))
    assert info["placement_bytes_in_lds"] == 2 and info["variant"] == 4
    # a makespan bound between 65280 and 65535: exact with bytes, optimistic with nibbles
    dur2 = np.full(n, 100, np.int32)
    dur2[1] = 101                                             # no common factor to divide out
    dur2[0] += 65400 - int(dur2.sum())
    w2 = W.Workload("just below 16 bits", p, rp, ci, dur2, np.zeros((p, p), np.int32), mem, pl, rk)
    (z2, b2, pk2, f2), info2 = _with_env(env16, lambda: assert_parity(gpu_lib, w2))
    assert info2["variant"] == 4 and (z2[f2 == 0] > 65535 - 255).any()


def test_launch_shape_from_the_description_and_autotuning(gpu_lib):
    """A shape given with the description is used as given and changes no result; the autotuning helper returns
    an evaluator that is still right."""
    import torch
    from paper_2503_09357_amd import dagsched as ds
    w = W.gen_config(3, n_cand=64)
    want = oracle.evaluate_workload(w, 0, threads=8)
    pl, rk = torch.from_numpy(w.placement).cuda(), torch.from_numpy(w.rank).cuda()
    shape = dict(cand_per_block=2, ring_slots=16, feeders=1, placement_mode=0, block_threads=256)
    with ds.Evaluator.for_workload(w, shape=shape) as ev:
        info = ev.info()
        assert (info["cand_per_block"], info["ring_slots"], info["feeders"], info["placement_bytes_in_lds"],
                info["block_threads"]) == (2, 16, 1, 0, 256)
        got = [t.cpu().numpy() for t in ev.evaluate(pl, rk)]
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
    # a shape that is not built: the int32 kernel answers, with the same results
    with ds.Evaluator.for_workload(w, shape=dict(ring_slots=32, placement_mode=1)) as ev:
        assert ev.info()["state_bits"] == 32
        got = [t.cpu().numpy() for t in ev.evaluate(pl, rk)]
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
    ev, best_shape = ds.Evaluator.autotuned(lambda s: ds.Evaluator.for_workload(w, shape=s), pl, rk)
    try:
        assert ev.info()["state_bits"] == 16
        got = [t.cpu().numpy() for t in ev.evaluate(pl, rk)]
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
    finally:
        ev.close()


def test_randomized_problems_and_launch_shapes(gpu_lib):
    """Many small random problems (sizes, machine counts, fan-in, durations, delays, static memory and limits, both
    layouts, malformed and cyclic candidates), each under a random launch shape: every kernel instantiation that
    the shapes reach must give the oracle's bits."""
    import torch
    from paper_2503_09357_amd import dagsched as ds
    seen = set()
    for case in range(250):
        rng = np.random.default_rng(90000 + case)
        n = int(rng.integers(1, 400)) if rng.random() < 0.9 else int(rng.integers(400, 3000))
        p, fanin, c = int(rng.integers(1, 65)), int(rng.integers(1, 11)), int(rng.integers(1, 120))
        layout = int(rng.integers(0, 2))
        w = W.random_instance(rng, n, p, c, max_fanin=fanin, max_dur=int(rng.integers(1, 400)) if rng.random() < 0.8 else 200000,
                              max_comm=int(rng.integers(0, 200)) if rng.random() < 0.8 else 3000, frac_arbitrary=0.3, frac_bad=0.15,
                              dup_prob=0.05 * int(rng.integers(0, 2)))
        if rng.random() < 0.5:
            w.weight = rng.integers(0, 50, n).astype(np.int64)
            w.mem_limit = rng.integers(-5, 400, p).astype(np.int64)
        shape = None
        if rng.random() < 0.75:
            mode = int(rng.integers(-1, 3))
            if mode == 2 and p > 16:
                mode = 1
            ring = int(rng.choice([0, 8, 16, 32])) if mode == 0 else int(rng.choice([0, 4, 8])) if mode > 0 else 0
            feeders = int(rng.integers(0, 4))
            if ring == 4 and feeders == 3:
                feeders = 2
            pseg = 1
            while pseg < p:
                pseg *= 2
            g = int(rng.choice([0, 1, 2, 4, 8, 16, 32, 64]))
            shape = dict(cand_per_block=g if g <= 64 // pseg else 0, ring_slots=ring, feeders=feeders,
                         placement_mode=mode, block_threads=int(rng.choice([0, 0, 384, 512, 1024])),
                         state_bits=int(rng.choice([0, 0, 16, 32])))
        pl, rk = w.placement, w.rank
        if layout == 1:
            pl, rk = np.ascontiguousarray(pl.T), np.ascontiguousarray(rk.T)
        with ds.Evaluator.for_workload(w, layout=layout, shape=shape) as ev:
            info = ev.info()
            got = [t.cpu().numpy() for t in ev.evaluate(torch.from_numpy(pl).cuda(), torch.from_numpy(rk).cuda())]
        want = oracle.evaluate_workload(w, layout, threads=8)
        for name, a, b in zip(("makespan", "bubble", "peak_mem", "flags"), got, want):
            assert np.array_equal(a, b), (name, case, n, p, fanin, c, layout, shape, info)
        seen.add((info["state_bits"], info["kernel_kind"], info["placement_bytes_in_lds"], info["feeders"], info["ring_slots"]))
    assert len(seen) >= 25, sorted(seen)                      # the sweep does reach many instantiations


def test_thirty_two_bit_end_times(gpu_lib):
    """Times that cannot stay below 65535: the same kernel with 32-bit end times on chip (variant 5), chosen by
    the library from the lower bound on the makespan, or asked for; always exact, no fallback list."""
    import torch
    from paper_2503_09357_amd import dagsched as ds
    rng = np.random.default_rng(32)
    cases = []
    for cfg, c in ((2, 300), (3, 60), (4, 40)):
        w = W.gen_config(cfg, n_cand=c)
        w.dur = (w.dur.astype(np.int64) * 211 + 7).astype(np.int32)      # no common factor, nothing fits 16 bits
        w.comm = (w.comm.astype(np.int64) * 50).astype(np.int32)
        cases.append((w, None))
    big = W.random_instance(rng, 400, 16, 60, max_fanin=7, max_dur=60000, max_comm=250, frac_arbitrary=0.3, frac_bad=0.2)
    big.weight = rng.integers(0, 50, 400).astype(np.int64)
    big.mem_limit = rng.integers(400, 1500, 16).astype(np.int64)
    cases += [(big, None), (big, dict(placement_mode=2)), (big, dict(placement_mode=0, ring_slots=16, feeders=3))]
    small = W.random_instance(rng, 90, 3, 50, max_fanin=2, frac_arbitrary=0.4, frac_bad=0.2)
    cases.append((small, dict(state_bits=32)))                            # asked for although 16 bits would do
    for w, shape in cases:
        with ds.Evaluator.for_workload(w, shape=shape) as ev:
            info = ev.info()
            got = [t.cpu().numpy() for t in ev.evaluate(torch.from_numpy(w.placement).cuda(), torch.from_numpy(w.rank).cuda())]
        assert info["variant"] == 5 and info["state_bits"] == 32, (w.name, shape, info)
        want = oracle.evaluate_workload(w, 0, threads=8)
        for name, a, b in zip(("makespan", "bubble", "peak_mem", "flags"), got, want):
            assert np.array_equal(a, b), (name, w.name, shape, info)
        if w.name.startswith("cfg"):
            assert (got[0][got[3] == 0] > 65535).all()
    # delays above 255 or durations above 65534 (after the common factor is divided out): wide ops, in which the
    # relaxer looks the delays up and durations reach 256 * 65535 - 1
    wide = []
    for cfg, c in ((2, 300), (3, 60), (4, 40)):
        w = W.gen_config(cfg, n_cand=c)
        w.dur = (w.dur.astype(np.int64) * 997 + rng.integers(0, 900, w.n_nodes)).astype(np.int32)
        w.comm = (w.comm.astype(np.int64) * 431 + 3).astype(np.int32)
        wide.append((w, None))
    r1 = W.random_instance(rng, 333, 7, 64, max_fanin=6, max_dur=900000, max_comm=50000, frac_arbitrary=0.3, frac_bad=0.2)
    r2 = W.random_instance(rng, 100, 64, 64, max_fanin=2, max_dur=70000, max_comm=300, frac_arbitrary=0.3, frac_bad=0.2)
    r3 = W.random_instance(rng, 60, 5, 30, max_dur=9, max_comm=300)          # long delays alone
    r1.dur[:6] = [65535, 131071, 65534, 131070, 196605, 16776959]        # around the multiples of 65535; the largest one
    wide += [(r1, None), (r1, dict(placement_mode=0, ring_slots=16, feeders=3)), (r2, None), (r3, None)]
    for w, shape in wide:
        with ds.Evaluator.for_workload(w, shape=shape) as ev:
            info = ev.info()
            got = [t.cpu().numpy() for t in ev.evaluate(torch.from_numpy(w.placement).cuda(), torch.from_numpy(w.rank).cuda())]
        assert info["variant"] == 5 and info["wide_ops"] == 1, (w.name, shape, info)
        want = oracle.evaluate_workload(w, 0, threads=8)
        for name, a, b in zip(("makespan", "bubble", "peak_mem", "flags"), got, want):
            assert np.array_equal(a, b), (name, w.name, shape, info)
    # a duration beyond 256 * 65535 - 1: the int32 kernel
    w = W.random_instance(rng, 50, 4, 20, max_dur=70001, zero_dur=False)
    w.dur[0] = 256 * 65535
    (z, b, pk, f), info = assert_parity(gpu_lib, w)
    assert info["variant"] in (1, 2)


def test_sixteen_bit_overflow_falls_back(gpu_lib):
    """End times that leave the 16-bit range: the ring kernel must hand exactly those candidates to the
    int32 kernel.  A long chain on few machines whose makespan straddles 65535 for different orders."""
    rng = np.random.default_rng(77)
    n, p = 600, 3
    rp, ci = W.random_dag(rng, n, 2, window=30)
    dur = rng.integers(60, 160, n).astype(np.int32)          # sum ~ 66000, so z crosses 65535 with few machines
    comm = rng.integers(1, 200, (p, p)).astype(np.int32)
    mem = rng.integers(-9, 10, n).astype(np.int64)
    pl, rk = W.list_schedules(rp, ci, p, 300, 4242)
    pl1, rk1 = W.list_schedules(rp, ci, 1, 100, 99)          # every third candidate runs everything on machine 0
    pl[::3], rk[::3] = pl1, rk1
    w = W.Workload("straddles 16 bits", p, rp, ci, dur, comm, mem, pl, rk)
    env16 = {"state_bits": 16}                 # (left alone the library would take 32-bit end times here)
    (z, b, pk, f), info = _with_env(env16, lambda: assert_parity(gpu_lib, w))
    assert info["state_bits"] == 16 and info["variant"] == 4        # optimistic ring kernel
    assert (z[f == 0] > 65535).any() and (z[f == 0] < 65535).any()
    # a common factor in every duration and delay is divided out before the 16-bit test
    w2 = W.Workload("scaled by 1000", p, rp, ci, dur * 1000, comm * 1000, mem, pl, rk)
    (z2, b2, pk2, f2), info2 = _with_env(env16, lambda: assert_parity(gpu_lib, w2))
    assert info2["time_scale"] == 1000 and (z2[f == 0] == 1000 * z[f == 0].astype(np.int64)).all()


def test_fallback_count_is_reported(gpu_lib):
    """dagsched_last_fallbacks: how many candidates of the last evaluate went to the int32 kernel one by one.  In an
    optimistic 16-bit run those are the well-formed, acyclic candidates whose end times reach the 16-bit range."""
    import torch
    rng = np.random.default_rng(77)
    n, p = 600, 3
    rp, ci = W.random_dag(rng, n, 2, window=30)
    dur = rng.integers(60, 160, n).astype(np.int32)
    comm = rng.integers(1, 200, (p, p)).astype(np.int32)
    pl, rk = W.list_schedules(rp, ci, p, 300, 4242)
    pl1, rk1 = W.list_schedules(rp, ci, 1, 100, 99)
    pl[::3], rk[::3] = pl1, rk1
    w = W.Workload("straddles 16 bits", p, rp, ci, dur, comm, rng.integers(-9, 10, n).astype(np.int64), pl, rk)
    zo, _, _, fo = oracle.evaluate_workload(w)
    dev = torch.device("cuda", 0)
    with gpu_lib.Evaluator.for_workload(w, shape={"state_bits": 16}) as ev:
        assert ev.info()["variant"] == 4
        z, _, _, f = ev.evaluate(torch.from_numpy(w.placement).to(dev), torch.from_numpy(w.rank).to(dev))
        n_fb = ev.last_fallbacks()
        assert (z.cpu().numpy() == zo).all() and (f.cpu().numpy() == fo).all()
        # an end time of 65535 or more cannot be held: those candidates must have gone over, and only feasible ones can
        assert int((zo >= 65535).sum()) <= n_fb <= int((fo == 0).sum()) and 0 < n_fb < w.n_cand, n_fb
        z2, _, _, f2 = ev.evaluate(torch.from_numpy(w.placement[1::3].copy()).to(dev), torch.from_numpy(w.rank[1::3].copy()).to(dev))
        n_fb2 = ev.last_fallbacks()
        assert n_fb2 <= n_fb and (z2.cpu().numpy() == zo[1::3]).all()
    with gpu_lib.Evaluator.for_workload(w) as ev:             # 32-bit state: nothing to hand over
        ev.evaluate(torch.from_numpy(w.placement).to(dev), torch.from_numpy(w.rank).to(dev))
        assert ev.info()["variant"] == 5 and ev.last_fallbacks() == 0


def test_two_live_handles_on_one_kernel_instantiation(gpu_lib):
    """Distinct handles are independent.  Two problems of different size that take the same kernel instantiation
    (same machines, same shape; the larger one needs more than 48 KB of LDS, the smaller one a few KB) are made one
    after the other and evaluated alternately: the kernel's LDS allowance belongs to the function, and the handle
    made second must not take away what the first one needs."""
    import torch
    rng = np.random.default_rng(4711)
    shape = {"feeders": 2, "ring_slots": 8, "placement_mode": 1, "cand_per_block": 8, "preds_per_op": 4}
    big = W.random_instance(rng, 3500, 8, 70, max_fanin=4, frac_arbitrary=0.2, frac_bad=0.1)
    small = W.random_instance(rng, 90, 8, 50, max_fanin=4, frac_arbitrary=0.2, frac_bad=0.1)
    want = {id(w): oracle.evaluate_workload(w) for w in (big, small)}
    dev = torch.device("cuda", 0)
    with gpu_lib.Evaluator.for_workload(big, shape=shape) as eb, gpu_lib.Evaluator.for_workload(small, shape=shape) as es:
        ib, is_ = eb.info(), es.info()
        assert ib["lds_bytes"] > 48 * 1024 > is_["lds_bytes"], (ib, is_)
        for k in ("variant", "cand_per_block", "ring_slots", "feeders", "placement_bytes_in_lds", "kernel_kind", "state_bits"):
            assert ib[k] == is_[k], (k, ib, is_)
        tens = {id(w): (torch.from_numpy(w.placement).to(dev), torch.from_numpy(w.rank).to(dev)) for w in (big, small)}
        for turn in range(3):
            for ev, w in ((eb, big), (es, small)):
                out = ev.evaluate(*tens[id(w)])
                torch.cuda.synchronize()
                for name, a, o in zip(("makespan", "bubble", "peak_mem", "flags"), out, want[id(w)]):
                    assert (a.cpu().numpy() == o).all(), (name, w.name, turn)


def _layered_workload(rng, n, p, n_cand, span, extra_edges=()):
    """A DAG whose node ids are a topological order and whose edges reach at most `span` ids back (plus the given
    extra edges), list-scheduled candidates, some of them then made cyclic or malformed."""
    src, dst = [], []
    for v in range(1, n):
        for u in rng.choice(np.arange(max(0, v - span), v), size=min(v, span, int(rng.integers(0, 4))), replace=False):
            src.append(int(u)); dst.append(v)
    for u, v in extra_edges:
        src.append(u); dst.append(v)
    rp, ci = W.csr_from_edges(n, src, dst)
    pl, rk = W.list_schedules(rp, ci, p, n_cand, int(rng.integers(0, 2 ** 62)))
    for c in range(0, n_cand, 5):                            # every fifth candidate: arbitrary orders (mostly cyclic)
        for j in range(p):
            idx = np.nonzero(pl[c] == j)[0]
            rk[c, idx] = rng.permutation(len(idx))
    if n_cand > 8:
        pl[3, n // 2] = p
        rk[7, n // 3] = -1
        rk[8, 0] = rk[8, n - 1] if pl[8, 0] == pl[8, n - 1] else rk[8, 0] + n
    return W.Workload("layered n=%d p=%d span=%d" % (n, p, span), p, rp, ci, rng.integers(0, 9, n).astype(np.int32),
                      rng.integers(0, 6, (p, p)).astype(np.int32), rng.integers(-5, 6, n).astype(np.int64), pl, rk)


def test_window_of_end_time_cells(gpu_lib):
    """Graphs whose edges are short in the order of the node ids can be evaluated with a window of named end-time
    cells per candidate instead of a cell per operation.  The library takes that mode by itself on the layered
    workload; here it is also forced, with windows that fit, windows far too small (candidates whose schedule does not
    fit go to the int32 kernel: the results stay the oracle's, the count says how many went), a single long-range edge
    that no small window can hold, all kernel kinds, several candidates per wavefront, weights and limits."""
    import torch
    rng = np.random.default_rng(5150)
    dev = torch.device("cuda", 0)
    w5 = W.gen_config(5, n_cand=40)
    (z, b, pk, f), info = assert_parity(gpu_lib, w5, repeats=2)
    assert info["window_log2"] == 12 and info["variant"] == 4, info
    (z, b, pk, f), info = _with_env({"window_cells": -1}, lambda: assert_parity(gpu_lib, w5))
    assert info["window_log2"] == 0
    (z, b, pk, f), info = assert_parity(gpu_lib, dataclasses_replace(w5, placement=w5.placement[:9], rank=w5.rank[:9]), layout=1)
    assert info["window_log2"] == 12
    # a window far too small for the layered workload: most candidates miss; they are evaluated again by the 16-bit
    # kernel with a cell per operation (a 32-bit cell per operation does not fit the LDS here), whose own range stops
    # would go on to the int32 kernel
    w5few = dataclasses_replace(w5, placement=w5.placement[:12], rank=w5.rank[:12])
    want5 = oracle.evaluate_workload(w5few, threads=8)
    for shape in ({"window_cells": 1024}, {"window_cells": 512, "ring_slots": 8}):
        with gpu_lib.Evaluator.for_workload(w5few, shape=shape) as ev:
            got = ev.evaluate(torch.from_numpy(w5few.placement).to(dev), torch.from_numpy(w5few.rank).to(dev))
            assert ev.last_fallbacks() > 0 and ev.info()["window_log2"] == int(np.log2(shape["window_cells"]))
            for a, o in zip(got, want5):
                assert np.array_equal(a.cpu().numpy(), o), shape
    seen_fallbacks = 0
    for n, p, span, cells, extra in ((700, 5, 20, 256, ()), (700, 5, 20, 32, ()), (1500, 16, 60, 1024, ()),
                                     (1500, 16, 60, 64, ()), (900, 64, 30, 512, ()), (400, 1, 10, 64, ()),
                                     (1200, 7, 15, 128, ((0, 1199), (3, 900))), (333, 3, 400, 512, ()), (2000, 33, 8, 8, ())):
        w = _layered_workload(rng, n, p, 45, span, extra)
        for shape in ({"window_cells": cells}, {"window_cells": cells, "preds_per_op": 4, "ring_slots": 16, "feeders": 3}):
            _say("%s window %d %s" % (w.name, cells, shape))
            want = oracle.evaluate_workload(w, threads=8)
            with gpu_lib.Evaluator.for_workload(w, shape=shape) as ev:
                info = ev.info()
                assert info["window_log2"] == int(np.log2(cells)) and info["variant"] == 4, info
                got = ev.evaluate(torch.from_numpy(w.placement).to(dev), torch.from_numpy(w.rank).to(dev))
                n_fb = ev.last_fallbacks()
                for name, a, o in zip(("makespan", "bubble", "peak_mem", "flags"), got, want):
                    bad = np.nonzero(np.asarray(a.cpu().numpy() != o).reshape(len(o), -1).any(axis=1))[0]
                    assert len(bad) == 0, "%s differs at %s (%s, %d fallbacks)" % (name, bad[:8], info, n_fb)
            if cells - 3 >= n:                               # every operation has a cell of its own: nothing can be missed
                assert n_fb == 0, (w.name, cells, n_fb)
            if extra:
                assert n_fb > 0
            seen_fallbacks += n_fb
    assert seen_fallbacks > 0
    # with static memory and limits (the accountant reads the lists of the ingest launch)
    w = _layered_workload(rng, 800, 6, 60, 25)
    w = dataclasses_replace(w, weight=rng.integers(0, 20, 800).astype(np.int64), mem_limit=np.array([1500] + [10 ** 9] * 5, dtype=np.int64))
    (z, b, pk, f), info = _with_env({"window_cells": 256}, lambda: assert_parity(gpu_lib, w))
    assert info["window_log2"] == 8 and 16 in set(f.tolist())
    # end times that need 32 bits: cells of 64 bits, same protocol (before: such a problem of this size went to the
    # int32 kernel, one wavefront per candidate with its state in HBM)
    w5big = dataclasses_replace(w5, dur=(w5.dur * 37 + 11).astype(np.int32), comm=(w5.comm * 30).astype(np.int32),
                                placement=w5.placement[:12], rank=w5.rank[:12])
    (z, b, pk, f), info = assert_parity(gpu_lib, w5big, repeats=2)
    assert info["window_log2"] == 12 and info["state_bits"] == 32 and info["variant"] == 4 and int(z.max()) > 65535, info
    for n, p, span, cells in ((900, 7, 25, 256), (900, 7, 25, 16), (1300, 64, 40, 512), (500, 2, 12, 128)):
        w = _layered_workload(rng, n, p, 45, span)
        w = dataclasses_replace(w, dur=(w.dur * 211).astype(np.int32))
        for shape in ({"window_cells": cells, "state_bits": 32}, {"window_cells": cells, "state_bits": 32, "preds_per_op": 4}):
            _say("%s window %d of 64-bit cells %s" % (w.name, cells, shape))
            (z, b, pk, f), info = _with_env(shape, lambda: assert_parity(gpu_lib, w, repeats=2))
            assert info["window_log2"] == int(np.log2(cells)) and info["state_bits"] == 32, info
    # node ids that are no topological order: the mode is not taken, whatever the shape asks for
    wr = W.random_instance(rng, 300, 4, 20)
    (z, b, pk, f), info = _with_env({"window_cells": 128}, lambda: assert_parity(gpu_lib, wr))
    assert info["window_log2"] == 0


def test_large_delays(gpu_lib):
    rng = np.random.default_rng(5)
    w = W.random_instance(rng, 120, 5, 30, max_comm=4000, max_dur=977)
    (z, b, pk, f), info = assert_parity(gpu_lib, w)
    assert info["variant"] == 5 and info["wide_ops"] == 1
    (z, b, pk, f), info = _with_env({"kernel": 1}, lambda: assert_parity(gpu_lib, w))
    assert info["variant"] in (1, 2)


def test_many_op_parts_use_the_general_kernel(gpu_lib):
    """The 16-bit kernel counts the op parts of a lane in 16 bits: a graph with 65536 parts or more (here 40000
    operations of up to twelve predecessors each) must be left to the int32 kernel."""
    rng = np.random.default_rng(11)
    n, p = 40000, 6
    rp, ci = W.random_dag(rng, n, 12, window=400)
    dur = rng.integers(0, 2, n).astype(np.int32)             # short operations: hardly any edge is implied by a longer path
    comm = rng.integers(3, 6, (p, p)).astype(np.int32)
    mem = rng.integers(-3, 4, n).astype(np.int64)
    pl, rk = W.list_schedules(rp, ci, p, 5, 1234)
    w = W.Workload("many parts", p, rp, ci, dur, comm, mem, pl, rk)
    (z, b, pk, f), info = assert_parity(gpu_lib, w)
    assert info["state_bits"] == 32 and (f == 0).all()


# --------------------------------------------------------------------------- static memory and limits (eq. (16))

@pytest.mark.parametrize("force_general", [0, 1])
def test_static_memory_and_limits(gpu_lib, force_general):
    """Base level = static memory placed on the machine; OVER_MEMORY is tested last.  The limits are set at a
    quantile of the unlimited peaks so that both outcomes occur."""
    import dataclasses
    rng = np.random.default_rng(1616)
    cases = [W.gen_config(1, n_cand=200), W.gen_config(2, n_cand=300), W.gen_config(4, n_cand=9), W.gen_config(5, n_cand=3),
             W.random_instance(rng, 150, 6, 80, max_fanin=7, frac_arbitrary=0.3, frac_bad=0.3)]
    seen = set()
    for w in cases:
        weight = rng.integers(0, 1000, w.n_nodes).astype(np.int64)
        zo, bo, pko, fo = oracle.Problem(w.n_devices, w.row_ptr, w.col_idx, w.dur, w.comm, w.mem_delta,
                                         weight=weight).evaluate(w.placement, w.rank, threads=8)
        ok = fo == 0
        limit = pko[ok].max(axis=0).astype(np.int64)             # loose everywhere ...
        limit[0] = int(np.median(pko[ok][:, 0]))                 # ... but tight on machine 0
        w2 = dataclasses.replace(w, name=w.name + " + weights", weight=weight)
        w3 = dataclasses.replace(w, name=w.name + " + weights + limits", weight=weight, mem_limit=limit)
        env = {"kernel": 1} if force_general else {}
        (z2, b2, pk2, f2), _ = _with_env(env, lambda: assert_parity(gpu_lib, w2))
        assert (f2 == fo).all() and (pk2 == pko).all()
        (z3, b3, pk3, f3), _ = _with_env(env, lambda: assert_parity(gpu_lib, w3))
        seen.update(int(x) for x in f3)
        assert (f3[~ok] == fo[~ok]).all()            # the new flag never hides another one
        (z4, b4, pk4, f4), _ = _with_env(env, lambda: assert_parity(gpu_lib, w3, layout=1))
        assert (f4 == f3).all()
    assert {0, 16} <= seen


# --------------------------------------------------------------------------- missing channels (eqs. (9)-(10))

@pytest.mark.parametrize("env", [{}, {"kernel": 1}, {"state_bits": 32}])
def test_missing_channels(gpu_lib, env):
    """comm entry -1: the pair has no channel; a candidate with a message over it is NO_CHANNEL, after the flags of
    malformed candidates and before every other one.  Random clusters on random instances (a third of the pairs
    missing down to a few), a chain-shaped cluster under the pipelines, a few missing pairs under config 4."""
    import dataclasses
    rng = np.random.default_rng(910)
    seen = {}

    def run(w, layouts=(0,)):
        for layout in layouts:
            (z, b, pk, f), _ = _with_env(env, lambda: assert_parity(gpu_lib, w, layout=layout))
            for x in f:
                seen[int(x)] = seen.get(int(x), 0) + 1
        return f

    for trial in range(6):
        p = int(rng.integers(2, 9))
        w = W.random_instance(rng, int(rng.integers(20, 300)), p, 120, max_fanin=4, frac_bad=0.2)
        missing = (rng.random((p, p)) < (0.35, 0.1, 0.03)[trial % 3]) & ~np.eye(p, dtype=bool)
        comm = np.where(missing, oracle.NO_CHANNEL, w.comm).astype(np.int32)
        np.fill_diagonal(comm, oracle.NO_CHANNEL if trial % 2 else 0)
        limit = np.full(p, 3, dtype=np.int64) if trial % 3 == 0 else None          # OVER_MEMORY comes after NO_CHANNEL
        run(dataclasses.replace(w, name=w.name + " missing channels", comm=comm, mem_limit=limit), layouts=(0, 1))
    for cfg, n in ((1, 300), (2, 200)):                                             # pipelines: stage s on machine s
        w = W.gen_config(cfg, n_cand=n)
        p = w.n_devices
        near = np.abs(np.arange(p)[:, None] - np.arange(p)[None, :]) == 1
        chain = np.where(near, w.comm, oracle.NO_CHANNEL).astype(np.int32)
        f_full = oracle.evaluate_workload(w)[3]
        assert (run(dataclasses.replace(w, name=w.name + " chain cluster", comm=chain)) == f_full).all()
        cut = chain.copy(); cut[2, 1] = oracle.NO_CHANNEL
        assert (run(dataclasses.replace(w, name=w.name + " cut chain", comm=cut)) == ds_flag_no_channel()).all()
    w = W.gen_config(4, n_cand=24)                                                  # a placement per candidate
    comm = w.comm.copy()
    comm[3, 17] = comm[30, 2] = oracle.NO_CHANNEL
    f = run(dataclasses.replace(w, name=w.name + " two pairs missing", comm=comm))
    assert 0 < (f == ds_flag_no_channel()).sum()
    assert seen.get(0, 0) > 100 and seen.get(32, 0) > 100 and seen.get(1, 0) > 20 and seen.get(2, 0) and seen.get(4, 0), seen


def ds_flag_no_channel():
    from paper_2503_09357_amd import dagsched
    assert dagsched.FLAG_NO_CHANNEL == oracle.FLAG_NO_CHANNEL and dagsched.NO_CHANNEL == oracle.NO_CHANNEL
    return dagsched.FLAG_NO_CHANNEL


def test_memory_limit_on_an_empty_machine(gpu_lib):
    """A machine that runs nothing has level 0; a negative limit on it still flags the candidate."""
    import dataclasses
    rng = np.random.default_rng(1617)
    rp, ci = W.random_dag(rng, 40, 2, window=8)
    pl, rk = W.list_schedules(rp, ci, 3, 50, 7)                # machines 0..2 used, machine 3 always empty
    w = W.Workload("empty machine", 4, rp, ci, rng.integers(1, 9, 40).astype(np.int32),
                   rng.integers(1, 5, (4, 4)).astype(np.int32), rng.integers(-3, 4, 40).astype(np.int64), pl, rk)
    big = np.full(4, 10**9, dtype=np.int64)
    for lim3, want in ((0, 0), (-1, 16)):
        lim = big.copy()
        lim[3] = lim3
        (z, b, pk, f), _ = assert_parity(gpu_lib, dataclasses.replace(w, mem_limit=lim))
        assert (f == want).all()



def test_shortcut_edges_next_to_longer_paths(gpu_lib):
    """Wide operations whose predecessors are also reachable through longer paths: the fast kernel may leave such
    an edge out of its ops only when the path's intermediate durations cover the largest channel delay.  Durations
    of 0, 1, 2 and 50 against delays up to 60 put many edges on either side of that line."""
    rng = np.random.default_rng(8080)
    for trial in range(4):
        n, p = 220, 5
        src, dst = [], []
        for v in range(1, n):
            for u in rng.choice(np.arange(max(0, v - 12), v), size=min(v, int(rng.integers(1, 4))), replace=False):
                src.append(int(u)); dst.append(v)
        preds = {v: set() for v in range(n)}
        for u, v in zip(src, dst):
            preds[v].add(u)
        for v in range(2, n):                                  # shortcuts from predecessors of predecessors (and theirs)
            anc = set()
            for u in preds[v]:
                anc |= preds[u]
                for t in preds[u]:
                    anc |= preds[t]
            for u in sorted(anc - preds[v])[: int(rng.integers(0, 6))]:
                src.append(u); dst.append(v)
        rp, ci = W.csr_from_edges(n, src, dst)
        dur = rng.choice([0, 1, 2, 50], size=n, p=[0.2, 0.3, 0.3, 0.2]).astype(np.int32)
        comm = rng.integers(0, 61, (p, p)).astype(np.int32)
        mem = rng.integers(-5, 6, n).astype(np.int64)
        pl, rk = W.list_schedules(rp, ci, p, 120, 1000 + trial)
        w = W.Workload("shortcut edges %d" % trial, p, rp, ci, dur, comm, mem, pl, rk)
        assert (np.diff(W.csr_from_edges(n, dst, src)[0]) > 4).sum() > 20      # plenty of wide operations
        (z, b, pk, f), info = assert_parity(gpu_lib, w)
        assert info["state_bits"] == 16 and (f == 0).all()
