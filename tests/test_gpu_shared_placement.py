"""Parity of the shared-placement kernel (candidates that place alike and differ in the orders only, the regime of
Sec. V's pipeline experiments) against the CPU oracle, through the C-ABI.  The hint never changes a result: every
case is compared element by element with the oracle, and candidates that do not keep the promise are among them."""
from __future__ import annotations

import dataclasses

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W
from test_gpu_parity import _say, _with_env, assert_parity

pytestmark = pytest.mark.gpu

SHARED = {"ignore_shared_placement": 0}          # the library's default, said aloud


def _forced(waves):
    """The library keeps handles for small batches on the ring kernel; naming the number of relaxing wavefronts per
    workgroup makes it take the shared-placement kernel whatever the batch size."""
    return dict(SHARED, static_waves=waves)
STATIC = 6                                            # dagsched_get_info: the shared-placement kernel


def _fixed_placement_instance(rng, n, p, n_cand, max_fanin=3, max_dur=9, max_comm=5, used=None, strangers=0):
    """Random DAG, one random placement (machines >= `used` stay empty), list-scheduled orders; then a third of the
    candidates get arbitrary per-machine permutations (mostly cyclic), some are malformed, and `strangers` of them
    move one operation to another machine, re-ranked properly (feasible, but not the shared placement)."""
    rp, ci = W.random_dag(rng, n, max_fanin, dup_prob=0.05)
    used = p if used is None else used
    fixed = rng.integers(0, used, n).astype(np.int32)
    pl, rk = W.list_schedules(rp, ci, p, n_cand, int(rng.integers(0, 2 ** 62)), fixed_placement=fixed)
    for c in range(n_cand):
        r = rng.random()
        if r < 0.3:
            for j in range(p):
                idx = np.nonzero(pl[c] == j)[0]
                rk[c, idx] = rng.permutation(len(idx))
        elif r < 0.45:
            v = int(rng.integers(0, n))
            how = int(rng.integers(0, 5))
            if how == 0:
                pl[c, v] = -1 - int(rng.integers(0, 3))
            elif how == 1:
                pl[c, v] = p + int(rng.integers(0, 3))
            elif how == 2:
                rk[c, v] = -1 - int(rng.integers(0, 3))
            elif how == 3:
                rk[c, v] = rk[c, v] + 1 + int(rng.integers(0, n))
            else:
                rk[c, v] = rk[c, int(rng.integers(0, n))]
    for c in rng.choice(n_cand, size=min(strangers, n_cand), replace=False):
        v = int(rng.integers(0, n))
        old, new = int(pl[c, v]), int((pl[c, v] + 1 + rng.integers(0, p - 1)) % p) if p > 1 else int(pl[c, v])
        if new == old or (pl[c] < 0).any() or (pl[c] >= p).any():
            continue
        rk[c, (pl[c] == old) & (rk[c] > rk[c, v])] -= 1          # close the gap it leaves
        pl[c, v] = new
        rk[c, v] = int((pl[c] == new).sum()) - 1                 # last on its new machine (may or may not be acyclic)
    w = W.Workload("shared placement n=%d p=%d" % (n, p), p, rp, ci, rng.integers(0, max_dur + 1, n).astype(np.int32),
                   rng.integers(0, max_comm + 1, (p, p)).astype(np.int32), rng.integers(-6, 7, n).astype(np.int64), pl, rk)
    return w, fixed


def _run(ds, w, fixed, layout=0, want_variant=STATIC, waves=1):
    import torch
    dev = torch.device("cuda", 0)
    _say("%s | N=%d E=%d P=%d C=%d layout=%d" % (w.name, w.n_nodes, w.n_edges, w.n_devices, w.n_cand, layout))
    pl, rk = (w.placement, w.rank) if layout == 0 else (np.ascontiguousarray(w.placement.T), np.ascontiguousarray(w.rank.T))

    def go():
        with ds.Evaluator.for_workload(w, max_candidates=max(1, w.n_cand), layout=layout, shared_placement=fixed) as ev:
            outs = []
            for _ in range(2):
                out = ev.evaluate(torch.from_numpy(pl).to(dev), torch.from_numpy(rk).to(dev))
                torch.cuda.synchronize()
                outs.append(tuple(t.cpu().numpy() for t in out))
            return outs, ev.info()

    outs, info = _with_env(_forced(waves), go)
    assert info["variant"] in (want_variant if isinstance(want_variant, tuple) else (want_variant,)), info
    assert all((a == b).all() for a, b in zip(*outs)), "evaluation is not deterministic"
    z, b, pk, f = outs[0]
    zo, bo, pko, fo = oracle.evaluate_workload(w, layout, threads=8)
    bad = np.nonzero(f != fo)[0]
    assert len(bad) == 0, "flags differ at %s: gpu %s oracle %s (%s)" % (bad[:8], f[bad[:8]], fo[bad[:8]], info)
    bad = np.nonzero(z != zo)[0]
    assert len(bad) == 0, "makespan differs at %s: gpu %s oracle %s (%s)" % (bad[:8], z[bad[:8]], zo[bad[:8]], info)
    assert (b == bo).all() and pk.shape == pko.shape and (pk == pko).all()
    return f, info


@pytest.mark.parametrize("cfg,c,waves", [(1, 1024, 1), (1, 1024, 4), (2, 3000, 2), (2, 3000, 5), (2, 65536, 0)])
def test_pipeline_configurations(gpu_lib, cfg, c, waves):
    """for_workload finds the shared placement by itself ("auto"), as bench.py does; at full size the library takes
    the shared-placement kernel by itself (waves = 0), the smaller batches are made to."""
    w = W.gen_config(cfg, n_cand=c)
    env = _forced(waves) if waves else SHARED
    (z, b, pk, f), info = _with_env(env, lambda: assert_parity(gpu_lib, w))
    assert info["variant"] == STATIC, info
    if cfg == 2:
        marked = np.zeros(w.n_cand, bool)
        marked[w.meta["cyclic"][w.meta["cyclic"] < c]] = True
        assert ((f == 1) == marked).all()
    (z1, b1, pk1, f1), info = _with_env(_forced(waves or 2), lambda: assert_parity(gpu_lib, dataclasses.replace(
        w, placement=w.placement[:257], rank=w.rank[:257]), layout=1))
    assert info["variant"] == STATIC and (f1 == f[:257]).all()
    if not waves:                                             # the same handle parameters as bench.py: the ring kernel for small batches
        _, info = _with_env(SHARED, lambda: assert_parity(gpu_lib, W.gen_config(1, n_cand=1024)))
        assert info["variant"] == 3, info


def test_random_problems_with_malformed_cyclic_and_stranger_candidates(gpu_lib):
    rng = np.random.default_rng(606)
    seen = {}
    for trial in range(24):
        p = int(rng.choice([1, 2, 3, 4, 5, 8, 13, 16, 31, 64]))
        n = int(rng.choice([1, 2, 7, 33, 64, 130, 257, 700, 1501]))
        w, fixed = _fixed_placement_instance(rng, n, p, int(rng.choice([1, 9, 70, 300])), max_fanin=int(rng.integers(1, 5)),
                                             used=max(1, p - int(rng.integers(0, 3))), strangers=int(rng.choice([0, 0, 3, 20])))
        if trial % 4 == 1:
            w = dataclasses.replace(w, weight=rng.integers(0, 50, n).astype(np.int64), mem_limit=rng.integers(20, 400, p).astype(np.int64))
        if trial % 4 == 2:
            w = dataclasses.replace(w, dur=(w.dur * 12).astype(np.int32), comm=(w.comm * 18).astype(np.int32))   # gcd 6
        g = 64 // (1 << (p - 1).bit_length())                 # candidates per relaxing wavefront
        fits = [wv for wv in (1, 2, 3, 4, 8) if g * wv <= 64 and 25 * n + g * wv * (4 * n + 40) + 6000 <= 160 * 1024]
        waves = fits[trial % 5 % len(fits)]
        f, info = _run(gpu_lib, w, fixed, layout=trial % 2, waves=waves)
        for x in f:
            seen[int(x)] = seen.get(int(x), 0) + 1
    assert all(seen.get(k, 0) > 10 for k in (0, 1, 2, 4, 16)), seen


def test_largest_problems_the_kernel_takes(gpu_lib):
    """Tables and one wavefront's candidates just fit the LDS: 5000 operations on 64 machines (one candidate per
    wavefront), 3600 on 16 (four); a ragged candidate count, so the last batch of a workgroup is partly empty."""
    rng = np.random.default_rng(611)
    for n, p, c in ((5000, 64, 37), (3600, 16, 61), (1000, 3, 333)):
        w, fixed = _fixed_placement_instance(rng, n, p, c, max_fanin=3, strangers=2)
        f, info = _run(gpu_lib, w, fixed, waves=1)
        assert (f == 0).sum() > c // 3, (n, p, np.bincount(f))


def test_every_candidate_breaks_the_promise(gpu_lib):
    """A hint that is simply wrong: all candidates are evaluated by the int32 kernel, results as always."""
    rng = np.random.default_rng(607)
    w = W.random_instance(rng, 120, 5, 90, frac_bad=0.2)
    f, info = _run(gpu_lib, w, np.zeros(w.n_nodes, np.int32))
    assert (f == 0).sum() > 20


def test_problems_the_kernel_does_not_take(gpu_lib):
    """More than four distinct predecessors, a delay or a makespan bound beyond the format: the hint is ignored."""
    rng = np.random.default_rng(608)
    w, fixed = _fixed_placement_instance(rng, 90, 4, 40, max_fanin=7)
    _, info = _run(gpu_lib, w, fixed, want_variant=3)
    w, fixed = _fixed_placement_instance(rng, 90, 4, 40, max_comm=300)
    w.comm[0, 1] = 300
    _, info = _run(gpu_lib, w, fixed, want_variant=5)
    w, fixed = _fixed_placement_instance(rng, 400, 4, 40, max_dur=400)
    _, info = _run(gpu_lib, w, fixed, want_variant=(4, 5))
    with pytest.raises(gpu_lib.DagschedError):
        bad = fixed.copy(); bad[3] = 4
        gpu_lib.Evaluator.for_workload(w, shared_placement=bad)


def test_with_missing_channels_and_through_the_search_calls(gpu_lib):
    import torch
    rng = np.random.default_rng(609)
    w, fixed = _fixed_placement_instance(rng, 200, 6, 150, strangers=30)
    comm = w.comm.copy()
    comm[0, 1] = comm[4, 2] = oracle.NO_CHANNEL
    f, _ = _run(gpu_lib, dataclasses.replace(w, comm=comm), fixed)
    assert (f == 32).sum() > 0
