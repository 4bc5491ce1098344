"""The allocation-free entry point dagsched_schedule_static against dagsched_schedule, through the C-ABI: same
start times, end times and flag, bit for bit, on two calls in a row of which the second has the smaller input (the
static scratch then still holds the larger call's rows), and again in the other order."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W

pytestmark = pytest.mark.gpu


def _cases(rng, n, p):
    """A feasible candidate, a cyclic one, one with a bad rank and one with a bad placement."""
    w = W.random_instance(rng, n, p, 6, max_fanin=4, frac_arbitrary=0.0, frac_bad=0.0)
    pl, rk = w.placement.copy(), w.rank.copy()
    for j in range(p):                                       # candidate 1: every machine's order reversed
        idx = np.nonzero(pl[1] == j)[0]
        rk[1, idx] = len(idx) - 1 - rk[1, idx]
    rk[2, 0] = rk[2, 0] + n
    pl[3, n // 2] = p
    return w, pl, rk


def test_schedule_static_matches_schedule(gpu_lib):
    import torch
    ds = gpu_lib
    dev = torch.device("cuda", 0)
    rng = np.random.default_rng(20250309)
    big, small = _cases(rng, 3001, 7), _cases(rng, 77, 3)
    seen_flags = set()
    with ds.Evaluator.for_workload(big[0], max_candidates=1) as eb, ds.Evaluator.for_workload(small[0], max_candidates=1) as es:
        for order in ((eb, big), (es, small)), ((es, small), (eb, big)), ((eb, big), (es, small)):
            for ev, (w, pl, rk) in order:
                prob = oracle.Problem.of(w)
                for c in range(pl.shape[0]):
                    print("[no-alloc] N=%d P=%d candidate %d" % (w.n_nodes, w.n_devices, c), flush=True)
                    tp, tr = torch.from_numpy(pl[c]).to(dev), torch.from_numpy(rk[c]).to(dev)
                    s0, e0, f0 = ev.schedule(tp, tr)
                    s1, e1, f1 = ev.schedule(tp, tr, static_scratch=True)
                    torch.cuda.synchronize()
                    assert int(f0[0]) == int(f1[0])
                    assert torch.equal(s0, s1) and torch.equal(e0, e1)
                    flag_o, so, eo, _, _ = prob.schedule(pl[c], rk[c])
                    assert int(f1[0]) == flag_o
                    if flag_o == 0:
                        assert (s1.cpu().numpy() == so).all() and (e1.cpu().numpy() == eo).all()
                    else:
                        assert (s1 == -1).all() and (e1 == -1).all()
                    seen_flags.add(flag_o)
    assert {0, 1, 2, 4} <= seen_flags, seen_flags


def test_schedule_static_refuses_what_the_scratch_cannot_hold(gpu_lib):
    import torch
    ds = gpu_lib
    dev = torch.device("cuda", 0)
    n = ds.STATIC_MAX_NODES + 1
    rp, ci = W.csr_from_edges(n, list(range(n - 1)), list(range(1, n)))
    with ds.Evaluator(2, rp, ci, np.ones(n, np.int32), np.ones((2, 2), np.int32), np.zeros(n, np.int64), 1) as ev:
        pl = torch.zeros(n, dtype=torch.int32, device=dev)
        rk = torch.arange(n, dtype=torch.int32, device=dev)
        s0, e0, f0 = ev.schedule(pl, rk)
        torch.cuda.synchronize()
        assert int(f0[0]) == 0 and int(e0[-1]) == n
        with pytest.raises(ds.DagschedError) as err:
            ev.schedule(pl, rk, static_scratch=True)
        assert err.value.code == ds.ESCRATCH and "static scratch" in str(err.value)
