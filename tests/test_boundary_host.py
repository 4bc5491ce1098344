"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
description check returns the documented codes (the same codes the oracle's problem check returns)."""
from __future__ import annotations

import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import _build, dagsched
from paper_2503_09357_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dagsched.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dagsched_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(_build.ensure_hip())
    names = _declared_symbols()
    assert set(names) == set(dagsched.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror_texts():
    lib = dagsched.load(import_torch_first=False)
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(lib.dagsched_strerror(code)) > 0


def test_validate_codes_match_oracle_problem_check():
    rp, ci = W.csr_from_edges(3, [0, 1], [1, 2])
    base = dict(n_devices=2, row_ptr=rp, col_idx=ci, dur=[1, 2, 3], comm=[[0, 1], [1, 0]], mem_delta=[0, 0, 0])
    big = 2 ** 31 - 1
    rp_cyc, ci_cyc = W.csr_from_edges(3, [0, 1, 2], [1, 2, 0])
    cases = [
        ({}, dagsched.OK),
        ({"dur": [1, -2, 3]}, dagsched.EINVAL),
        ({"comm": [[0, -2], [1, 0]]}, dagsched.EINVAL),
        ({"comm": [[0, -1], [-1, 0]]}, dagsched.OK),                    # -1: the pair has no channel (eq. (10))
        ({"dur": [big, 0, 0], "comm": [[0, -1], [-1, 0]]}, dagsched.OK),
        ({"comm": [[-5, 1], [1, -9]]}, dagsched.OK),
        ({"row_ptr": rp_cyc, "col_idx": ci_cyc}, dagsched.ECYCLE),
        ({"row_ptr": np.array([0, 1, 2, 2]), "col_idx": np.array([0, 2])}, dagsched.EINVAL),
        ({"row_ptr": np.array([0, 1, 2, 2]), "col_idx": np.array([1, 3])}, dagsched.EINVAL),
        ({"row_ptr": np.array([0, 2, 1, 2]), "col_idx": np.array([1, 2])}, dagsched.EINVAL),
        ({"dur": [big, 0, 0], "comm": [[0, 0], [0, 0]]}, dagsched.OK),
        ({"dur": [big, 1, 0], "comm": [[0, 0], [0, 0]]}, dagsched.EOVERFLOW),
        ({"dur": [big - 2, 0, 0], "comm": [[0, 1], [0, 0]]}, dagsched.OK),
        ({"dur": [big - 1, 0, 0], "comm": [[0, 1], [0, 0]]}, dagsched.EOVERFLOW),
    ]
    for change, want in cases:
        args = dict(base, **change)
        assert dagsched.validate(**args) == want, change
        prob = oracle.Problem(args["n_devices"], args["row_ptr"], args["col_idx"], args["dur"], args["comm"],
                              args["mem_delta"])
        assert prob.check() == want, change
    # arguments only the boundary has
    assert dagsched.validate(**base, max_candidates=0) == dagsched.EINVAL
    assert dagsched.validate(**base, layout=7) == dagsched.EINVAL
    assert dagsched.validate(**dict(base, n_devices=65, comm=np.zeros((65, 65)))) == dagsched.EINVAL
    assert dagsched.validate(**dict(base, n_devices=0)) == dagsched.EINVAL
    assert dagsched.load(import_torch_first=False).dagsched_validate(None) == dagsched.EINVAL
    # null array pointer
    d = dagsched._HostProblem(2, rp, ci, [1, 2, 3], [[0, 1], [1, 0]], [0, 0, 0], 1, 0, 0)
    d.desc.dur = None
    assert dagsched.load(import_torch_first=False).dagsched_validate(ctypes.byref(d.desc)) == dagsched.EINVAL


def test_validate_accepts_all_configs():
    for cfg in (1, 2, 3, 4, 5):
        w = W.gen_config(cfg, n_cand=1)
        assert dagsched.validate(w.n_devices, w.row_ptr, w.col_idx, w.dur, w.comm, w.mem_delta) == dagsched.OK


def test_generators_are_seeded_and_prefix_consistent():
    a = W.gen_config(4, n_cand=6)
    b = W.gen_config(4, n_cand=3)
    assert (a.placement[:3] == b.placement).all() and (a.rank[:3] == b.rank).all()
    assert (a.dur == b.dur).all() and (a.col_idx == b.col_idx).all()
    c = W.gen_config(4, n_cand=3, seed=123)
    assert not (c.placement == b.placement).all()
    for cfg, (n, e, p) in {1: (64, 80, 4), 2: (768, 960, 8), 3: (6144, 7040, 16), 4: (11712, 25360, 32)}.items():
        w = W.gen_config(cfg, n_cand=2)
        assert (w.n_nodes, w.n_edges, w.n_devices) == (n, e, p)
    w = W.gen_config(5, n_cand=1)
    assert w.n_nodes == 50000 and w.n_devices == 64 and 120000 < w.n_edges < 130000


def test_validate_checks_static_memory():
    rp, ci = W.csr_from_edges(3, [0, 1], [1, 2])
    args = dict(n_devices=2, row_ptr=rp, col_idx=ci, dur=[1, 1, 1], comm=[[0, 1], [1, 0]], mem_delta=[0, 0, 0])
    ds = dagsched
    assert ds.validate(**args, weight=[0, 5, 7], mem_limit=[-3, 10]) == 0      # limits may be anything
    assert ds.validate(**args, weight=[0, -1, 7]) == -1                        # W_i >= 0
    with pytest.raises(ValueError):
        ds.validate(**args, weight=[1, 2])
    with pytest.raises(ValueError):
        ds.validate(**args, mem_limit=[1, 2, 3])



def test_validate_checks_the_launch_shape():
    rp, ci = W.csr_from_edges(3, [0, 1], [1, 2])
    args = dict(n_devices=2, row_ptr=rp, col_idx=ci, dur=[1, 1, 1], comm=[[0, 1], [1, 0]], mem_delta=[0, 0, 0])
    ds = dagsched
    assert ds.validate(**args, shape={}) == 0
    assert ds.validate(**args, shape=dict(cand_per_block=8, ring_slots=16, feeders=3, placement_mode=0, block_threads=512)) == 0
    for bad in (dict(cand_per_block=3), dict(cand_per_block=128), dict(ring_slots=5), dict(feeders=5), dict(feeders=-1),
                dict(placement_mode=3), dict(placement_mode=-2), dict(block_threads=100), dict(block_threads=2048)):
        assert ds.validate(**args, shape=bad) == -1, bad


def test_validate_checks_the_shared_placement_hint():
    rp, ci = W.csr_from_edges(3, [0, 1], [1, 2])
    args = dict(n_devices=2, row_ptr=rp, col_idx=ci, dur=[1, 1, 1], comm=[[0, 1], [1, 0]], mem_delta=[0, 0, 0])
    assert dagsched.validate(**args, shared_placement=[0, 1, 1]) == 0
    assert dagsched.validate(**args, shared_placement=[0, 2, 1]) == -1
    assert dagsched.validate(**args, shared_placement=[0, -1, 1]) == -1
    with pytest.raises(ValueError):
        dagsched.validate(**args, shared_placement=[0, 1])


def test_bench_refuses_more_than_one_gpu_and_reads_the_committed_counters():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    sys.path.insert(0, root)
    import bench
    w = W.gen_config(4, n_cand=1)
    per_cand = 8 * w.n_nodes + 16 + 8 * w.n_devices
    assert bench.algorithmic_bytes(w) - per_cand == 4 * (w.n_nodes + 1) + 4 * w.n_edges + 12 * w.n_nodes + 4 * w.n_devices ** 2
    t = bench.measured_traffic(4)                    # None once the kernel sources changed after the counters were taken
    assert t is None or t > 0
    assert bench.measured_traffic(99) is None


def test_plan_of_the_five_workloads():
    """dagsched_plan (host only): the variant and shape dagsched_create would take on an MI355X.  The pipelines with
    their shared placement as a hint: the small one stays on the ring kernel, the zero-bubble one takes the
    shared-placement kernel, the bidirectional one does not fit it; the MoE and the layered graph run optimistically
    in 16 bits; every shape fits the LDS, and a shape asked for is the shape planned."""
    from paper_2503_09357_amd import workloads as W
    full = {1: 1024, 2: 65536, 3: 16384, 4: 4096, 5: 1024}
    want = {1: 3, 2: 6, 3: 3, 4: 4, 5: 4}
    for cfg in (1, 2, 3, 4, 5):
        w = W.gen_config(cfg, n_cand=2)
        hint = w.placement[0] if cfg <= 3 else None
        args = (w.n_devices, w.row_ptr, w.col_idx, w.dur, w.comm, w.mem_delta)
        info = dagsched.plan(*args, max_candidates=full[cfg], shared_placement=hint)
        assert info["variant"] == want[cfg], (cfg, info)
        assert 0 < info["lds_bytes"] <= 160 * 1024 and info["block_threads"] % 64 == 0 and info["state_bits"] == 16
        assert info["cand_per_block"] * (1 if info["variant"] == 6 else w.n_devices) <= 64 * max(1, info["block_threads"] // 128)
        no_hint = dagsched.plan(*args, max_candidates=full[cfg], shared_placement=hint, shape={"ignore_shared_placement": 1})
        assert no_hint["variant"] in (3, 4), (cfg, no_hint)
        forced = dagsched.plan(*args, max_candidates=full[cfg], shape={"kernel": 1})
        assert forced["variant"] in (1, 2) and forced["state_bits"] == 32
        if cfg in (1, 2):
            shaped = dagsched.plan(*args, max_candidates=full[cfg], shape={"feeders": 1, "ring_slots": 4, "placement_mode": 1, "cand_per_block": 2})
            assert (shaped["feeders"], shaped["ring_slots"], shaped["placement_bytes_in_lds"], shaped["cand_per_block"]) == (1, 4, 1, 2)
        small_gpu = dagsched.plan(*args, max_candidates=full[cfg], lds_bytes=64 * 1024, n_cu=8)
        assert small_gpu["lds_bytes"] <= 64 * 1024
    # a bad description is answered as dagsched_validate answers it
    w = W.gen_config(1, n_cand=1)
    with pytest.raises(dagsched.DagschedError) as e:
        dagsched.plan(w.n_devices, w.row_ptr, w.col_idx, -w.dur, w.comm, w.mem_delta)
    assert e.value.code == dagsched.EINVAL


def test_plan_takes_the_window_of_end_time_cells_only_where_it_is_sound():
    """Host logic of the window mode: taken by itself on a large graph whose node ids are a topological order with
    short edges (the layered workload: 4096 cells for edges of at most 499 ids), never when the ids are no
    topological order, never when the caller forbids it, with the caller's cell count when one is given, only
    while every cell name fits 16 bits (N + 3 N / (K - 3) + 1 <= 65535), and with 64-bit cells when the end times
    need 32 bits."""
    from paper_2503_09357_amd import workloads as W
    w = W.gen_config(5, n_cand=2)
    args = (w.n_devices, w.row_ptr, w.col_idx, w.dur, w.comm, w.mem_delta)
    src, dst = W.edges_from_csr(w.row_ptr, w.col_idx)
    assert (src < dst).all() and int((dst - src).max()) == 499
    info = dagsched.plan(*args, max_candidates=1024)
    assert info["window_log2"] == 12 and info["variant"] == 4 and info["lds_bytes"] < 48 * 1024 and info["placement_bytes_in_lds"] == 0
    assert dagsched.plan(*args, max_candidates=1024, shape={"window_cells": -1})["window_log2"] == 0
    assert dagsched.plan(*args, max_candidates=1024, shape={"window_cells": 8192})["window_log2"] == 13
    # 50000 operations in periods of 13 names of 16 cells: names up to 61540 fit; in periods of 5 of 8 they do not
    assert dagsched.plan(*args, max_candidates=1024, shape={"window_cells": 16})["window_log2"] == 4
    assert dagsched.plan(*args, max_candidates=1024, shape={"window_cells": 8})["window_log2"] == 0
    for bad in (3, 100, 65536, -2):                          # a power of two from 8 to 32768, 0 or -1
        with pytest.raises(dagsched.DagschedError):
            dagsched.plan(*args, max_candidates=1024, shape={"window_cells": bad})
    # 32-bit end times: the same window with cells of 64 bits (twice the LDS of the 16-bit window, not 200 KB)
    wide = dagsched.plan(*args, max_candidates=1024, shape={"state_bits": 32})
    assert wide["window_log2"] == 12 and wide["state_bits"] == 32 and wide["variant"] == 4 and wide["lds_bytes"] < 64 * 1024
    big = (w.n_devices, w.row_ptr, w.col_idx, (w.dur * 37 + 11).astype(np.int32), (w.comm * 30).astype(np.int32), w.mem_delta)
    info = dagsched.plan(*big, max_candidates=1024)
    assert info["window_log2"] == 12 and info["state_bits"] == 32 and info["variant"] == 4
    assert dagsched.plan(*big, max_candidates=1024, shape={"window_cells": -1})["variant"] in (1, 2)   # else: the int32 kernel
    # the same graph with its ids reversed is no topological order: declined, also when asked for
    n = w.n_nodes
    rp, ci = W.csr_from_edges(n, n - 1 - dst, n - 1 - src)
    rev = (w.n_devices, rp, ci, w.dur[::-1].copy(), w.comm, w.mem_delta[::-1].copy())
    assert dagsched.plan(*rev, max_candidates=1024)["window_log2"] == 0
    assert dagsched.plan(*rev, max_candidates=1024, shape={"window_cells": 4096})["window_log2"] == 0
    # a small layered graph: not by itself (nothing to gain), but on request
    rng = np.random.default_rng(11)
    s2, d2 = [], []
    for v in range(1, 600):
        for u in rng.choice(np.arange(max(0, v - 9), v), size=min(v, 2), replace=False):
            s2.append(int(u)); d2.append(v)
    rp, ci = W.csr_from_edges(600, s2, d2)
    small = (4, rp, ci, np.ones(600, np.int32), np.ones((4, 4), np.int32), np.zeros(600, np.int64))
    assert dagsched.plan(*small, max_candidates=64)["window_log2"] == 0
    assert dagsched.plan(*small, max_candidates=64, shape={"window_cells": 128})["window_log2"] == 7
    # the MoE graph is numbered micro-batch by micro-batch: an operation 1021 ids on lies in another micro-batch at any
    # depth, no window has a margin.  Renumbered level by level its edges are short (64 ids once the implied ones are
    # dropped) and the margin is there, but its levels are narrow (19 operations for 32 machines) and most schedules
    # would miss a window of 1024 cells: not taken by itself either, only on request
    w4 = W.gen_config(4, n_cand=2)
    args4 = (w4.n_devices, w4.row_ptr, w4.col_idx, w4.dur, w4.comm, w4.mem_delta)
    assert dagsched.plan(*args4, max_candidates=4096)["window_log2"] == 0
    s4, d4 = W.edges_from_csr(w4.row_ptr, w4.col_idx)
    lvl = np.zeros(w4.n_nodes, np.int64)
    for u, v in sorted(zip(s4.tolist(), d4.tolist())):
        lvl[v] = max(lvl[v], lvl[u] + 1)
    by_level = np.lexsort((np.arange(w4.n_nodes), lvl))
    new_id = np.empty(w4.n_nodes, np.int64)
    new_id[by_level] = np.arange(w4.n_nodes)
    rp, ci = W.csr_from_edges(w4.n_nodes, new_id[s4], new_id[d4])
    lev4 = (w4.n_devices, rp, ci, w4.dur[by_level].copy(), w4.comm, w4.mem_delta[by_level].copy())
    assert dagsched.plan(*lev4, max_candidates=4096)["window_log2"] == 0
    assert dagsched.plan(*lev4, max_candidates=4096, shape={"window_cells": 4096})["window_log2"] == 12
