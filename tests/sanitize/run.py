#!/usr/bin/env python3
"""Host-side sanitizer run (AddressSanitizer + UndefinedBehaviorSanitizer).

Builds tests/sanitize/driver.cpp together with the library's source (host pass instrumented, device pass untouched)
and the two C oracles, all with clang's -fsanitize=address,undefined, writes the five workloads' descriptions with a
few candidates each plus some random and some malformed problems to a temporary directory, and runs the driver over
them: dagsched_validate and dagsched_plan (the description checks and the planning of kernel variant and launch
shape: the index arithmetic on caller arrays), the evaluation oracle with and without channel contention, the
coarsening oracle.  No GPU is needed or touched.  Not collected by pytest (minutes of compilation); run by hand:

    python tests/sanitize/run.py

Exit status 0 = no finding.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

from paper_2503_09357_amd import workloads as W  # noqa: E402

SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def dump(path, w, n_cand, max_candidates, shared):
    pl, rk = w.placement[:n_cand], w.rank[:n_cand]
    er = W.fcfs_edge_ranks(w.row_ptr, w.col_idx, w.n_devices, pl, rk)
    weight = np.arange(w.n_nodes, dtype=np.int64) % 7 if w.weight is None else w.weight
    limit = np.full(w.n_devices, 10 ** 12, np.int64) if w.mem_limit is None else w.mem_limit
    with open(path, "wb") as f:
        np.array([w.n_nodes, w.n_edges, w.n_devices, len(pl), int(shared), max_candidates], np.int32).tofile(f)
        for a, dt in ((w.row_ptr, np.int32), (w.col_idx, np.int32), (w.dur, np.int32), (np.asarray(w.comm).reshape(-1), np.int32),
                      (w.mem_delta, np.int64), (weight, np.int64), (limit, np.int64), (pl, np.int32), (rk, np.int32), (er, np.int32)):
            np.ascontiguousarray(a, dtype=dt).tofile(f)


def main() -> int:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/llvm/bin/clang"
    tmp = tempfile.mkdtemp(prefix="dagsched_san_")
    objs = []
    for src in ("dagsched_oracle.c", "coarsen_oracle.c"):
        obj = os.path.join(tmp, src[:-2] + ".o")
        subprocess.check_call([clang, "-O1", "-g", "-std=c11", *SAN, "-c", os.path.join(ROOT, "oracle", src), "-o", obj])
        objs.append(obj)
    exe = os.path.join(tmp, "driver")
    host_san = [x for flag in SAN for x in ("-Xarch_host", flag)]
    lib_obj, drv_obj = os.path.join(tmp, "dagsched.o"), os.path.join(tmp, "driver.o")
    print("building (device code is compiled too: a few minutes) ...", flush=True)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host_san,
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-function",
                           "-I", os.path.join(ROOT, "include"), "-c",
                           os.path.join(ROOT, "paper_2503_09357_amd", "csrc", "dagsched.hip"), "-o", lib_obj])
    subprocess.check_call([clang + "++", "-O1", "-g", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
                           os.path.join(HERE, "driver.cpp"), "-o", drv_obj])
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "--hip-link", "-fno-gpu-sanitize", *SAN, lib_obj, drv_obj, *objs, "-o", exe])
    files = []
    full = {1: 1024, 2: 65536, 3: 16384, 4: 4096, 5: 1024}
    for cfg in (1, 2, 3, 4, 5):
        w = W.gen_config(cfg, n_cand=6)
        path = os.path.join(tmp, "cfg%d.bin" % cfg)
        dump(path, w, 6, full[cfg], cfg <= 3)
        files.append(path)
    rng = np.random.default_rng(12345)
    for i in range(12):
        p = int(rng.choice([1, 2, 7, 16, 33, 64]))
        n = int(rng.choice([1, 2, 65, 300, 1201]))
        w = W.random_instance(rng, n, p, 12, max_fanin=int(rng.integers(0, 7)), max_comm=int(rng.choice([0, 5, 300, 70000])),
                              max_dur=int(rng.choice([1, 9, 70000])), frac_arbitrary=0.3, frac_bad=0.3, dup_prob=0.1)
        path = os.path.join(tmp, "random%d.bin" % i)
        dump(path, w, 12, int(rng.choice([1, 12, 5000])), False)
        files.append(path)
    # malformed descriptions: a cycle, an index out of range, a negative duration, a comm entry below -1
    w = W.random_instance(rng, 40, 3, 4)
    for j, breaker in enumerate(("cycle", "index", "dur", "comm")):
        w2 = W.Workload(w.name, 3, w.row_ptr.copy(), w.col_idx.copy(), w.dur.copy(), np.asarray(w.comm).copy(), w.mem_delta, w.placement, w.rank)
        if breaker == "cycle":
            src, dst = W.edges_from_csr(w.row_ptr, w.col_idx)
            rp, ci = W.csr_from_edges(40, list(src) + [int(dst[0])], list(dst) + [int(src[0])])
            w2 = W.Workload(w.name, 3, rp, ci, w.dur, w.comm, w.mem_delta, w.placement, w.rank)
        elif breaker == "index":
            w2.col_idx[0] = 40
        elif breaker == "dur":
            w2.dur[3] = -1
        else:
            w2.comm[0, 1] = -2
        path = os.path.join(tmp, "bad%d.bin" % j)
        try:
            dump(path, w2, 4, 4, False)
        except Exception:                                     # (the generator of channel orders may refuse a broken graph)
            continue
        files.append(path)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    rc = subprocess.call([exe, *files], env=env)
    print("sanitized run: exit status %d" % rc)
    shutil.rmtree(tmp, ignore_errors=True)
    return rc


if __name__ == "__main__":
    sys.exit(main())
