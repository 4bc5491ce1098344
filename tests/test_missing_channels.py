"""Pins for missing communication channels (eqs. (9)-(10) of Sec. III): a machine pair outside the channel set C
carries the comm entry -1, and a candidate that needs a message over it is infeasible (flag NO_CHANNEL).

The oracle walks the edges; the checks here take the equations as printed instead: with one-hot allocations X
(eq. (6)), sum over the edges of x_{i1,j1} * x_{i2,j2} is the matrix X[src]^T X[dst], and eq. (10) wants it to be
zero on every pair outside C."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2503_09357_amd import workloads as W


def _edges(w):
    src = np.repeat(np.arange(w.n_nodes), np.diff(w.row_ptr))
    return src, np.asarray(w.col_idx)


def _uses_missing_pair(w, comm, pl):
    """eqs. (9)-(10) as a matrix product; only called for placements inside [0, P)."""
    P = w.n_devices
    X = np.zeros((w.n_nodes, P), dtype=np.int64)
    X[np.arange(w.n_nodes), pl] = 1
    src, dst = _edges(w)
    z = X[src].T @ X[dst]                                  # z[j1, j2] = number of messages from j1 to j2
    outside = (np.asarray(comm) == oracle.NO_CHANNEL) & ~np.eye(P, dtype=bool)
    return bool((z[outside] > 0).any())


def _with_comm(w, comm):
    return dataclasses.replace(w, comm=np.ascontiguousarray(comm, dtype=np.int32))


def test_flag_is_the_product_form_of_eqs_9_and_10_and_unused_pairs_change_nothing():
    rng = np.random.Generator(np.random.PCG64(910))
    seen = {0: 0, 1: 0, 2: 0, 4: 0, 32: 0}
    for trial in range(30):
        p = int(rng.integers(2, 7))
        w = W.random_instance(rng, int(rng.integers(6, 40)), p, 40)
        missing = (rng.random((p, p)) < rng.choice([0.1, 0.3, 0.6])) & ~np.eye(p, dtype=bool)
        comm = np.where(missing, oracle.NO_CHANNEL, w.comm)
        if trial % 2:
            np.fill_diagonal(comm, oracle.NO_CHANNEL)                         # a machine needs no channel to itself
        z0, b0, k0, f0 = oracle.evaluate_workload(w)                         # every pair connected
        z1, b1, k1, f1 = oracle.evaluate_workload(_with_comm(w, comm))
        # the delay written on a pair that no message uses is never read: two other fillers give the same
        z2, b2, k2, f2 = oracle.evaluate_workload(_with_comm(w, np.where(missing, 0, w.comm)))
        z3, b3, k3, f3 = oracle.evaluate_workload(_with_comm(w, np.where(missing, 77, w.comm)))
        for c in range(w.n_cand):
            if f0[c] in (oracle.FLAG_BAD_PLACEMENT, oracle.FLAG_BAD_RANK):
                assert f1[c] == f0[c]                                         # malformed stays malformed
            elif _uses_missing_pair(w, comm, w.placement[c]):
                assert f1[c] == oracle.FLAG_NO_CHANNEL
                assert z1[c] == -1 and b1[c] == -1 and (k1[c] == -1).all()
            else:
                for a, b in ((z0, z1), (b0, b1), (k0, k1), (f0, f1), (z2, z1), (z3, z1), (f2, f1), (f3, f1)):
                    assert (a[c] == b[c]).all()
            seen[int(f1[c])] = seen.get(int(f1[c]), 0) + 1
    assert min(seen[k] for k in (0, 1, 32)) > 20 and seen[2] > 0 and seen[4] > 0, seen


def test_pipeline_on_a_chain_shaped_cluster():
    """A pipeline with stage s on machine s sends activations s -> s+1 and gradients s+1 -> s, nothing else."""
    p, m = 4, 6
    w = W.uniform_pipeline(p, m, 2, 3, 1, "1f1b")
    full = oracle.evaluate_workload(w)
    assert full[3][0] == 0
    idx = np.arange(p)
    both = np.full((p, p), oracle.NO_CHANNEL)
    both[idx[:-1], idx[1:]] = 1
    both[idx[1:], idx[:-1]] = 1
    got = oracle.evaluate_workload(_with_comm(w, both))
    assert all((a == b).all() for a, b in zip(full, got))
    forward_only = both.copy()
    forward_only[idx[1:], idx[:-1]] = oracle.NO_CHANNEL                      # gradients cannot travel
    assert oracle.evaluate_workload(_with_comm(w, forward_only))[3][0] == oracle.FLAG_NO_CHANNEL
    for a in range(p - 1):                                                   # each single link is needed
        one = both.copy(); one[a, a + 1] = oracle.NO_CHANNEL
        assert oracle.evaluate_workload(_with_comm(w, one))[3][0] == oracle.FLAG_NO_CHANNEL
        one = both.copy(); one[a + 1, a] = oracle.NO_CHANNEL
        assert oracle.evaluate_workload(_with_comm(w, one))[3][0] == oracle.FLAG_NO_CHANNEL
    # the direction matters: a link 2 -> 0 does not help a message 0 -> 2
    rp, ci = W.csr_from_edges(2, [0], [1])
    comm = np.array([[0, 0, -1], [0, 0, 0], [5, 0, 0]])
    prob = oracle.Problem(3, rp, ci, [1, 1], comm, [0, 0])
    fl = prob.evaluate(np.array([[0, 2], [2, 0], [0, 1]]), np.zeros((3, 2), np.int32))
    assert fl[3].tolist() == [oracle.FLAG_NO_CHANNEL, 0, 0] and fl[0].tolist() == [-1, 7, 2]
    # no messages at all on one machine: a cluster without any channel is fine
    none = np.full((p, p), oracle.NO_CHANNEL)
    order = np.argsort(full[0][0] * 0 + oracle.Problem.of(w).schedule(w.placement[0], w.rank[0])[1], kind="stable")
    rk = np.empty(w.n_nodes, np.int32); rk[order] = np.arange(w.n_nodes)
    z, b, k, f = oracle.Problem.of(_with_comm(w, none)).evaluate(np.zeros((1, w.n_nodes), np.int32), rk[None])
    assert f[0] == 0 and z[0] == w.dur.sum() and b[0] == (p - 1) * w.dur.sum()


def test_flag_precedence_with_missing_channels():
    w = W.uniform_pipeline(3, 4, 2, 3, 1, "1f1b")
    comm = w.comm.copy(); comm[0, 1] = oracle.NO_CHANNEL
    w1 = dataclasses.replace(_with_comm(w, comm), mem_limit=np.zeros(3, np.int64))
    prob = oracle.Problem.of(w1)
    pl0, rk0 = w.placement[0], w.rank[0]
    ids = w.meta["ids"]

    def flag(pl, rk):
        return int(prob.evaluate(pl[None], rk[None])[3][0])

    assert flag(pl0, rk0) == oracle.FLAG_NO_CHANNEL                           # before OVER_MEMORY (limit 0 everywhere)
    rk = rk0.copy(); f_, b_ = ids[("F", 1, 1)], ids[("B", 1, 1)]
    rk[f_], rk[b_] = rk[b_], rk[f_]
    assert flag(pl0, rk) == oracle.FLAG_NO_CHANNEL                            # before CYCLIC
    rk = rk0.copy(); rk[3] = -1
    assert flag(pl0, rk) == oracle.FLAG_BAD_RANK                              # after BAD_RANK
    pl = pl0.copy(); pl[3] = 3
    assert flag(pl, rk0) == oracle.FLAG_BAD_PLACEMENT                         # after BAD_PLACEMENT
    # with the link back, the same limits give OVER_MEMORY
    assert int(oracle.Problem.of(dataclasses.replace(w, mem_limit=np.zeros(3, np.int64))).evaluate(
        pl0[None], rk0[None])[3][0]) == oracle.FLAG_OVER_MEMORY


def test_problem_checks_with_missing_channels():
    rp, ci = W.csr_from_edges(3, [0, 1], [1, 2])
    big = 2 ** 31 - 1

    def code(dur, comm):
        return oracle.Problem(2, rp, ci, dur, comm, [0, 0, 0]).check()

    assert code([1, 2, 3], [[0, -1], [1, 0]]) == oracle.OK
    assert code([1, 2, 3], [[0, -1], [-1, 0]]) == oracle.OK
    assert code([1, 2, 3], [[0, -2], [1, 0]]) == oracle.EINVAL
    assert code([big, 0, 0], [[0, -1], [-1, 0]]) == oracle.OK                 # -1 is not a delay: no part of the bound
    assert code([big - 1, 0, 0], [[0, -1], [1, 0]]) == oracle.EOVERFLOW
