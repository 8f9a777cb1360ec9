"""Pins for the CPU oracle's list-scheduling simulator (Sec. 3.4; no GPU)."""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def batch_of(n, edges, labels=None):
    """One graph with the given edge list, contracted by `labels` (identity if None)."""
    src = np.array([e[0] for e in edges], np.int64)
    dst = np.array([e[1] for e in edges], np.int64)
    order = np.lexsort((dst, src))
    src, dst = src[order], dst[order]
    rp = np.zeros(n + 1, np.int32)
    np.add.at(rp, src + 1, 1)
    rp = np.cumsum(rp).astype(np.int32)
    g = wl.BaseGraph(n, n, rp, dst.astype(np.int32), np.zeros((n, 16), np.float32))
    lab = np.arange(n, dtype=np.int32) if labels is None else np.asarray(labels, np.int32)
    w = wl.custom("sim", wl.ModelSpec(16, 32, 1, "f32"), [g], [lab.reshape(1, n)], seed=0)
    return orc.contract(w)


def two_phase(b, c, t, x, C, D):
    """A second formulation: first the processing order by Kahn's algorithm with the queue
    discipline (tensors that are produced go on the channel before the next op is taken), then
    one pass over that order computing done = max(resource free, predecessors done) + duration."""
    n0, n1 = int(b.node_off[c]), int(b.node_off[c + 1])
    G = n1 - n0
    succ = [list(b.out_col[b.out_rowptr[n0 + v]:b.out_rowptr[n0 + v + 1]] - n0) for v in range(G)]
    pred = [list(b.in_col[b.in_rowptr[n0 + v]:b.in_rowptr[n0 + v + 1]] - n0) for v in range(G)]
    is_ar = [x[n0 + v] >= 0 for v in range(G)]
    left = [len(p) for p in pred]
    ops = [v for v in range(G) if left[v] == 0 and not is_ar[v]]
    ars = [v for v in range(G) if left[v] == 0 and is_ar[v]]
    order = []
    while ops or ars:
        u = ars.pop(0) if ars else ops.pop(0)
        order.append(u)
        for w_ in succ[u]:
            left[w_] -= 1
            if left[w_] == 0:
                (ars if is_ar[w_] else ops).append(w_)
    if len(order) < G:
        return float("inf")
    done = {}
    free = {False: 0.0, True: 0.0}
    for u in order:
        dur = float(np.float32(C)) * float(x[n0 + u]) + float(np.float32(D)) if is_ar[u] else float(t[n0 + u])
        start = max([free[is_ar[u]]] + [done[p] for p in pred[u]])
        done[u] = start + dur
        free[is_ar[u]] = done[u]
    return float(np.float32(max(free.values())))


def test_chain_is_the_sum_of_times():
    n = 9
    b = batch_of(n, [(i, i + 1) for i in range(n - 1)])
    t = np.arange(1, n + 1, dtype=np.float32) * 0.25
    x = -np.ones(n, np.float32)
    assert orc.simulate(b, t, x, 1.0, 1.0)[0] == np.float32(t.sum())


def test_ops_only_cost_the_sum_of_times_whatever_the_graph():
    g = wl.random_dag(3, 40, 0.15, 16)
    w = wl.custom("s", wl.ModelSpec(16, 32, 1, "f32"), [g], [np.arange(g.n, dtype=np.int32).reshape(1, -1)], seed=0)
    b = orc.contract(w)
    t = (np.arange(g.n) % 7 + 1).astype(np.float32)
    got = orc.simulate(b, t, -np.ones(g.n, np.float32), 0.1, 0.2)[0]
    assert got == np.float32(t.sum())


def test_one_all_reduce_behind_a_chain_overlaps_with_the_rest():
    # a>b>c, tensor r produced by b
    b = batch_of(4, [(0, 1), (1, 2), (1, 3)])
    t = np.array([2, 3, 4, 0], np.float32)
    x = np.array([-1, -1, -1, 10], np.float32)
    assert orc.simulate(b, t, x, 0.1, 0.5)[0] == np.float32(max(2 + 3 + 4, 2 + 3 + 0.1 * 10 + 0.5))   # hidden
    assert orc.simulate(b, t, x, 1.0, 0.5)[0] == np.float32(2 + 3 + 1.0 * 10 + 0.5)                    # exposed


def test_two_tensors_queue_on_the_channel():
    # a>b ; r1 produced by a, r2 by b
    b = batch_of(4, [(0, 1), (0, 2), (1, 3)])
    t = np.array([1, 2, 0, 0], np.float32)
    x = np.array([-1, -1, 8, 2], np.float32)
    C, D = 0.5, 0.25
    t1_done = 1 + C * 8 + D            # starts when a is done
    r2_start = max(1 + 2, t1_done)     # produced at 3, channel busy until t1_done
    assert orc.simulate(b, t, x, C, D)[0] == np.float32(r2_start + C * 2 + D)


def test_ring_all_reduce_closed_form():
    # T = 2 (N-1) x / (B N) for a ring of N devices and link bandwidth B (Sec. 3.1)
    N, B = 8, 12.5
    b = batch_of(1, [])
    x = np.array([100.0], np.float32)
    got = orc.simulate(b, np.zeros(1, np.float32), x, 2 * (N - 1) / (B * N), 0.0)[0]
    assert abs(got - 2 * (N - 1) * 100.0 / (B * N)) <= 1e-5 * got


def test_an_op_behind_an_all_reduce_waits_for_it():
    # a > r > u (u applies the reduced gradient), a > c
    b = batch_of(4, [(0, 1), (0, 3), (1, 2)])
    t = np.array([1, 0, 2, 3], np.float32)       # node 1 is the all-reduce
    x = np.array([-1, 6, -1, -1], np.float32)
    # order: a (0..1); r on the channel 1..1+6+1 = 8; queue after a: c (node 3), then u (node 2)
    # released when r is processed: c runs 1..4, u starts at max(4, 8) = 8, done 10
    assert orc.simulate(b, t, x, 1.0, 1.0)[0] == np.float32(10.0)


def test_a_cyclic_module_costs_infinity():
    # 0>1>2>3 with nodes 0 and 2 fused: the quotient has the cycle {0,2} > 1 > {0,2}
    b = batch_of(4, [(0, 1), (1, 2), (2, 3)], labels=[0, 1, 0, 3])
    assert b.ntot == 3
    got = orc.simulate(b, np.ones(3, np.float32), -np.ones(3, np.float32), 1.0, 1.0)[0]
    assert np.isinf(got)


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_against_the_two_phase_formulation(seed):
    g = wl.random_dag(seed, 60, 0.08, 16)
    labs = np.stack([np.arange(g.n), wl.random_labels(seed + 5, g.n, 45)[0], wl.random_labels(seed + 9, g.n, 30)[0]])
    w = wl.custom("s", wl.ModelSpec(16, 32, 1, "f32"), [g], [labs.astype(np.int32)], seed=0)
    b = orc.contract(w)
    rng = wl.Rng(seed, 11)
    t = (rng.uniform(b.ntot) * 3 + 0.1).astype(np.float32)
    x = np.where(rng.uniform(b.ntot) < 0.3, rng.uniform(b.ntot) * 20, -1.0).astype(np.float32)
    got = orc.simulate(b, t, x, 0.37, 0.11)
    for c in range(b.n_cand):
        want = two_phase(b, c, t, x, 0.37, 0.11)
        assert (np.isinf(want) and np.isinf(got[c])) or abs(got[c] - want) <= 1e-6 * max(1.0, abs(want)), (c, got[c], want)


def test_hand_worked_example():
    vals = {}
    for line in open(os.path.join(GOLD, "simulate_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = [float(z) for z in v]
    e = vals["edges"]
    b = batch_of(int(vals["n"][0]), [(int(e[i]), int(e[i + 1])) for i in range(0, len(e), 2)])
    got = orc.simulate(b, np.array(vals["op_time"], np.float32), np.array(vals["ar_size"], np.float32),
                       vals["c"][0], vals["d"][0])[0]
    assert got == np.float32(vals["cost"][0])
