"""Pins for the CPU oracle's backtracking search (Alg. 1; no GPU)."""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from oracle import search as osr
from paper_2209_12769_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def cost_fn_of(g, model, weights, t, x, c, d):
    def f(labels):
        labels = np.asarray(labels, np.int32)
        w = wl.custom("s", model, [g], [labels], weights=weights)
        return orc.cost(w, t, x, c, d)
    return f


def chain_case(m, est):
    X = np.zeros((m, 16), np.float32)
    X[:, 2] = 1.0 + np.arange(m) / 4.0
    rp, ci = wl._csr_from_edges(m, np.arange(m - 1), np.arange(1, m))
    g = wl.BaseGraph(m, m, rp, ci, X)
    model = wl.ModelSpec(16, 32, 1, "f32")
    wt = wl.make_weights(model, 0)
    wt = wl.Weights(np.zeros_like(wt.layers), np.zeros_like(wt.biases),
                    np.concatenate([np.zeros(wt.head.size - 1, np.float32), [np.float32(est)]]))
    return g, model, wt


def test_generator_is_splitmix64():
    # first output of splitmix64 seeded with 0 (published test vector of the algorithm)
    assert osr.mix(0) == 0xE220A8397B1DCDAF
    assert osr.draw(1, 2, 3, 4) == osr.mix((osr.mix(1 ^ osr.mix((2 << 32) + 3)) + 4 * 0xD1342543DE82EF95) & ((1 << 64) - 1))
    assert osr.draw(1, 2, 3, 4) != osr.draw(1, 2, 4, 4) != osr.draw(1, 3, 3, 4)


def test_random_apply_merges_only_along_its_own_kind():
    w = wl.make("cfg1", 1)
    g = w.graphs[0]
    h = np.arange(g.n, dtype=np.int32)
    assert np.array_equal(osr.random_apply(g, h, 0, 0, 5, 0, 0), h)
    for n in (1, 4, 9):
        a = osr.random_apply(g, h, 0, n, 5, 1, 0)
        assert np.array_equal(a[g.n_op:], h[g.n_op:])                       # tensors untouched
        assert g.n - n <= len(np.unique(a)) <= g.n
        b = osr.random_apply(g, h, 1, n, 5, 1, 1)
        assert np.array_equal(b[:g.n_op], h[:g.n_op])                       # ops untouched
        assert g.n - n <= len(np.unique(b)) <= g.n
        runs = b[g.n_op:]
        # buckets are contiguous in production order
        assert len(np.unique(runs)) == 1 + int(np.sum(runs[1:] != runs[:-1]))
    # an op merge joins the two ends of a dependency
    a = osr.random_apply(g, h, 0, 1, 5, 1, 0)
    merged = [np.nonzero(a == l)[0] for l in np.unique(a) if np.sum(a == l) == 2]
    assert len(merged) == 1
    u, v = merged[0]
    assert v in g.col[g.rowptr[u]:g.rowptr[u + 1]]


def test_beta_zero_never_changes_the_module():
    w = wl.make("cfg1", 1)
    g = w.graphs[0]
    t, x = wl.profile_of(w)
    f = cost_fn_of(g, w.model, w.weights, t, x, 0.02, 0.01)
    r = osr.search(g, f, alpha=1.0, beta=0, seed=3, max_unchanged=11, parents=1)
    assert np.array_equal(r.labels_opt, np.arange(g.n))
    assert r.cost_opt == r.cost_in and r.improved == 0
    assert r.evaluated == 12 and r.valid == 12 and r.enqueued == 12 and r.steps == 6     # 11 rounded up to a whole step


def test_chain_with_a_cheap_estimator_ends_fully_fused():
    g, model, wt = chain_case(6, 0.5)
    t, x = wl.profile_of(wl.custom("c", model, [g], [np.arange(6, dtype=np.int32).reshape(1, 6)], weights=wt))
    f = cost_fn_of(g, model, wt, t, x, 0.0, 0.0)
    r = osr.search(g, f, alpha=1.5, beta=3, seed=1, max_unchanged=200, parents=2)
    assert r.cost_in == np.float32(np.sum(t.astype(np.float64)))
    assert r.cost_opt == 0.5 and len(np.unique(r.labels_opt)) == 1


def test_invariants_of_the_result():
    w = wl.make("cfg1", 1)
    w.weights.head[-1] += 0.2
    g = w.graphs[0]
    t, x = wl.profile_of(w)
    f = cost_fn_of(g, w.model, w.weights, t, x, 0.05, 0.02)
    r = osr.search(g, f, alpha=1.05, beta=4, seed=7, max_unchanged=60, parents=4, keep_trace=True)
    assert r.cost_opt <= r.cost_in and np.isfinite(r.cost_opt)
    assert f(r.labels_opt.reshape(1, -1))[0] == np.float32(r.cost_opt)
    best = [tr[3] for tr in r.trace]
    assert all(b1 <= b0 for b0, b1 in zip(best, best[1:]))
    lab = r.labels_opt
    # every op group is connected through dependencies inside the group; buckets are contiguous
    for l in np.unique(lab[:g.n_op]):
        mem = set(np.nonzero(lab == l)[0].tolist())
        seen, todo = set(), [min(mem)]
        while todo:
            u = todo.pop()
            if u in seen:
                continue
            seen.add(u)
            for v in g.col[g.rowptr[u]:g.rowptr[u + 1]]:
                if v in mem:
                    todo.append(int(v))
            for p in range(g.n):
                if p in mem and u in g.col[g.rowptr[p]:g.rowptr[p + 1]]:
                    todo.append(p)
        assert seen == mem
    runs = lab[g.n_op:]
    assert len(np.unique(runs)) == 1 + int(np.sum(runs[1:] != runs[:-1]))
    assert not (set(lab[:g.n_op].tolist()) & set(runs.tolist()))
    assert r.improved >= 1 and r.valid <= r.evaluated


def test_same_seed_same_search_other_seed_other_search():
    g, model, wt = chain_case(8, 0.75)
    t, x = wl.profile_of(wl.custom("c", model, [g], [np.arange(8, dtype=np.int32).reshape(1, 8)], weights=wt))
    f = cost_fn_of(g, model, wt, t, x, 0.0, 0.0)
    a = osr.search(g, f, 1.2, 2, 11, max_unchanged=30, keep_trace=True)
    b = osr.search(g, f, 1.2, 2, 11, max_unchanged=30, keep_trace=True)
    c = osr.search(g, f, 1.2, 2, 12, max_unchanged=30, keep_trace=True)
    assert a.trace == b.trace and a.trace != c.trace


def test_hand_worked_queue_discipline():
    rec = {}
    with open(os.path.join(GOLD, "search_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            rec[k] = [float(z) for z in v]
    script = [rec["cost_in"][0]] + rec["children"]
    pos = [0]

    def f(labels):
        out = script[pos[0]:pos[0] + len(labels)]
        pos[0] += len(labels)
        return np.array(out, np.float32)

    g, _, _ = chain_case(4, 1.0)
    r = osr.search(g, f, alpha=rec["alpha"][0], beta=2, seed=0, max_unchanged=1000, parents=1, max_steps=3,
                   keep_trace=True)
    assert r.cost_opt == rec["cost_opt"][0] and r.steps == rec["steps"][0]
    assert (r.evaluated, r.valid, r.enqueued, r.improved) == tuple(
        int(rec[k][0]) for k in ("evaluated", "valid", "enqueued", "improved"))
    assert r.trace[-1][4] == rec["final_unchanged"][0] and r.trace[-1][5] == rec["final_queue"][0]


def star_with_tail(k):
    """Ops 0..k-1 all feed op k (a centre with k predecessors), and k feeds k+1: k + 2 computation ops."""
    n = k + 2
    src = np.concatenate([np.arange(k), [k]])
    dst = np.concatenate([np.full(k, k), [k + 1]])
    rp, ci = wl._csr_from_edges(n, src, dst)
    return wl.BaseGraph(n, n, rp, ci, np.zeros((n, 16), np.float32))


def test_the_two_draws_of_op_fusion_have_the_distributions_their_definitions_give():
    # One application on the unfused star: the paper's draw picks one of the k + 2 ops uniformly and then
    # one of its predecessors, so the tail dependency (k -> k+1) is fused with probability 1 / (k + 2),
    # a given leaf with probability 1 / (k + 2) * 1 / k, and nothing happens (a leaf was picked, it has no
    # predecessor) with probability k / (k + 2).  Drawing a dependency of the base module uniformly fuses
    # the tail with probability 1 / (k + 1) and always fuses something.
    k = 4
    g = star_with_tail(k)
    h = np.arange(g.n, dtype=np.int32)
    trials = 6000
    tail = {"op": 0, "dependency": 0}
    nothing = {"op": 0, "dependency": 0}
    leaf0 = {"op": 0, "dependency": 0}
    for mode in ("op", "dependency"):
        for s in range(trials):
            a = osr.random_apply(g, h, 0, 1, 17, s, 0, op_draw=mode)
            tail[mode] += a[k] == a[k + 1]
            leaf0[mode] += a[0] == a[k]
            nothing[mode] += np.array_equal(a, h)
    def close(count, p):
        return abs(count / trials - p) < 4.0 * np.sqrt(p * (1 - p) / trials) + 1e-9
    assert close(tail["op"], 1 / (k + 2)) and close(nothing["op"], k / (k + 2)) and close(leaf0["op"], 1 / (k + 2) / k)
    assert close(tail["dependency"], 1 / (k + 1)) and nothing["dependency"] == 0 and close(leaf0["dependency"], 1 / (k + 1))


def test_the_papers_draw_sees_the_current_module():
    # after the centre has absorbed leaf 0, the centre's group has k - 1 predecessors left, the module has
    # k + 1 ops, and the op that is drawn is a group, whichever of its members one looks at
    k = 3
    g = star_with_tail(k)
    h = np.arange(g.n, dtype=np.int32)
    h[0] = h[k]
    assert osr.current_op_groups(g, h).tolist() == [k, 1, 2, k + 1]          # order of smallest member: {0, k}, 1, 2, k+1
    assert osr.current_predecessors(g, h, k).tolist() == [1, 2]
    assert osr.current_predecessors(g, h, k + 1).tolist() == [k]
    assert osr.current_predecessors(g, h, 1).tolist() == []
    # n applications never touch tensors and only ever merge along dependencies of the current module
    w = wl.make("cfg1", 1)
    gg = w.graphs[0]
    hh = np.arange(gg.n, dtype=np.int32)
    a = osr.random_apply(gg, hh, 0, 12, 3, 0, 0, op_draw="op")
    assert np.array_equal(a[gg.n_op:], hh[gg.n_op:]) and len(np.unique(a)) < gg.n
    src, dst = osr.op_edges(gg)
    for l in np.unique(a[:gg.n_op]):
        mem = np.nonzero(a == l)[0]
        if len(mem) > 1:                                                     # connected through fused dependencies
            inside = (a[src] == l) & (a[dst] == l)
            assert inside.sum() >= len(mem) - 1
    # a whole search runs with it and keeps the invariants of the result
    g2, model, wt = chain_case(8, 0.25)
    t = g2.X[:, 2].copy()
    x = np.full(g2.n, -1.0, np.float32)
    res = osr.search(g2, cost_fn_of(g2, model, wt, t, x, 0.0, 0.0), alpha=1.05, beta=3, seed=2, max_unchanged=60,
                     op_draw="op")
    assert res.cost_opt <= res.cost_in and res.evaluated > 0
