"""Pins for the CPU oracle's contraction (no GPU).

Each test checks the oracle against something other than itself: the base
graph itself, closed forms, the dense quotient computed with numpy matrices,
a hand-worked fixture, or invariants that a dropped term / wrong index /
transposed operand would break.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _one(g, labels, F=None, bf16=False):
    labels = np.asarray(labels, dtype=np.int32).reshape(1, -1) if np.ndim(labels) == 1 else np.asarray(labels, np.int32)
    model = wl.ModelSpec(g.X.shape[1], 8, 1, "f32")
    w = wl.custom("t", model, [g], [labels])
    return orc.contract(w, bf16=bf16), w


def _dense(g):
    A = np.zeros((g.n, g.n), dtype=np.int64)
    for u in range(g.n):
        A[u, g.col[g.rowptr[u]:g.rowptr[u + 1]]] = 1
    return A


def _canonical_P(labels):
    """Membership matrix with groups numbered by ascending smallest member
    (computed independently of the oracle, by sorting the minima)."""
    labels = np.asarray(labels)
    labs = sorted(set(labels.tolist()), key=lambda L: int(np.min(np.nonzero(labels == L)[0])))
    P = np.zeros((len(labels), len(labs)), dtype=np.int64)
    for j, L in enumerate(labs):
        P[labels == L, j] = 1
    return P


def _check_against_dense(g, labels, b, c=0):
    P = _canonical_P(labels)
    G = P.shape[1]
    Q = (P.T @ _dense(g) @ P > 0).astype(np.int64)
    np.fill_diagonal(Q, 0)
    n0, n1 = b.node_off[c], b.node_off[c + 1]
    assert n1 - n0 == G
    assert np.array_equal(b.new_id[c * g.n:(c + 1) * g.n], np.argmax(P, axis=1))
    for r in range(G):
        oc = b.out_col[b.out_rowptr[n0 + r]:b.out_rowptr[n0 + r + 1]] - n0
        ic = b.in_col[b.in_rowptr[n0 + r]:b.in_rowptr[n0 + r + 1]] - n0
        assert np.array_equal(oc, np.nonzero(Q[r])[0]), (r, oc)
        assert np.array_equal(ic, np.nonzero(Q[:, r])[0]), (r, ic)
    assert b.edge_off[c + 1] - b.edge_off[c] == Q.sum()
    Xc = P.T.astype(np.float64) @ g.X.astype(np.float64)
    np.testing.assert_allclose(b.Xc[n0:n1], Xc, rtol=1e-6, atol=0)
    assert np.array_equal(b.cnt[n0:n1], P.sum(axis=0))


def _set_partitions(n):
    """All set partitions of {0..n-1} as restricted-growth strings."""
    def rec(prefix, m):
        if len(prefix) == n:
            yield list(prefix)
            return
        for v in range(m + 1):
            prefix.append(v)
            yield from rec(prefix, max(m, v + 1))
            prefix.pop()
    yield from rec([], 0)


def test_identity_partition_reproduces_base_graph():
    for seed, n in [(1, 16), (2, 60), (3, 200)]:
        g = wl.random_dag(seed, n, 0.1, 5)
        perm = wl.Rng(seed, 9).permutation(n)          # distinct arbitrary labels
        b, _ = _one(g, perm)
        assert b.ntot == n and b.etot == g.e
        assert np.array_equal(b.new_id, np.arange(n))
        assert np.array_equal(b.out_rowptr, g.rowptr)
        assert np.array_equal(b.out_col, g.col)
        At = sp.csr_matrix((np.ones(g.e), g.col, g.rowptr), shape=(n, n)).T.tocsr()
        At.sort_indices()
        assert np.array_equal(b.in_rowptr, At.indptr)
        assert np.array_equal(b.in_col, At.indices)
        assert np.array_equal(b.Xc, g.X)
        assert np.all(b.cnt == 1)


def test_single_group_gives_one_node():
    g = wl.random_dag(4, 40, 0.2, 6)
    b, _ = _one(g, np.full(g.n, 17))
    assert b.ntot == 1 and b.etot == 0
    assert np.array_equal(b.out_rowptr, [0, 0]) and np.array_equal(b.in_rowptr, [0, 0])
    np.testing.assert_allclose(b.Xc[0], g.X.astype(np.float64).sum(axis=0), rtol=1e-6)
    assert b.cnt[0] == g.n


def test_all_partitions_of_tiny_graphs_match_dense_quotient():
    for seed in (11, 12):
        g = wl.random_dag(seed, 6, 0.45, 3)
        parts = list(_set_partitions(6))
        assert len(parts) == 203                         # Bell(6)
        # labels need not be canonical: map block k to label (5 - k)
        labs = np.array([[5 - k for k in p] for p in parts], dtype=np.int32)
        b, _ = _one(g, labs)
        for c, p in enumerate(labs):
            _check_against_dense(g, p, b, c)


def test_random_labelings_match_dense_quotient():
    for seed, n, k in [(21, 16, 5), (22, 16, 11), (23, 12, 3), (24, 30, 9)]:
        g = wl.random_dag(seed, n, 0.25, 4)
        labs = wl.random_labels(seed, n, k, C=8)
        b, _ = _one(g, labs)
        for c in range(8):
            _check_against_dense(g, labs[c], b, c)


def test_hand_worked_example():
    f = {}
    for line in open(os.path.join(GOLD, "contract_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        f[k] = np.array([float(x) for x in v])
    n = int(f["n"][0])
    g = wl.BaseGraph(n, n, f["rowptr"].astype(np.int32), f["col"].astype(np.int32),
                     f["X"].reshape(n, 2).astype(np.float32))
    b, _ = _one(g, f["labels"].astype(np.int32))
    assert b.ntot == int(f["G"][0])
    assert np.array_equal(b.new_id, f["new_id"].astype(np.int32))
    assert np.array_equal(b.out_rowptr, f["out_rowptr"].astype(np.int32))
    assert np.array_equal(b.out_col, f["out_col"].astype(np.int32))
    assert np.array_equal(b.in_rowptr, f["in_rowptr"].astype(np.int32))
    assert np.array_equal(b.in_col, f["in_col"].astype(np.int32))
    assert np.array_equal(b.Xc.reshape(-1), f["Xc"].astype(np.float32))
    assert np.array_equal(b.cnt, f["cnt"].astype(np.int32))


def test_feature_sums_are_conserved_and_exact_for_integers():
    g = wl.random_dag(31, 120, 0.05, 7, integer_features=True)
    labs = wl.random_labels(31, g.n, 25, C=4)
    b, _ = _one(g, labs)
    for c in range(4):
        n0, n1 = b.node_off[c], b.node_off[c + 1]
        assert np.array_equal(b.Xc[n0:n1].sum(axis=0), g.X.sum(axis=0))      # small integers: exact
    g2 = wl.random_dag(32, 120, 0.05, 7)
    b2, _ = _one(g2, labs)
    for c in range(4):
        n0, n1 = b2.node_off[c], b2.node_off[c + 1]
        np.testing.assert_allclose(b2.Xc[n0:n1].astype(np.float64).sum(axis=0),
                                   g2.X.astype(np.float64).sum(axis=0), rtol=1e-6)


def test_label_bijection_leaves_output_unchanged():
    g = wl.random_dag(41, 50, 0.1, 3)
    lab = wl.random_labels(41, g.n, 12)[0]
    perm = wl.Rng(41, 5).permutation(g.n).astype(np.int32)
    b1, _ = _one(g, lab)
    b2, _ = _one(g, perm[lab])
    for k in ("node_off", "edge_off", "new_id", "out_rowptr", "out_col", "in_rowptr", "in_col", "Xc"):
        assert np.array_equal(getattr(b1, k), getattr(b2, k)), k


def test_in_and_out_lists_hold_the_same_edges_and_never_grow():
    w = wl.make("cfg2", 6)
    b = orc.contract(w)
    g = w.graphs[0]
    for c in range(w.n_cand):
        n0, n1 = b.node_off[c], b.node_off[c + 1]
        e0, e1 = b.edge_off[c], b.edge_off[c + 1]
        assert e1 - e0 <= g.e and n1 - n0 <= g.n
        src = np.repeat(np.arange(n0, n1), np.diff(b.out_rowptr[n0:n1 + 1]))
        fwd = set(zip(src.tolist(), b.out_col[e0:e1].tolist()))
        dst = np.repeat(np.arange(n0, n1), np.diff(b.in_rowptr[n0:n1 + 1]))
        bwd = set(zip(b.in_col[e0:e1].tolist(), dst.tolist()))
        assert fwd == bwd and len(fwd) == e1 - e0
        assert all(n0 <= t < n1 for _, t in fwd)
        # interval partitions of a topological order keep the quotient acyclic: all edges go up
        assert all(s < t for s, t in fwd)


def test_batch_layout_is_the_concatenation_of_single_runs():
    w = wl.make("cfg5", 6, n_graphs=3, n_lo=30, n_hi=80)
    b = orc.contract(w, bf16=False)
    assert b.node_off[0] == 0 and b.edge_off[0] == 0
    for c in range(w.n_cand):
        s = orc.contract(w.subset([c]), bf16=False)
        n0, e0 = b.node_off[c], b.edge_off[c]
        assert b.node_off[c + 1] - n0 == s.ntot and b.edge_off[c + 1] - e0 == s.etot
        assert np.array_equal(b.out_rowptr[n0:n0 + s.ntot + 1] - e0, s.out_rowptr)
        assert np.array_equal(b.in_rowptr[n0:n0 + s.ntot + 1] - e0, s.in_rowptr)
        assert np.array_equal(b.out_col[e0:e0 + s.etot] - n0, s.out_col)
        assert np.array_equal(b.in_col[e0:e0 + s.etot] - n0, s.in_col)
        assert np.array_equal(b.Xc[n0:n0 + s.ntot], s.Xc)
        assert np.array_equal(b.new_id[w.cand_off[c]:w.cand_off[c + 1]], s.new_id)


def test_out_of_range_label_is_an_error():
    g = wl.random_dag(51, 10, 0.3, 2)
    lab = np.arange(10, dtype=np.int32)
    lab[3] = 10
    with pytest.raises(ValueError):
        _one(g, lab)
    lab[3] = -1
    with pytest.raises(ValueError):
        _one(g, lab)


def test_bf16_rounding_matches_the_library_conversion():
    torch = pytest.importorskip("torch")
    rng = wl.Rng(61, 0)
    x = (rng.normal(20000) * np.exp(rng.uniform(20000) * 40 - 20)).astype(np.float32)
    ties = np.array([1.00390625, 1.01171875, -1.00390625, 3.0, 0.0, 65280.0 * 2 ** 100], dtype=np.float32)
    x = np.concatenate([x, ties])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(orc.round_bf16(x), want)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to the even mantissa (1.0)
    assert orc.round_bf16(np.array([1.00390625], np.float32))[0] == 1.0
    assert orc.round_bf16(np.array([1.01171875], np.float32))[0] == 1.015625


def test_bf16_mode_rounds_the_contracted_features_once():
    g = wl.random_dag(71, 40, 0.1, 4)
    lab = wl.random_labels(71, g.n, 9)
    b32, _ = _one(g, lab, bf16=False)
    b16, _ = _one(g, lab, bf16=True)
    assert np.array_equal(b16.Xc, orc.round_bf16(b32.Xc))
    assert np.array_equal(b16.out_col, b32.out_col)
