"""Pins for the CPU oracle's forward pass (no GPU).

The oracle is compared with a dense-adjacency float64 evaluation written with
numpy matrices, with closed forms for special weights, with a hand-worked
fixture, and with invariants (node relabelling, partition invariance of the
sum readout).
"""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _dense_forward(A, X, model, wt):
    """Dense float64 evaluation: H' = ReLU(H Ws + Din^-1 A^T H Win + Dout^-1 A H Wout + b),
    r = 1^T H_L, then the three-layer head."""
    A = A.astype(np.float64)
    h = X.astype(np.float64)
    din = A.sum(axis=0)
    dout = A.sum(axis=1)
    inv_in = np.where(din > 0, 1.0 / np.maximum(din, 1), 0.0)
    inv_out = np.where(dout > 0, 1.0 / np.maximum(dout, 1), 0.0)
    off = 0
    d = model.F
    Hh = model.H
    for l in range(model.L):
        W = wt.layers[off:off + 3 * d * Hh].astype(np.float64).reshape(3 * d, Hh)
        off += 3 * d * Hh
        b = wt.biases[l * Hh:(l + 1) * Hh].astype(np.float64)
        hin = inv_in[:, None] * (A.T @ h)
        hout = inv_out[:, None] * (A @ h)
        h = np.maximum(h @ W[:d] + hin @ W[d:2 * d] + hout @ W[2 * d:] + b, 0.0)
        d = Hh
    r = h.sum(axis=0)
    hd = wt.head.astype(np.float64)
    W1 = hd[:Hh * Hh].reshape(Hh, Hh)
    b1 = hd[Hh * Hh:Hh * Hh + Hh]
    o = Hh * Hh + Hh
    W2 = hd[o:o + Hh * Hh].reshape(Hh, Hh)
    b2 = hd[o + Hh * Hh:o + Hh * Hh + Hh]
    o = o + Hh * Hh + Hh
    w3 = hd[o:o + Hh]
    b3 = hd[o + Hh]
    z1 = np.maximum(r @ W1 + b1, 0.0)
    z2 = np.maximum(z1 @ W2 + b2, 0.0)
    return float(z2 @ w3 + b3), h, r


def _dense_adj(b, c=0):
    n0, n1 = b.node_off[c], b.node_off[c + 1]
    G = n1 - n0
    A = np.zeros((G, G))
    for r in range(G):
        A[r, b.out_col[b.out_rowptr[n0 + r]:b.out_rowptr[n0 + r + 1]] - n0] = 1
    return A


def test_dense_adjacency_brute_force_on_small_graphs():
    for seed, n, k, F, H, L in [(1, 16, 16, 5, 7, 2), (2, 16, 6, 4, 8, 3), (3, 9, 4, 3, 5, 1), (4, 14, 9, 6, 6, 4)]:
        g = wl.random_dag(seed, n, 0.3, F)
        model = wl.ModelSpec(F, H, L, "f32")
        labs = wl.random_labels(seed, n, k, C=5)
        w = wl.custom("t", model, [g], [labs], seed=seed, std=0.4)
        b = orc.contract(w)
        pred, h_last, ro = orc.gnn_forward(b, model, w.weights, want_hidden=True)
        for c in range(5):
            n0, n1 = b.node_off[c], b.node_off[c + 1]
            t, h, r = _dense_forward(_dense_adj(b, c), b.Xc[n0:n1], model, w.weights)
            np.testing.assert_allclose(h_last[n0:n1], h, rtol=2e-6, atol=1e-6)
            np.testing.assert_allclose(ro[c], r, rtol=2e-6, atol=1e-6)
            assert abs(pred[c] - t) <= 5e-6 * max(abs(t), 1.0), (seed, c, pred[c], t)


def test_hand_worked_example():
    f = {}
    for line in open(os.path.join(GOLD, "gnn_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        f[k] = np.array([float(x) for x in v], dtype=np.float32)
    g = wl.BaseGraph(2, 2, np.array([0, 1, 1], np.int32), np.array([1], np.int32), f["x"].reshape(2, 1))
    model = wl.ModelSpec(1, 1, 1, "f32")
    w = wl.custom("t", model, [g], [np.array([[0, 1]], np.int32)], wl.Weights(f["layers"], f["biases"], f["head"]))
    assert orc.evaluate(w)[0] == f["pred"][0]


def test_mean_not_sum_over_neighbours():
    # star: nodes 0,1,2 feed node 3; Win = 1 elsewhere 0 => h(3) = mean(1,2,6) = 3, others 0
    g = wl.BaseGraph(4, 4, np.array([0, 1, 2, 3, 3], np.int32), np.array([3, 3, 3], np.int32),
                     np.array([[1], [2], [6], [100]], np.float32))
    model = wl.ModelSpec(1, 1, 1, "f32")
    head = np.array([1, 0, 1, 0, 1, 0], np.float32)
    w = wl.custom("t", model, [g], [np.arange(4, dtype=np.int32)[None]],
                  wl.Weights(np.array([0, 1, 0], np.float32), np.zeros(1, np.float32), head))
    assert orc.evaluate(w)[0] == 3.0
    # Wout = 1: nodes 0,1,2 each see successor 3 (mean 100), node 3 has none => 300
    w.weights = wl.Weights(np.array([0, 0, 1], np.float32), np.zeros(1, np.float32), head)
    assert orc.evaluate(w)[0] == 300.0


def test_zero_weights_give_the_bias_only_output():
    g = wl.random_dag(5, 30, 0.2, 6)
    model = wl.ModelSpec(6, 8, 3, "f32")
    labs = wl.random_labels(5, g.n, 11, C=3)
    wt = wl.make_weights(model, 3, 0.5)
    wt.layers[:] = 0.0
    w = wl.custom("t", model, [g], [labs], wt)
    b = orc.contract(w)
    pred, h_last, ro = orc.gnn_forward(b, model, wt, want_hidden=True)
    H = model.H
    bl = np.maximum(wt.biases[(model.L - 1) * H:].astype(np.float64), 0)
    hd = wt.head.astype(np.float64)
    for c in range(3):
        G = b.node_off[c + 1] - b.node_off[c]
        r = G * bl
        np.testing.assert_allclose(ro[c], r, rtol=1e-6)
        z1 = np.maximum(r @ hd[:H * H].reshape(H, H) + hd[H * H:H * H + H], 0)
        o = H * H + H
        z2 = np.maximum(z1 @ hd[o:o + H * H].reshape(H, H) + hd[o + H * H:o + H * H + H], 0)
        t = z2 @ hd[o + H * H + H:o + H * H + 2 * H] + hd[-1]
        assert abs(pred[c] - t) <= 2e-6 * max(1.0, abs(t))


def test_identity_self_weights_make_readout_partition_invariant():
    F = H = 6
    g = wl.random_dag(6, 40, 0.15, F)
    model = wl.ModelSpec(F, H, 3, "f32")
    wt = wl.make_weights(model, 1, 0.3)
    wt.layers[:] = 0.0
    wt.biases[:] = 0.0
    for l in range(model.L):
        W = wt.layers[l * 3 * H * H:(l + 1) * 3 * H * H].reshape(3 * H, H)
        W[:H] = np.eye(H)
    labs = np.stack([wl.random_labels(6, g.n, 7)[0], wl.random_labels(7, g.n, 23)[0], np.arange(g.n, dtype=np.int32)])
    w = wl.custom("t", model, [g], [labs], wt)
    b = orc.contract(w)
    pred, h_last, ro = orc.gnn_forward(b, model, wt, want_hidden=True)
    np.testing.assert_allclose(h_last, b.Xc, rtol=0, atol=0)          # non-negative features pass ReLU unchanged
    colsum = g.X.astype(np.float64).sum(axis=0)
    for c in range(3):
        np.testing.assert_allclose(ro[c], colsum, rtol=1e-6)
    assert abs(pred[0] - pred[1]) <= 1e-5 * abs(pred[0]) and abs(pred[0] - pred[2]) <= 1e-5 * abs(pred[0])


def test_edgeless_graph_is_a_per_node_mlp():
    n, F, H = 12, 4, 5
    rng = wl.Rng(8, 0)
    g = wl.BaseGraph(n, n, np.zeros(n + 1, np.int32), np.zeros(0, np.int32), rng.uniform(n * F).reshape(n, F).astype(np.float32))
    model = wl.ModelSpec(F, H, 2, "f32")
    w = wl.custom("t", model, [g], [np.arange(n, dtype=np.int32)[None]], seed=2, std=0.5)
    b = orc.contract(w)
    _, h_last, _ = orc.gnn_forward(b, model, w.weights, want_hidden=True)
    W0 = w.weights.layers[:3 * F * H].astype(np.float64).reshape(3 * F, H)[:F]
    W1 = w.weights.layers[3 * F * H:].astype(np.float64).reshape(3 * H, H)[:H]
    b0, b1 = w.weights.biases[:H].astype(np.float64), w.weights.biases[H:].astype(np.float64)
    want = np.maximum(np.maximum(g.X.astype(np.float64) @ W0 + b0, 0) @ W1 + b1, 0)
    np.testing.assert_allclose(h_last, want, rtol=2e-6, atol=1e-6)


def test_node_relabelling_leaves_the_prediction_unchanged():
    w = wl.make("cfg1")
    g = w.graphs[0]
    base = orc.evaluate(w)[0]
    for s in range(3):
        perm = wl.Rng(90 + s, 0).permutation(g.n)       # new index of old node v is perm[v]
        inv = np.argsort(perm)
        src = np.repeat(np.arange(g.n), np.diff(g.rowptr))
        rowptr, col = wl._csr_from_edges(g.n, perm[src], perm[g.col])
        g2 = wl.BaseGraph(g.n, g.n, rowptr, col, g.X[inv])
        w2 = wl.custom("p", w.model, [g2], [w.group_id[inv][None]], w.weights)
        t = orc.evaluate(w2)[0]
        assert abs(t - base) <= 1e-6 * abs(base), (t, base)


def test_bf16_mode_is_exact_on_representable_data_and_close_otherwise():
    # small integers and dyadic weights: nothing is rounded, so both modes agree bit for bit
    n, F, H = 10, 4, 4
    g = wl.random_dag(9, n, 0.3, F, integer_features=True)
    model = wl.ModelSpec(F, H, 1, "bf16")
    wt = wl.make_weights(model, 4, 1.0)
    for a in (wt.layers, wt.biases, wt.head):
        a[:] = np.round(a * 2) / 2          # multiples of 0.5
    # degrees 1,2,4 keep means dyadic: use a chain graph instead of the random one
    rp = np.minimum(np.arange(n + 1), n - 1).astype(np.int32)
    g = wl.BaseGraph(n, n, rp, np.arange(1, n, dtype=np.int32), g.X)
    w = wl.custom("t", model, [g], [np.arange(n, dtype=np.int32)[None]], wt)
    assert orc.evaluate(w, bf16=True)[0] == orc.evaluate(w, bf16=False)[0]
    # random data: bf16 storage stays within a few 2^-9 relative steps of fp32 storage
    w3 = wl.make("cfg3", 4)
    a, b = orc.evaluate(w3, bf16=True), orc.evaluate(w3, bf16=False)
    assert np.all(np.abs(a - b) <= 2e-2 * np.maximum(np.abs(b), 1e-3 * np.median(np.abs(b))))
    assert not np.array_equal(a, b)


def test_oracle_is_deterministic():
    w = wl.make("cfg2", 3)
    assert np.array_equal(orc.evaluate(w), orc.evaluate(w))
