"""Pins for the CPU oracle's forward pass with attention coefficients (no GPU).

The oracle walks neighbour lists; it is compared with a dense masked-softmax float64
evaluation written with numpy matrices, with the closed form for zero attention vectors
(plain mean over the neighbourhood), with a single-node graph, with a hand-worked fixture,
and with invariants (node relabelling; destination vector zero makes the source vector
irrelevant).
"""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _head(r, wt, H):
    hd = wt.head.astype(np.float64)
    W1, b1 = hd[:H * H].reshape(H, H), hd[H * H:H * H + H]
    o = H * H + H
    W2, b2 = hd[o:o + H * H].reshape(H, H), hd[o + H * H:o + H * H + H]
    o += H * H + H
    w3, b3 = hd[o:o + H], hd[o + H]
    z1 = np.maximum(r @ W1 + b1, 0.0)
    z2 = np.maximum(z1 @ W2 + b2, 0.0)
    return float(z2 @ w3 + b3)


def _dense_attention_forward(A, X, model, wt, uniform=False):
    """M = I + A^T + A counts how often j is in the list N_i = (i, predecessors, successors).
    Per head: S_ij = LeakyReLU(s_i + t_j); P = M * exp(S - rowmax); gamma = P / rowsum(P);
    E = ReLU(gamma Z_head + b).  With uniform=True gamma = M / rowsum(M)."""
    A = A.astype(np.float64)
    n = A.shape[0]
    M = np.eye(n) + A.T + A
    h = X.astype(np.float64)
    H, K = model.H, model.heads
    Dh = H // K
    off = 0
    d = model.F
    for l in range(model.L):
        W = wt.layers[off:off + d * H].astype(np.float64).reshape(d, H)
        off += d * H
        a_src = wt.att[2 * H * l:2 * H * l + H].astype(np.float64)
        a_dst = wt.att[2 * H * l + H:2 * H * (l + 1)].astype(np.float64)
        b = wt.biases[l * H:(l + 1) * H].astype(np.float64)
        Z = h @ W
        out = np.zeros((n, H))
        for k in range(K):
            cols = slice(k * Dh, (k + 1) * Dh)
            if uniform:
                G = M / M.sum(axis=1, keepdims=True)
            else:
                s = Z[:, cols] @ a_src[cols]
                t = Z[:, cols] @ a_dst[cols]
                S = s[:, None] + t[None, :]
                S = np.where(S > 0, S, 0.2 * S)
                S = np.where(M > 0, S, -np.inf)
                P = M * np.exp(S - S.max(axis=1, keepdims=True))
                G = P / P.sum(axis=1, keepdims=True)
            out[:, cols] = G @ Z[:, cols]
        h = np.maximum(out + b, 0.0)
        d = H
    return _head(h.sum(axis=0), wt, H), h


def _dense_adj(b, c=0):
    n0, n1 = b.node_off[c], b.node_off[c + 1]
    G = n1 - n0
    A = np.zeros((G, G))
    for r in range(G):
        A[r, b.out_col[b.out_rowptr[n0 + r]:b.out_rowptr[n0 + r + 1]] - n0] = 1
    return A


def _case(seed, n, p, F, H, L, K, groups, C=1, std=None):
    g = wl.random_dag(seed, n, p, F)
    labs = wl.random_labels(seed + 1, g.n, groups, C=C)
    m = wl.ModelSpec(F, H, L, "f32", "attention", K)
    return wl.custom("att", m, [g], [labs], seed=seed, std=std)


@pytest.mark.parametrize("seed,n,p,F,H,L,K,groups", [(1, 14, 0.25, 4, 8, 2, 2, 9), (2, 16, 0.4, 8, 16, 3, 4, 6),
                                                      (3, 12, 0.15, 3, 6, 1, 1, 12), (4, 16, 0.5, 4, 8, 2, 8, 5)])
def test_against_dense_masked_softmax(seed, n, p, F, H, L, K, groups):
    w = _case(seed, n, p, F, H, L, K, groups, C=2, std=0.6)
    b = orc.contract(w)
    pred, h_last, _ = orc.gnn_forward(b, w.model, w.weights, want_hidden=True)
    for c in range(w.n_cand):
        A = _dense_adj(b, c)
        n0, n1 = b.node_off[c], b.node_off[c + 1]
        want, h = _dense_attention_forward(A, b.Xc[n0:n1], w.model, w.weights)
        np.testing.assert_allclose(h_last[n0:n1], h, rtol=2e-6, atol=1e-7)
        assert abs(pred[c] - want) <= 2e-6 * max(1.0, abs(want))


def test_quotients_with_two_cycles_count_a_neighbour_twice():
    # arbitrary partitions make u>v and v>u both edges of the quotient: v is then twice in N_u
    w = _case(7, 16, 0.5, 4, 8, 2, 2, 4, C=3, std=0.6)
    b = orc.contract(w)
    twice = 0
    for c in range(w.n_cand):
        A = _dense_adj(b, c)
        twice += int(((A > 0) & (A.T > 0)).sum())
    assert twice > 0
    pred = orc.gnn_forward(b, w.model, w.weights)
    for c in range(w.n_cand):
        n0, n1 = b.node_off[c], b.node_off[c + 1]
        want, _ = _dense_attention_forward(_dense_adj(b, c), b.Xc[n0:n1], w.model, w.weights)
        assert abs(pred[c] - want) <= 2e-6 * max(1.0, abs(want))


def test_zero_attention_vectors_give_the_plain_mean_over_the_neighbourhood():
    w = _case(5, 15, 0.3, 4, 8, 2, 2, 8, std=0.5)
    w.weights.att[:] = 0.0
    b = orc.contract(w)
    pred, h_last, _ = orc.gnn_forward(b, w.model, w.weights, want_hidden=True)
    want, h = _dense_attention_forward(_dense_adj(b), b.Xc, w.model, w.weights, uniform=True)
    np.testing.assert_allclose(h_last, h, rtol=2e-6, atol=1e-7)
    assert abs(pred[0] - want) <= 2e-6 * max(1.0, abs(want))


def test_zero_destination_vector_makes_the_source_vector_irrelevant():
    # u_ij = LeakyReLU(s_i) does not depend on j: uniform coefficients whatever a_src is
    w = _case(6, 15, 0.3, 4, 8, 2, 4, 8, std=0.5)
    H = w.model.H
    for l in range(w.model.L):
        w.weights.att[2 * H * l + H:2 * H * (l + 1)] = 0.0
    b = orc.contract(w)
    got = orc.gnn_forward(b, w.model, w.weights)
    want, _ = _dense_attention_forward(_dense_adj(b), b.Xc, w.model, w.weights, uniform=True)
    assert abs(got[0] - want) <= 2e-6 * max(1.0, abs(want))


def test_single_node_graph_is_a_plain_network():
    F, H = 5, 8
    g = wl.BaseGraph(1, 1, np.array([0, 0], np.int32), np.zeros(0, np.int32),
                     np.arange(1, F + 1, dtype=np.float32).reshape(1, F) / 4)
    m = wl.ModelSpec(F, H, 2, "f32", "attention", 2)
    w = wl.custom("one", m, [g], [np.zeros((1, 1), np.int32)], seed=11, std=0.4)
    got = orc.evaluate(w)[0]
    h = g.X.astype(np.float64)[0]
    off, d = 0, F
    for l in range(2):
        W = w.weights.layers[off:off + d * H].astype(np.float64).reshape(d, H)
        off += d * H
        h = np.maximum(h @ W + w.weights.biases[l * H:(l + 1) * H], 0.0)      # gamma_ii = 1
        d = H
    want = _head(h, w.weights, H)
    assert abs(got - want) <= 2e-6 * max(1.0, abs(want))


def test_node_relabelling_does_not_change_the_prediction():
    g = wl.random_dag(21, 18, 0.3, 4)
    labs = wl.random_labels(22, g.n, 18, C=1)          # identity-sized partition: every node its own group
    labs[0] = np.arange(g.n)
    m = wl.ModelSpec(4, 8, 2, "f32", "attention", 2)
    w = wl.custom("perm", m, [g], [labs], seed=3, std=0.5)
    base = orc.evaluate(w)[0]
    # reverse the numbering: edges i>j become (n-1-i)>(n-1-j)
    n = g.n
    src = np.repeat(np.arange(n), np.diff(g.rowptr))
    dst = g.col
    order = np.lexsort((n - 1 - dst, n - 1 - src))
    s2, d2 = (n - 1 - src)[order], (n - 1 - dst)[order]
    rp = np.zeros(n + 1, np.int32)
    np.add.at(rp, s2 + 1, 1)
    rp = np.cumsum(rp).astype(np.int32)
    g2 = wl.BaseGraph(n, n, rp, d2.astype(np.int32), g.X[::-1].copy())
    w2 = wl.custom("perm2", m, [g2], [labs], weights=w.weights)
    assert abs(orc.evaluate(w2)[0] - base) <= 2e-6 * max(1.0, abs(base))


def test_hand_worked_example():
    vals = {}
    for line in open(os.path.join(GOLD, "attention_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array([float(x) for x in v], np.float32)
    g = wl.BaseGraph(2, 2, np.array([0, 1, 1], np.int32), np.array([1], np.int32), vals["x"].reshape(2, 1))
    m = wl.ModelSpec(1, 2, 1, "f32", "attention", 2)
    wt = wl.Weights(vals["layers"], vals["biases"], vals["head"], vals["att"])
    w = wl.custom("gold", m, [g], [np.arange(2, dtype=np.int32).reshape(1, 2)], weights=wt)
    got = orc.evaluate(w)[0]
    assert abs(got - float(vals["pred"][0])) <= 1e-6
    # with the edge reversed the lists are (a, b) and (b, a) again (predecessor and successor swap
    # roles but both are neighbours): the same value
    g2 = wl.BaseGraph(2, 2, np.array([0, 0, 1], np.int32), np.array([0], np.int32), vals["x"].reshape(2, 1))
    w2 = wl.custom("gold2", m, [g2], [np.arange(2, dtype=np.int32).reshape(1, 2)], weights=wt)
    assert abs(orc.evaluate(w2)[0] - float(vals["pred"][0])) <= 1e-6


def test_bf16_storage_points():
    # with bf16 storage z, the activations, W and the head matrices are bf16 values
    w = _case(9, 14, 0.3, 8, 16, 2, 2, 9, std=0.5)
    b = orc.contract(w, True)
    _, h_last, _ = orc.gnn_forward(b, w.model, w.weights, bf16=True, want_hidden=True)
    assert np.array_equal(h_last, orc.round_bf16(h_last))
    p32 = orc.gnn_forward(orc.contract(w, False), w.model, w.weights, bf16=False)
    p16 = orc.gnn_forward(b, w.model, w.weights, bf16=True)
    assert abs(p32[0] - p16[0]) <= 5e-2 * max(1.0, abs(p32[0]))
