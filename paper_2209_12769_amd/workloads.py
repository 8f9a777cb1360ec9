"""Seeded synthetic inputs for the fusion-candidate evaluator.

This module only *draws* inputs: base training DAGs (compute ops plus gradient
all-reduce tensor nodes), per-candidate fusion labels (op-fusion groups and
tensor buckets) and model weights.  It holds none of the evaluator's own
arithmetic (no contraction, no message passing): both the CPU oracle's tests
and the GPU tests call it so that they see identical inputs, and neither of
those two sides imports the other.

A candidate is what the strategy search hands to its cost model: the base
module plus an op-fusion strategy and a tensor-fusion strategy (Sec. 3.2 of
the paper).  Here that is a label per base node; nodes with equal labels are
fused.  The paper's real workloads are HLO modules of ResNet50, BERT,
Transformer ... (Sec. 6.1); they are not available, so the generators below
stand in for them, taking their shape: thousands of instructions (Sec. 2.4),
many small gradient tensors (Sec. 2.3).

All randomness comes from one counter-based generator (splitmix64 finaliser
over seed/stream/counter), written out here so the draws do not depend on any
library's distribution code.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function applied element-wise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


class Rng:
    """Counter-based generator: value k of stream (seed, stream) is
    splitmix(splitmix(seed*2^20 + stream) + k)."""

    def __init__(self, seed: int, stream: int = 0):
        key = np.array([(int(seed) << 20) + int(stream)], dtype=np.uint64)
        self._key = _splitmix(key)[0]
        self._ctr = 0

    def u64(self, n: int) -> np.ndarray:
        n = int(n)
        c = np.arange(self._ctr, self._ctr + n, dtype=np.uint64)
        self._ctr += n
        with np.errstate(over="ignore"):
            return _splitmix(c * np.uint64(0xD1342543DE82EF95) + self._key)

    def uniform(self, n: int) -> np.ndarray:
        """float64 in [0, 1) with 53 random bits."""
        return (self.u64(n) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)

    def integers(self, lo: int, hi: int, n: int) -> np.ndarray:
        """int64 uniform on [lo, hi] inclusive."""
        span = int(hi) - int(lo) + 1
        return (np.floor(self.uniform(n) * span).astype(np.int64)) + int(lo)

    def normal(self, n: int) -> np.ndarray:
        """Standard normal by Box-Muller (cosine branch only)."""
        u1 = 1.0 - self.uniform(n)          # (0, 1]
        u2 = self.uniform(n)
        return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)

    def permutation(self, n: int) -> np.ndarray:
        return np.argsort(self.u64(n), kind="stable").astype(np.int64)


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclass
class BaseGraph:
    """One base training DAG in CSR form (row = source op, col = consumer),
    rows sorted, no self loops, no duplicate edges.  Nodes 0..n_op-1 are
    compute ops in a topological order; nodes n_op..n-1 are gradient
    all-reduce tensors in order of production."""
    n: int
    n_op: int
    rowptr: np.ndarray      # int32 [n+1]
    col: np.ndarray         # int32 [E]
    X: np.ndarray           # float32 [n, F]

    @property
    def n_ar(self) -> int:
        return self.n - self.n_op

    @property
    def e(self) -> int:
        return int(self.col.shape[0])


@dataclass
class ModelSpec:
    F: int
    H: int
    L: int
    dtype: str              # "f32" | "bf16"
    agg: str = "mean"       # "mean": in/out mean aggregation; "attention": K-head attention over N_i
    heads: int = 1          # K (attention only); H must be a multiple of K


@dataclass
class Weights:
    """fp32 master weights.  layers = concat over l of W^l row-major [3d, H]
    (row blocks: self, in-mean, out-mean); biases = concat of b^l [H];
    head = W1[H,H] | b1[H] | W2[H,H] | b2[H] | w3[H] | b3[1], W row-major
    [in, out].  With attention aggregation W^l is [d, H] and att = concat over l
    of a_src^l[H] | a_dst^l[H] (head k owns columns k*H/K .. (k+1)*H/K)."""
    layers: np.ndarray
    biases: np.ndarray
    head: np.ndarray
    att: Optional[np.ndarray] = None


@dataclass
class Workload:
    name: str
    model: ModelSpec
    graphs: List[BaseGraph]
    cand_graph: np.ndarray      # int32 [C] index into graphs
    cand_off: np.ndarray        # int64 [C+1] offsets into group_id
    group_id: np.ndarray        # int32 [sum N_b(c)] labels in [0, N_b(c))
    weights: Weights
    note: str = ""

    @property
    def n_cand(self) -> int:
        return int(self.cand_graph.shape[0])

    def g_node_off(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([g.n for g in self.graphs])]).astype(np.int32)

    def g_edge_off(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([g.e for g in self.graphs])]).astype(np.int32)

    def cat_rowptr(self) -> np.ndarray:
        """Concatenation of the per-graph rowptr arrays, each of length n+1 and
        each starting at 0 (graph b's array starts at g_node_off[b] + b)."""
        return np.concatenate([g.rowptr for g in self.graphs]).astype(np.int32)

    def cat_col(self) -> np.ndarray:
        return np.concatenate([g.col for g in self.graphs]).astype(np.int32)

    def cat_X(self) -> np.ndarray:
        return np.ascontiguousarray(np.concatenate([g.X for g in self.graphs], axis=0), dtype=np.float32)

    def subset(self, idx: Sequence[int]) -> "Workload":
        """Workload restricted to the given candidates (same graphs, weights)."""
        idx = np.asarray(idx, dtype=np.int64)
        parts = [self.group_id[self.cand_off[i]:self.cand_off[i + 1]] for i in idx]
        sizes = np.array([p.shape[0] for p in parts], dtype=np.int64)
        return Workload(self.name + f"[{len(idx)}]", self.model, self.graphs,
                        self.cand_graph[idx].copy(),
                        np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64),
                        np.concatenate(parts).astype(np.int32) if len(parts) else np.zeros(0, np.int32),
                        self.weights, self.note)


# --------------------------------------------------------------------------
# graph assembly helpers
# --------------------------------------------------------------------------
def _csr_from_edges(n: int, src: np.ndarray, dst: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Sorted, duplicate-free, loop-free CSR from an edge list."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keep = src != dst
    key = np.unique(src[keep] * n + dst[keep])
    s = key // n
    d = key % n
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, s + 1, 1)
    rowptr = np.cumsum(rowptr)
    return rowptr.astype(np.int32), d.astype(np.int32)


def _features(rng: Rng, n: int, n_op: int, F: int, ar_bytes: Optional[np.ndarray]) -> np.ndarray:
    """Feature rows.  All entries ~U(0,1); when ar_bytes is given, column 0 of
    an all-reduce node is its tensor size in MiB (linear, so that fused sizes
    add up, Sec. 2.3) and column 1 flags the node kind (1 = all-reduce)."""
    X = rng.uniform(n * F).reshape(n, F)
    if ar_bytes is not None:
        X[:n_op, 1] = 0.0
        X[n_op:, 1] = 1.0
        X[n_op:, 0] = ar_bytes / float(1 << 20)
    return X.astype(np.float32)


def _log_uniform(rng: Rng, n: int, lo: float, hi: float) -> np.ndarray:
    return np.exp(math.log(lo) + rng.uniform(n) * (math.log(hi) - math.log(lo)))


class _DagBuilder:
    """Forward ops are appended with explicit predecessor lists; backward()
    then derives the gradient ops and the all-reduce tensors."""

    def __init__(self):
        self.preds: List[List[int]] = []
        self.params: List[int] = []

    def op(self, preds: Sequence[int], params: int = 0) -> int:
        self.preds.append(list(preds))
        self.params.append(params)
        return len(self.preds) - 1

    def chain(self, prev: int, n: int) -> int:
        for _ in range(n):
            prev = self.op([prev])
        return prev

    def training_dag(self) -> Tuple[int, int, np.ndarray, np.ndarray]:
        """Returns (n, n_op, src, dst).  For forward op i (visited last to
        first) a gradient op B_i consumes the gradient ops of i's consumers and
        i's first input activation; an op with parameters also gets a
        weight-gradient op fed by the same upstream gradients and activation,
        and that op produces one all-reduce tensor per parameter tensor."""
        nf = len(self.preds)
        succ: List[List[int]] = [[] for _ in range(nf)]
        src: List[int] = []
        dst: List[int] = []
        for i, ps in enumerate(self.preds):
            for p in ps:
                succ[p].append(i)
                src.append(p)
                dst.append(i)
        nxt = nf
        bid = [-1] * nf
        ar_prod: List[int] = []
        for i in range(nf - 1, -1, -1):
            ups = [bid[j] for j in succ[i]] if succ[i] else [i]
            act = self.preds[i][0] if self.preds[i] else i
            b = nxt
            nxt += 1
            bid[i] = b
            for u in ups:
                src.append(u)
                dst.append(b)
            src.append(act)
            dst.append(b)
            if self.params[i] > 0:
                g = nxt
                nxt += 1
                for u in ups:
                    src.append(u)
                    dst.append(g)
                src.append(act)
                dst.append(g)
                ar_prod.extend([g] * self.params[i])
        n_op = nxt
        for k, g in enumerate(ar_prod):
            src.append(g)
            dst.append(n_op + k)
        return n_op + len(ar_prod), n_op, np.array(src), np.array(dst)


def _resnet50_dag() -> Tuple[int, int, np.ndarray, np.ndarray]:
    b = _DagBuilder()

    def conv_bn(x: int, relu: bool) -> int:
        x = b.op([x], params=1)         # conv weight
        x = b.op([x])                   # batch statistics
        x = b.op([x], params=2)         # scale / shift
        if relu:
            x = b.op([x])
        return x

    x = b.op([])                        # input
    x = conv_bn(x, True)
    x = b.op([x])                       # max-pool
    for stage, blocks in enumerate([3, 4, 6, 3]):
        for k in range(blocks):
            inp = x
            y = conv_bn(inp, True)
            y = conv_bn(y, True)
            y = conv_bn(y, False)       # a residual skip spans every 3 convs
            skip = conv_bn(inp, False) if k == 0 else inp
            x = b.op([y, skip])         # add
            x = b.op([x])               # relu
    x = b.op([x])                       # global pool
    x = b.op([x], params=1)             # fc weight
    x = b.op([x], params=1)             # fc bias
    x = b.op([x])                       # loss
    return b.training_dag()


def _transformer_dag(blocks: int, ew: int, embed_params: int, tail_params: int) -> Tuple[int, int, np.ndarray, np.ndarray]:
    """Post-LN transformer encoder stack.  `ew` elementwise ops (casts,
    broadcasts, reshapes ...) are inserted after each major op so that a block
    has the instruction count of a real HLO module."""
    b = _DagBuilder()

    def dense(x: int) -> int:
        x = b.op([x], params=1)         # matmul weight
        x = b.op([x], params=1)         # bias add
        return b.chain(x, ew)

    def layer_norm(x: int) -> int:
        m = b.op([x])                   # mean
        v = b.op([x, m])                # variance
        y = b.op([x, m, v])             # normalise
        y = b.op([y], params=2)         # scale / shift
        return b.chain(y, ew)

    x = b.op([])
    for _ in range(max(embed_params - 2, 0)):
        x = b.op([x], params=1)         # embedding tables
    if embed_params >= 2:
        x = b.op([x], params=2)         # embedding layer norm
    x = b.chain(x, ew)
    for _ in range(blocks):
        q = dense(x)
        k = dense(x)
        v = dense(x)                    # x feeds q, k, v and the residual: fan-out 4
        s = b.op([q, k])                # scores
        s = b.chain(s, 3 + ew)          # scale, mask, softmax, dropout
        c = b.op([s, v])                # context
        c = b.chain(c, ew)
        o = dense(c)
        o = b.op([o])                   # dropout
        r = b.op([x, o])                # residual add
        z = layer_norm(r)
        f = dense(z)
        f = b.op([f])                   # gelu
        f = dense(f)
        f = b.op([f])                   # dropout
        r = b.op([z, f])
        x = layer_norm(r)
    for _ in range(tail_params):
        x = b.op([x], params=1)         # pooler / classifier
    x = b.op([x])                       # loss
    return b.training_dag()


# --------------------------------------------------------------------------
# partitions
# --------------------------------------------------------------------------
def _run_starts_uniform(rng: Rng, C: int, n: int, kmax: int) -> np.ndarray:
    """bool [C, n]: start flags of consecutive runs with lengths ~U{1..kmax}."""
    lens = rng.integers(1, kmax, C * n).reshape(C, n)
    pos = np.cumsum(lens, axis=1) - lens            # start positions of runs
    flags = np.zeros((C, n), dtype=bool)
    rows = np.repeat(np.arange(C), n).reshape(C, n)
    ok = pos < n
    flags[rows[ok], pos[ok]] = True
    return flags


def _run_starts_geometric(rng: Rng, C: int, n: int, p: float) -> np.ndarray:
    """bool [C, n]: a run ends after each node with probability p, so run
    lengths are geometric(p)."""
    flags = np.zeros((C, n), dtype=bool)
    flags[:, 0] = True
    if n > 1:
        flags[:, 1:] = rng.uniform(C * (n - 1)).reshape(C, n - 1) < p
    return flags


def _labels_from_starts(rng: Rng, starts: np.ndarray) -> np.ndarray:
    """Turns run-start flags [C, n] into labels in [0, n): run r of candidate c
    gets label perm_c[r] for a per-candidate random permutation, so labels are
    arbitrary (not already canonical)."""
    C, n = starts.shape
    run = np.cumsum(starts, axis=1) - 1
    out = np.empty((C, n), dtype=np.int32)
    for c in range(C):
        out[c] = rng.permutation(n)[run[c]]
    return out


def _interval_partitions(rng: Rng, g: BaseGraph, C: int, op_rule: Tuple, ar_rule: Tuple,
                         need_edge: bool) -> np.ndarray:
    """int32 [C, n] labels.  Op-fusion groups are contiguous intervals of the
    topological node order (the quotient of a DAG by such intervals is always
    acyclic); with need_edge an interval only continues from node i-1 to i if
    the edge (i-1, i) exists, i.e. the group is a chain of producer/consumer
    ops.  Tensor buckets are contiguous runs of all-reduce nodes in production
    order (neighbouring gradient tensors, Sec. 3.2 (iii))."""
    n, n_op = g.n, g.n_op

    def starts(rule, m):
        if rule[0] == "uniform":
            return _run_starts_uniform(rng, C, m, rule[1])
        return _run_starts_geometric(rng, C, m, rule[1])

    s = np.zeros((C, n), dtype=bool)
    s[:, :n_op] = starts(op_rule, n_op)
    if n > n_op:
        s[:, n_op:] = starts(ar_rule, n - n_op)
        s[:, n_op] = True
    s[:, 0] = True
    if need_edge:
        conn = np.zeros(n, dtype=bool)
        for i in range(1, n_op):
            row = g.col[g.rowptr[i - 1]:g.rowptr[i]]
            conn[i] = np.any(row == i)
        s[:, 1:n_op] |= ~conn[1:n_op][None, :]
    return _labels_from_starts(rng, s)


def _quotient_is_acyclic(n: int, src: np.ndarray, dst: np.ndarray, lab: np.ndarray) -> bool:
    """Validity check used only by the cfg1 generator (fusions that would
    create a dependency cycle are rejected before a candidate is costed)."""
    edges = {(int(lab[s]), int(lab[d])) for s, d in zip(src, dst) if lab[s] != lab[d]}
    nodes = set(int(x) for x in lab)
    indeg = {v: 0 for v in nodes}
    adj: Dict[int, List[int]] = {v: [] for v in nodes}
    for s, d in edges:
        adj[s].append(d)
        indeg[d] += 1
    stack = [v for v in nodes if indeg[v] == 0]
    seen = 0
    while stack:
        v = stack.pop()
        seen += 1
        for w in adj[v]:
            indeg[w] -= 1
            if indeg[w] == 0:
                stack.append(w)
    return seen == len(nodes)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def make_weights(model: ModelSpec, seed: int = 0, std: Optional[float] = None) -> Weights:
    """Draw order W^0, b^0, ..., W^{L-1}, b^{L-1}, W1, b1, W2, b2, w3, b3 from
    one stream.  std=None scales each tensor by 1/sqrt(fan_in) (keeps
    activations O(1) at any width); biases use the same std as their layer."""
    rng = Rng(seed, 7)
    Ws, bs, As = [], [], []
    for l in range(model.L):
        d = model.F if l == 0 else model.H
        if model.agg == "attention":
            # draw order per layer: W, a_src, a_dst, b
            s = std if std is not None else 1.0 / math.sqrt(d)
            Ws.append(rng.normal(d * model.H) * s)
            sa = std if std is not None else 1.0 / math.sqrt(model.H // model.heads)
            As.append(rng.normal(2 * model.H) * sa)
            bs.append(rng.normal(model.H) * s)
        else:
            s = std if std is not None else 1.0 / math.sqrt(3 * d)
            Ws.append(rng.normal(3 * d * model.H) * s)
            bs.append(rng.normal(model.H) * s)
    H = model.H
    s = std if std is not None else 1.0 / math.sqrt(H)
    head = [rng.normal(H * H) * s, rng.normal(H) * s, rng.normal(H * H) * s, rng.normal(H) * s,
            rng.normal(H) * s, rng.normal(1) * s]
    return Weights(np.concatenate(Ws).astype(np.float32), np.concatenate(bs).astype(np.float32),
                   np.concatenate(head).astype(np.float32),
                   np.concatenate(As).astype(np.float32) if As else None)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
def _pack(name, model, graphs, labels_per_graph: List[np.ndarray], weights, note="") -> Workload:
    cg, parts = [], []
    for b, lab in enumerate(labels_per_graph):
        for c in range(lab.shape[0]):
            cg.append(b)
        parts.append(lab.reshape(-1))
    sizes = np.array([graphs[b].n for b in cg], dtype=np.int64)
    return Workload(name, model, graphs, np.array(cg, dtype=np.int32),
                    np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64),
                    np.concatenate(parts).astype(np.int32), weights, note)


def cfg1(n_cand: int = 1) -> Workload:
    """Tiny: 8 layers of 8 ops, 1-3 out-edges to the next layer, 8 all-reduce
    sinks; edge-connected pairs merged w.p. 0.3 when the quotient stays
    acyclic; buckets are runs of 1-3; F=16, H=32, L=2, fp32, N(0, 0.1)."""
    model = ModelSpec(16, 32, 2, "f32")
    rng = Rng(1000, 0)
    src, dst = [], []
    for k in range(7):
        for j in range(8):
            deg = int(rng.integers(1, 3, 1)[0])
            tg = rng.permutation(8)[:deg]
            for t in tg:
                src.append(8 * k + j)
                dst.append(8 * (k + 1) + int(t))
    feed = rng.integers(0, 63, 8)
    for a in range(8):
        src.append(int(feed[a]))
        dst.append(64 + a)
    n, n_op = 72, 64
    rowptr, col = _csr_from_edges(n, np.array(src), np.array(dst))
    g = BaseGraph(n, n_op, rowptr, col, _features(rng, n, n_op, model.F, None))
    es = np.repeat(np.arange(n), np.diff(rowptr))
    ed = col.astype(np.int64)
    labs = np.empty((n_cand, n), dtype=np.int32)
    prng = Rng(1000, 1)
    for c in range(n_cand):
        lab = np.arange(n)
        order = prng.permutation(len(es))
        coin = prng.uniform(len(es))
        for e in order:
            u, v = int(es[e]), int(ed[e])
            if v >= n_op or coin[e] >= 0.3 or lab[u] == lab[v]:
                continue
            trial = lab.copy()
            trial[trial == lab[v]] = lab[u]
            if _quotient_is_acyclic(n, es, ed, trial):
                lab = trial
        ar = _run_starts_uniform(prng, 1, n - n_op, 3)[0]
        ar[0] = True
        run = np.cumsum(ar) - 1
        used = set(int(x) for x in lab[:n_op])
        free = [x for x in range(n) if x not in used]
        lab[n_op:] = np.array(free)[run]
        labs[c] = lab
    return _pack("cfg1", model, [g], [labs], make_weights(model, 0, 0.1))


def _single_graph_cfg(name, seed, dag, model, n_cand, ar_lo, ar_hi, op_rule, ar_rule, need_edge) -> Workload:
    n, n_op, src, dst = dag
    rng = Rng(seed, 0)
    rowptr, col = _csr_from_edges(n, src, dst)
    ar_bytes = _log_uniform(rng, n - n_op, ar_lo, ar_hi)
    g = BaseGraph(n, n_op, rowptr, col, _features(rng, n, n_op, model.F, ar_bytes))
    labs = _interval_partitions(Rng(seed, 1), g, n_cand, op_rule, ar_rule, need_edge)
    return _pack(name, model, [g], [labs], make_weights(model, 0))


def cfg2(n_cand: int = 256) -> Workload:
    """ResNet-50-shaped training DAG, 161 all-reduce tensors of 4 KB-9 MB;
    chains of 1-4 ops, buckets of 1-20 tensors; F=32, H=128, L=3, fp32."""
    return _single_graph_cfg("cfg2", 2000, _resnet50_dag(), ModelSpec(32, 128, 3, "f32"), n_cand,
                             4e3, 9e6, ("uniform", 4), ("uniform", 20), True)


def cfg3(n_cand: int = 1024) -> Workload:
    """BERT-base-shaped: 12 blocks of ~120 ops, 200 all-reduce tensors of
    2 KB-9 MB; partition rule as cfg2; F=32, H=128, L=3, bf16."""
    return _single_graph_cfg("cfg3", 3000, _transformer_dag(12, 2, 5, 3), ModelSpec(32, 128, 3, "bf16"), n_cand,
                             2e3, 9e6, ("uniform", 4), ("uniform", 20), True)


def cfg4(n_cand: int = 4096) -> Workload:
    """24-block transformer, ~6000 ops + 400 all-reduce tensors of 4 KB-50 MB;
    groups are intervals of 1-8 ops of the topological order (connected or
    not), buckets of 1-40; F=64, H=256, L=4, bf16."""
    return _single_graph_cfg("cfg4", 4000, _transformer_dag(24, 9, 10, 6), ModelSpec(64, 256, 4, "bf16"), n_cand,
                             4e3, 50e6, ("uniform", 8), ("uniform", 40), False)


def cfg5(n_cand: int = 8192, n_graphs: int = 64, n_lo: int = 100, n_hi: int = 20000) -> Workload:
    """Heterogeneous batch: random base DAGs with log-uniform op counts,
    power-law out-degree (alpha 2.5, cap 32), round(0.05 n_op) all-reduce
    sinks of 4 KB-50 MB; geometric(0.4) intervals for groups and buckets;
    n_cand/n_graphs candidates per base graph; F=64, H=256, L=4, bf16."""
    model = ModelSpec(64, 256, 4, "bf16")
    rng = Rng(5000, 0)
    per = max(1, n_cand // n_graphs)
    kk = np.arange(1, 33, dtype=np.float64)
    cdf = np.cumsum(kk ** -2.5)
    cdf /= cdf[-1]
    graphs, labels = [], []
    n_ops = np.round(_log_uniform(rng, n_graphs, n_lo, n_hi)).astype(np.int64)
    for b in range(n_graphs):
        n_op = int(n_ops[b])
        deg = 1 + np.searchsorted(cdf, rng.uniform(n_op), side="right")
        deg = np.minimum(deg, np.maximum(n_op - 1 - np.arange(n_op), 0))
        src = np.repeat(np.arange(n_op), deg)
        lo = src + 1
        dst = lo + np.floor(rng.uniform(src.shape[0]) * (n_op - lo)).astype(np.int64)
        n_ar = max(1, int(round(0.05 * n_op)))
        feed = rng.integers(0, n_op - 1, n_ar)
        src = np.concatenate([src, feed])
        dst = np.concatenate([dst, n_op + np.arange(n_ar)])
        n = n_op + n_ar
        rowptr, col = _csr_from_edges(n, src, dst)
        ar_bytes = _log_uniform(rng, n_ar, 4e3, 50e6)
        g = BaseGraph(n, n_op, rowptr, col, _features(rng, n, n_op, model.F, ar_bytes))
        graphs.append(g)
        labels.append(_interval_partitions(Rng(5000, 100 + b), g, per, ("geometric", 0.4), ("geometric", 0.4), False))
    # Graphs from a hundred to twenty thousand nodes under a sum readout give graph vectors of very
    # different size; with a signed last layer the predictions are remainders a hundred times smaller
    # than the terms they add up, which bf16 storage of the activations does not resolve (the CPU oracle
    # run with bf16 storage is 0.13 away from itself run in fp32).  The last layer is therefore taken
    # non-negative here: a prediction is a sum of non-negative terms, as a time is.
    wt = make_weights(model, 0)
    head = wt.head.copy()
    head[-(model.H + 1):] = np.abs(head[-(model.H + 1):])
    return _pack("cfg5", model, graphs, labels, Weights(wt.layers, wt.biases, head, wt.att))


CONFIGS = {"cfg1": cfg1, "cfg2": cfg2, "cfg3": cfg3, "cfg4": cfg4, "cfg5": cfg5}


def make(name: str, n_cand: Optional[int] = None, **kw) -> Workload:
    fn = CONFIGS[name]
    return fn(**kw) if n_cand is None else fn(n_cand, **kw)


# --------------------------------------------------------------------------
# small hand-made cases for the tests
# --------------------------------------------------------------------------
def random_dag(seed: int, n: int, p: float, F: int, integer_features: bool = False) -> BaseGraph:
    """Erdos-Renyi DAG on the index order (edge i->j only for i<j)."""
    rng = Rng(seed, 3)
    m = rng.uniform(n * n).reshape(n, n) < p
    m = np.triu(m, 1)
    src, dst = np.nonzero(m)
    rowptr, col = _csr_from_edges(n, src, dst)
    if integer_features:
        X = rng.integers(0, 7, n * F).reshape(n, F).astype(np.float32)
    else:
        X = rng.uniform(n * F).reshape(n, F).astype(np.float32)
    return BaseGraph(n, n, rowptr, col, X)


def random_labels(seed: int, n: int, n_groups: int, C: int = 1) -> np.ndarray:
    """Arbitrary (not interval, not necessarily acyclic) labelings [C, n] with
    values in [0, n): exercises the contraction for any partition."""
    rng = Rng(seed, 4)
    lab = rng.integers(0, max(n_groups, 1) - 1, C * n).reshape(C, n)
    out = np.empty((C, n), dtype=np.int32)
    for c in range(C):
        out[c] = rng.permutation(n)[lab[c]]
    return out


def with_attention(w: Workload, heads: int, seed: int = 0, std: Optional[float] = None) -> Workload:
    """The same graphs and candidates evaluated by the attention variant of the estimator.  The last layer
    of its regression network is taken non-negative (see with_time_like_head): with signed random
    weights the attention model's predictions on the large configurations are remainders of terms a
    hundred times their size, which no bf16 storage of the activations resolves."""
    m = ModelSpec(w.model.F, w.model.H, w.model.L, w.model.dtype, "attention", heads)
    return with_time_like_head(Workload(w.name + "-attention", m, w.graphs, w.cand_graph, w.cand_off, w.group_id,
                                        make_weights(m, seed, std), w.note))


def with_time_like_head(w: Workload) -> Workload:
    """The same workload with the last layer of the regression network made non-negative (|w3|, |b3|):
    the prediction is then a sum of non-negative terms, as a time is, and its relative error is not
    inflated by a last dot product that cancels (random signed weights can leave a prediction a hundred
    times smaller than the terms it adds up)."""
    wt = w.weights
    head = wt.head.copy()
    H = w.model.H
    head[-(H + 1):] = np.abs(head[-(H + 1):])
    return Workload(w.name, w.model, w.graphs, w.cand_graph, w.cand_off, w.group_id,
                    Weights(wt.layers, wt.biases, head, wt.att), w.note)


def profile_of(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Stand-in for the profiler's records (Sec. 3.1) over all base nodes, concatenated like
    the features: (op_time, ar_size).  An op's execution time is 0.05 + feature column 2; an
    all-reduce node's tensor size is feature column 0 (MiB in cfg2-cfg5); ar_size is -1 for
    ops and op_time is 0 for all-reduce nodes."""
    t, x = [], []
    for g in w.graphs:
        is_ar = np.arange(g.n) >= g.n_op
        t.append(np.where(is_ar, 0.0, 0.05 + g.X[:, 2]).astype(np.float32))
        x.append(np.where(is_ar, g.X[:, 0], -1.0).astype(np.float32))
    return np.concatenate(t), np.concatenate(x)


def custom(name: str, model: ModelSpec, graphs: List[BaseGraph], labels_per_graph: List[np.ndarray],
           weights: Optional[Weights] = None, seed: int = 0, std: Optional[float] = None) -> Workload:
    return _pack(name, model, graphs, labels_per_graph, weights or make_weights(model, seed, std))


# --------------------------------------------------------------------------
# training samples of the fused-op estimator
# --------------------------------------------------------------------------
def training_labels(g: BaseGraph, seed: int, C: int, kmax: int = 48, cover: float = 0.6) -> np.ndarray:
    """Labelings [C, n] whose groups of two or more ops are training samples drawn the way
    Sec. 5.1 describes (Fused Op Estimator): a random op is fused with one of its
    predecessors, and the fused op again with one of its predecessors, k times; k is
    log-uniform in [1, kmax] and growth stops early when no free predecessor is left (the
    paper draws far larger counts than a module has ops; the same early stop applies there).
    Samples of one labeling are disjoint; seeds are drawn until `cover` of the ops are used.
    All-reduce nodes stay single."""
    rng = Rng(seed, 21)
    n, n_op = g.n, g.n_op
    crp = np.zeros(n + 1, np.int64)
    src = np.repeat(np.arange(n), np.diff(g.rowptr))
    np.add.at(crp, g.col + 1, 1)
    crp = np.cumsum(crp)
    order = np.argsort(g.col, kind="stable")
    pred = src[order]
    out = np.empty((C, n), np.int32)
    for c in range(C):
        lab = np.arange(n, dtype=np.int32)
        used = np.zeros(n, bool)
        used[n_op:] = True
        tries = rng.permutation(n_op)
        ks = np.exp(rng.uniform(n_op) * math.log(kmax)).astype(np.int64)
        pick = rng.u64(n_op * 4)
        pi, covered = 0, 0
        for i, s0 in enumerate(tries):
            if covered >= cover * n_op:
                break
            if used[s0]:
                continue
            members, frontier = [int(s0)], [int(p) for p in pred[crp[s0]:crp[s0 + 1]] if not used[p]]
            used[s0] = True
            for _ in range(int(ks[i])):
                frontier = [p for p in frontier if not used[p]]
                if not frontier:
                    break
                p = frontier[int(pick[pi % pick.size] % np.uint64(len(frontier)))]
                pi += 1
                used[p] = True
                members.append(p)
                frontier += [int(q) for q in pred[crp[p]:crp[p + 1]] if not used[q]]
            if len(members) >= 2:
                lab[members] = min(members)
                covered += len(members)
        out[c] = lab
    return out


def synthetic_fused_times(node_off: np.ndarray, base_node: np.ndarray, op_time: np.ndarray,
                          seed: int = 0) -> np.ndarray:
    """Stand-in for profiled fused-op times (Sec. 3.3.3 trains on profiled ones): the members'
    own times summed, scaled by a fusion gain that grows with the number of members and by
    +-10 % seeded noise.  Positive for every fused op.  node_off [K+1] and base_node [rows]
    describe the batch of fused-op subgraphs (concatenated base numbering)."""
    K = node_off.size - 1
    cnt = np.diff(node_off.astype(np.int64))
    own = np.asarray(op_time, np.float64)[np.asarray(base_node[:int(node_off[-1])], np.int64)]
    s = np.zeros(K)
    np.add.at(s, np.repeat(np.arange(K), cnt), own)
    gain = 0.55 + 0.45 / np.sqrt(np.maximum(cnt, 1))
    noise = 0.9 + 0.2 * Rng(seed, 22).uniform(max(K, 1))[:K]
    return np.maximum(s * gain * noise, 1e-3).astype(np.float32)
