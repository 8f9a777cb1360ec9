"""TEST INFRASTRUCTURE ONLY -- the backtracking search of the paper (Alg. 1, Sec. 4) over
fusion strategies, written out step by step on the CPU with the oracle's Cost(H).

A strategy is a labelling of the base nodes (equal labels = one fused op or one fused gradient
tensor); H_in is the all-singleton labelling.  Q is a priority queue by cost; per dequeued H
every optimisation method s draws n = Random(0, beta) and applies itself n times
(RandomApply); a valid H' replaces H_opt when cheaper (the counter of unchanged evaluations
restarts) and is enqueued when Cost(H') <= alpha * Cost(H_opt); the search ends when Q is empty
or the counter reaches its limit.

Choices of this build where the paper is silent or where this build's scope cuts in:
  * H_opt starts as H_in; the counter counts evaluated valid candidates.
  * Methods: (i) op fusion and (iii) tensor fusion.  (ii) duplicates an op, which is not a
    partition of the node set, and is left out.
  * (i) one application, as the paper words it (op_draw = "op"): draw a computation op of the
    CURRENT module uniformly (a group of the labelling, groups taken in the order of their
    smallest member), then one of its predecessor ops in the current module uniformly (the
    groups of computation ops with a dependency into it, same order); the predecessor joins
    the op.  An op without predecessors leaves the module as it is.  One 64-bit draw serves
    both: the low 32 bits pick the op, the high 32 bits the predecessor.
    The alternative (op_draw = "dependency", the default of the device driver, which has both): draw a dependency
    u -> v between two computation ops of the BASE module uniformly; if its ends are in
    different groups, the group of u joins the group of v.  It needs no view of the current
    module between applications, but it is a different distribution: ops with many
    predecessors are chosen more often, and a dependency inside a group changes nothing.
  * (iii) one application: draw an all-reduce node a and a side uniformly; the nearest bucket on
    that side in production order, if any, joins the bucket of a.
  * Validity: the module must be acyclic (its cost is finite); op kinds that must not be fused
    do not exist in the synthetic modules.
  * Random(0, beta) is an integer uniform on [0, beta].
  * Batching: up to `parents` entries are dequeued per step (ascending cost, then age) and their
    children are costed together, then handled in order; parents = 1 is the paper's loop.
  * Equal costs dequeue oldest first; a queue above `max_queue` entries drops its most expensive.
  * All draws come from one counter-based generator keyed by (seed, step, child):
    key = mix(seed ^ mix(step * 2^32 + child)), draw d = mix(key + d * 0xD1342543DE82EF95),
    mix = splitmix64's output function; draw 0 gives n, draws 1.. the applications.

Pins (tests/test_oracle_search.py): beta = 0 (every child equals its parent: the evaluation
count and the unchanged optimum follow in closed form), a chain whose optimum is known,
invariants of every H_opt (finite cost, groups connected through fused dependencies, buckets
contiguous), monotone best cost, the queue discipline against a hand-worked trace
(tests/golden/search_example.txt).  That the paper's own implementation draws its mutations
this way: parity unpinned.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Tuple

import numpy as np

_M = (1 << 64) - 1


def mix(x: int) -> int:
    """splitmix64 output function on a 64-bit integer."""
    z = (x + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def draw(seed: int, step: int, child: int, d: int) -> int:
    key = mix((seed ^ mix(((step << 32) + child) & _M)) & _M)
    return mix((key + d * 0xD1342543DE82EF95) & _M)


def op_edges(g) -> Tuple[np.ndarray, np.ndarray]:
    """Dependencies between two computation ops, in CSR order."""
    src = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    dst = g.col.astype(np.int64)
    keep = (src < g.n_op) & (dst < g.n_op)
    return src[keep], dst[keep]


def current_op_groups(g, lab: np.ndarray) -> np.ndarray:
    """Labels of the computation ops of the current module, in the order of their smallest member."""
    ops = lab[:g.n_op]
    _, first = np.unique(ops, return_index=True)
    return ops[np.sort(first)]


def current_predecessors(g, lab: np.ndarray, group: int, pred_lists=None) -> np.ndarray:
    """Labels of the computation ops of the current module with a dependency into `group`, in the
    order of their smallest member."""
    src, dst = op_edges(g)
    into = (lab[dst] == group) & (lab[src] != group)
    cand = set(lab[src[into]].tolist())
    order = current_op_groups(g, lab)
    return np.array([l for l in order if l in cand], dtype=lab.dtype)


def random_apply(g, labels: np.ndarray, method: int, n: int, seed: int, step: int, child: int,
                 op_draw: str = "dependency") -> np.ndarray:
    """RandomApply(H, s, n): method 0 = op fusion, 1 = tensor fusion; draws 1..n of the child's stream."""
    lab = labels.copy()
    if method == 0 and op_draw == "op":
        for i in range(n):
            r = draw(seed, step, child, 1 + i)
            groups = current_op_groups(g, lab)
            if len(groups) == 0:
                continue
            op = groups[(r & 0xFFFFFFFF) % len(groups)]
            preds = current_predecessors(g, lab, op)
            if len(preds) == 0:
                continue
            p_ = preds[(r >> 32) % len(preds)]
            lab[lab == p_] = op
    elif method == 0:
        src, dst = op_edges(g)
        for i in range(n):
            r = draw(seed, step, child, 1 + i)
            if len(src) == 0:
                continue
            k = r % len(src)
            lu, lv = lab[src[k]], lab[dst[k]]
            if lu != lv:
                lab[lab == lu] = lv
    else:
        n_ar = g.n - g.n_op
        for i in range(n):
            r = draw(seed, step, child, 1 + i)
            if n_ar == 0:
                continue
            a = g.n_op + (r % n_ar)
            side = 1 if (r >> 32) & 1 else -1
            b = a + side
            while g.n_op <= b < g.n and lab[b] == lab[a]:
                b += side
            if g.n_op <= b < g.n:
                lab[lab == lab[b]] = lab[a]
    return lab


@dataclass
class SearchResult:
    labels_opt: np.ndarray
    cost_in: float
    cost_opt: float
    steps: int = 0
    evaluated: int = 0
    valid: int = 0
    enqueued: int = 0
    improved: int = 0
    trace: List[Tuple] = field(default_factory=list)


def search(g, cost_fn: Callable[[np.ndarray], np.ndarray], alpha: float, beta: int, seed: int,
           max_unchanged: int = 1000, parents: int = 1, max_steps: int = 1 << 30, max_queue: int = 1 << 30,
           keep_trace: bool = False, op_draw: str = "dependency") -> SearchResult:
    """cost_fn maps labels [C, n] (int32) to float32 costs [C] (+inf = invalid)."""
    h_in = np.arange(g.n, dtype=np.int32)
    cost_in = np.float32(cost_fn(h_in.reshape(1, -1))[0])
    res = SearchResult(h_in.copy(), float(cost_in), float(cost_in))
    cost_opt = cost_in
    heap: List[Tuple[float, int, np.ndarray]] = [(float(cost_in), 0, h_in)]
    next_id, unchanged, step = 1, 0, 0
    while heap and unchanged < max_unchanged and step < max_steps:
        ps = [heapq.heappop(heap) for _ in range(min(parents, len(heap)))]
        kids = []
        for pi, (_, _, lab) in enumerate(ps):
            for s in range(2):
                j = 2 * pi + s
                n = draw(seed, step, j, 0) % (beta + 1)
                kids.append(random_apply(g, lab, s, n, seed, step, j, op_draw))
        costs = np.asarray(cost_fn(np.stack(kids).astype(np.int32)), dtype=np.float32)
        for j, c in enumerate(costs):
            res.evaluated += 1
            if not np.isfinite(c):
                continue
            res.valid += 1
            if c < cost_opt:
                cost_opt = c
                res.labels_opt = kids[j].copy()
                res.improved += 1
                unchanged = 0
            else:
                unchanged += 1
            if float(c) <= float(np.float32(alpha)) * float(cost_opt):
                heapq.heappush(heap, (float(c), next_id, kids[j]))
                next_id += 1
                res.enqueued += 1
            if keep_trace:
                res.trace.append((step, j, float(c), float(cost_opt), unchanged, len(heap)))
        if len(heap) > max_queue:
            heap = heapq.nsmallest(max_queue, heap)
            heapq.heapify(heap)
        step += 1
    res.steps = step
    res.cost_opt = float(cost_opt)
    return res
