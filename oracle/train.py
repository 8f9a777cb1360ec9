"""CPU oracle of estimator training (test infrastructure only; numpy, fp64 throughout).

What it follows
  * The estimator of Sec. 3.3 in the reading the forward oracle takes: L layers
        h'[v] = ReLU([h[v] | mean over predecessors | mean over successors] W + b),
    the sum of the final embeddings over the ops of each fused op (Sec. 3.3.1, second
    equation), and the regression network z1 = ReLU(r W1 + b1), z2 = ReLU(z1 W2 + b2),
    y = z2 . w3 + b3 (Sec. 3.3.2).
  * Model training, Sec. 3.3.3: graph network and regression network are trained together,
    supervised, on a set G of fused ops with profiled times y'; Eq. (1) is the loss and Adam
    the optimiser.  Eq. (1) as printed is the logarithm of a squared difference, which has
    no minimum at a perfect fit; the reading taken here is the mean squared difference of
    the logarithms,
        L(theta) = 1/|G| * sum_g (log max(y_g, floor) - log y'_g)^2 ,
    where the floor keeps the logarithm defined when the linear output is not positive; a
    sample below the floor contributes its loss but no gradient.
  * Adam as published (Kingma & Ba): m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2,
    theta -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps), t counted from 1.

The gradient is the hand-derived reverse pass of exactly these formulas, one statement per
formula, with no fusion or reordering.  Pins (tests/test_oracle_train.py): central finite
differences of the loss for every parameter tensor, reverse-mode differentiation of an
independently written forward pass by a library (torch.autograd, fp64), closed forms of the
loss, the library's Adam, and the constant-gradient closed form of Adam.  Where a pre-activation
is closer to zero than single precision resolves, a single-precision pass may take the ReLU
derivative from either side; undecided_units() lists such units and the `flip` argument takes the
other side, pinned by moving a unit just across zero.

Nothing in the product package imports this module, and it shares no code with the HIP path.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np


@dataclass
class Params:
    """fp64 copies of the estimator's parameters in the layout of the C interface."""
    W: List[np.ndarray]      # per layer [3d, H]
    b: List[np.ndarray]      # per layer [H]
    W1: np.ndarray
    b1: np.ndarray
    W2: np.ndarray
    b2: np.ndarray
    w3: np.ndarray
    b3: np.ndarray           # [1]

    def flat(self) -> np.ndarray:
        """W_layers | b_layers | head, the order of the C interface."""
        parts = [w.ravel() for w in self.W] + [x.ravel() for x in self.b]
        parts += [self.W1.ravel(), self.b1, self.W2.ravel(), self.b2, self.w3, self.b3]
        return np.concatenate(parts)

    @staticmethod
    def shapes(F: int, H: int, L: int):
        s = [(3 * (F if l == 0 else H), H) for l in range(L)] + [(H,)] * L
        return s + [(H, H), (H,), (H, H), (H,), (H,), (1,)]

    @staticmethod
    def from_flat(theta: np.ndarray, F: int, H: int, L: int) -> "Params":
        out, o = [], 0
        for s in Params.shapes(F, H, L):
            n = int(np.prod(s))
            out.append(np.array(theta[o:o + n], dtype=np.float64).reshape(s))
            o += n
        assert o == theta.size
        return Params(out[:L], out[L:2 * L], *out[2 * L:])

    @staticmethod
    def from_weights(weights, F: int, H: int, L: int) -> "Params":
        theta = np.concatenate([np.asarray(weights.layers, np.float64).ravel(),
                                np.asarray(weights.biases, np.float64).ravel(),
                                np.asarray(weights.head, np.float64).ravel()])
        return Params.from_flat(theta, F, H, L)


def _edges(rowptr: np.ndarray, col: np.ndarray, n: int) -> Tuple[np.ndarray, np.ndarray]:
    """(owner, neighbour) of every list entry of a CSR structure with n rows."""
    deg = np.diff(np.asarray(rowptr[:n + 1], np.int64))
    return np.repeat(np.arange(n), deg), np.asarray(col[:int(rowptr[n])], np.int64)


def _mean_of_neighbours(h: np.ndarray, own: np.ndarray, nb: np.ndarray, n: int) -> np.ndarray:
    s = np.zeros((n, h.shape[1]))
    np.add.at(s, own, h[nb])
    deg = np.bincount(own, minlength=n).astype(np.float64)
    return s / np.maximum(deg, 1.0)[:, None]


def forward(batch, p: Params):
    """Returns (y [B], cache) for a block-diagonal batch (oracle.Batch)."""
    n, B = batch.ntot, batch.n_cand
    pin = _edges(batch.in_rowptr, batch.in_col, n)     # v <- its predecessors
    pout = _edges(batch.out_rowptr, batch.out_col, n)  # v <- its successors
    h = np.asarray(batch.Xc[:n], np.float64)
    hs, mps, mss = [h], [], []
    for W, b in zip(p.W, p.b):
        mp = _mean_of_neighbours(h, pin[0], pin[1], n)
        ms = _mean_of_neighbours(h, pout[0], pout[1], n)
        h = np.maximum(np.concatenate([h, mp, ms], axis=1) @ W + b, 0.0)
        hs.append(h)
        mps.append(mp)
        mss.append(ms)
    gid = np.repeat(np.arange(B), np.diff(np.asarray(batch.node_off, np.int64)))
    r = np.zeros((B, h.shape[1]))
    np.add.at(r, gid, h)
    z1 = np.maximum(r @ p.W1 + p.b1, 0.0)
    z2 = np.maximum(z1 @ p.W2 + p.b2, 0.0)
    y = z2 @ p.w3 + p.b3[0]
    return y, dict(hs=hs, mps=mps, mss=mss, gid=gid, r=r, z1=z1, z2=z2, pin=pin, pout=pout)


def loss_of(y: np.ndarray, target: np.ndarray, floor: float) -> float:
    """Eq. (1) in the reading of the header."""
    if y.size == 0:
        return 0.0
    d = np.log(np.maximum(y, floor)) - np.log(np.asarray(target, np.float64))
    return float(np.mean(d * d))


def undecided_units(batch, p: Params, rel: float):
    """Units (layer, row, column) whose pre-activation lies within rel * (largest magnitude in
    that layer) of zero, top layer first; the two hidden layers of the regression network count
    as layers L (z1) and L + 1 (z2), their rows are samples.  An fp32 forward pass cannot tell
    which side of zero such a unit is on, so its ReLU derivative may legitimately be taken either
    way; loss_and_gradients(flip=...) gives the other choice."""
    _, c = forward(batch, p)
    out = []
    L = len(p.W)
    for l, Z in ((L + 1, c["z1"] @ p.W2 + p.b2), (L, c["r"] @ p.W1 + p.b1)):
        if Z.size:
            r, j = np.nonzero(np.abs(Z) < rel * np.abs(Z).max())
            out += [(l, int(a), int(b)) for a, b in zip(r, j)]
    for l in range(L - 1, -1, -1):
        Z = np.concatenate([c["hs"][l], c["mps"][l], c["mss"][l]], axis=1) @ p.W[l] + p.b[l]
        r, j = np.nonzero(np.abs(Z) < rel * np.abs(Z).max())
        out += [(l, int(a), int(b)) for a, b in zip(r, j)]
    return out


def loss_and_gradients(batch, target: np.ndarray, p: Params, floor: float = 1e-6, flip=()):
    """(loss, y, gradient as Params) of Eq. (1) over the batch.  `flip` lists units (layer, row,
    column) whose ReLU derivative is taken from the other side of zero (see undecided_units);
    the forward values are not touched."""
    y, c = forward(batch, p)
    B, n = batch.n_cand, batch.ntot
    t = np.asarray(target, np.float64)
    loss = loss_of(y, t, floor)
    # dL/dy: 2/|G| (log y - log y') / y above the floor, nothing below it
    yc = np.maximum(y, floor)
    dy = np.where(y > floor, 2.0 / max(B, 1) * (np.log(yc) - np.log(t)) / yc, 0.0)
    # regression network
    L = len(p.W)
    on2, on1 = c["z2"] > 0, c["z1"] > 0
    for (fl, fr, fc) in flip:
        if fl == L + 1:
            on2[fr, fc] = not on2[fr, fc]
        elif fl == L:
            on1[fr, fc] = not on1[fr, fc]
    gw3 = c["z2"].T @ dy
    gb3 = np.array([dy.sum()])
    dz2 = np.outer(dy, p.w3) * on2
    gW2 = c["z1"].T @ dz2
    gb2 = dz2.sum(axis=0)
    dz1 = (dz2 @ p.W2.T) * on1
    gW1 = c["r"].T @ dz1
    gb1 = dz1.sum(axis=0)
    dr = dz1 @ p.W1.T
    # the sum over the ops of a fused op hands its gradient to every one of them
    G = dr[c["gid"]]
    gW: List[Optional[np.ndarray]] = [None] * L
    gb: List[Optional[np.ndarray]] = [None] * L
    pin, pout = c["pin"], c["pout"]
    indeg = np.maximum(np.bincount(pin[0], minlength=n), 1).astype(np.float64)
    outdeg = np.maximum(np.bincount(pout[0], minlength=n), 1).astype(np.float64)
    for l in range(L - 1, -1, -1):
        h, hn = c["hs"][l], c["hs"][l + 1]
        d = h.shape[1]
        on = hn > 0
        for (fl, fr, fc) in flip:
            if fl == l:
                on[fr, fc] = not on[fr, fc]
        dZ = G * on
        A = np.concatenate([h, c["mps"][l], c["mss"][l]], axis=1)
        gW[l] = A.T @ dZ
        gb[l] = dZ.sum(axis=0)
        if l == 0:
            break
        dA = dZ @ p.W[l].T
        G = dA[:, :d].copy()
        # mean over predecessors of v: each predecessor u receives dA_pred[v] / indeg(v)
        np.add.at(G, pin[1], (dA[:, d:2 * d] / indeg[:, None])[pin[0]])
        np.add.at(G, pout[1], (dA[:, 2 * d:] / outdeg[:, None])[pout[0]])
    return loss, y, Params(gW, gb, gW1, gb1, gW2, gb2, gw3, gb3)


def adam_step(theta: np.ndarray, g: np.ndarray, m: np.ndarray, v: np.ndarray, t: int, lr: float, beta1: float,
              beta2: float, eps: float):
    """One Adam update; t is the 1-based count of this step.  Returns (theta, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m, v


def train(batches, targets, p: Params, F: int, H: int, L: int, lr: float, beta1: float = 0.9, beta2: float = 0.999,
          eps: float = 1e-8, floor: float = 1e-6):
    """One Adam step per (batch, target) pair, in order.  Returns (params, losses)."""
    theta = p.flat()
    m = np.zeros_like(theta)
    v = np.zeros_like(theta)
    losses = []
    for t, (bt, tg) in enumerate(zip(batches, targets), start=1):
        loss, _, g = loss_and_gradients(bt, tg, Params.from_flat(theta, F, H, L), floor)
        theta, m, v = adam_step(theta, g.flat(), m, v, t, lr, beta1, beta2, eps)
        losses.append(loss)
    return Params.from_flat(theta, F, H, L), losses
