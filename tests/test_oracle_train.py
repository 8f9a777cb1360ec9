"""Pins for the CPU oracle of estimator training (Sec. 3.3.3, Eq. (1), Adam; no GPU).

The hand-derived reverse pass is checked against two things that do not share its formulas:
central finite differences of the loss, and a library's reverse-mode differentiation of a
forward pass written a second way (dense normalised adjacency matrices instead of
per-list sums).  The loss and the optimiser are checked against closed forms and against the
library's Adam."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from oracle import train as ot
from paper_2209_12769_amd import workloads as wl


def tiny_case(seed, F=4, H=8, L=3, n=12, groups=4, C=3):
    """A few random DAGs contracted by arbitrary labels: a batch of C small graphs."""
    g = wl.random_dag(seed, n, 0.35, F)
    model = wl.ModelSpec(F, H, L, "f32")
    w = wl.custom("t", model, [g], [wl.random_labels(seed, n, groups, C)], seed=seed, std=0.4)
    w.weights.head[-1] += 1.5                       # estimates mostly positive
    b = orc.contract(w)
    p = ot.Params.from_weights(w.weights, F, H, L)
    y, _ = ot.forward(b, p)
    p.b3[0] += max(0.0, 1.0 - y.min())              # every estimate at least 1: no sample at the floor
    rng = np.random.default_rng(seed)
    target = rng.uniform(0.5, 3.0, b.n_cand)
    return b, p, target, model


def fused_case(seed, F=16, H=32, L=2):
    """Samples the way training draws them: fused-op subgraphs of a ResNet-shaped module."""
    base = wl.make("cfg2", 1)
    model = wl.ModelSpec(base.model.F, H, L, "f32")
    w = wl.custom("s", model, base.graphs, [wl.training_labels(base.graphs[0], seed, 2, kmax=12)], seed=seed)
    w.weights.head[-1] += 1.0
    t, x = wl.profile_of(w)
    fo, _, member = orc.fused_ops(w, orc.contract(w), x)
    return fo, ot.Params.from_weights(w.weights, model.F, H, L), wl.synthetic_fused_times(fo.node_off, member, t, seed), model


def test_loss_closed_forms():
    t = np.array([0.5, 2.0, 7.0])
    assert ot.loss_of(t.copy(), t, 1e-6) == 0.0
    assert ot.loss_of(np.e * t, t, 1e-6) == pytest.approx(1.0, rel=1e-14)
    assert ot.loss_of(t / np.e ** 2, t, 1e-6) == pytest.approx(4.0, rel=1e-14)
    # below the floor the floor is what the logarithm sees
    assert ot.loss_of(np.array([-3.0]), np.array([1.0]), 1e-3) == pytest.approx(np.log(1e-3) ** 2, rel=1e-14)
    assert ot.loss_of(np.zeros(0), np.zeros(0), 1e-6) == 0.0


def test_forward_matches_the_forward_oracle():
    b, p, _, model = tiny_case(3, F=16, H=32, L=2)
    w = wl.Weights(np.concatenate([x.ravel() for x in p.W]).astype(np.float32),
                   np.concatenate(p.b).astype(np.float32),
                   np.concatenate([p.W1.ravel(), p.b1, p.W2.ravel(), p.b2, p.w3, p.b3]).astype(np.float32))
    y, _ = ot.forward(b, p)
    np.testing.assert_allclose(y, orc.gnn_forward(b, model, w), rtol=2e-6, atol=1e-6)


@pytest.mark.parametrize("seed", [1, 2, 5])
def test_gradient_against_finite_differences(seed):
    b, p, target, model = tiny_case(seed)
    loss, y, g = ot.loss_and_gradients(b, target, p)
    assert (y > 1e-3).all()                          # no sample sits at the floor's kink
    theta, gf = p.flat(), g.flat()
    F, H, L = model.F, model.H, model.L

    def f(th):
        yy, _ = ot.forward(b, ot.Params.from_flat(th, F, H, L))
        return ot.loss_of(yy, target, 1e-6)

    assert f(theta) == pytest.approx(loss, rel=1e-14)
    rng = np.random.default_rng(seed)
    # every tensor gets probed: walk the tensors and take a few coordinates of each
    o, worst = 0, 0.0
    for shp in ot.Params.shapes(F, H, L):
        nel = int(np.prod(shp))
        for i in o + rng.choice(nel, size=min(nel, 12), replace=False):
            h = 1e-6
            e = np.zeros_like(theta)
            e[i] = h
            fd = (f(theta + e) - f(theta - e)) / (2 * h)
            worst = max(worst, abs(fd - gf[i]) / max(1e-4, abs(fd), abs(gf[i])))
        o += nel
    # a ReLU unit within h of zero would show as an O(1) mismatch; smooth points agree to ~1e-8
    assert worst < 1e-5


def _torch_forward(batch, tp, F, H, L):
    """Second formulation: dense row-normalised adjacency matrices, plain matmuls."""
    n, B = batch.ntot, batch.n_cand
    Ain = torch.zeros(n, n, dtype=torch.float64)
    Aout = torch.zeros(n, n, dtype=torch.float64)
    for v in range(n):
        for k in range(batch.in_rowptr[v], batch.in_rowptr[v + 1]):
            Ain[v, batch.in_col[k]] += 1.0
        for k in range(batch.out_rowptr[v], batch.out_rowptr[v + 1]):
            Aout[v, batch.out_col[k]] += 1.0
    Ain = Ain / Ain.sum(1, keepdim=True).clamp(min=1.0)
    Aout = Aout / Aout.sum(1, keepdim=True).clamp(min=1.0)
    S = torch.zeros(B, n, dtype=torch.float64)
    for c in range(B):
        S[c, batch.node_off[c]:batch.node_off[c + 1]] = 1.0
    h = torch.tensor(np.asarray(batch.Xc[:n], np.float64))
    for l in range(L):
        h = torch.relu(torch.cat([h, Ain @ h, Aout @ h], dim=1) @ tp[l] + tp[L + l])
    W1, b1, W2, b2, w3, b3 = tp[2 * L:]
    z2 = torch.relu(torch.relu(S @ h @ W1 + b1) @ W2 + b2)
    return z2 @ w3 + b3


@pytest.mark.parametrize("case", ["tiny", "fused"])
def test_gradient_against_library_autodiff(case):
    if case == "tiny":
        b, p, target, model = tiny_case(7, F=8, H=16, L=3, n=20, groups=6, C=4)
    else:
        b, p, target, model = fused_case(4)
        assert b.n_cand > 20 and b.etot > 0
    F, H, L = model.F, model.H, model.L
    loss, y, g = ot.loss_and_gradients(b, target, p)
    tp = [torch.tensor(x, dtype=torch.float64, requires_grad=True)
          for x in p.W + p.b + [p.W1, p.b1, p.W2, p.b2, p.w3, p.b3]]
    ty = _torch_forward(b, tp, F, H, L)
    tl = ((torch.log(ty.clamp(min=1e-6)) - torch.log(torch.tensor(np.asarray(target, np.float64)))) ** 2).mean()
    tl.backward()
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    assert loss == pytest.approx(float(tl.detach()), rel=1e-11)
    tg = np.concatenate([x.grad.numpy().ravel() for x in tp])
    np.testing.assert_allclose(g.flat(), tg, rtol=1e-9, atol=1e-12 * max(1.0, np.abs(tg).max()))
    assert np.abs(tg).max() > 0


def test_sample_below_floor_has_loss_but_no_gradient():
    b, p, target, model = tiny_case(2)
    p.b3[0] = -50.0                                   # every estimate far below zero
    loss, y, g = ot.loss_and_gradients(b, target, p, floor=1e-3)
    assert (y < 0).all()
    assert loss == pytest.approx(np.mean((np.log(1e-3) - np.log(target)) ** 2), rel=1e-13)
    assert not g.flat().any()


def test_flipped_unit_is_the_derivative_from_the_other_side():
    # put one pre-activation a hair above zero, then a hair below: the gradient just below equals
    # the gradient just above with that unit's ReLU derivative flipped, and the two differ clearly
    b, p, target, model = tiny_case(4)
    l, row, col = 1, 3, 2
    _, c = ot.forward(b, p)
    Z = np.concatenate([c["hs"][l], c["mps"][l], c["mss"][l]], axis=1) @ p.W[l] + p.b[l]
    # moving the bias moves the whole column; the probed unit is the only one that crosses zero
    others = np.delete(Z[:, col], row)
    assert np.abs(others - Z[row, col]).min() > 1e-6
    base = p.b[l][col] - Z[row, col]
    p.b[l][col] = base + 1e-11
    assert ot.undecided_units(b, p, 1e-9) == [(l, row, col)]
    _, _, g_above = ot.loss_and_gradients(b, target, p)
    _, _, g_above_flipped = ot.loss_and_gradients(b, target, p, flip=[(l, row, col)])
    p.b[l][col] = base - 1e-11
    _, _, g_below = ot.loss_and_gradients(b, target, p)
    scale = np.abs(g_below.flat()).max()
    assert np.abs(g_above_flipped.flat() - g_below.flat()).max() < 1e-8 * scale
    assert np.abs(g_above.flat() - g_below.flat()).max() > 1e-4 * scale


def test_adam_constant_gradient_closed_form():
    # with the same gradient at every step the bias-corrected moments are g and g^2: each step
    # moves by lr * g / (|g| + eps), whatever the betas
    g = np.array([0.3, -2.0, 1e-4, 0.0])
    th, m, v = np.zeros(4), np.zeros(4), np.zeros(4)
    for t in range(1, 8):
        th, m, v = ot.adam_step(th, g, m, v, t, 0.01, 0.9, 0.999, 1e-8)
        np.testing.assert_allclose(th, -t * 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12, atol=0)


def test_adam_against_library():
    rng = np.random.default_rng(0)
    th0 = rng.normal(size=50)
    gs = rng.normal(size=(6, 50)) * np.exp(rng.normal(size=(6, 50)) * 3)
    tp = torch.tensor(th0.copy(), requires_grad=True)
    opt = torch.optim.Adam([tp], lr=3e-3, betas=(0.8, 0.95), eps=1e-6)
    th, m, v = th0.copy(), np.zeros(50), np.zeros(50)
    for t, g in enumerate(gs, start=1):
        tp.grad = torch.tensor(g.copy())
        opt.step()
        th, m, v = ot.adam_step(th, g, m, v, t, 3e-3, 0.8, 0.95, 1e-6)
        np.testing.assert_allclose(th, tp.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_training_lowers_the_loss_on_fused_op_samples():
    b, p, target, model = fused_case(1)
    trained, losses = ot.train([b] * 30, [target] * 30, p, model.F, model.H, model.L, lr=2e-3)
    assert losses[-1] < 0.5 * losses[0]
    final, _, _ = ot.loss_and_gradients(b, target, trained)
    assert final < losses[0]


def test_training_labels_are_disjoint_connected_samples():
    base = wl.make("cfg2", 1)
    g = base.graphs[0]
    lab = wl.training_labels(g, 9, 3, kmax=16)
    assert (lab[:, g.n_op:] == np.arange(g.n_op, g.n)).all()      # all-reduce nodes stay single
    src = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    for c in range(3):
        ids, cnt = np.unique(lab[c], return_counts=True)
        assert (cnt >= 2).sum() > 10
        for gid in ids[cnt >= 2]:
            mem = np.nonzero(lab[c] == gid)[0]
            assert gid == mem.min()
            # grown along predecessor edges: weakly connected through edges inside the group
            inside = np.isin(src, mem) & np.isin(g.col, mem)
            reach, frontier = {int(mem[0])}, [int(mem[0])]
            adj = {}
            for u, v in zip(src[inside], g.col[inside]):
                adj.setdefault(int(u), []).append(int(v))
                adj.setdefault(int(v), []).append(int(u))
            while frontier:
                x = frontier.pop()
                for y in adj.get(x, []):
                    if y not in reach:
                        reach.add(y)
                        frontier.append(y)
            assert len(reach) == mem.size
