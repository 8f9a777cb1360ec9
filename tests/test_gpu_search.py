"""GPU parity of the backtracking search (Alg. 1) against the CPU oracle's search, through the
C ABI.  The search takes decisions on floating-point costs, so the comparison of whole runs uses
estimators whose output is exact on both sides (zero matrices, the prediction is the last bias):
every cost is then a sum of fp32 inputs accumulated in fp64 in a fixed order, identical bit for
bit, and the two searches must take the same path: same counters, same best cost, same H_opt.
With a real estimator the paths may part where two costs are within the estimator's tolerance;
there the result is checked on its own: H_opt costed by the oracle agrees with the reported cost."""
import numpy as np
import pytest

from oracle import oracle as orc
from oracle import search as osr
from paper_2209_12769_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_12769_amd import binding
    binding.lib()
    return binding


def constant_estimator(model, value):
    wt = wl.make_weights(model, 0)
    return wl.Weights(np.zeros_like(wt.layers), np.zeros_like(wt.biases),
                      np.concatenate([np.zeros(wt.head.size - 1, np.float32), [np.float32(value)]]), wt.att)


def oracle_cost_fn(g, model, weights, t, x, c, d):
    def f(labels):
        w = wl.custom("s", model, [g], [np.asarray(labels, np.int32)], weights=weights)
        return orc.cost(w, t, x, c, d)
    return f


def gpu_search(B, g, model, weights, t, x, parents, **kw):
    ident = np.tile(np.arange(g.n, dtype=np.int32), (2 * parents, 1))
    w = wl.custom("s", model, [g], [ident], weights=weights)        # sizes the context for 2 * parents candidates
    ev = B.evaluator_for(w)
    ev.set_profile(t, x)
    labels, r = ev.search(0, g.n, parents=parents, **kw)
    ev.close()
    return labels, r


def same_run(r, ref, labels, tag):
    got = (r.cost_in, r.cost_opt, r.steps, r.evaluated, r.valid, r.enqueued, r.improved)
    want = (np.float32(ref.cost_in), np.float32(ref.cost_opt), ref.steps, ref.evaluated, ref.valid, ref.enqueued,
            ref.improved)
    assert got == want, (tag, got, want)
    assert np.array_equal(labels, ref.labels_opt), tag


@pytest.mark.parametrize("name,est,alpha,beta,parents,limit", [
    ("cfg1", 0.04, 1.05, 4, 1, 60), ("cfg1", 0.04, 1.2, 6, 8, 150), ("cfg2", 0.03, 1.02, 8, 16, 200),
    ("cfg3", 0.02, 1.01, 12, 8, 100)])
def test_same_path_as_the_oracle_with_an_exact_estimator(B, name, est, alpha, beta, parents, limit):
    base = wl.make(name, 1)
    g, model = base.graphs[0], base.model
    wt = constant_estimator(model, est)
    t, x = wl.profile_of(base)
    kw = dict(alpha=alpha, beta=beta, seed=5, max_unchanged=limit, max_steps=40)
    ref = osr.search(g, oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01), parents=parents, **kw)
    labels, r = gpu_search(B, g, model, wt, t, x, parents, ar_c=0.02, ar_d=0.01, **kw)
    same_run(r, ref, labels, name)
    assert r.improved >= 1 and r.cost_opt < r.cost_in
    print(f"[search] {name} P={parents}: {r.evaluated} evaluated, {r.valid} valid, cost {r.cost_in:.4f} -> "
          f"{r.cost_opt:.4f}, {len(np.unique(labels))} groups of {g.n}", flush=True)


@pytest.mark.parametrize("name,est,alpha,beta,parents,limit", [
    ("cfg1", 0.04, 1.05, 4, 1, 60), ("cfg1", 0.04, 1.2, 6, 8, 150), ("cfg2", 0.03, 1.02, 8, 16, 200)])
def test_same_path_as_the_oracle_with_the_papers_op_draw(B, name, est, alpha, beta, parents, limit):
    """Method (i) as the paper words it: an op of the current module, then one of its current predecessors."""
    base = wl.make(name, 1)
    g, model = base.graphs[0], base.model
    wt = constant_estimator(model, est)
    t, x = wl.profile_of(base)
    kw = dict(alpha=alpha, beta=beta, seed=7, max_unchanged=limit, max_steps=30)
    ref = osr.search(g, oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01), parents=parents, op_draw="op", **kw)
    labels, r = gpu_search(B, g, model, wt, t, x, parents, ar_c=0.02, ar_d=0.01, op_draw=B.DC_DRAW_OP, **kw)
    same_run(r, ref, labels, name)
    other = osr.search(g, oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01), parents=parents, **kw)
    assert not np.array_equal(other.labels_opt, ref.labels_opt) or other.evaluated != ref.evaluated   # the draws differ
    assert r.improved >= 1 and r.cost_opt < r.cost_in
    print(f"[search, op draw] {name} P={parents}: {r.evaluated} evaluated, {r.valid} valid, cost {r.cost_in:.4f} -> "
          f"{r.cost_opt:.4f}, {len(np.unique(labels))} groups of {g.n}", flush=True)


def test_queue_limit_and_beta_zero(B):
    base = wl.make("cfg1", 1)
    g, model = base.graphs[0], base.model
    wt = constant_estimator(model, 0.04)
    t, x = wl.profile_of(base)
    f = oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01)
    kw = dict(alpha=1.3, beta=3, seed=9, max_unchanged=80, max_steps=25)
    ref = osr.search(g, f, parents=4, max_queue=5, **kw)
    labels, r = gpu_search(B, g, model, wt, t, x, 4, ar_c=0.02, ar_d=0.01, max_queue=5, **kw)
    same_run(r, ref, labels, "max_queue")
    assert r.queued <= 5
    kw = dict(alpha=1.0, beta=0, seed=3, max_unchanged=11)
    ref = osr.search(g, f, parents=1, **kw)
    labels, r = gpu_search(B, g, model, wt, t, x, 1, ar_c=0.02, ar_d=0.01, **kw)
    same_run(r, ref, labels, "beta0")
    assert r.evaluated == 12 and np.array_equal(labels, np.arange(g.n))


@pytest.mark.parametrize("name,tol", [("cfg2", 1e-5), ("cfg3", 2e-2)])
def test_result_with_a_real_estimator_stands_on_its_own(B, name, tol):
    base = wl.make(name, 1)
    g, model = base.graphs[0], base.model
    wt = base.weights
    wt.head[-1] += 0.3
    t, x = wl.profile_of(base)
    labels, r = gpu_search(B, g, model, wt, t, x, 16, alpha=1.05, beta=8, seed=2, ar_c=0.02, ar_d=0.01,
                           max_unchanged=300, max_steps=12)
    assert r.cost_opt <= r.cost_in and 0 < r.valid <= r.evaluated
    f = oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01)
    want_in = f(np.arange(g.n, dtype=np.int32).reshape(1, -1))[0]
    want_opt = f(labels.reshape(1, -1))[0]
    assert abs(r.cost_in - want_in) <= tol * want_in
    assert abs(r.cost_opt - want_opt) <= tol * want_opt
    print(f"[search] {name} real estimator: cost {r.cost_in:.4f} -> {r.cost_opt:.4f} in {r.steps} steps", flush=True)


@pytest.mark.timeout(300)
def test_largest_base_graph(B):
    # 65535 nodes: the mutation kernel keeps 128 KB of labels in LDS, the modules walk in global memory
    from test_gpu_parity import largest_graph
    g = largest_graph(16)
    model = wl.ModelSpec(16, 32, 1, "f32")
    wt = constant_estimator(model, 0.03)
    base = wl.custom("largest", model, [g], [np.arange(g.n, dtype=np.int32).reshape(1, g.n)], weights=wt)
    t, x = wl.profile_of(base)
    kw = dict(alpha=1.01, beta=40, seed=4, max_unchanged=1000, max_steps=4)
    ref = osr.search(g, oracle_cost_fn(g, model, wt, t, x, 0.02, 0.01), parents=2, **kw)
    labels, r = gpu_search(B, g, model, wt, t, x, 2, ar_c=0.02, ar_d=0.01, **kw)
    same_run(r, ref, labels, "largest")
    assert r.evaluated >= 8 and r.valid >= 1


def test_bad_arguments(B):
    base = wl.make("cfg1", 2)
    t, x = wl.profile_of(base)
    ev = B.evaluator_for(base)
    with pytest.raises(B.DiscoError) as e:
        ev.search(0, 72, alpha=1.1, beta=2, seed=0, ar_c=0.1, ar_d=0.1)
    assert e.value.status == B.DC_ERR_INVALID_ARG            # no profile
    ev.set_profile(t, x)
    for kw, want in ((dict(alpha=0.9), B.DC_ERR_INVALID_ARG), (dict(beta=-1), B.DC_ERR_INVALID_ARG),
                     (dict(op_draw=2), B.DC_ERR_INVALID_ARG),
                     (dict(parents=0), B.DC_ERR_INVALID_ARG), (dict(parents=2), B.DC_ERR_CAPACITY)):
        args = dict(alpha=1.1, beta=2, seed=0, ar_c=0.1, ar_d=0.1, parents=1)
        args.update(kw)
        with pytest.raises(B.DiscoError) as e:
            ev.search(0, 72, **args)
        assert e.value.status == want, kw
    with pytest.raises(B.DiscoError) as e:
        ev.search(3, 72, alpha=1.1, beta=2, seed=0, ar_c=0.1, ar_d=0.1)
    assert e.value.status == B.DC_ERR_INVALID_ARG
    ev.close()
