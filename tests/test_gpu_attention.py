"""GPU parity of the attention variant of the estimator (Sec. 3.3.1 with attention
coefficients, graph-attention reading) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}     # against the plain oracle (fp32 storage, fp64 accumulation)
MIRROR_TOL = 6e-3                      # bf16 path against the oracle with the same bf16 storage points


def check(got, w, tag):
    want = orc.evaluate(w)
    err = rel_err(got, want)
    print(f"[attention] {tag} max rel err vs plain oracle {err.max():.3e}", flush=True)
    assert err.max() <= TOL[w.model.dtype]
    if w.model.dtype == "bf16":
        err = rel_err(got, orc.evaluate(w, bf16=True))
        print(f"[attention] {tag} max rel err vs oracle with bf16 storage points {err.max():.3e}", flush=True)
        assert err.max() <= MIRROR_TOL


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_12769_amd import binding
    binding.lib()
    return binding


def rel_err(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    floor = 1e-3 * float(np.median(np.abs(ref))) if ref.size else 0.0
    return np.abs(got - ref) / np.maximum(np.maximum(np.abs(ref), floor), 1e-30)


def run(B, w):
    ev = B.evaluator_for(w)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    pred = ev.eval_candidates(cg, co, gid).cpu().numpy()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    again = ev.eval_candidates(cg, co, gid).cpu().numpy()
    assert np.array_equal(pred, again)
    ev.close()
    return pred


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F,H,L,K", [(16, 32, 2, 4), (32, 64, 1, 2), (16, 128, 2, 8), (64, 256, 2, 4), (16, 512, 1, 1),
                                     (48, 64, 3, 8)])
def test_small_batches_every_width(B, dtype, F, H, L, K):
    g = wl.random_dag(7, 300, 0.02, F)
    labs = wl.random_labels(8, g.n, 90, C=7)
    w = wl.custom(f"att-{dtype}-{F}-{H}-{L}-{K}", wl.ModelSpec(F, H, L, dtype, "attention", K), [g], [labs], seed=3)
    if dtype == "bf16":
        # random signed weights let the last dot product cancel to a hundredth of its terms, where bf16
        # storage alone (the oracle with bf16 storage points against the plain one) is 3e-2 off; the
        # 2e-2 bound is about predictions that are sums of like-signed terms, as times are
        w = wl.with_time_like_head(w)
    check(run(B, w), w, w.name)


def test_long_neighbour_lists_and_two_cycles(B):
    # few groups on a dense graph: lists far longer than a lane group, neighbours that are both
    # predecessor and successor
    g = wl.random_dag(11, 500, 0.05, 16)
    labs = np.concatenate([wl.random_labels(12, g.n, 6, C=2), wl.random_labels(13, g.n, 60, C=2)])
    w = wl.custom("att-dense", wl.ModelSpec(16, 64, 2, "f32", "attention", 4), [g], [labs], seed=5)
    got = run(B, w)
    want = orc.evaluate(w)
    assert rel_err(got, want).max() <= TOL["f32"]


def test_zero_attention_vectors_equal_uniform_coefficients(B):
    g = wl.random_dag(17, 200, 0.03, 16)
    labs = wl.random_labels(18, g.n, 70, C=3)
    w = wl.custom("att-zero", wl.ModelSpec(16, 64, 2, "f32", "attention", 4), [g], [labs], seed=6)
    w.weights.att[:] = 0.0
    got = run(B, w)
    want = orc.evaluate(w)
    assert rel_err(got, want).max() <= TOL["f32"]


@pytest.mark.parametrize("name,n,heads", [("cfg1", 3, 4), ("cfg2", 64, 4), ("cfg3", 48, 8), ("cfg4", 12, 4)])
def test_configurations_with_attention(B, name, n, heads):
    w = wl.with_attention(wl.make(name, n), heads)
    check(run(B, w), w, f"{w.name} C={w.n_cand}")


def test_config_errors(B):
    for H, K in [(48, 4), (64, 3), (64, 16), (1024, 4)]:
        cfg = B.DcConfig(16, H, 1, B.DC_F32, 4, 100, 100, 0, 0, B.DC_AGG_ATTENTION, K)
        st, h = B.dc_create(cfg)
        assert st in (B.DC_ERR_UNSUPPORTED, B.DC_ERR_INVALID_ARG) and not h
    # the two weight calls are tied to the kind of context
    ev = B.Evaluator(16, 32, 1, "f32", 4, 100, 100)
    z = np.zeros(3 * 16 * 32 + 4 * 32 * 32 + 1000, np.float32)
    assert B.dc_set_attention_weights(ev.ctx, z, z, z, z) == B.DC_ERR_INVALID_ARG
    ev.close()
    ev = B.Evaluator(16, 32, 1, "f32", 4, 100, 100, agg="attention", heads=2)
    assert B.dc_set_weights(ev.ctx, z, z, z) == B.DC_ERR_INVALID_ARG
    ev.close()
