"""GPU parity of the list-scheduling simulator (Sec. 3.4) against the CPU oracle, through the
C ABI.  Both sides add fp64 times in the order the rules fix, so the costs must agree bit for bit."""
import numpy as np
import pytest

from oracle import oracle as orc
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


def times_of(ref, F):
    """Synthetic per-node inputs from the contracted features: all-reduce nodes are those whose
    kind column (feature 1) is positive, their size is the summed size column (feature 0, MiB);
    computation nodes take 0.05 + the sum of their members' third feature as execution time."""
    is_ar = ref.Xc[:, 1] > 0
    ar_size = np.where(is_ar, ref.Xc[:, 0], -1.0).astype(np.float32)
    op_time = np.where(is_ar, 0.0, 0.05 + ref.Xc[:, 2]).astype(np.float32)
    return op_time, ar_size


def run(B, w, ref, op_time, ar_size, c, d):
    import torch
    ev = B.evaluator_for(w)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    nb = int(w.cand_off[-1])
    geo = w.g_edge_off()
    eb = int(sum(int(geo[b + 1] - geo[b]) for b in w.cand_graph))
    batch = ev.alloc_batch(w.n_cand, nb, nb, eb)
    ev.contract_graphs(cg, co, gid, batch)
    t = torch.from_numpy(op_time).to(ev.device)
    x = torch.from_numpy(ar_size).to(ev.device)
    cost = ev.simulate(batch, t, x, c, d).cpu().numpy()
    st = ev.check()
    again = ev.simulate(batch, t, x, c, d).cpu().numpy()
    assert np.array_equal(cost, again)
    ev.close()
    return cost, st


@pytest.mark.parametrize("name,n", [("cfg1", 5), ("cfg2", 256), ("cfg3", 128), ("cfg4", 64)])
def test_configurations(B, name, n):
    w = wl.make(name, n)
    ref = orc.contract(w, False)
    op_time, ar_size = times_of(ref, w.model.F)
    if name == "cfg1":                       # cfg1's features are all uniform noise: mark its 8 sinks by hand
        deg_out = np.diff(ref.out_rowptr)
        ar_size = np.where(deg_out == 0, ref.Xc[:, 0] * 10, -1.0).astype(np.float32)
        op_time = (0.05 + ref.Xc[:, 2]).astype(np.float32)
    assert (ar_size >= 0).any() and (ar_size < 0).any()
    for c, d in ((0.02, 0.01), (0.5, 0.3)):
        want = orc.simulate(ref, op_time, ar_size, c, d)
        got, st = run(B, w, ref, op_time, ar_size, c, d)
        assert st == B.DC_OK
        assert np.array_equal(got, want), (name, c, d, np.abs(got - want).max())
    print(f"[simulate] {name} C={w.n_cand} cost range {want.min():.3f} .. {want.max():.3f}", flush=True)


def test_cycles_give_infinity_and_large_graphs_use_the_global_path(B):
    # arbitrary partitions of a dense DAG: most quotients are cyclic; the identity partition is not
    g = wl.random_dag(11, 700, 0.02, 16)
    labs = np.concatenate([np.arange(g.n, dtype=np.int32).reshape(1, -1), wl.random_labels(12, g.n, 300, C=2),
                           wl.random_labels(13, g.n, 650, C=2)])
    w = wl.custom("sim-cyc", wl.ModelSpec(16, 32, 1, "f32"), [g], [labs], seed=1)
    ref = orc.contract(w, False)
    rng = wl.Rng(5, 11)
    op_time = (rng.uniform(ref.ntot) + 0.1).astype(np.float32)
    ar_size = np.where(rng.uniform(ref.ntot) < 0.2, rng.uniform(ref.ntot) * 8, -1.0).astype(np.float32)
    want = orc.simulate(ref, op_time, ar_size, 0.25, 0.05)
    assert np.isinf(want).any() and np.isfinite(want).any()
    got, st = run(B, w, ref, op_time, ar_size, 0.25, 0.05)
    assert st == B.DC_OK
    assert np.array_equal(got, want)
    # a contracted graph of several thousand nodes does not fit the 80 KB a wave has on chip: same
    # result through slices of global memory (identity and coarse partitions of a 5000-node DAG)
    gb = wl.random_dag(23, 5000, 0.0006, 16)
    labsb = np.concatenate([np.arange(gb.n, dtype=np.int32).reshape(1, -1), wl.random_labels(24, gb.n, 4000, C=1),
                            wl.random_labels(25, gb.n, 900, C=1)])
    big = wl.custom("sim-big", wl.ModelSpec(16, 32, 1, "f32"), [gb], [labsb], seed=1)
    refb = orc.contract(big, False)
    need = [24 * int(refb.node_off[c + 1] - refb.node_off[c]) + 2 * int(refb.edge_off[c + 1] - refb.edge_off[c])
            for c in range(big.n_cand)]
    assert max(need) > 80 * 1024 > min(need)
    rng = wl.Rng(6, 11)
    t2 = (rng.uniform(refb.ntot) + 0.1).astype(np.float32)
    x2 = np.where(rng.uniform(refb.ntot) < 0.15, rng.uniform(refb.ntot) * 8, -1.0).astype(np.float32)
    wantb = orc.simulate(refb, t2, x2, 0.1, 0.02)
    assert np.isfinite(wantb).any()
    gotb, st = run(B, big, refb, t2, x2, 0.1, 0.02)
    assert st == B.DC_OK
    assert np.array_equal(gotb, wantb)
