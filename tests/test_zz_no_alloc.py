"""dc_simulate_static, the simulator entry point that allocates nothing (for callers under graph
capture or in loops that must not call hipMalloc), against dc_simulate through the C ABI: the same
costs bit for bit on two calls in a row, the second on a smaller batch, with modules that are walked
in LDS and modules that are walked in the library's own device array."""
import numpy as np
import pytest

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


def batch_with_large_and_small_modules(n_cand):
    """cfg4's module under fusion strategies that leave it nearly unfused (6.5 k nodes: too large for LDS,
    walked in global memory) next to ordinary candidates (1.4 k nodes, walked in LDS)."""
    w = wl.make("cfg4", n_cand)
    g = w.graphs[0]
    labs = w.group_id.reshape(n_cand, g.n).copy()
    labs[::3] = np.arange(g.n, dtype=np.int32)             # every third candidate: the unfused module
    labs[1::6, :200] = labs[1::6, 0:1]                     # and some with one large group in front
    return wl.custom("static", w.model, w.graphs, [labs], seed=0)


def run_both(B, w, ev):
    import torch
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    nb = int(w.cand_off[-1])
    eb = w.n_cand * w.graphs[0].e
    batch = ev.alloc_batch(w.n_cand, nb, nb, eb)
    ev.contract_graphs(cg, co, gid, batch)
    ntot, etot = ev.last_totals()
    Xc = batch.Xc[:ntot].float()
    is_ar = Xc[:, 1] > 0
    ar_size = torch.where(is_ar, Xc[:, 0], torch.full_like(Xc[:, 0], -1.0)).contiguous()
    op_time = torch.where(is_ar, torch.zeros_like(Xc[:, 2]), 0.05 + Xc[:, 2]).contiguous()
    want = ev.simulate(batch, op_time, ar_size, 0.02, 0.01).clone()
    assert ev.check() == B.DC_OK
    got = torch.full((w.n_cand,), -7.0, dtype=torch.float32, device=ev.device)
    st_dev = torch.full((1,), -1, dtype=torch.int32, device=ev.device)
    sizes = np.diff(batch.node_off.cpu().numpy()[:w.n_cand + 1])
    esizes = np.diff(batch.edge_off.cpu().numpy()[:w.n_cand + 1])
    st = B.dc_simulate_static(batch.c, int(sizes.max()), int(esizes.max()), op_time.data_ptr(), ar_size.data_ptr(),
                              0.02, 0.01, got.data_ptr(), st_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == B.DC_OK, B.dc_simulate_static_error()
    torch.cuda.synchronize()
    assert int(st_dev.item()) == B.DC_OK
    assert torch.equal(got, want), (got - want).abs().max()
    assert torch.isfinite(want).all()
    return int(sizes.max()), int((24 * sizes + 2 * esizes).max())


def test_static_simulator_equals_the_context_one_on_two_calls_in_a_row(B):
    big = batch_with_large_and_small_modules(48)
    small = big.subset(range(5, 16))
    ev = B.evaluator_for(big)
    largest, need = run_both(B, big, ev)
    assert largest > 6000 and need > 80 * 1024          # the global-memory walk was exercised
    run_both(B, small, ev)                              # second call, smaller input, same device array
    run_both(B, big, ev)
    ev.close()


def test_static_simulator_rejects_modules_beyond_its_limit_on_the_host(B):
    w = wl.make("cfg2", 2)
    ev = B.evaluator_for(w)
    batch = ev.alloc_batch(2, 10, 10, 10)
    st = B.dc_simulate_static(batch.c, 20000, 40000, 1, 1, 0.0, 0.0, 1, None, 0)
    assert st == B.DC_ERR_CAPACITY and "256 KiB" in B.dc_simulate_static_error()
    assert B.dc_simulate_static(batch.c, 70000, 10, 1, 1, 0.0, 0.0, 1, None, 0) == B.DC_ERR_CAPACITY
    assert B.dc_simulate_static(batch.c, -1, 10, 1, 1, 0.0, 0.0, 1, None, 0) == B.DC_ERR_INVALID_ARG
    ev.close()
