"""GPU parity of the Cost(H) composition (Secs. 3.1, 3.3, 3.4) against the CPU oracle, through
the C ABI: times and tensor sizes of every node of the candidate modules (dc_module_times) and
the end-to-end time (dc_cost_candidates).

Tensor sizes, profiled times and the classification of every node are exact; the estimate of a
fused op is floating point (rel 1e-5 fp32, 2e-2 bf16 against the plain oracle -- fp32 storage,
fp64 accumulation -- measured against max(|estimate|, 1e-3 of the median estimate); the bf16 path
is held to a tighter bound against the oracle run with the device's bf16 storage points).  The schedule's order does not depend on the durations, so the cost is a
fixed max-plus expression of them and inherits their relative tolerance."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}     # against the plain oracle
MIRROR_TOL = 8e-3                      # bf16 path against the oracle with bf16 storage points.  The device also rounds
                                       # the per-fused-op sums and the regression network's hidden layers to bf16, which
                                       # that oracle mode does not: measured 5.7e-3 on the configurations


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2209_12769_amd import binding
    binding.lib()
    return binding


def positive(w):
    """The same workload with the last bias of the regression network raised by one, so that
    most estimates are positive and the clamp at zero does not hide them."""
    wt = w.weights
    head = wt.head.copy()
    head[-1] += 1.0
    return wl.Workload(w.name, w.model, w.graphs, w.cand_graph, w.cand_off, w.group_id,
                       wl.Weights(wt.layers, wt.biases, head, wt.att), w.note)


def sizes(w):
    nb = int(w.cand_off[-1])
    geo = w.g_edge_off()
    eb = int(sum(int(geo[b + 1] - geo[b]) for b in w.cand_graph))
    return nb, eb


def gpu_module_times(B, w, t, x, which=0):
    """-> op_time, ar_size, node_off, (fused ops the estimator ran on, their rows, their edges), fused ops that
    repeated one of those, status"""
    ev = B.evaluator_for(w)
    ev.select_kernels(which)
    ev.set_profile(t, x)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    nb, eb = sizes(w)
    batch = ev.alloc_batch(w.n_cand, nb, nb, eb)
    op_time, ar_size = ev.module_times(cg, co, gid, batch)
    st = ev.check()
    ntot, _ = ev.last_totals()
    counts = ev.last_fused_ops()
    repeats = ev.last_fused_op_repeats()
    out = (op_time[:ntot].cpu().numpy(), ar_size[:ntot].cpu().numpy(), batch.node_off.cpu().numpy(), counts, repeats, st)
    ev.close()
    return out


def distinct_fused_ops(w, ref_b, fo, cnode):
    """Fused ops of the batch up to repetition (same base graph, same members): how many there are, their rows,
    their edges, and how many fused ops repeat an earlier one."""
    cand = np.searchsorted(ref_b.node_off, cnode, side="right") - 1
    seen = set()
    K = M = E = 0
    for k in range(fo.n_cand):
        key = (int(w.cand_graph[cand[k]]), fo.new_id[fo.node_off[k]:fo.node_off[k + 1]].tobytes())
        if key not in seen:
            seen.add(key)
            K += 1
            M += int(fo.node_off[k + 1] - fo.node_off[k])
            E += int(fo.edge_off[k + 1] - fo.edge_off[k])
    return (K, M, E), fo.n_cand - K


def gpu_cost(B, w, t, x, c, d):
    ev = B.evaluator_for(w)
    ev.set_profile(t, x)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    cost = ev.cost_candidates(cg, co, gid, c, d).cpu().numpy()
    st = ev.check()
    again = ev.cost_candidates(cg, co, gid, c, d).cpu().numpy()
    assert np.array_equal(cost, again, equal_nan=True)
    ev.close()
    return cost, st


def check_times(w, got_t, got_x, ref_b, t, x, mirror=True):
    want_t, want_x, fo, cnode, fo_pred = orc.module_times(w, ref_b, t, x, want_fused=True)
    assert np.array_equal(got_x, want_x)
    fused = np.zeros(ref_b.ntot, bool)
    fused[cnode] = True
    assert np.array_equal(got_t[~fused], want_t[~fused])
    if fo.n_cand:
        floor = 1e-3 * float(np.median(np.abs(fo_pred)))
        scale = np.maximum(np.abs(fo_pred), floor)
        err = np.abs(got_t[cnode] - want_t[cnode]) / scale
        assert err.max() <= TOL[w.model.dtype], (w.name, err.max(), int(err.argmax()))
        if w.model.dtype == "bf16" and mirror:
            mir_t = orc.module_times(w, ref_b, t, x, bf16=True)[0]
            merr = np.abs(got_t[cnode] - mir_t[cnode]) / scale
            print(f"[module_times] {w.name} max rel err vs oracle with bf16 storage points {merr.max():.2e}", flush=True)
            assert merr.max() <= MIRROR_TOL, (w.name, merr.max())
        return float(err.max()), fo, fo_pred
    return 0.0, fo, fo_pred


@pytest.mark.parametrize("name,n", [("cfg1", 5), ("cfg2", 48), ("cfg3", 40), ("cfg4", 12), ("cfg5", 12)])
def test_module_times_of_the_configurations(B, name, n):
    w = positive(wl.make(name, n, n_graphs=12) if name == "cfg5" else wl.make(name, n))
    t, x = wl.profile_of(w)
    ref_b = orc.contract(w)
    got_t, got_x, node_off, counts, repeats, st = gpu_module_times(B, w, t, x)
    assert st == B.DC_OK
    assert np.array_equal(node_off, ref_b.node_off)
    err, fo, fo_pred = check_times(w, got_t, got_x, ref_b, t, x)
    cnode = orc.module_times(w, ref_b, t, x, want_fused=True)[3]
    assert (counts, repeats) == distinct_fused_ops(w, ref_b, fo, cnode)
    assert np.mean(fo_pred > 0) > 0.5
    print(f"[module_times] {name} C={n}: {fo.n_cand} fused ops, {fo.ntot} rows, {fo.etot} edges, "
          f"max rel err {err:.2e}", flush=True)


@pytest.mark.parametrize("name,n", [("cfg1", 5), ("cfg2", 48), ("cfg3", 40), ("cfg4", 12)])
def test_cost_of_the_configurations(B, name, n):
    w = positive(wl.make(name, n))
    t, x = wl.profile_of(w)
    for c, d in ((0.02, 0.01), (0.5, 0.3)):
        want = orc.cost(w, t, x, c, d)
        got, st = gpu_cost(B, w, t, x, c, d)
        assert st == B.DC_OK
        assert np.all(np.isfinite(want)) and np.all(np.isfinite(got))
        err = np.abs(got - want) / np.abs(want)
        assert err.max() <= TOL[w.model.dtype], (name, c, d, err.max())
        if w.model.dtype == "bf16":
            mir = orc.cost(w, t, x, c, d, bf16=True)
            assert np.max(np.abs(got - mir) / np.abs(mir)) <= MIRROR_TOL
    print(f"[cost] {name} C={n}: cost {want.min():.3f} .. {want.max():.3f}, max rel err {err.max():.2e}", flush=True)


def test_a_repeated_fused_op_takes_the_first_ones_estimate_bit_for_bit(B):
    """Fused ops of one batch with the same base graph and the same members are estimated once: the times of
    every node equal, bit for bit, those of a pass that runs the estimator on every fused op; the counts are
    those of the oracle's batch up to repetition.  Cases: candidates that share most groups (cfg4, cfg3),
    the same candidate three times over, and two base graphs with the same edges but other features under the
    same labels (equal member lists that must not be taken for each other)."""
    cases = [positive(wl.make("cfg4", 24)), positive(wl.make("cfg3", 40))]
    w3 = wl.make("cfg3", 2)
    n = w3.graphs[0].n
    lab = w3.group_id.reshape(2, n)
    cases.append(positive(wl.custom("thrice", w3.model, w3.graphs, [np.concatenate([lab[:1]] * 3 + [lab[1:]])])))
    g0 = w3.graphs[0]
    g1 = wl.BaseGraph(g0.n, g0.n_op, g0.rowptr, g0.col, (g0.X[::-1] * 0.5 + 0.25).astype(np.float32).copy())
    cases.append(positive(wl.custom("twins", w3.model, [g0, g1], [lab, lab])))
    for w in cases:
        t, x = wl.profile_of(w)
        ref_b = orc.contract(w)
        once = gpu_module_times(B, w, t, x)
        every = gpu_module_times(B, w, t, x, B.DC_KERNELS_EVERY_FUSED_OP)
        assert once[5] == B.DC_OK and every[5] == B.DC_OK
        assert np.array_equal(once[0], every[0]) and np.array_equal(once[1], every[1]), w.name
        _, _, fo, cnode, _ = orc.module_times(w, ref_b, t, x, want_fused=True)
        assert every[3] == (fo.n_cand, fo.ntot, fo.etot) and every[4] == 0
        want = distinct_fused_ops(w, ref_b, fo, cnode)
        assert (once[3], once[4]) == want, (w.name, once[3], once[4], want)
        print(f"[repeats] {w.name}: {fo.n_cand} fused ops, {want[0][0]} up to repetition", flush=True)
        if w.name == "thrice":
            assert want[1] >= 2 * (fo.n_cand // 4)
        if w.name == "twins":
            assert want[0][0] >= 2 * len({fo.new_id[fo.node_off[k]:fo.node_off[k + 1]].tobytes() for k in range(fo.n_cand)}) - 0
        c_once, st1 = gpu_cost(B, w, t, x, 0.02, 0.01)
        ev = B.evaluator_for(w)
        ev.select_kernels(B.DC_KERNELS_EVERY_FUSED_OP)
        ev.set_profile(t, x)
        c_every = ev.cost_candidates(ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id),
                                     0.02, 0.01).cpu().numpy()
        assert ev.check() == B.DC_OK and st1 == B.DC_OK
        ev.close()
        assert np.array_equal(c_once, c_every, equal_nan=True), w.name


def test_cost_is_the_simulator_on_the_module_times(B):
    import torch
    w = positive(wl.make("cfg3", 24))
    t, x = wl.profile_of(w)
    ev = B.evaluator_for(w)
    ev.set_profile(t, x)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    nb, eb = sizes(w)
    batch = ev.alloc_batch(w.n_cand, nb, nb, eb)
    op_time, ar_size = ev.module_times(cg, co, gid, batch)
    two_step = ev.simulate(batch, op_time, ar_size, 0.02, 0.01).cpu().numpy()
    one_call = ev.cost_candidates(cg, co, gid, 0.02, 0.01).cpu().numpy()
    assert ev.check() == B.DC_OK
    assert np.array_equal(two_step, one_call)
    # and the simulator's own parity: the oracle on the device's times gives the same bits
    ref_b = orc.contract(w)
    ntot = ref_b.ntot
    want = orc.simulate(ref_b, op_time[:ntot].cpu().numpy(), ar_size[:ntot].cpu().numpy(), 0.02, 0.01)
    assert np.array_equal(one_call, want)
    ev.close()


@pytest.mark.timeout(300)
def test_full_size_batch_sampled_and_deterministic(B):
    # the launch `bench.py --cost` times: 4096 candidates of cfg4 through dc_cost_candidates; sampled
    # candidates against the oracle, the whole vector against a second run (inside gpu_cost)
    w = positive(wl.make("cfg4", 4096))
    t, x = wl.profile_of(w)
    got, st = gpu_cost(B, w, t, x, 0.02, 0.01)
    assert st == B.DC_OK and np.isfinite(got).all()
    sample = [0, 1777, 4095]
    want = orc.cost(w.subset(sample), t, x, 0.02, 0.01)
    err = np.abs(got[sample] - want) / np.abs(want)
    print(f"[cost full size] sampled max rel err {err.max():.2e}", flush=True)
    assert err.max() <= TOL["bf16"]


def test_cost_is_capturable_in_a_hip_graph_and_replays_identically(B):
    """dc_cost_candidates only enqueues kernels on the caller's stream (the sizes of the fused-op batch stay
    on the device), so it can be captured; every replay must reproduce the eager costs bit for bit."""
    import torch
    w = positive(wl.make("cfg3", 24))
    t, x = wl.profile_of(w)
    ev = B.evaluator_for(w)
    ev.set_profile(t, x)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    cost = torch.empty(w.n_cand, dtype=torch.float32, device=ev.device)
    eager = ev.cost_candidates(cg, co, gid, 0.02, 0.01, cost).clone()
    torch.cuda.synchronize()
    assert ev.check() == B.DC_OK
    side = torch.cuda.Stream(device=ev.device)
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ev.cost_candidates(cg, co, gid, 0.02, 0.01, cost)           # warm-up on the capture stream
        torch.cuda.current_stream().synchronize()
        with torch.cuda.graph(graph, stream=side):
            ev.cost_candidates(cg, co, gid, 0.02, 0.01, cost)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        cost.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(cost, eager), f"replay {rep}"
        again = ev.cost_candidates(cg, co, gid, 0.02, 0.01).clone()
        torch.cuda.synchronize()
        assert torch.equal(again, eager)
    assert ev.check() == B.DC_OK
    ev.close()


def test_attention_estimator(B):
    w = positive(wl.with_attention(wl.make("cfg3", 16), 4))
    t, x = wl.profile_of(w)
    ref_b = orc.contract(w)
    got_t, got_x, _, _, _, st = gpu_module_times(B, w, t, x)
    assert st == B.DC_OK
    err, fo, _ = check_times(w, got_t, got_x, ref_b, t, x)
    want = orc.cost(w, t, x, 0.02, 0.01)
    got, st = gpu_cost(B, w, t, x, 0.02, 0.01)
    assert st == B.DC_OK and np.max(np.abs(got - want) / np.abs(want)) <= TOL["bf16"]
    print(f"[module_times] attention: {fo.n_cand} fused ops, max rel err {err:.2e}", flush=True)


def edge_case_workload(dtype):
    """One random DAG of 300 ops and 12 tensors with: the all-singleton partition (no fused op),
    all ops in one group, one group that mixes an op with a tensor, arbitrary labels (cyclic
    quotients), and all tensors in one bucket."""
    n_op, n_ar = 300, 12
    g0 = wl.random_dag(77, n_op, 0.02, 32)
    rng = wl.Rng(77, 11)
    src = np.concatenate([np.repeat(np.arange(n_op), np.diff(g0.rowptr)), rng.integers(0, n_op - 1, n_ar)])
    dst = np.concatenate([g0.col, n_op + np.arange(n_ar)])
    rp, ci = wl._csr_from_edges(n_op + n_ar, src, dst)
    n = n_op + n_ar
    g = wl.BaseGraph(n, n_op, rp, ci, rng.uniform(n * 32).reshape(n, 32).astype(np.float32))
    labs = np.empty((6, n), np.int32)
    labs[0] = np.arange(n)
    labs[1] = np.arange(n)
    labs[1, :n_op] = 0
    labs[2] = np.arange(n)
    labs[2, n_op] = 5
    labs[3, :n_op] = wl.random_labels(5, n_op, 40, 1)[0]
    labs[3, n_op:] = np.arange(n_op, n)
    labs[4, :n_op] = wl.random_labels(6, n_op, 150, 1)[0]
    labs[4, n_op:] = n_op
    labs[5] = np.arange(n)
    labs[5, n_op:] = n - 1
    return positive(wl.custom("edge", wl.ModelSpec(32, 64, 2, dtype), [g], [labs], seed=3))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_cases(B, dtype):
    w = edge_case_workload(dtype)
    t, x = wl.profile_of(w)
    ref_b = orc.contract(w)
    got_t, got_x, _, counts, _, st = gpu_module_times(B, w, t, x)
    assert st == B.DC_OK
    # the sum over 300 member rows is rounded to bf16 before the regression network, a rounding point the
    # oracle's bf16 mode does not have: the bound against the plain oracle holds, the tighter one is not asked
    check_times(w, got_t, got_x, ref_b, t, x, mirror=False)
    want = orc.cost(w, t, x, 0.1, 0.05)
    got, st = gpu_cost(B, w, t, x, 0.1, 0.05)
    assert st == B.DC_OK
    assert np.array_equal(np.isinf(got), np.isinf(want))
    assert np.isinf(want[2]) and np.isfinite(want[0]) and np.isfinite(want[5])
    fin = np.isfinite(want)
    assert np.max(np.abs(got[fin] - want[fin]) / np.abs(want[fin])) <= TOL[dtype]
    assert got[0] == want[0]                 # no estimator involved: exact
    assert got[5] == want[5]


def test_no_fused_op_at_all(B):
    w = wl.make("cfg2", 3)
    n = w.graphs[0].n
    w = wl.custom("id", w.model, w.graphs, [np.tile(np.arange(n, dtype=np.int32), (3, 1))])
    t, x = wl.profile_of(w)
    got_t, got_x, _, counts, repeats, st = gpu_module_times(B, w, t, x)
    assert st == B.DC_OK and counts == (0, 0, 0) and repeats == 0
    assert np.array_equal(got_t, np.tile(t, 3)) and np.array_equal(got_x, np.tile(x, 3))
    got, st = gpu_cost(B, w, t, x, 0.02, 0.01)
    assert st == B.DC_OK and np.array_equal(got, orc.cost(w, t, x, 0.02, 0.01))


def test_call_order_and_limits(B):
    w = wl.make("cfg1", 2)
    t, x = wl.profile_of(w)
    ev = B.evaluator_for(w)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    with pytest.raises(B.DiscoError) as e:
        ev.cost_candidates(cg, co, gid, 0.1, 0.1)
    assert e.value.status == B.DC_ERR_INVALID_ARG          # no profile yet
    ev.set_profile(t, x)
    ev.cost_candidates(cg, co, gid, 0.1, 0.1)
    assert ev.check() == B.DC_OK
    ev.set_base_graphs(w.g_node_off(), w.g_edge_off(), w.cat_rowptr(), w.cat_col(), w.cat_X())
    with pytest.raises(B.DiscoError) as e:                 # new graphs discard the profile
        ev.cost_candidates(cg, co, gid, 0.1, 0.1)
    assert e.value.status == B.DC_ERR_INVALID_ARG
    ev.close()
    # a context whose estimator scratch is smaller than the base graphs cannot take the cost path
    small = B.evaluator_for(w, max_nodes=40, max_edges=100)
    with pytest.raises(B.DiscoError) as e:
        small.set_profile(t, x)
    assert e.value.status == B.DC_ERR_CAPACITY
    small.close()
    # rows that are not strictly ascending
    g = w.graphs[0]
    col = g.col.copy()
    u = int(np.argmax(np.diff(g.rowptr) >= 2))
    s = g.rowptr[u]
    col[s], col[s + 1] = col[s + 1], col[s]
    w2 = wl.custom("unsorted", w.model, [wl.BaseGraph(g.n, g.n_op, g.rowptr, col, g.X)],
                   [w.group_id.reshape(w.n_cand, g.n)])
    ev = B.evaluator_for(w2)
    with pytest.raises(B.DiscoError) as e:
        ev.set_profile(t, x)
    assert e.value.status == B.DC_ERR_BAD_GRAPH
    ev.close()


def test_layers_on_a_fused_op_batch_equal_the_separate_kernels(B):
    """The fused-op batches run the same fused layer kernel as the candidate modules (millions of rows in
    tiny graphs: nearly every neighbour list has at most one entry).  dc_select_kernels can make a context
    run the neighbour means and the node update as separate kernels instead: the same arithmetic in the
    same order, so the costs agree bit for bit."""
    w = positive(wl.make("cfg4", 24))
    t, x = wl.profile_of(w)

    def run(which=0):
        ev = B.evaluator_for(w)
        ev.select_kernels(which)
        ev.set_profile(t, x)
        cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
        cost = ev.cost_candidates(cg, co, gid, 0.02, 0.01).cpu().numpy()
        assert ev.check() == B.DC_OK
        counts = ev.last_fused_ops()
        ev.close()
        return cost, counts

    dma, counts = run()
    reg, counts2 = run(B.DC_KERNELS_SEPARATE_LAYERS)
    assert counts == counts2 and counts[0] > 1000
    assert np.isfinite(dma).all()
    assert np.array_equal(dma, reg), np.abs(dma - reg).max()
