#!/usr/bin/env python3
"""Benchmark of the fusion-candidate evaluator on one MI355X.

A step is one pass of the whole hot path (dc_eval_candidates: contraction of
every candidate, all message-passing layers, readout and head) over one batch
of synthetic candidates that is already resident in HBM.  Prints one JSON line:
candidates/s, the roofline position of the dominant kernel (timed live with HIP
events on the launch stream) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0           # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def algorithmic_work(w, ntot, etot, fused_readout=False):
    """Bytes / flops each kernel family must move or compute per step (what the
    method needs, not what an implementation happens to touch)."""
    m = w.model
    s = 2 if m.dtype == "bf16" else 4
    nb = int(w.cand_off[-1])
    C = w.n_cand
    base = sum(4 * (g.n + 1) + 4 * g.e + 4 * g.n * m.F for g in w.graphs)       # read once per batch
    contract = 4 * nb + 4 * nb + ntot * m.F * s + 2 * 4 * (ntot + C + etot) + base
    if getattr(m, "agg", "mean") == "attention":
        # per layer: z = h W (dense), score terms from z, weighted sums over N_i (z read once, h' written)
        pf = pb = sb = ab = 0
        d = m.F
        for _ in range(m.L):
            pf += 2 * ntot * d * m.H
            pb += ntot * (d + m.H) * s + d * m.H * s
            sb += ntot * m.H * s + 2 * 4 * ntot * m.heads
            ab += 2 * ntot * m.H * s + 2 * 4 * (ntot + etot) + 4 * ntot * m.heads
            d = m.H
        return {"contract": {"bytes": contract}, "attention_project": {"flops": pf, "bytes": pb},
                "attention_scores": {"bytes": sb}, "attention_aggregate": {"bytes": ab},
                "readout_head": {"bytes": ntot * m.H * s}}
    agg_b, upd_f, upd_b = 0, 0, 0
    fus = {"fused_layer": [0, 0], "layer256": [0, 0], "layer256_d64": [0, 0]}
    d = m.F
    readout_b = ntot * m.H * s
    for l in range(m.L):
        bulk = m.dtype == "bf16" and m.H == 256 and d in (256, 64)
        fused = m.dtype == "bf16" and m.H in (128, 256) and d % 64 == 0
        idx = 2 * 4 * (ntot + etot)
        flops = 2 * ntot * 3 * d * m.H
        if fused:       # means never leave the chip: read h, write h', read the neighbour lists and W
            k = fus[("layer256" if d == 256 else "layer256_d64") if bulk else "fused_layer"]
            k[0] += flops
            out_b = ntot * m.H * s
            if bulk and fused_readout and l == m.L - 1:
                # the last layer leaves column sums per 64 rows and graph instead of its rows; the readout reads those
                out_b = readout_b = (ntot // 64 + C) * m.H * 4
            k[1] += ntot * d * s + out_b + idx + 3 * d * m.H * s
        else:           # read h, write both means; then read [h|h_in|h_out] and W, write h'
            agg_b += ntot * d * s + 2 * ntot * d * s + idx
            upd_f += flops
            upd_b += ntot * (3 * d + m.H) * s + 3 * d * m.H * s
        d = m.H
    return {"contract": {"bytes": contract}, "aggregate": {"bytes": agg_b},
            "update": {"flops": upd_f, "bytes": upd_b},
            "fused_layer": {"flops": fus["fused_layer"][0], "bytes": fus["fused_layer"][1]},
            "layer256": {"flops": fus["layer256"][0], "bytes": fus["layer256"][1]},
            "layer256_d64": {"flops": fus["layer256_d64"][0], "bytes": fus["layer256_d64"][1]},
            "readout_head": {"bytes": readout_b}}


def long_list_stats(ev, w, cg, co, gid, ntot, etot, torch):
    """(number of (row, direction) pairs with more than five neighbours -- the layer kernel gathers up to five
    itself --, their neighbour count in all) of the contracted batch: what the pre-pass of the bulk layer kernel
    serves.  Outside the timed region."""
    batch = ev.alloc_batch(w.n_cand, int(w.cand_off[-1]), ntot, etot)
    ev.contract_graphs(cg, co, gid, batch)
    torch.cuda.synchronize()
    pairs = entries = 0
    for rp in (batch.in_rowptr, batch.out_rowptr):
        deg = (rp[1:ntot + 1] - rp[:ntot]).to(torch.int64)
        long = deg > 5
        pairs += int(long.sum())
        entries += int(deg[long].sum())
    del batch
    return pairs, entries


def pre_pass_work(w, pairs, entries):
    """Bytes the pre-pass must move per step: every neighbour row its lists name (2 bytes x d), the mean it
    writes per list, the neighbour numbers (4 bytes each) and per list its row number and list bounds."""
    m, by, d = w.model, 0, w.model.F
    for _ in range(m.L):
        by += entries * d * 2 + pairs * d * 2 + 4 * entries + 12 * pairs
        d = m.H
    return {"bytes": by}


def read_traffic(workload, kernel):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    recorded in profiles/traffic_<workload>.txt as '<kernel>_traffic_bytes_per_launch: N'."""
    p = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(p):
        return None
    for line in open(p):
        if line.startswith(f"{kernel}_traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def host_cores():
    """Threads the oracle may use: the host's CPU count, capped by the share the environment grants
    (OMP_NUM_THREADS is set to the machine's CPU share on the GPU machines)."""
    n = os.cpu_count() or 1
    try:
        n = min(n, len(os.sched_getaffinity(0)))
    except (AttributeError, OSError):
        pass
    cap = os.environ.get("OMP_NUM_THREADS", "")
    if cap.isdigit() and int(cap) > 0:
        n = min(n, int(cap))
    return max(1, n)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, seconds_target=8.0):
    """The oracle (contract + forward) timed on this host: one instance on one core, then one
    independent single-threaded instance per core on disjoint candidate slices (measured aggregate).
    Both on evenly spaced samples of the workload's candidates, sized for about `seconds_target`
    seconds of wall time each."""
    from oracle import oracle as orc
    probe = w.subset([0])
    t0 = time.perf_counter()
    orc.evaluate(probe)
    per = max(time.perf_counter() - t0, 1e-4)
    n1 = int(max(1, min(w.n_cand, seconds_target / per)))
    idx = np.linspace(0, w.n_cand - 1, n1).astype(np.int64)
    t0 = time.perf_counter()
    orc.evaluate(w.subset(idx))
    dt1 = time.perf_counter() - t0
    cores = host_cores()
    nc = int(max(cores, min(w.n_cand, cores * seconds_target / per)))
    nc = min(nc, w.n_cand)
    idx = np.unique(np.linspace(0, w.n_cand - 1, nc).astype(np.int64))
    t0 = time.perf_counter()
    orc.evaluate_parallel(w, False, cores, idx)
    dtc = time.perf_counter() - t0
    return {"value": len(idx) / dtc, "unit": "candidates/s", "cores": min(cores, len(idx)), "kind": "oracle",
            "sample": f"{len(idx)} of {w.n_cand} candidates of {w.name}, evenly spaced, contract+forward, one "
                      f"single-threaded oracle instance per core on disjoint slices, {dtc:.1f} s wall",
            "single_core": {"value": n1 / dt1, "cores": 1,
                            "sample": f"{n1} candidates, one instance, {dt1:.1f} s"},
            "cpu_model": cpu_model(), "host_cpus": os.cpu_count()}


def simulate_bench(args, w, B, torch):
    """Times dc_simulate alone: the batch is contracted once, then K simulator passes."""
    ev = B.evaluator_for(w)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    nb = int(w.cand_off[-1])
    geo = w.g_edge_off()
    eb = int(sum(int(geo[b + 1] - geo[b]) for b in w.cand_graph))
    batch = ev.alloc_batch(w.n_cand, nb, nb, eb)
    ev.contract_graphs(cg, co, gid, batch)
    ntot, etot = ev.last_totals()
    Xc = batch.Xc[:ntot].float()
    is_ar = Xc[:, 1] > 0
    ar_size = torch.where(is_ar, Xc[:, 0], torch.full_like(Xc[:, 0], -1.0)).contiguous()
    op_time = torch.where(is_ar, torch.zeros_like(Xc[:, 2]), 0.05 + Xc[:, 2]).contiguous()
    cost = torch.empty(w.n_cand, dtype=torch.float32, device=ev.device)
    for _ in range(args.warmup):
        ev.simulate(batch, op_time, ar_size, 0.02, 0.01, cost)
    torch.cuda.synchronize()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev.simulate(batch, op_time, ar_size, 0.02, 0.01, cost)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out = {"metric": "fusion candidates simulated/sec (list scheduling + all-reduce channel) on 1 MI355X",
           "value": round(w.n_cand * args.steps / dt, 1), "unit": "candidates/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": w.name, "candidates": w.n_cand, "contracted_nodes": ntot, "contracted_edges": etot,
                      "finite": int(torch.isfinite(cost).sum().item())}}
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        n = w.n_cand                          # the simulator is cheap on the CPU: time the whole batch
        ref = orc.contract(w, False)
        ar = np.where(ref.Xc[:, 1] > 0, ref.Xc[:, 0], -1.0).astype(np.float32)
        tt = np.where(ref.Xc[:, 1] > 0, 0.0, 0.05 + ref.Xc[:, 2]).astype(np.float32)
        t0 = time.perf_counter()
        orc.simulate(ref, tt, ar, 0.02, 0.01)
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n / cdt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
                               "sample": f"all {n} candidates, simulator only (contraction not timed), {cdt:.3f} s"}
    ev.close()
    print(json.dumps(out), flush=True)


def cost_bench(args, w, B, torch):
    """Times dc_cost_candidates: contraction, the estimator on the fused ops (once per distinct fused op of the
    batch; --every-fused-op: on each of them), per-node times, list scheduling.  Profiled data are synthetic
    (workloads.profile_of)."""
    from paper_2209_12769_amd import workloads as wl
    t_base, x_base = wl.profile_of(w)
    w.weights.head[-1] += 1.0                 # random weights: keeps most estimates above the clamp at zero
    ev = B.evaluator_for(w)
    if args.every_fused_op:
        ev.select_kernels(B.DC_KERNELS_EVERY_FUSED_OP)
    ev.set_profile(t_base, x_base)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    cost = torch.empty(w.n_cand, dtype=torch.float32, device=ev.device)
    ar_c, ar_d = 0.02, 0.01
    for _ in range(args.warmup):
        ev.cost_candidates(cg, co, gid, ar_c, ar_d, cost)
    torch.cuda.synchronize()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    ntot, etot = ev.last_totals()
    K, M, E = ev.last_fused_ops()
    repeats = ev.last_fused_op_repeats()
    ev.profile_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev.cost_candidates(cg, co, gid, ar_c, ar_d, cost)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fam = ev.profile_end()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    work = algorithmic_work(w, M, E)          # the layer kernels run on the fused-op batch
    m = w.model
    s = 2 if m.dtype == "bf16" else 4
    work["fused_op_head"] = {"flops": 2 * 2 * K * m.H * m.H, "bytes": M * m.H * s + 5 * K * m.H * s}
    # list scheduling: the module's lists in both directions, a time, a size and a completion time per node
    work["simulate"] = {"bytes": 8 * (ntot + etot) + 12 * ntot}
    kernels = {}
    for name, (ms_total, launches) in fam.items():
        if launches == 0:
            continue
        per = ms_total / args.steps
        k = {"ms_per_step": round(per, 4), "launches_per_step": launches / args.steps}
        if per > 0 and name in work and work[name].get("bytes"):
            k["GB/s"] = round(work[name]["bytes"] / (per * 1e-3) / 1e9, 1)
        if per > 0 and name in work and work[name].get("flops"):
            k["TFLOP/s"] = round(work[name]["flops"] / (per * 1e-3) / 1e12, 2)
        kernels[name] = k
    # the message-passing layers as a whole: the layer kernels charged with the pre-pass (means of rows with
    # long neighbour lists) and the descriptor build they cannot run without
    layer_keys = [k for k in ("layer256", "layer256_d64", "fused_layer", "aggregate", "update", "aggregate_heavy",
                              "build_desc") if k in kernels]
    if layer_keys:
        ms = sum(kernels[k]["ms_per_step"] for k in layer_keys)
        fl = sum(work[k].get("flops", 0) for k in layer_keys if k in work)
        by = sum(work[k].get("bytes", 0) for k in layer_keys if k in work)
        kernels["layer_total"] = {"ms_per_step": round(ms, 4), "parts": layer_keys,
                                  "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 2), "GB/s": round(by / (ms * 1e-3) / 1e9, 1),
                                  "frac_of_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS[w.model.dtype], 4)}
    dom = max((n for n in kernels if n != "layer_total"), key=lambda n: kernels[n]["ms_per_step"])
    if "TFLOP/s" in kernels[dom]:
        peak = PEAK_MFMA_TFLOPS[m.dtype]
        ach = kernels[dom]["TFLOP/s"]
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": round(ach / peak, 4), "traffic": read_traffic(w.name + ("_cost_every_fused_op" if args.every_fused_op else "_cost"), dom)}
    else:
        ach = kernels[dom].get("GB/s", 0.0)
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": read_traffic(w.name + ("_cost_every_fused_op" if args.every_fused_op else "_cost"), dom)}
    roof["avg_launch_ms"] = round(kernels[dom]["ms_per_step"] / max(kernels[dom]["launches_per_step"], 1), 4)
    out = {"metric": "fusion candidates costed/sec (contraction + estimator on the fused ops + list scheduling) "
                     "on 1 MI355X",
           "value": round(w.n_cand * args.steps / dt, 1), "unit": "candidates/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": m.dtype, "data": "synthetic",
           "config": {"workload": w.name, "candidates": w.n_cand, "contracted_nodes": ntot, "contracted_edges": etot,
                      "fused_ops": K + repeats, "fused_ops_estimated": K, "fused_ops_repeating_an_estimated_one": repeats,
                      "fused_op_rows": M, "fused_op_edges": E, "F": m.F, "H": m.H, "L": m.L,
                      "finite": int(torch.isfinite(cost).sum().item())},
           "roofline": roof, "kernels": kernels}
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        n = min(w.n_cand, 6 if w.name in ("cfg4", "cfg5") else 32)
        sub = w.subset(np.linspace(0, w.n_cand - 1, n).astype(np.int64))
        t0 = time.perf_counter()
        orc.cost(sub, t_base, x_base, ar_c, ar_d)
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n / cdt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
                               "sample": f"{n} of {w.n_cand} candidates of {w.name}, evenly spaced, {cdt:.1f} s"}
    ev.close()
    print(json.dumps(out), flush=True)


def search_bench(args, w, B, torch):
    """Times dc_search (Alg. 1 with batched steps) on the workload's first base graph: every step mutates
    `parents` queue entries twice on the device, costs the children in one dc_cost_candidates call and
    updates the queue on the host.  A step here is one search step; value = candidates costed per second."""
    from paper_2209_12769_amd import workloads as wl
    g = w.graphs[0]
    P = max(1, (args.n_cand or 4096) // 2)
    ident = np.tile(np.arange(g.n, dtype=np.int32), (2 * P, 1))
    wt = w.weights
    wt.head[-1] += 1.0
    ws = wl.custom(w.name, w.model, [g], [ident], weights=wt)
    t_base, x_base = wl.profile_of(ws)
    ev = B.evaluator_for(ws)
    ev.set_profile(t_base, x_base)
    kw = dict(alpha=1.05, beta=16, seed=1, ar_c=0.02, ar_d=0.01, max_unchanged=1 << 30, parents=P, max_queue=4 * P,
              op_draw=B.DC_DRAW_OP if args.op_draw == "op" else B.DC_DRAW_DEPENDENCY)
    ev.search(0, g.n, max_steps=args.warmup, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    labels, r = ev.search(0, g.n, max_steps=args.steps, **kw)
    dt = time.perf_counter() - t0
    out = {"metric": "fusion candidates generated and costed/sec inside the backtracking search (Alg. 1) on 1 MI355X",
           "value": round(r.evaluated / dt, 1), "unit": "candidates/s", "n_gpus": 1, "steps": int(r.steps),
           "warmup": args.warmup, "ms_per_step": round(dt / max(r.steps, 1) * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": w.model.dtype, "data": "synthetic",
           "config": {"workload": w.name, "base_nodes": g.n, "parents_per_step": P, "alpha": 1.05, "beta": 16,
                      "op_draw": args.op_draw, "evaluated": int(r.evaluated), "valid": int(r.valid), "enqueued": int(r.enqueued),
                      "improved": int(r.improved), "cost_in": r.cost_in, "cost_opt": r.cost_opt,
                      "groups_opt": int(len(np.unique(labels))),
                      "note": "includes the set-up of the call (first cost of H_in, buffers) and one stream "
                              "synchronisation per step"}}
    ev.close()
    print(json.dumps(out), flush=True)


def train_bench(args, w, B, torch):
    """Times dc_train_step (Sec. 3.3.3): forward with kept activations, loss of Eq. (1), reverse pass and one
    Adam update over one resident batch of fused-op samples.  The samples are drawn the way Sec. 5.1 describes
    (workloads.training_labels) on the workload's base graph; the profiled times they are fitted to are
    synthetic (workloads.synthetic_fused_times).  fp32."""
    from paper_2209_12769_amd import workloads as wl
    g = w.graphs[0]
    C = args.n_cand or 128
    model = wl.ModelSpec(w.model.F, w.model.H, w.model.L, "f32")
    ws = wl.custom(w.name + "-train", model, [g], [wl.training_labels(g, 1, C)], seed=0)
    ws.weights.head[-1] += 1.0
    nb = int(ws.cand_off[-1])
    eb = g.e * C
    ev = B.Evaluator(model.F, model.H, model.L, "f32", nb // 2 + 1, nb, eb)
    ev.set_base_graphs(ws.g_node_off(), ws.g_edge_off(), ws.cat_rowptr(), ws.cat_col(), ws.cat_X())
    ev.set_weights(ws.weights)
    t_base, x_base = wl.profile_of(ws)
    ev.set_profile(t_base, x_base)
    cg, co, gid = ev.to_device(ws.cand_graph), ev.to_device(ws.cand_off), ev.to_device(ws.group_id)
    batch = ev.fused_op_batch(cg, co, gid, ev.alloc_batch(nb // 2 + 1, nb, nb, eb))
    K, M, E = ev.last_fused_ops()
    target_h = wl.synthetic_fused_times(batch.node_off[:K + 1].cpu().numpy(), batch.new_id[:M].cpu().numpy(), t_base)
    target = torch.from_numpy(target_h).to(ev.device)
    ev.train_begin(1e-4, K, M)
    loss = torch.empty(1, dtype=torch.float32, device=ev.device)
    first = None
    for _ in range(args.warmup):
        ev.train_step(batch, target, loss)
        if first is None:
            first = float(loss.cpu()[0])
    torch.cuda.synchronize()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    ev.profile_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev.train_step(batch, target, loss)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fam = ev.profile_end()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    F, H, L = model.F, model.H, model.L
    dims = [F] + [H] * (L - 1)
    gemm = sum(2 * M * 3 * d * H for d in dims)                     # one product with every layer's [3d, H] matrix
    work = {"train_update": {"flops": gemm, "bytes": sum(M * (3 * d + H) * 4 for d in dims)},
            "train_wgrad": {"flops": gemm, "bytes": sum(M * (3 * d + H) * 4 for d in dims)},
            "train_dgrad": {"flops": 2 * M * 3 * H * H * (L - 1), "bytes": (L - 1) * M * 4 * H * 4},
            "train_aggregate": {"bytes": sum((2 * E + 2 * M) * d * 4 for d in dims)},      # gathered rows + both means
            "train_gather_back": {"bytes": (L - 1) * ((M + 2 * E) * H * 4 + 2 * M * H * 4)}}
    kernels = {}
    for name, (ms_total, launches) in fam.items():
        if launches == 0:
            continue
        per = ms_total / args.steps
        k = {"ms_per_step": round(per, 4), "launches_per_step": launches / args.steps}
        if per > 0 and name in work and work[name].get("bytes"):
            k["GB/s"] = round(work[name]["bytes"] / (per * 1e-3) / 1e9, 1)
        if per > 0 and name in work and work[name].get("flops"):
            k["TFLOP/s"] = round(work[name]["flops"] / (per * 1e-3) / 1e12, 2)
        kernels[name] = k
    # the message-passing layers as a whole: the layer kernels charged with the pre-pass (means of rows with
    # long neighbour lists) and the descriptor build they cannot run without
    layer_keys = [k for k in ("layer256", "layer256_d64", "fused_layer", "aggregate", "update", "aggregate_heavy",
                              "build_desc") if k in kernels]
    if layer_keys:
        ms = sum(kernels[k]["ms_per_step"] for k in layer_keys)
        fl = sum(work[k].get("flops", 0) for k in layer_keys if k in work)
        by = sum(work[k].get("bytes", 0) for k in layer_keys if k in work)
        kernels["layer_total"] = {"ms_per_step": round(ms, 4), "parts": layer_keys,
                                  "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 2), "GB/s": round(by / (ms * 1e-3) / 1e9, 1),
                                  "frac_of_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS[w.model.dtype], 4)}
    dom = max((n for n in kernels if n != "layer_total"), key=lambda n: kernels[n]["ms_per_step"])
    if "TFLOP/s" in kernels[dom]:
        ach = kernels[dom]["TFLOP/s"]
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_TFLOPS["f32"], "unit": "TFLOP/s",
                "frac": round(ach / PEAK_MFMA_TFLOPS["f32"], 4), "traffic": read_traffic(w.name + "_train", dom)}
    else:
        ach = kernels[dom].get("GB/s", 0.0)
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": read_traffic(w.name + "_train", dom)}
    roof["avg_launch_ms"] = round(kernels[dom]["ms_per_step"] / max(kernels[dom]["launches_per_step"], 1), 4)
    out = {"metric": "fused-op samples trained/sec (forward + loss + reverse pass + Adam) on 1 MI355X",
           "value": round(K * args.steps / dt, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": ws.name, "labelings": C, "samples": K, "rows": M, "edges": E, "F": F, "H": H, "L": L,
                      "params": ev.num_params(), "loss_first": first, "loss_last": float(loss.cpu()[0])},
           "roofline": roof, "kernels": kernels}
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        from oracle import train as ot
        from threadpoolctl import threadpool_info
        n = min(C, 128)               # about 15 s of numpy
        sub = wl.custom("s", model, [g], [ws.group_id.reshape(C, g.n)[:n]], weights=ws.weights)
        fo, _, member = orc.fused_ops(sub, orc.contract(sub), x_base)
        tg = wl.synthetic_fused_times(fo.node_off, member, t_base)
        p0 = ot.Params.from_weights(ws.weights, F, H, L)
        t0 = time.perf_counter()
        ot.train([fo], [tg], p0, F, H, L, lr=1e-4)
        cdt = time.perf_counter() - t0
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        out["cpu_baseline"] = {"value": fo.n_cand / cdt, "unit": "samples/s", "cores": threads, "kind": "oracle",
                               "sample": f"one training step on the {fo.n_cand} samples ({fo.ntot} rows) of the first "
                                         f"{n} of {C} labelings, {cdt:.1f} s"}
    ev.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--n-cand", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--aggregator", default="mean", choices=["mean", "attention"],
                    help="mean: in/out mean aggregation (the headline path); attention: K-head attention coefficients")
    ap.add_argument("--heads", type=int, default=4)
    ap.add_argument("--simulate", action="store_true",
                    help="instead of the estimator, time the list-scheduling simulator (dc_simulate) on the "
                         "contracted batch; per-node times and tensor sizes are synthetic (from the features)")
    ap.add_argument("--cost", action="store_true",
                    help="instead of one estimate per module, time Cost(H) as the paper composes it "
                         "(dc_cost_candidates): estimator on the fused ops, profiled single ops, simulator")
    ap.add_argument("--every-fused-op", action="store_true",
                    help="with --cost: run the estimator on every fused op, also on those that repeat an earlier one "
                         "of the batch (default: once per distinct fused op)")
    ap.add_argument("--search", action="store_true",
                    help="time the backtracking search (dc_search) on the workload's base graph; "
                         "--n-cand children per step, --steps search steps")
    ap.add_argument("--op-draw", default="dependency", choices=["dependency", "op"],
                    help="with --search: how op fusion draws (a dependency of the base module, or the paper's "
                         "op of the current module and one of its predecessors)")
    ap.add_argument("--train", action="store_true",
                    help="time dc_train_step (estimator training, fp32) on samples drawn on the workload's base "
                         "graph; --n-cand = number of labelings the samples are drawn from")
    ap.add_argument("--kernels", type=int, default=0,
                    help="dc_select_kernels value (0: defaults; 1: neighbour means and node update as separate kernels)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run five element-wise copies (y = -x, fp32) of MIB MiB each: "
                         "a kernel of known HBM traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; candidates are independent, so more GPUs would each take a "
              "slice of the batch, but that is not part of this build. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        x = torch.ones(n, dtype=torch.float32, device="cuda:0")
        y = torch.empty_like(x)
        for _ in range(5):
            torch.neg(x, out=y)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_mib": args.copy_calibration, "launches": 5,
                          "read_bytes_per_launch": n * 4, "write_bytes_per_launch": n * 4}))
        return
    from paper_2209_12769_amd import binding as B
    from paper_2209_12769_amd import workloads as wl

    w = wl.make(args.workload, 1 if (args.search or args.train) else args.n_cand)
    if args.train:
        train_bench(args, w, B, torch)
        return
    if args.simulate:
        simulate_bench(args, w, B, torch)
        return
    if args.aggregator == "attention":
        w = wl.with_attention(w, args.heads)
    if args.cost:
        cost_bench(args, w, B, torch)
        return
    if args.search:
        search_bench(args, w, B, torch)
        return
    ev = B.evaluator_for(w)
    ev.select_kernels(args.kernels)
    cg, co, gid = ev.to_device(w.cand_graph), ev.to_device(w.cand_off), ev.to_device(w.group_id)
    pred = torch.empty(w.n_cand, dtype=torch.float32, device=ev.device)
    for _ in range(args.warmup):
        ev.eval_candidates(cg, co, gid, pred)
    torch.cuda.synchronize()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)
    ntot, etot = ev.last_totals()

    ev.profile_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev.eval_candidates(cg, co, gid, pred)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fam = ev.profile_end()
    assert ev.check() == B.DC_OK, B.dc_last_error(ev.ctx)

    work = algorithmic_work(w, ntot, etot, fused_readout=args.kernels == 0 and args.aggregator == "mean")
    if fam.get("aggregate_heavy", (0, 0))[1] > 0 and args.kernels == 0:
        pairs, entries = long_list_stats(ev, w, cg, co, gid, ntot, etot, torch)
        work["aggregate_heavy"] = pre_pass_work(w, pairs, entries)
    fam["contract_all"] = (sum(fam[k][0] for k in ("prep_scan", "contract", "finalize")), fam["contract"][1])
    contract_parts = {k: round(fam[k][0] / args.steps, 4) for k in ("prep_scan", "contract", "finalize")}
    kernels = {}
    for name, key in (("contract", "contract_all"), ("aggregate", "aggregate"), ("update", "update"),
                      ("fused_layer", "fused_layer"), ("layer256", "layer256"), ("layer256_d64", "layer256_d64"),
                      ("aggregate_heavy", "aggregate_heavy"), ("build_desc", "build_desc"),
                      ("attention_project", "attention_project"), ("attention_scores", "attention_scores"),
                      ("attention_aggregate", "attention_aggregate"),
                      ("readout_head", "readout_head")):
        ms_total, launches = fam[key]
        if launches == 0:
            continue
        per_step_ms = ms_total / args.steps
        k = {"ms_per_step": round(per_step_ms, 4), "launches_per_step": launches / args.steps}
        if per_step_ms > 0 and name in work:
            k["GB/s"] = round(work[name]["bytes"] / (per_step_ms * 1e-3) / 1e9, 1)
            if "flops" in work[name]:
                k["TFLOP/s"] = round(work[name]["flops"] / (per_step_ms * 1e-3) / 1e12, 2)
        if name == "contract":
            k["parts_ms"] = contract_parts          # candidate check + scan, per-candidate contraction, placement + feature sums
        kernels[name] = k
    # the message-passing layers as a whole: the layer kernels charged with the pre-pass (means of rows with
    # long neighbour lists) and the descriptor build they cannot run without
    layer_keys = [k for k in ("layer256", "layer256_d64", "fused_layer", "aggregate", "update", "aggregate_heavy",
                              "build_desc") if k in kernels]
    if layer_keys:
        ms = sum(kernels[k]["ms_per_step"] for k in layer_keys)
        fl = sum(work[k].get("flops", 0) for k in layer_keys if k in work)
        by = sum(work[k].get("bytes", 0) for k in layer_keys if k in work)
        kernels["layer_total"] = {"ms_per_step": round(ms, 4), "parts": layer_keys,
                                  "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 2), "GB/s": round(by / (ms * 1e-3) / 1e9, 1),
                                  "frac_of_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS[w.model.dtype], 4)}
    dom = max((n for n in kernels if n != "layer_total"), key=lambda n: kernels[n]["ms_per_step"])
    if dom in ("update", "fused_layer", "layer256", "layer256_d64", "attention_project"):
        peak = PEAK_MFMA_TFLOPS[w.model.dtype]
        ach = kernels[dom].get("TFLOP/s", 0.0)
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": round(ach / peak, 4), "traffic": read_traffic(w.name, dom),
                "avg_launch_ms": round(kernels[dom]["ms_per_step"] / max(kernels[dom]["launches_per_step"], 1), 4)}
    else:
        ach = kernels[dom].get("GB/s", 0.0)
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": read_traffic(w.name, dom),
                "avg_launch_ms": round(kernels[dom]["ms_per_step"] / max(kernels[dom]["launches_per_step"], 1), 4)}

    out = {
        "metric": "fusion candidates evaluated/sec (contract+GNN) on 1 MI355X",
        "value": round(w.n_cand * args.steps / dt, 1),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.model.dtype, "data": "synthetic",
        "config": {"workload": w.name, "candidates": w.n_cand, "base_graphs": len(w.graphs),
                   "base_nodes": int(np.mean([g.n for g in w.graphs])), "contracted_nodes": ntot,
                   "contracted_edges": etot, "F": w.model.F, "H": w.model.H, "L": w.model.L,
                   "aggregator": args.aggregator, **({"heads": args.heads} if args.aggregator == "attention" else {})},
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    ev.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
