"""ctypes front end of the CPU oracle (test infrastructure only).

Loads oracle/dc_oracle.cpp, compiled with g++ into oracle/_build/.  Nothing in
the product package imports this module; it knows nothing of the HIP library.
Only argument marshalling happens here: every number comes out of the C++.

Every function computes the definition: fp32 storage, fp64 accumulation, one rounding.  The
optional argument `bf16=True` additionally rounds features, activations, neighbour means and
matrices to bf16 where a bf16 device path stores them; it is a diagnostic second mode that a test
has to ask for, never the default.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dc_oracle.cpp")
# DC_ORACLE_SANITIZE=1 in the environment selects a build with the address and undefined-behaviour
# sanitizers (host code only); the process must then run with the sanitizer runtime preloaded.
_SANITIZE = os.environ.get("DC_ORACLE_SANITIZE", "") == "1"
_SO = os.path.join(_HERE, "_build", "libdc_oracle_san.so" if _SANITIZE else "libdc_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    os.makedirs(os.path.dirname(_SO), exist_ok=True)
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
        if _SANITIZE else ["-O2"]
    subprocess.check_call(["g++", *flags, "-std=c++17", "-shared", "-fPIC", "-o", _SO, _SRC])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
        _lib.orc_contract_batch.restype = C.c_int
        _lib.orc_gnn_forward.restype = None
        _lib.orc_simulate.restype = None
        _lib.orc_fused_op_batch.restype = C.c_int64
        _lib.orc_module_times.restype = None
        _lib.orc_round_bf16.restype = None
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Batch:
    """Block-diagonal batch of contracted graphs (global numbering)."""
    n_cand: int
    F: int
    node_off: np.ndarray
    edge_off: np.ndarray
    new_id: np.ndarray
    out_rowptr: np.ndarray
    out_col: np.ndarray
    in_rowptr: np.ndarray
    in_col: np.ndarray
    Xc: np.ndarray
    cnt: np.ndarray

    @property
    def ntot(self) -> int:
        return int(self.node_off[-1])

    @property
    def etot(self) -> int:
        return int(self.edge_off[-1])


def round_bf16(x: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(x, dtype=np.float32).copy()
    _load().orc_round_bf16(_p(y), C.c_int64(y.size))
    return y


def contract(w, bf16: bool = False) -> Batch:
    """Contracts all candidates of workload `w` (a workloads.Workload)."""
    lib = _load()
    bf16 = bool(bf16)
    F = w.model.F
    gno, geo = w.g_node_off(), w.g_edge_off()
    rowptr, col, X = w.cat_rowptr(), w.cat_col(), w.cat_X()
    cand_graph = np.ascontiguousarray(w.cand_graph, dtype=np.int32)
    cand_off = np.ascontiguousarray(w.cand_off, dtype=np.int64)
    label = np.ascontiguousarray(w.group_id, dtype=np.int32)
    Cn = w.n_cand
    cap_n = int(cand_off[-1])
    cap_e = int(sum(int(geo[b + 1] - geo[b]) for b in cand_graph))
    node_off = np.zeros(Cn + 1, np.int32)
    edge_off = np.zeros(Cn + 1, np.int32)
    new_id = np.zeros(max(cap_n, 1), np.int32)
    orp = np.zeros(cap_n + 1, np.int32)
    irp = np.zeros(cap_n + 1, np.int32)
    oc = np.zeros(max(cap_e, 1), np.int32)
    ic = np.zeros(max(cap_e, 1), np.int32)
    Xc = np.zeros((max(cap_n, 1), F), np.float32)
    cnt = np.zeros(max(cap_n, 1), np.int32)
    rc = lib.orc_contract_batch(C.c_int(len(w.graphs)), _p(gno), _p(geo), _p(rowptr), _p(col), _p(X), C.c_int(F),
                                C.c_int(Cn), _p(cand_graph), _p(cand_off), _p(label), C.c_int(int(bf16)),
                                C.c_int64(cap_n), C.c_int64(cap_e),
                                _p(node_off), _p(edge_off), _p(new_id), _p(orp), _p(oc), _p(irp), _p(ic),
                                _p(Xc), _p(cnt))
    if rc != 0:
        raise ValueError(f"oracle contraction failed with status {rc}")
    nt, et = int(node_off[-1]), int(edge_off[-1])
    return Batch(Cn, F, node_off, edge_off, new_id[:cap_n], orp[:nt + 1], oc[:et], irp[:nt + 1], ic[:et],
                 Xc[:nt], cnt[:nt])


def gnn_forward(b: Batch, model, weights, bf16: bool = False, want_hidden: bool = False):
    """Predicted time per candidate; with want_hidden also (h_last, readout)."""
    lib = _load()
    bf16 = bool(bf16)
    pred = np.zeros(b.n_cand, np.float32)
    h_last = np.zeros((max(b.ntot, 1), model.H), np.float32) if want_hidden else None
    ro = np.zeros((max(b.n_cand, 1), model.H), np.float32) if want_hidden else None
    Wl = np.ascontiguousarray(weights.layers, dtype=np.float32)
    bl = np.ascontiguousarray(weights.biases, dtype=np.float32)
    hd = np.ascontiguousarray(weights.head, dtype=np.float32)
    Xc = np.ascontiguousarray(b.Xc, dtype=np.float32)
    if getattr(model, "agg", "mean") == "attention":
        at = np.ascontiguousarray(weights.att, dtype=np.float32)
        lib.orc_gnn_forward_attn(C.c_int(b.n_cand), _p(b.node_off), _p(b.out_rowptr), _p(b.out_col),
                                 _p(b.in_rowptr), _p(b.in_col), _p(Xc), C.c_int(model.F), C.c_int(model.H),
                                 C.c_int(model.L), C.c_int(model.heads), C.c_int(int(bf16)), _p(Wl), _p(at), _p(bl),
                                 _p(hd), _p(pred), _p(h_last), _p(ro))
    else:
        lib.orc_gnn_forward(C.c_int(b.n_cand), _p(b.node_off), _p(b.out_rowptr), _p(b.out_col),
                            _p(b.in_rowptr), _p(b.in_col), _p(Xc), C.c_int(model.F), C.c_int(model.H),
                            C.c_int(model.L), C.c_int(int(bf16)), _p(Wl), _p(bl), _p(hd),
                            _p(pred), _p(h_last), _p(ro))
    if want_hidden:
        return pred, h_last[:b.ntot], ro[:b.n_cand]
    return pred


def simulate(b: Batch, op_time: np.ndarray, ar_size: np.ndarray, ar_c: float, ar_d: float) -> np.ndarray:
    """End-to-end time per candidate by list scheduling on one device plus a serial all-reduce
    channel; +inf where the contracted graph has a cycle."""
    lib = _load()
    cost = np.zeros(b.n_cand, np.float32)
    t = np.ascontiguousarray(op_time, dtype=np.float32)
    x = np.ascontiguousarray(ar_size, dtype=np.float32)
    lib.orc_simulate(C.c_int(b.n_cand), _p(b.node_off), _p(b.out_rowptr), _p(b.out_col), _p(b.in_rowptr),
                     _p(b.in_col), _p(t), _p(x), C.c_float(ar_c), C.c_float(ar_d), _p(cost))
    return cost


def fused_ops(w, b: Batch, ar_size_base: np.ndarray, bf16: bool = False):
    """The fused ops (groups of two or more computation ops) of every candidate of `w`, each
    as the subgraph of its members: returns (batch with one graph per fused op, contracted
    node of each fused op, base node of each row).  `b` is contract(w)."""
    lib = _load()
    bf16 = bool(bf16)
    F = w.model.F
    gno, geo = w.g_node_off(), w.g_edge_off()
    rowptr, col, X = w.cat_rowptr(), w.cat_col(), w.cat_X()
    cand_graph = np.ascontiguousarray(w.cand_graph, dtype=np.int32)
    cand_off = np.ascontiguousarray(w.cand_off, dtype=np.int64)
    x = np.ascontiguousarray(ar_size_base, dtype=np.float32)
    cap_n = int(cand_off[-1])
    cap_g = cap_n // 2 + 1
    cap_e = int(sum(int(geo[g + 1] - geo[g]) for g in cand_graph))
    node_off = np.zeros(cap_g + 1, np.int32)
    edge_off = np.zeros(cap_g + 1, np.int32)
    cnode = np.zeros(cap_g, np.int32)
    member = np.zeros(max(cap_n, 1), np.int32)
    orp = np.zeros(cap_n + 1, np.int32)
    irp = np.zeros(cap_n + 1, np.int32)
    oc = np.zeros(max(cap_e, 1), np.int32)
    ic = np.zeros(max(cap_e, 1), np.int32)
    Xf = np.zeros((max(cap_n, 1), F), np.float32)
    new_id = np.ascontiguousarray(b.new_id, dtype=np.int32)
    K = lib.orc_fused_op_batch(_p(gno), _p(geo), _p(rowptr), _p(col), _p(X), C.c_int(F), _p(x), C.c_int(w.n_cand),
                               _p(cand_graph), _p(cand_off), _p(new_id), _p(b.node_off), C.c_int(int(bf16)),
                               C.c_int64(cap_g), C.c_int64(cap_n), C.c_int64(cap_e), _p(node_off), _p(edge_off),
                               _p(cnode), _p(member), _p(orp), _p(oc), _p(irp), _p(ic), _p(Xf))
    if K < 0:
        raise ValueError(f"oracle fused-op extraction failed with status {K}")
    K = int(K)
    nt, et = int(node_off[K]), int(edge_off[K])
    fo = Batch(K, F, node_off[:K + 1], edge_off[:K + 1], member[:nt], orp[:nt + 1], oc[:et], irp[:nt + 1], ic[:et],
               Xf[:nt], np.diff(node_off[:K + 1]).astype(np.int32))
    return fo, cnode[:K], member[:nt]


def module_times(w, b: Batch, op_time_base: np.ndarray, ar_size_base: np.ndarray, bf16: bool = False,
                 want_fused: bool = False):
    """Per node of the contracted batch `b` = contract(w): execution time (profiled for single
    ops, estimated for fused ops, clamped at zero) and all-reduce tensor size (sum over the
    members of a bucket; negative for computation nodes)."""
    lib = _load()
    fo, cnode, _ = fused_ops(w, b, ar_size_base, bf16)
    fo_pred = gnn_forward(fo, w.model, w.weights, bf16) if fo.n_cand > 0 else np.zeros(0, np.float32)
    t = np.ascontiguousarray(op_time_base, dtype=np.float32)
    x = np.ascontiguousarray(ar_size_base, dtype=np.float32)
    cand_graph = np.ascontiguousarray(w.cand_graph, dtype=np.int32)
    cand_off = np.ascontiguousarray(w.cand_off, dtype=np.int64)
    new_id = np.ascontiguousarray(b.new_id, dtype=np.int32)
    gno = w.g_node_off()
    op_time = np.zeros(max(b.ntot, 1), np.float32)
    ar_size = np.zeros(max(b.ntot, 1), np.float32)
    cn = np.ascontiguousarray(cnode, dtype=np.int32)
    fp = np.ascontiguousarray(fo_pred, dtype=np.float32)
    lib.orc_module_times(_p(gno), _p(t), _p(x), C.c_int(w.n_cand), _p(cand_graph), _p(cand_off), _p(new_id),
                         _p(b.node_off), C.c_int64(fo.n_cand), _p(cn), _p(fp), _p(op_time), _p(ar_size))
    if want_fused:
        return op_time[:b.ntot], ar_size[:b.ntot], fo, cnode, fo_pred
    return op_time[:b.ntot], ar_size[:b.ntot]


def cost(w, op_time_base: np.ndarray, ar_size_base: np.ndarray, ar_c: float, ar_d: float,
         bf16: bool = False) -> np.ndarray:
    """Cost(H) per candidate: contraction, times of all nodes of the module, list scheduling."""
    b = contract(w, bf16)
    op_time, ar_size = module_times(w, b, op_time_base, ar_size_base, bf16)
    return simulate(b, op_time, ar_size, ar_c, ar_d)


def evaluate(w, bf16: bool = False) -> np.ndarray:
    """contract + forward: one predicted time per candidate of workload w."""
    return gnn_forward(contract(w, bf16), w.model, w.weights, bf16)


def evaluate_parallel(w, bf16: bool = False, threads: Optional[int] = None, idx=None) -> np.ndarray:
    """contract + forward with one independent, single-threaded oracle instance per thread, each on
    its own disjoint slice of the candidates (`idx`: the candidates wanted, default all).  The
    instances share nothing but the read-only inputs; the C++ runs outside the interpreter lock."""
    from concurrent.futures import ThreadPoolExecutor
    idx = np.arange(w.n_cand) if idx is None else np.asarray(idx, dtype=np.int64)
    if idx.size == 0:
        return np.zeros(0, np.float32)
    threads = max(1, min(int(threads or os.cpu_count() or 1), idx.size))
    parts = [p for p in np.array_split(idx, threads) if p.size]
    with ThreadPoolExecutor(len(parts)) as ex:
        outs = list(ex.map(lambda p: evaluate(w.subset(p), bf16), parts))
    return np.concatenate(outs)
