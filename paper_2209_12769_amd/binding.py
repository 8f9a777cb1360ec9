"""ctypes binding of libdisco.so -- argument marshalling only.

The module-level functions carry the names of the C ABI (include/disco.h) and
pass raw pointers; every step of the evaluation runs in the HIP kernels.
PyTorch is used for device memory and streams only.  There is no fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdisco.so")

DC_OK = 0
DC_ERR_INVALID_ARG = 1
DC_ERR_BAD_GRAPH = 2
DC_ERR_BAD_PARTITION = 3
DC_ERR_CAPACITY = 4
DC_ERR_OOM = 5
DC_ERR_HIP = 6
DC_ERR_UNSUPPORTED = 7
DC_F32 = 0
DC_BF16 = 1
DC_AGG_MEAN = 0
DC_AGG_ATTENTION = 1
DC_KERNELS_SEPARATE_LAYERS = 1
DC_KERNELS_EVERY_FUSED_OP = 2
DC_DRAW_DEPENDENCY, DC_DRAW_OP = 0, 1
STATUS_NAMES = {0: "DC_OK", 1: "DC_ERR_INVALID_ARG", 2: "DC_ERR_BAD_GRAPH", 3: "DC_ERR_BAD_PARTITION",
                4: "DC_ERR_CAPACITY", 5: "DC_ERR_OOM", 6: "DC_ERR_HIP", 7: "DC_ERR_UNSUPPORTED"}


class DcConfig(C.Structure):
    _fields_ = [("F", C.c_int32), ("H", C.c_int32), ("L", C.c_int32), ("dtype", C.c_int32),
                ("max_cand", C.c_int64), ("max_base_nodes", C.c_int64), ("max_base_edges", C.c_int64),
                ("max_nodes", C.c_int64), ("max_edges", C.c_int64),
                ("aggregator", C.c_int32), ("heads", C.c_int32)]


class DcBatch(C.Structure):
    _fields_ = [("n_cand", C.c_int32), ("cap_nodes", C.c_int64), ("cap_edges", C.c_int64),
                ("node_off", C.c_void_p), ("edge_off", C.c_void_p), ("new_id", C.c_void_p),
                ("out_rowptr", C.c_void_p), ("out_col", C.c_void_p), ("in_rowptr", C.c_void_p),
                ("in_col", C.c_void_p), ("Xc", C.c_void_p)]


class DcSearchParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("beta", C.c_int32), ("max_unchanged", C.c_int32), ("parents", C.c_int32),
                ("max_queue", C.c_int32), ("max_steps", C.c_int64), ("seed", C.c_uint64),
                ("ar_c", C.c_float), ("ar_d", C.c_float), ("op_draw", C.c_int32)]


class DcSearchResult(C.Structure):
    _fields_ = [("cost_in", C.c_float), ("cost_opt", C.c_float), ("steps", C.c_int64), ("evaluated", C.c_int64),
                ("valid", C.c_int64), ("enqueued", C.c_int64), ("improved", C.c_int64), ("queued", C.c_int64),
                ("unchanged", C.c_int64)]


class DcTrainParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("floor", C.c_float), ("max_samples", C.c_int64), ("max_rows", C.c_int64)]


class DiscoError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {detail}")


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2209_12769_amd.build)")
        # torch first: the process must hold one HIP runtime, the one that owns the tensors whose pointers
        # cross this boundary; loaded afterwards, libdisco.so binds to it instead of bringing a second copy
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, fp = C.c_void_p, C.c_int32, C.POINTER(C.c_float)
        L.dc_create.argtypes = [C.POINTER(vp), C.POINTER(DcConfig)]
        L.dc_destroy.argtypes = [vp]
        L.dc_workspace_bytes.argtypes = [C.POINTER(DcConfig)]
        L.dc_workspace_bytes.restype = C.c_size_t
        L.dc_set_weights.argtypes = [vp, vp, vp, vp, vp]
        L.dc_set_attention_weights.argtypes = [vp, vp, vp, vp, vp, vp]
        L.dc_set_base_graphs.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.dc_contract_graphs.argtypes = [vp, i32, vp, vp, vp, C.POINTER(DcBatch), vp]
        L.dc_gnn_forward.argtypes = [vp, C.POINTER(DcBatch), vp, vp]
        L.dc_eval_candidates.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.dc_simulate.argtypes = [vp, C.POINTER(DcBatch), vp, vp, C.c_float, C.c_float, vp, vp]
        L.dc_simulate_static.argtypes = [C.POINTER(DcBatch), i32, i32, vp, vp, C.c_float, C.c_float, vp, vp, vp]
        L.dc_simulate_static.restype = i32
        L.dc_simulate_static_error.argtypes = []
        L.dc_simulate_static_error.restype = C.c_char_p
        L.dc_set_profile.argtypes = [vp, vp, vp, vp]
        L.dc_module_times.argtypes = [vp, i32, vp, vp, vp, C.POINTER(DcBatch), vp, vp, vp]
        L.dc_cost_candidates.argtypes = [vp, i32, vp, vp, vp, C.c_float, C.c_float, vp, vp]
        L.dc_last_fused_ops.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64), vp]
        L.dc_last_fused_op_repeats.argtypes = [vp, C.POINTER(C.c_int64), vp]
        L.dc_search.argtypes = [vp, i32, C.POINTER(DcSearchParams), vp, C.POINTER(DcSearchResult), vp]
        L.dc_num_params.argtypes = [vp]
        L.dc_num_params.restype = C.c_int64
        L.dc_train_begin.argtypes = [vp, C.POINTER(DcTrainParams), vp]
        L.dc_fused_op_batch.argtypes = [vp, i32, vp, vp, vp, C.POINTER(DcBatch), vp]
        L.dc_loss_gradients.argtypes = [vp, C.POINTER(DcBatch), vp, vp, vp, vp, vp]
        L.dc_train_step.argtypes = [vp, C.POINTER(DcBatch), vp, vp, vp]
        L.dc_get_weights.argtypes = [vp, vp, vp, vp, vp]
        L.dc_check.argtypes = [vp, vp]
        L.dc_select_kernels.argtypes = [vp, i32]
        L.dc_last_totals.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), vp]
        L.dc_last_error.argtypes = [vp]
        L.dc_last_error.restype = C.c_char_p
        L.dc_profile_begin.argtypes = [vp]
        L.dc_profile_end.argtypes = [vp, C.POINTER(C.c_char_p), fp, C.POINTER(i32), i32]
        for n in ("dc_create", "dc_destroy", "dc_set_weights", "dc_set_attention_weights", "dc_set_base_graphs", "dc_contract_graphs",
                  "dc_gnn_forward", "dc_eval_candidates", "dc_simulate", "dc_check", "dc_last_totals", "dc_profile_begin",
                  "dc_profile_end", "dc_set_profile", "dc_module_times", "dc_cost_candidates", "dc_last_fused_ops",
                  "dc_last_fused_op_repeats", "dc_search",
                  "dc_train_begin", "dc_select_kernels", "dc_fused_op_batch", "dc_loss_gradients", "dc_train_step", "dc_get_weights"):
            getattr(L, n).restype = i32
        _lib = L
    return _lib


# ---- the C ABI, name for name -------------------------------------------------
def dc_workspace_bytes(cfg: DcConfig) -> int:
    return int(lib().dc_workspace_bytes(C.byref(cfg)))


def dc_create(cfg: DcConfig) -> Tuple[int, Optional[int]]:
    h = C.c_void_p()
    st = lib().dc_create(C.byref(h), C.byref(cfg))
    return st, h.value


def dc_destroy(ctx: int) -> int:
    return lib().dc_destroy(ctx)


def dc_set_weights(ctx, W_layers: np.ndarray, b_layers: np.ndarray, head: np.ndarray, stream: int = 0) -> int:
    return lib().dc_set_weights(ctx, W_layers.ctypes.data, b_layers.ctypes.data, head.ctypes.data, stream)


def dc_set_attention_weights(ctx, W_layers: np.ndarray, att: np.ndarray, b_layers: np.ndarray, head: np.ndarray,
                             stream: int = 0) -> int:
    return lib().dc_set_attention_weights(ctx, W_layers.ctypes.data, att.ctypes.data, b_layers.ctypes.data,
                                          head.ctypes.data, stream)


def dc_set_base_graphs(ctx, n_graphs, g_node_off, g_edge_off, rowptr, col, X, stream: int = 0) -> int:
    return lib().dc_set_base_graphs(ctx, n_graphs, g_node_off.ctypes.data, g_edge_off.ctypes.data,
                                    rowptr.ctypes.data, col.ctypes.data if col.size else None, X.ctypes.data, stream)


def dc_contract_graphs(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, batch: DcBatch, stream: int = 0) -> int:
    return lib().dc_contract_graphs(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, C.byref(batch), stream)


def dc_gnn_forward(ctx, batch: DcBatch, pred_ptr, stream: int = 0) -> int:
    return lib().dc_gnn_forward(ctx, C.byref(batch), pred_ptr, stream)


def dc_eval_candidates(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, pred_ptr, stream: int = 0) -> int:
    return lib().dc_eval_candidates(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, pred_ptr, stream)


def dc_simulate(ctx, batch: DcBatch, op_time_ptr, ar_size_ptr, ar_c: float, ar_d: float, cost_ptr,
                stream: int = 0) -> int:
    return lib().dc_simulate(ctx, C.byref(batch), op_time_ptr, ar_size_ptr, ar_c, ar_d, cost_ptr, stream)


def dc_set_profile(ctx, op_time: np.ndarray, ar_size: np.ndarray, stream: int = 0) -> int:
    return lib().dc_set_profile(ctx, op_time.ctypes.data, ar_size.ctypes.data, stream)


def dc_module_times(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, batch: DcBatch, op_time_ptr, ar_size_ptr,
                    stream: int = 0) -> int:
    return lib().dc_module_times(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, C.byref(batch), op_time_ptr,
                                 ar_size_ptr, stream)


def dc_cost_candidates(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, ar_c: float, ar_d: float, cost_ptr,
                       stream: int = 0) -> int:
    return lib().dc_cost_candidates(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, ar_c, ar_d, cost_ptr,
                                    stream)


def dc_last_fused_ops(ctx, stream: int = 0) -> Tuple[int, int, int, int]:
    k, m, e = C.c_int64(), C.c_int64(), C.c_int64()
    st = lib().dc_last_fused_ops(ctx, C.byref(k), C.byref(m), C.byref(e), stream)
    return st, k.value, m.value, e.value


def dc_last_fused_op_repeats(ctx, stream: int = 0) -> Tuple[int, int]:
    n = C.c_int64()
    st = lib().dc_last_fused_op_repeats(ctx, C.byref(n), stream)
    return st, n.value


def dc_search(ctx, graph: int, params: DcSearchParams, labels_opt: Optional[np.ndarray], res: DcSearchResult,
              stream: int = 0) -> int:
    return lib().dc_search(ctx, graph, C.byref(params), None if labels_opt is None else labels_opt.ctypes.data,
                           C.byref(res), stream)


def dc_num_params(ctx) -> int:
    return int(lib().dc_num_params(ctx))


def dc_train_begin(ctx, params: DcTrainParams, stream: int = 0) -> int:
    return lib().dc_train_begin(ctx, C.byref(params), stream)


def dc_fused_op_batch(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, batch: DcBatch, stream: int = 0) -> int:
    return lib().dc_fused_op_batch(ctx, n_cand, cand_graph_ptr, cand_off_ptr, group_id_ptr, C.byref(batch), stream)


def dc_loss_gradients(ctx, batch: DcBatch, target_ptr, loss_ptr, pred_ptr, grad_ptr, stream: int = 0) -> int:
    return lib().dc_loss_gradients(ctx, C.byref(batch), target_ptr, loss_ptr, pred_ptr, grad_ptr, stream)


def dc_train_step(ctx, batch: DcBatch, target_ptr, loss_ptr, stream: int = 0) -> int:
    return lib().dc_train_step(ctx, C.byref(batch), target_ptr, loss_ptr, stream)


def dc_get_weights(ctx, W_layers: np.ndarray, b_layers: np.ndarray, head: np.ndarray, stream: int = 0) -> int:
    return lib().dc_get_weights(ctx, W_layers.ctypes.data, b_layers.ctypes.data, head.ctypes.data, stream)


def dc_check(ctx, stream: int = 0) -> int:
    return lib().dc_check(ctx, stream)


def dc_simulate_static(batch: DcBatch, max_module_nodes: int, max_module_edges: int, op_time_ptr, ar_size_ptr,
                       ar_c: float, ar_d: float, cost_ptr, dev_status_ptr, stream: int = 0) -> int:
    return lib().dc_simulate_static(C.byref(batch), max_module_nodes, max_module_edges, op_time_ptr, ar_size_ptr,
                                    ar_c, ar_d, cost_ptr, dev_status_ptr, stream)


def dc_simulate_static_error() -> str:
    return lib().dc_simulate_static_error().decode()


def dc_select_kernels(ctx, which: int) -> int:
    return lib().dc_select_kernels(ctx, which)


def dc_last_totals(ctx, stream: int = 0) -> Tuple[int, int, int]:
    n, e = C.c_int64(), C.c_int64()
    st = lib().dc_last_totals(ctx, C.byref(n), C.byref(e), stream)
    return st, n.value, e.value


def dc_last_error(ctx) -> str:
    return lib().dc_last_error(ctx).decode()


def dc_profile_begin(ctx) -> int:
    return lib().dc_profile_begin(ctx)


def dc_profile_end(ctx) -> Dict[str, Tuple[float, int]]:
    cap = 32
    names = (C.c_char_p * cap)()
    ms = (C.c_float * cap)()
    cnt = (C.c_int32 * cap)()
    n = lib().dc_profile_end(ctx, names, ms, cnt, cap)
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(min(n, cap))}


# ---- convenience wrapper over torch device memory --------------------------------
@dataclass
class DeviceBatch:
    """Device arrays of one dc_batch (torch tensors own the memory)."""
    c: DcBatch
    node_off: "object"
    edge_off: "object"
    new_id: "object"
    out_rowptr: "object"
    out_col: "object"
    in_rowptr: "object"
    in_col: "object"
    Xc: "object"


class Evaluator:
    """Owns one dc_ctx.  Methods move pointers across the C ABI; nothing is computed in Python."""

    def __init__(self, F: int, H: int, L: int, dtype: str, max_cand: int, max_base_nodes: int, max_base_edges: int,
                 max_nodes: int = 0, max_edges: int = 0, device: str = "cuda:0", agg: str = "mean", heads: int = 1):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = DcConfig(F, H, L, DC_BF16 if dtype == "bf16" else DC_F32, max_cand, max_base_nodes,
                            max_base_edges, max_nodes, max_edges,
                            DC_AGG_ATTENTION if agg == "attention" else DC_AGG_MEAN, heads)
        self.dtype = dtype
        self.agg = agg
        st, h = dc_create(self.cfg)
        if st != DC_OK:
            raise DiscoError(st, "dc_create")
        self.ctx = h

    def close(self):
        if getattr(self, "ctx", None):
            dc_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _ok(self, st: int, what: str):
        if st != DC_OK:
            raise DiscoError(st, f"{what}: {dc_last_error(self.ctx)}")

    def set_weights(self, weights):
        W = np.ascontiguousarray(weights.layers, dtype=np.float32)
        b = np.ascontiguousarray(weights.biases, dtype=np.float32)
        hd = np.ascontiguousarray(weights.head, dtype=np.float32)
        if self.agg == "attention":
            at = np.ascontiguousarray(weights.att, dtype=np.float32)
            self._ok(dc_set_attention_weights(self.ctx, W, at, b, hd, self._stream()), "dc_set_attention_weights")
        else:
            self._ok(dc_set_weights(self.ctx, W, b, hd, self._stream()), "dc_set_weights")

    def set_base_graphs(self, g_node_off, g_edge_off, rowptr, col, X):
        gno = np.ascontiguousarray(g_node_off, dtype=np.int32)
        geo = np.ascontiguousarray(g_edge_off, dtype=np.int32)
        rp = np.ascontiguousarray(rowptr, dtype=np.int32)
        ci = np.ascontiguousarray(col, dtype=np.int32)
        Xf = np.ascontiguousarray(X, dtype=np.float32)
        self._ok(dc_set_base_graphs(self.ctx, len(gno) - 1, gno, geo, rp, ci, Xf, self._stream()), "dc_set_base_graphs")

    def to_device(self, a: np.ndarray):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.device)

    def alloc_batch(self, n_cand: int, n_labels: int, cap_nodes: int, cap_edges: int) -> DeviceBatch:
        t = self.torch
        i32 = dict(dtype=t.int32, device=self.device)
        node_off = t.empty(n_cand + 1, **i32)
        edge_off = t.empty(n_cand + 1, **i32)
        new_id = t.empty(max(n_labels, 1), **i32)
        orp = t.empty(cap_nodes + 1, **i32)
        irp = t.empty(cap_nodes + 1, **i32)
        oc = t.empty(max(cap_edges, 1), **i32)
        ic = t.empty(max(cap_edges, 1), **i32)
        Xc = t.empty((max(cap_nodes, 1), self.cfg.F), dtype=t.bfloat16 if self.dtype == "bf16" else t.float32,
                     device=self.device)
        c = DcBatch(n_cand, cap_nodes, cap_edges, node_off.data_ptr(), edge_off.data_ptr(), new_id.data_ptr(),
                    orp.data_ptr(), oc.data_ptr(), irp.data_ptr(), ic.data_ptr(), Xc.data_ptr())
        return DeviceBatch(c, node_off, edge_off, new_id, orp, oc, irp, ic, Xc)

    def contract_graphs(self, cand_graph, cand_off, group_id, batch: DeviceBatch) -> DeviceBatch:
        n_cand = int(cand_graph.numel())
        self._ok(dc_contract_graphs(self.ctx, n_cand, cand_graph.data_ptr(), cand_off.data_ptr(),
                                    group_id.data_ptr(), batch.c, self._stream()), "dc_contract_graphs")
        return batch

    def gnn_forward(self, batch: DeviceBatch, pred=None):
        if pred is None:
            pred = self.torch.empty(max(batch.c.n_cand, 1), dtype=self.torch.float32, device=self.device)
        self._ok(dc_gnn_forward(self.ctx, batch.c, pred.data_ptr(), self._stream()), "dc_gnn_forward")
        return pred[:batch.c.n_cand]

    def simulate(self, batch: DeviceBatch, op_time, ar_size, ar_c: float, ar_d: float, cost=None):
        if cost is None:
            cost = self.torch.empty(max(batch.c.n_cand, 1), dtype=self.torch.float32, device=self.device)
        self._ok(dc_simulate(self.ctx, batch.c, op_time.data_ptr(), ar_size.data_ptr(), ar_c, ar_d,
                             cost.data_ptr(), self._stream()), "dc_simulate")
        return cost[:batch.c.n_cand]

    def eval_candidates(self, cand_graph, cand_off, group_id, pred=None):
        n_cand = int(cand_graph.numel())
        if pred is None:
            pred = self.torch.empty(max(n_cand, 1), dtype=self.torch.float32, device=self.device)
        self._ok(dc_eval_candidates(self.ctx, n_cand, cand_graph.data_ptr(), cand_off.data_ptr(),
                                    group_id.data_ptr(), pred.data_ptr(), self._stream()), "dc_eval_candidates")
        return pred[:n_cand]

    def set_profile(self, op_time: np.ndarray, ar_size: np.ndarray):
        t = np.ascontiguousarray(op_time, dtype=np.float32)
        x = np.ascontiguousarray(ar_size, dtype=np.float32)
        self._ok(dc_set_profile(self.ctx, t, x, self._stream()), "dc_set_profile")

    def module_times(self, cand_graph, cand_off, group_id, batch: DeviceBatch, op_time=None, ar_size=None):
        n_cand = int(cand_graph.numel())
        f32 = dict(dtype=self.torch.float32, device=self.device)
        if op_time is None:
            op_time = self.torch.empty(max(batch.c.cap_nodes, 1), **f32)
        if ar_size is None:
            ar_size = self.torch.empty(max(batch.c.cap_nodes, 1), **f32)
        self._ok(dc_module_times(self.ctx, n_cand, cand_graph.data_ptr(), cand_off.data_ptr(), group_id.data_ptr(),
                                 batch.c, op_time.data_ptr(), ar_size.data_ptr(), self._stream()), "dc_module_times")
        return op_time, ar_size

    def cost_candidates(self, cand_graph, cand_off, group_id, ar_c: float, ar_d: float, cost=None):
        n_cand = int(cand_graph.numel())
        if cost is None:
            cost = self.torch.empty(max(n_cand, 1), dtype=self.torch.float32, device=self.device)
        self._ok(dc_cost_candidates(self.ctx, n_cand, cand_graph.data_ptr(), cand_off.data_ptr(), group_id.data_ptr(),
                                    ar_c, ar_d, cost.data_ptr(), self._stream()), "dc_cost_candidates")
        return cost[:n_cand]

    def search(self, graph: int, n_nodes: int, alpha: float, beta: int, seed: int, ar_c: float, ar_d: float,
               max_unchanged: int = 1000, parents: int = 1, max_steps: int = 1 << 40, max_queue: int = 4096,
               op_draw: int = 0):
        """Alg. 1 on base graph `graph`; returns (labels_opt, DcSearchResult)."""
        p = DcSearchParams(alpha, beta, max_unchanged, parents, max_queue, max_steps, seed, ar_c, ar_d, op_draw)
        r = DcSearchResult()
        labels = np.zeros(n_nodes, np.int32)
        self._ok(dc_search(self.ctx, graph, p, labels, r, self._stream()), "dc_search")
        return labels, r

    # ---- training of the estimator ----
    def num_params(self) -> int:
        return dc_num_params(self.ctx)

    def train_begin(self, lr: float, max_samples: int, max_rows: int, beta1: float = 0.9, beta2: float = 0.999,
                    eps: float = 1e-8, floor: float = 1e-6):
        p = DcTrainParams(lr, beta1, beta2, eps, floor, max_samples, max_rows)
        self._ok(dc_train_begin(self.ctx, p, self._stream()), "dc_train_begin")

    def fused_op_batch(self, cand_graph, cand_off, group_id, batch: DeviceBatch) -> DeviceBatch:
        n_cand = int(cand_graph.numel())
        self._ok(dc_fused_op_batch(self.ctx, n_cand, cand_graph.data_ptr(), cand_off.data_ptr(), group_id.data_ptr(),
                                   batch.c, self._stream()), "dc_fused_op_batch")
        return batch

    def loss_gradients(self, batch: DeviceBatch, target, want_grad: bool = True):
        """(loss [1], pred [n], grad [num_params] or None), device tensors."""
        f32 = dict(dtype=self.torch.float32, device=self.device)
        loss = self.torch.empty(1, **f32)
        pred = self.torch.empty(max(batch.c.n_cand, 1), **f32)
        grad = self.torch.empty(max(self.num_params(), 1), **f32) if want_grad else None
        self._ok(dc_loss_gradients(self.ctx, batch.c, target.data_ptr(), loss.data_ptr(), pred.data_ptr(),
                                   grad.data_ptr() if want_grad else None, self._stream()), "dc_loss_gradients")
        return loss, pred[:batch.c.n_cand], grad

    def train_step(self, batch: DeviceBatch, target, loss=None):
        if loss is None:
            loss = self.torch.empty(1, dtype=self.torch.float32, device=self.device)
        self._ok(dc_train_step(self.ctx, batch.c, target.data_ptr(), loss.data_ptr(), self._stream()), "dc_train_step")
        return loss

    def get_weights(self):
        """(W_layers, b_layers, head) as host fp32 arrays in the layout of dc_set_weights."""
        c = self.cfg
        nW = sum(3 * (c.F if l == 0 else c.H) * c.H for l in range(c.L))
        W = np.empty(nW, np.float32)
        b = np.empty(c.L * c.H, np.float32)
        hd = np.empty(2 * c.H * c.H + 3 * c.H + 1, np.float32)
        self._ok(dc_get_weights(self.ctx, W, b, hd, self._stream()), "dc_get_weights")
        return W, b, hd

    def last_fused_ops(self) -> Tuple[int, int, int]:
        st, k, m, e = dc_last_fused_ops(self.ctx, self._stream())
        self._ok(st, "dc_last_fused_ops")
        return k, m, e

    def last_fused_op_repeats(self) -> int:
        st, n = dc_last_fused_op_repeats(self.ctx, self._stream())
        self._ok(st, "dc_last_fused_op_repeats")
        return n

    def check(self) -> int:
        return dc_check(self.ctx, self._stream())

    def select_kernels(self, which: int) -> None:
        st = dc_select_kernels(self.ctx, which)
        if st != DC_OK:
            raise DiscoError(st, "dc_select_kernels")

    def last_totals(self) -> Tuple[int, int]:
        st, n, e = dc_last_totals(self.ctx, self._stream())
        self._ok(st, "dc_last_totals")
        return n, e

    def profile_begin(self):
        self._ok(dc_profile_begin(self.ctx), "dc_profile_begin")

    def profile_end(self):
        return dc_profile_end(self.ctx)


def evaluator_for(w, slack: float = 1.0, max_nodes: int = 0, max_edges: int = 0, device: str = "cuda:0") -> Evaluator:
    """Evaluator sized for workload `w` (a workloads.Workload) with its base graphs and weights set."""
    geo = w.g_edge_off()
    nb = int(w.cand_off[-1])
    eb = int(sum(int(geo[b + 1] - geo[b]) for b in w.cand_graph))
    ev = Evaluator(w.model.F, w.model.H, w.model.L, w.model.dtype, max(w.n_cand, 1), max(int(nb * slack), 1),
                   max(int(eb * slack), 1), max_nodes, max_edges, device, getattr(w.model, "agg", "mean"),
                   getattr(w.model, "heads", 1))
    ev.set_base_graphs(w.g_node_off(), geo, w.cat_rowptr(), w.cat_col(), w.cat_X())
    ev.set_weights(w.weights)
    return ev
