"""ctypes binding of libomega_srpe.so: the same entry points as include/omega_srpe.h.

Only argument marshalling happens here.  PyTorch supplies device memory and the HIP
stream; every step of the path runs inside the library.  There is no fallback: if the
library has not been built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libomega_srpe.so")

OMG_OK, OMG_EINVAL, OMG_ERANGE, OMG_ENOMEM, OMG_ESTATE, OMG_EHIP, OMG_EUNSUPPORTED, OMG_ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7
OMG_HOST, OMG_DEVICE = 0, 1
OMG_F32, OMG_BF16 = 0, 1
OMG_SAGE_MEAN, OMG_GCN_SYM, OMG_GAT, OMG_GCNII = 0, 1, 2, 3
OMG_ACT_NONE, OMG_ACT_RELU, OMG_ACT_ELU = 0, 1, 2
OMG_MAX_LAYERS = 8

EXPORTS = [
    "omg_create", "omg_destroy", "omg_strerror", "omg_set_profiling", "omg_get_timing",
    "omg_build_computation_graph", "omg_graph_sizes", "omg_graph_export", "omg_graph_destroy",
    "omg_init_buffer", "omg_run_layer", "omg_gat_src_logits", "omg_gat_fold", "omg_serve_batch", "omg_last_graph_sizes",
    "omg_precompute_embeddings", "omg_set_policy", "omg_measure_read_rate",
    "omg_cgp_wire_width", "omg_cgp_partition_graph", "omg_cgp_local_aggregate", "omg_cgp_merge_mean",
    "omg_cgp_merge_update", "omg_debug_fail_allocation", "omg_debug_set_fused_sum_limit", "omg_debug_set_small_path", "omg_debug_set_gather_multi", "omg_run_layer_static", "omg_static_scratch_bytes",
]


class omg_base_csr(C.Structure):
    _fields_ = [("n_nodes", C.c_int64), ("indptr", C.c_void_p), ("indices", C.c_void_p)]


class omg_table(C.Structure):
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_int32), ("dim", C.c_int32),
                ("n_rows", C.c_int64), ("ld", C.c_int64)]


class omg_layer(C.Structure):
    _fields_ = [("model", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("heads", C.c_int32),
                ("act", C.c_int32), ("head_mean", C.c_int32), ("leaky_slope", C.c_float), ("aggregator", C.c_int32),
                ("W_self", C.c_void_p), ("W_nb", C.c_void_p), ("a_src", C.c_void_p), ("a_dst", C.c_void_p),
                ("bias", C.c_void_p), ("src_logits", C.c_void_p), ("agg_p", C.c_float), ("agg_eps", C.c_float),
                ("alpha", C.c_float), ("init_rows", C.c_void_p), ("init_ld", C.c_int64), ("fold", C.c_void_p)]


class omg_timing(C.Structure):
    _fields_ = [("build_ms", C.c_float), ("gather_ms", C.c_float * OMG_MAX_LAYERS),
                ("combine_ms", C.c_float * OMG_MAX_LAYERS), ("update_ms", C.c_float * OMG_MAX_LAYERS),
                ("total_ms", C.c_float)]


class OmegaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().omg_strerror(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} ({code})")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2501_08547_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_08547_amd.build` "
                           f"(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
    L.omg_create.argtypes = [C.POINTER(vp), C.POINTER(omg_base_csr), vp]
    L.omg_destroy.argtypes = [vp]
    L.omg_destroy.restype = None
    L.omg_strerror.argtypes = [C.c_int]
    L.omg_strerror.restype = C.c_char_p
    L.omg_set_profiling.argtypes = [vp, C.c_int]
    L.omg_get_timing.argtypes = [vp, C.POINTER(omg_timing)]
    L.omg_build_computation_graph.argtypes = [vp, i32, i64, vp, vp, C.c_int, u32, vp, i64, C.POINTER(vp)]
    L.omg_graph_sizes.argtypes = [vp, C.POINTER(i64 * 4)]
    L.omg_graph_export.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.omg_graph_destroy.argtypes = [vp]
    L.omg_graph_destroy.restype = None
    L.omg_init_buffer.argtypes = [vp, vp, C.POINTER(omg_table), vp, i64, vp, i64]
    L.omg_run_layer.argtypes = [vp, vp, C.c_int, C.POINTER(omg_table), vp, i64, C.POINTER(omg_layer), vp, i64]
    L.omg_run_layer_static.argtypes = L.omg_run_layer.argtypes
    L.omg_static_scratch_bytes.argtypes = []
    L.omg_static_scratch_bytes.restype = C.c_int64
    L.omg_gat_src_logits.argtypes = [vp, C.POINTER(omg_table), C.POINTER(omg_layer), vp]
    L.omg_gat_fold.argtypes = [vp, C.POINTER(omg_layer), vp]
    L.omg_serve_batch.argtypes = [vp, i32, C.POINTER(omg_table), C.POINTER(omg_layer), vp, i64, i32, i64, vp, vp,
                                  C.c_int, u32, vp, i64]
    L.omg_last_graph_sizes.argtypes = [vp, C.POINTER(i64 * 4)]
    L.omg_set_policy.argtypes = [vp, C.c_int, C.c_uint64, vp]
    L.omg_precompute_embeddings.argtypes = [vp, i32, C.POINTER(omg_table), C.POINTER(omg_layer), C.POINTER(omg_table)]
    L.omg_cgp_wire_width.argtypes = [C.POINTER(omg_layer)]
    L.omg_cgp_wire_width.restype = C.c_int64
    L.omg_cgp_partition_graph.argtypes = [vp, vp, vp, i32, i32, C.POINTER(vp)]
    L.omg_cgp_local_aggregate.argtypes = [vp, vp, C.c_int, C.POINTER(omg_table), vp, i64, C.POINTER(omg_layer), vp, i64,
                                          vp, i64]
    L.omg_cgp_merge_mean.argtypes = [vp, i64, i32, vp, i64, C.POINTER(omg_layer), vp, i64]
    L.omg_cgp_merge_update.argtypes = [vp, i64, i32, vp, i64, C.POINTER(omg_layer), vp, i64, vp, i64]
    L.omg_measure_read_rate.argtypes = [vp, vp, i64, i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_float)]
    L.omg_debug_set_fused_sum_limit.argtypes = [vp, i32]
    L.omg_debug_set_small_path.argtypes = [vp, i32]
    L.omg_debug_set_gather_multi.argtypes = [vp, i32]
    L.omg_debug_fail_allocation.argtypes = [i64]
    L.omg_debug_fail_allocation.restype = None
    for name in EXPORTS:
        fn = getattr(L, name)
        # without declared argument types ctypes would pass a Python int as a 32-bit C int: a truncated address
        if fn.argtypes is None:
            raise RuntimeError(f"binding.py declares no argument types for {name}")
        if name not in ("omg_destroy", "omg_graph_destroy", "omg_strerror", "omg_cgp_wire_width",
                        "omg_debug_fail_allocation", "omg_static_scratch_bytes"):
            fn.restype = C.c_int
    _lib = L
    return L


def cgp_wire_width(layer: omg_layer) -> int:
    return int(lib().omg_cgp_wire_width(C.byref(layer)))


def _check(rc: int, where: str):
    if rc != OMG_OK:
        raise OmegaError(rc, where)


def _ptr(t) -> Optional[int]:
    """Address of a torch tensor (device or host) or of a numpy array; None stays None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


_MODEL = {"sage": OMG_SAGE_MEAN, "gcn": OMG_GCN_SYM, "gat": OMG_GAT, "gcnii": OMG_GCNII}
_ACT = {"none": OMG_ACT_NONE, "relu": OMG_ACT_RELU, "elu": OMG_ACT_ELU}
_AGG = {"mean": 0, "sum": 1, "max": 2, "power": 3, "moment": 4}     # OMG_AGG_*
_DTYPE = {"f32": OMG_F32, "bf16": OMG_BF16}


def make_table(data, dtype: str, dim: int) -> omg_table:
    """data: 2-D device tensor (n_rows, ld); fp32 for "f32", int16/uint16/bfloat16 storage for "bf16"."""
    return omg_table(_ptr(data), _DTYPE[dtype], dim, data.shape[0], data.stride(0))


def make_layer(p, dev: dict, src_logits=None, init_rows=None, fold=None) -> omg_layer:
    """p: layer parameters (model, d_in, d_out, heads, act, head_mean, leaky_slope);
    dev: device tensors W_self, W_nb, a_src, a_dst, bias (missing ones None)."""
    return omg_layer(_MODEL[p.model], p.d_in, p.d_out, p.heads, _ACT[p.act], int(p.head_mean), float(p.leaky_slope),
                     _AGG[getattr(p, "aggregator", "mean")],
                     _ptr(dev.get("W_self")), _ptr(dev.get("W_nb")), _ptr(dev.get("a_src")), _ptr(dev.get("a_dst")),
                     _ptr(dev.get("bias")), _ptr(src_logits), float(getattr(p, "agg_p", 1.0)),
                     float(getattr(p, "agg_eps", 0.0)), float(getattr(p, "alpha", 0.0)), _ptr(init_rows),
                     0 if init_rows is None else init_rows.stride(0), _ptr(fold))


class Graph:
    """Owner of an omg_graph handle."""

    def __init__(self, ctx: "Context"):
        self.ctx = ctx
        self.handle = C.c_void_p(None)

    def sizes(self):
        s = (C.c_int64 * 4)()
        _check(lib().omg_graph_sizes(self.handle, C.byref(s)), "omg_graph_sizes")
        return dict(n_cand=s[0], n_target=s[1], rows_in=s[2], nnz_in=s[3])

    def export(self):
        s = self.sizes()
        cand = np.empty(s["n_cand"], np.int32)
        qdeg = np.empty(s["n_cand"], np.int32)
        targets = np.empty(s["n_target"], np.int32)
        indptr = np.empty(s["rows_in"] + 1, np.int64)
        cols = np.empty(s["nnz_in"], np.int32)
        cdeg = np.empty(s["nnz_in"], np.int32)
        _check(lib().omg_graph_export(self.handle, _ptr(cand), _ptr(qdeg), _ptr(targets), _ptr(indptr), _ptr(cols),
                                      _ptr(cdeg)), "omg_graph_export")
        return dict(cand=cand, qdeg=qdeg, targets=targets, indptr=indptr, cols=cols, cdeg=cdeg)

    def destroy(self):
        if self.handle:
            lib().omg_graph_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Context:
    """Owner of an omg_ctx handle.  indptr (int64) and indices (int32) are device tensors that
    must outlive the context."""

    def __init__(self, indptr, indices, stream: Optional[int] = None):
        L = lib()
        self._keep = (indptr, indices)
        csr = omg_base_csr(indptr.shape[0] - 1, _ptr(indptr), _ptr(indices))
        self.handle = C.c_void_p(None)
        _check(L.omg_create(C.byref(self.handle), C.byref(csr), stream), "omg_create")

    def close(self):
        if self.handle:
            lib().omg_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_policy(self, policy: str = "ratio", seed: int = 0, node_scores=None):
        """policy: "ratio" (the paper's) | "random" (seeded) | "score" (node_scores: fp32 device tensor [n_nodes],
        kept alive by this object)."""
        self._scores = node_scores
        _check(lib().omg_set_policy(self.handle, {"ratio": 0, "random": 1, "score": 2}[policy], seed, _ptr(node_scores)),
               "omg_set_policy")

    def debug_set_fused_sum_limit(self, limit: int):
        _check(lib().omg_debug_set_fused_sum_limit(self.handle, limit), "omg_debug_set_fused_sum_limit")

    def debug_set_small_path(self, on):
        _check(lib().omg_debug_set_small_path(self.handle, int(on)), "omg_debug_set_small_path")

    def debug_set_gather_multi(self, on: int):
        _check(lib().omg_debug_set_gather_multi(self.handle, int(on)), "omg_debug_set_gather_multi")

    def set_profiling(self, on):
        _check(lib().omg_set_profiling(self.handle, int(on)), "omg_set_profiling")

    def get_timing(self) -> omg_timing:
        t = omg_timing()
        _check(lib().omg_get_timing(self.handle, C.byref(t)), "omg_get_timing")
        return t

    def build_computation_graph(self, n_query: int, qe_query, qe_node, gamma_ppm: int, recompute_set=None,
                                graph: Optional[Graph] = None) -> Graph:
        """Edge arrays: int32 numpy arrays (host) or int32 device tensors."""
        where = OMG_HOST if isinstance(qe_query, np.ndarray) else OMG_DEVICE
        g = graph if graph is not None else Graph(self)
        n_r = 0 if recompute_set is None else int(recompute_set.shape[0])
        _check(lib().omg_build_computation_graph(self.handle, n_query, int(qe_query.shape[0]), _ptr(qe_query),
                                                 _ptr(qe_node), where, gamma_ppm, _ptr(recompute_set), n_r,
                                                 C.byref(g.handle)), "omg_build_computation_graph")
        return g

    def init_buffer(self, graph: Graph, features: omg_table, query_feats, buf0):
        _check(lib().omg_init_buffer(self.handle, graph.handle, C.byref(features), _ptr(query_feats),
                                     query_feats.stride(0), _ptr(buf0), buf0.stride(0)), "omg_init_buffer")

    def run_layer(self, graph: Graph, is_last: bool, table_prev: omg_table, buf_prev, layer: omg_layer, buf_out):
        _check(lib().omg_run_layer(self.handle, graph.handle, int(is_last), C.byref(table_prev), _ptr(buf_prev),
                                   buf_prev.stride(0), C.byref(layer), _ptr(buf_out), buf_out.stride(0)),
               "omg_run_layer")

    def run_layer_static(self, graph: Graph, is_last: bool, table_prev: omg_table, buf_prev, layer: omg_layer, buf_out):
        """omg_run_layer with its scratch in the library's static device array: allocates nothing."""
        _check(lib().omg_run_layer_static(self.handle, graph.handle, int(is_last), C.byref(table_prev), _ptr(buf_prev),
                                          buf_prev.stride(0), C.byref(layer), _ptr(buf_out), buf_out.stride(0)),
               "omg_run_layer_static")

    def gat_fold(self, layer: omg_layer, fold):
        """fold: fp32 device tensor of 2 x heads x d_in values (the layer's folded score vectors)."""
        _check(lib().omg_gat_fold(self.handle, C.byref(layer), _ptr(fold)), "omg_gat_fold")

    def gat_src_logits(self, table: omg_table, layer: omg_layer, logits):
        _check(lib().omg_gat_src_logits(self.handle, C.byref(table), C.byref(layer), _ptr(logits)),
               "omg_gat_src_logits")

    def serve_batch(self, tables: Sequence[omg_table], layers: Sequence[omg_layer], query_feats, n_query: int,
                    qe_query, qe_node, gamma_ppm: int, out):
        k = len(layers)
        where = OMG_HOST if isinstance(qe_query, np.ndarray) else OMG_DEVICE
        tarr = (omg_table * k)(*tables)
        larr = (omg_layer * k)(*layers)
        _check(lib().omg_serve_batch(self.handle, k, tarr, larr, _ptr(query_feats), query_feats.stride(0), n_query,
                                     int(qe_query.shape[0]), _ptr(qe_query), _ptr(qe_node), where, gamma_ppm,
                                     _ptr(out), out.stride(0)), "omg_serve_batch")

    def precompute_embeddings(self, features: omg_table, layers: Sequence[omg_layer], out_tables: Sequence[omg_table]):
        """Fills out_tables[l - 1] with layer l's output for every node of the training graph, l = 1..k-1."""
        k = len(layers)
        larr = (omg_layer * k)(*layers)
        oarr = (omg_table * max(1, k - 1))(*out_tables)
        _check(lib().omg_precompute_embeddings(self.handle, k, C.byref(features), larr, oarr), "omg_precompute_embeddings")

    # ---- computation graph parallelism (one partition's share; the merge)
    def cgp_partition_graph(self, graph: Graph, node_part, n_part: int, p: int, part_graph: Optional[Graph] = None) -> Graph:
        """node_part: int32 device tensor [n_nodes]."""
        g = part_graph if part_graph is not None else Graph(self)
        _check(lib().omg_cgp_partition_graph(self.handle, graph.handle, _ptr(node_part), n_part, p, C.byref(g.handle)),
               "omg_cgp_partition_graph")
        return g

    def cgp_local_aggregate(self, part_graph: Graph, is_last: bool, table_prev: omg_table, buf_prev, layer: omg_layer,
                            wire, row_mean=None):
        """wire: 2-D fp32 device tensor (n_rows, ld_wire): this partition's block of the record buffer."""
        _check(lib().omg_cgp_local_aggregate(self.handle, part_graph.handle, int(is_last), C.byref(table_prev),
                                             _ptr(buf_prev), buf_prev.stride(0), C.byref(layer), _ptr(row_mean),
                                             0 if row_mean is None else row_mean.stride(0), _ptr(wire), wire.stride(0)),
               "omg_cgp_local_aggregate")

    def cgp_merge_mean(self, wire, layer: omg_layer, row_mean):
        """wire: 3-D fp32 device tensor (n_part, n_rows, ld_wire), contiguous."""
        _check(lib().omg_cgp_merge_mean(self.handle, wire.shape[1], wire.shape[0], _ptr(wire), wire.stride(1),
                                        C.byref(layer), _ptr(row_mean), row_mean.stride(0)), "omg_cgp_merge_mean")

    def cgp_merge_update(self, wire, layer: omg_layer, buf_prev, buf_out):
        _check(lib().omg_cgp_merge_update(self.handle, wire.shape[1], wire.shape[0], _ptr(wire), wire.stride(1),
                                          C.byref(layer), _ptr(buf_prev), buf_prev.stride(0), _ptr(buf_out),
                                          buf_out.stride(0)), "omg_cgp_merge_update")

    def measure_read_rate(self, buffer, reps: int, blocks: int):
        """(bytes read, milliseconds) of a plain read sweep over a device tensor (measurement aid)."""
        nbytes, ms = C.c_double(0.0), C.c_float(0.0)
        _check(lib().omg_measure_read_rate(self.handle, _ptr(buffer), buffer.numel() * buffer.element_size(),
                                           reps, blocks, C.byref(nbytes), C.byref(ms)), "omg_measure_read_rate")
        return nbytes.value, ms.value

    def last_graph_sizes(self):
        s = (C.c_int64 * 4)()
        _check(lib().omg_last_graph_sizes(self.handle, C.byref(s)), "omg_last_graph_sizes")
        return dict(n_cand=s[0], n_target=s[1], rows_in=s[2], nnz_in=s[3])
