"""Plumbing: puts a workload's arrays into device memory (via PyTorch) and wraps them in the
structures the library takes.  No arithmetic of the method happens here."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from . import binding as B


def _dev(a: np.ndarray, device) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


@dataclass
class DeviceModel:
    ctx: B.Context
    indptr: torch.Tensor
    indices: torch.Tensor
    table_data: List[torch.Tensor]
    tables: List[B.omg_table]
    weights: List[dict]
    layers: List[B.omg_layer]
    params: list
    side: List[Optional[torch.Tensor]] = field(default_factory=list)

    def out_width(self) -> int:
        return self.params[-1].out_width

    def close(self):
        self.ctx.close()


def upload(built, device="cuda:0", stream: Optional[int] = None, gat_side_tables: bool = True) -> DeviceModel:
    """built: synth.configs.Built.  Creates the context on the current stream of `device`."""
    dev = torch.device(device)
    torch.cuda.set_device(dev)
    indptr = _dev(built.graph.indptr.astype(np.int64), dev)
    indices = _dev(built.graph.indices.astype(np.int32), dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    ctx = B.Context(indptr, indices, stream)
    table_data, tables = [], []
    for t in built.tables:
        d = _dev(t.data, dev)
        table_data.append(d)
        tables.append(B.make_table(d, t.dtype, t.dim))
    weights, layers, side = [], [], []
    for l, p in enumerate(built.layers):
        w = {k: _dev(getattr(p, k), dev) for k in ("W_self", "W_nb", "a_src", "a_dst", "bias")
             if getattr(p, k) is not None}
        weights.append(w)
        lay = B.make_layer(p, w)
        s = None
        if p.model == "gat" and gat_side_tables:
            # once per model: the folded score vectors and the stored rows' score halves
            w["fold"] = torch.empty(2 * p.heads * p.d_in, dtype=torch.float32, device=dev)
            ctx.gat_fold(lay, w["fold"])
            s = torch.empty((tables[l].n_rows, p.heads), dtype=torch.float32, device=dev)
            ctx.gat_src_logits(tables[l], lay, s)
            lay = B.make_layer(p, w, src_logits=s, fold=w["fold"])
        side.append(s)
        layers.append(lay)
    torch.cuda.synchronize(dev)
    return DeviceModel(ctx, indptr, indices, table_data, tables, weights, layers, list(built.layers), side)


def assemble(indptr: torch.Tensor, indices: torch.Tensor, tables, params, stream: Optional[int] = None,
             gat_side_tables: bool = True) -> DeviceModel:
    """Same as upload() for arrays that already are device tensors.  tables: list of
    (tensor (n_rows, ld), "f32" | "bf16", dim); params: layer parameters with host weights."""
    dev = indptr.device
    torch.cuda.set_device(dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    ctx = B.Context(indptr, indices, stream)
    table_data = [t for t, _, _ in tables]
    tabs = [B.make_table(t, dt, dim) for t, dt, dim in tables]
    weights, layers, side = [], [], []
    for l, p in enumerate(params):
        w = {k: _dev(getattr(p, k), dev) for k in ("W_self", "W_nb", "a_src", "a_dst", "bias")
             if getattr(p, k) is not None}
        weights.append(w)
        lay = B.make_layer(p, w)
        s = None
        if p.model == "gat" and gat_side_tables:
            # once per model: the folded score vectors and the stored rows' score halves
            w["fold"] = torch.empty(2 * p.heads * p.d_in, dtype=torch.float32, device=dev)
            ctx.gat_fold(lay, w["fold"])
            s = torch.empty((tabs[l].n_rows, p.heads), dtype=torch.float32, device=dev)
            ctx.gat_src_logits(tabs[l], lay, s)
            lay = B.make_layer(p, w, src_logits=s, fold=w["fold"])
        side.append(s)
        layers.append(lay)
    torch.cuda.synchronize(dev)
    return DeviceModel(ctx, indptr, indices, table_data, tabs, weights, layers, list(params), side)


def second_context(dm: DeviceModel, stream: int) -> DeviceModel:
    """Another context on `stream` over the same graph, tables and weights (nothing is copied): batches
    served through different contexts may overlap on the device."""
    ctx = B.Context(dm.indptr, dm.indices, stream)
    return DeviceModel(ctx, dm.indptr, dm.indices, dm.table_data, dm.tables, dm.weights, dm.layers, dm.params, dm.side)


def precompute_tables(dm: DeviceModel, dtypes: Optional[List[str]] = None) -> List[torch.Tensor]:
    """Overwrites the model's embedding tables (tables[1..k-1]) with embeddings computed by the library on
    the training graph (omg_precompute_embeddings), in the storage types they already have (or `dtypes`).
    Returns the new table tensors; GAT side tables are recomputed for them."""
    k = len(dm.layers)
    n = dm.indptr.shape[0] - 1
    plain = [B.make_layer(p, w) for p, w in zip(dm.params, dm.weights)]          # no side tables while precomputing
    new_data, new_tabs = [], []
    for l in range(1, k):
        dt = dtypes[l - 1] if dtypes is not None else ("f32" if dm.tables[l].dtype == B.OMG_F32 else "bf16")
        dim = dm.params[l - 1].out_width
        es = 4 if dt == "f32" else 2
        ld = -(-dim * es // 16) * 16 // es
        t = torch.zeros((n, ld), dtype=torch.float32 if dt == "f32" else torch.int16, device=dm.indptr.device)
        new_data.append(t)
        new_tabs.append(B.make_table(t, dt, dim))
    torch.cuda.synchronize()
    dm.ctx.precompute_embeddings(dm.tables[0], plain, new_tabs)
    for l in range(1, k):
        dm.table_data[l] = new_data[l - 1]
        dm.tables[l] = new_tabs[l - 1]
        p = dm.params[l]
        if p.model == "gat" and dm.side[l] is not None:
            s = torch.empty((n, p.heads), dtype=torch.float32, device=dm.indptr.device)
            lay = B.make_layer(p, dm.weights[l])
            dm.ctx.gat_src_logits(dm.tables[l], lay, s)
            dm.side[l] = s
            dm.layers[l] = B.make_layer(p, dm.weights[l], src_logits=s, fold=dm.weights[l].get("fold"))
    torch.cuda.synchronize()
    return new_data
