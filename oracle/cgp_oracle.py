"""CPU oracle for computation graph parallelism (Omega, arXiv 2501.08547, Sec. 6).  TEST INFRASTRUCTURE ONLY.

A plain fp64 statement of what ONE layer computes when the batch's computation graph is split over P
partitions by the partition of each edge's source: every partition aggregates the neighbours it holds
(local aggregation, Sec. 6.1, Eq. 3), the local aggregations of a destination are brought together (on
several GPUs: one all-to-all) and a merge function tailored to the aggregation turns them into the value
the unpartitioned layer would have computed, after which the layer's update runs as usual (Sec. 6.2).
Nothing here is shared with the GPU library, and nothing here receives values from it.  The layer
definitions themselves are srpe_oracle.layer_row's; this file restates only what Sec. 6 adds.

Steps, in the paper's order
  1. request partitioning: query q belongs to partition q mod P (queries are dealt out evenly); an edge
     belongs to the partition of its SOURCE; an existing node belongs to node_part[u]         (Sec. 6.1)
  2. partitioned computation graph of partition p: the rows of the batch's graph (all queries, all
     recompute targets: the targets are made known to every builder), each row holding only the edges
     whose source is in p, in the order they have in the whole graph                          (Sec. 6.1)
  3. local aggregation a_{v,p} over N_p(v)                                                    (Eq. 3)
  4. merge of {a_{v,p}}_p, then the update function                                           (Eq. 3, Sec. 6.2)

What a partition hands over for a destination (the "wire" record), per aggregation
  mean, sum      sum of the local messages, and their number
  max            element-wise maximum of the local messages (minus infinity where it holds none)
  power mean     sum of the local messages raised to p (Sec. 6.2); merge adds, divides by the total number of
                 messages and takes the 1/p-th power
  moments        first the mean of ALL messages of the destination is formed (a merge of local sums) and made
                 known to every partition; then as the power mean, on (message - mean)^n      (Sec. 6.2)
  softmax (GAT)  per head: the largest local score, the sum of exp(score - that maximum), and the sum of the
                 projected sources weighted by the same exponentials; merge rescales every partition's two sums
                 by exp(its maximum - the overall maximum), adds them and divides               (Sec. 6.2)
  GCN, GCNII     (reading; the paper does not discuss their normalisation) 1 / sqrt(d_u d_v) factors: the
                 source's part is applied locally, the destination's part and the self term by the merge, which
                 knows d_v as the total number of messages plus one

Readings where the paper is silent
  * q mod P for "evenly assigns partitions to every query node"
  * a freshly computed row used as a source lives in the partition of its node (the partition that
    merged and updated it), a query row in the query's partition
  * the per-builder recomputation policy (each builder choosing among its own candidates) is a choice of
    the recompute set and is not restated here: these functions take the batch's graph as given

Parity pins live in tests/test_oracle_pins.py (the merged result equals the unpartitioned layer for every
model and aggregation, closed-form softmax merges, stability with huge scores, partition structure).
Unpinned: nothing in this file.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from .srpe_oracle import LazyTable, OracleGraph, _act


@dataclass
class PartGraph:
    """Partition p's share of a computation graph: same rows, only the edges whose source is in p."""
    p: int
    indptr: np.ndarray   # int64 [rows_in + 1]
    cols: np.ndarray     # int32, tagged as in the whole graph
    cdeg: np.ndarray     # int32


def row_partitions(g: OracleGraph, node_part: np.ndarray, n_part: int) -> np.ndarray:
    """Partition of every freshly computed row: query q -> q mod P, target t -> node_part[t]."""
    q = np.arange(g.n_query, dtype=np.int64) % n_part
    return np.concatenate([q, np.asarray(node_part, dtype=np.int64)[g.T]])


def source_partitions(g: OracleGraph, node_part: np.ndarray, n_part: int) -> np.ndarray:
    """Partition of every edge of the whole graph = partition of its source (Sec. 6.1)."""
    rp = row_partitions(g, node_part, n_part)
    c = g.cols.astype(np.int64)
    out = np.empty(c.shape[0], dtype=np.int64)
    stored = c >= 0
    out[stored] = np.asarray(node_part, dtype=np.int64)[c[stored]]
    out[~stored] = rp[~c[~stored]]
    return out


def partition_graph(g: OracleGraph, node_part: np.ndarray, n_part: int, p: int) -> PartGraph:
    sp = source_partitions(g, node_part, n_part)
    indptr = np.zeros(g.rows_in + 1, dtype=np.int64)
    cols: List[int] = []
    cdeg: List[int] = []
    for v in range(g.rows_in):
        for e in range(int(g.indptr[v]), int(g.indptr[v + 1])):
            if sp[e] == p:
                cols.append(int(g.cols[e]))
                cdeg.append(int(g.cdeg[e]))
        indptr[v + 1] = len(cols)
    return PartGraph(p, indptr, np.asarray(cols, dtype=np.int32), np.asarray(cdeg, dtype=np.int32))


def _sources(pg: PartGraph, v: int, d_in: int, table_prev: LazyTable, buf_prev: np.ndarray) -> np.ndarray:
    c = pg.cols[pg.indptr[v]:pg.indptr[v + 1]].astype(np.int64)
    h = np.empty((c.shape[0], d_in))
    stored = c >= 0
    if stored.any():
        h[stored] = table_prev.rows(c[stored])
    if (~stored).any():
        h[~stored] = buf_prev[~c[~stored], :d_in]
    return h


def local_aggregation(layer, h_src: np.ndarray, deg_src: np.ndarray, h_dst: np.ndarray,
                      mean: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """a_{v,p} of Eq. 3 for one destination in one partition.  h_src (n_p, d_in): the local neighbours;
    deg_src their degrees; h_dst the destination's own input (the attention needs it; Sec. 6.2 has it
    all-gathered); mean: the destination's overall message mean (moments, second step)."""
    n = h_src.shape[0]
    d = h_src.shape[1]
    rec: Dict[str, np.ndarray] = {"count": np.float64(n)}
    if layer.model == "sage":
        kind = getattr(layer, "aggregator", "mean")
        if kind in ("mean", "sum"):
            rec["sum"] = h_src.sum(axis=0)
        elif kind == "max":
            rec["max"] = h_src.max(axis=0) if n else np.full(d, -np.inf)
        elif kind == "power":
            rec["sum"] = ((np.maximum(h_src, 0.0) + float(layer.agg_eps)) ** float(layer.agg_p)).sum(axis=0)
        elif kind == "moment":
            if mean is None:
                rec["sum"] = h_src.sum(axis=0)                       # first step: towards the overall mean
            else:
                rec["sum"] = ((h_src - mean[None, :]) ** int(layer.agg_p)).sum(axis=0)
        else:
            raise ValueError(kind)
        return rec
    if layer.model in ("gcn", "gcnii"):
        w = 1.0 / np.sqrt(np.asarray(deg_src, dtype=np.float64) + 1.0)
        rec["sum"] = (w[:, None] * h_src).sum(axis=0)
        return rec
    if layer.model == "gat":
        H = layer.heads
        dh = layer.d_out // H
        W = np.asarray(layer.W_nb, dtype=np.float64)
        a_s = np.asarray(layer.a_src, dtype=np.float64)
        a_d = np.asarray(layer.a_dst, dtype=np.float64)
        z_dst = (h_dst @ W).reshape(H, dh)
        if n == 0:
            rec["max"] = np.full(H, -np.inf)
            rec["expsum"] = np.zeros(H)
            rec["wsum"] = np.zeros((H, dh))
            return rec
        z = (h_src @ W).reshape(n, H, dh)
        e = (z * a_s[None]).sum(-1) + (z_dst * a_d).sum(-1)[None]
        e = np.where(e > 0.0, e, layer.leaky_slope * e)
        m = e.max(axis=0)
        w = np.exp(e - m[None])
        rec["max"] = m
        rec["expsum"] = w.sum(axis=0)
        rec["wsum"] = (w[:, :, None] * z).sum(axis=0)
        return rec
    raise ValueError(layer.model)


def merge(layer, recs: List[Dict[str, np.ndarray]]) -> np.ndarray:
    """The merge function of Eq. 3 for one destination: the P local aggregations -> what the aggregation
    over the whole neighbourhood gives.  For SAGE-style layers the aggregated vector; for GCN / GCNII the
    neighbour part of the normalised sum (without the self term); for GAT the (heads, d_head) attention
    output before the bias."""
    total = float(sum(float(r["count"]) for r in recs))
    if layer.model == "sage":
        kind = getattr(layer, "aggregator", "mean")
        if kind == "max":
            if total == 0:
                return np.zeros_like(recs[0]["max"])
            out = recs[0]["max"]
            for r in recs[1:]:
                out = np.maximum(out, r["max"])
            return out
        s = sum(r["sum"] for r in recs)
        if total == 0:
            return np.zeros_like(s)
        if kind == "sum":
            return s
        if kind == "mean":
            return s / total
        if kind == "power":
            return (s / total) ** (1.0 / float(layer.agg_p))
        if kind == "moment":
            c = s / total
            return np.sign(c) * np.abs(c) ** (1.0 / int(layer.agg_p))
        raise ValueError(kind)
    if layer.model in ("gcn", "gcnii"):
        return sum(r["sum"] for r in recs) / np.sqrt(total + 1.0)
    if layer.model == "gat":
        if total == 0:
            return np.zeros_like(recs[0]["wsum"])
        M = recs[0]["max"]
        for r in recs[1:]:
            M = np.maximum(M, r["max"])
        S = np.zeros_like(M)
        acc = np.zeros_like(recs[0]["wsum"])
        for r in recs:
            f = np.exp(r["max"] - M)                 # exp(-inf) = 0 for a partition that holds no neighbour
            S = S + f * r["expsum"]
            acc = acc + f[:, None] * r["wsum"]
        return acc / S[:, None]
    raise ValueError(layer.model)


def message_mean(recs: List[Dict[str, np.ndarray]]) -> np.ndarray:
    """Moments, first step: the mean of all of a destination's messages from the local sums."""
    total = float(sum(float(r["count"]) for r in recs))
    s = sum(r["sum"] for r in recs)
    return s / total if total else np.zeros_like(s)


def update(layer, h_self: np.ndarray, merged: np.ndarray, total_count: float,
           h0_self: Optional[np.ndarray] = None) -> np.ndarray:
    """U of Eq. 3: the layer's update applied to the destination's own input and the merged aggregation."""
    W = np.asarray(layer.W_nb, dtype=np.float64)
    b = np.asarray(layer.bias, dtype=np.float64)
    if layer.model == "sage":
        return _act(h_self @ np.asarray(layer.W_self, dtype=np.float64) + merged @ W + b, layer.act)
    if layer.model in ("gcn", "gcnii"):
        agg = h_self / (total_count + 1.0) + merged
        if layer.model == "gcnii":
            agg = (1.0 - float(layer.alpha)) * agg + float(layer.alpha) * np.asarray(h0_self, dtype=np.float64)
        return _act(agg @ W + b, layer.act)
    if layer.model == "gat":
        H = layer.heads
        out = merged + b.reshape(H, layer.d_out // H)
        return _act(out.mean(axis=0) if layer.head_mean else out.reshape(-1), layer.act)
    raise ValueError(layer.model)


def run_layer_cgp(g: OracleGraph, parts: List[PartGraph], layer, table_prev: LazyTable, buf_prev: np.ndarray,
                  is_last: bool, buf0: Optional[np.ndarray] = None, return_wire: bool = False):
    """One layer under CGP: local aggregations in every partition, merge, update (Eq. 3)."""
    n_rows = g.n_query if is_last else g.rows_in
    d = layer.d_in
    out = np.zeros((n_rows, layer.out_width))
    wire: List[List[Dict[str, np.ndarray]]] = []
    two_step = layer.model == "sage" and getattr(layer, "aggregator", "mean") == "moment"
    for v in range(n_rows):
        h_dst = buf_prev[v, :d]
        srcs = [(_sources(pg, v, d, table_prev, buf_prev), pg.cdeg[pg.indptr[v]:pg.indptr[v + 1]]) for pg in parts]
        mean = None
        if two_step:
            mean = message_mean([local_aggregation(layer, h, c, h_dst) for h, c in srcs])
        recs = [local_aggregation(layer, h, c, h_dst, mean) for h, c in srcs]
        total = float(sum(float(r["count"]) for r in recs))
        merged = merge(layer, recs)
        out[v] = update(layer, h_dst, merged, total, None if buf0 is None else buf0[v, :d])
        wire.append(recs)
    return (out, wire) if return_wire else out


def cgp_reference(g: OracleGraph, node_part: np.ndarray, n_part: int, tables: List[LazyTable], layers,
                  query_feats: np.ndarray) -> np.ndarray:
    """k layers under CGP over the batch's computation graph; returns h_q^(k) for the B queries."""
    from .srpe_oracle import initial_buffer
    parts = [partition_graph(g, node_part, n_part, p) for p in range(n_part)]
    k = len(layers)
    buf0 = initial_buffer(g, tables[0], query_feats)
    buf = buf0
    for l in range(1, k + 1):
        buf = run_layer_cgp(g, parts, layers[l - 1], tables[l - 1], buf, is_last=(l == k), buf0=buf0)
    return buf
