"""CPU oracle for SRPE serving (Omega, arXiv 2501.08547).  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the serving path computes, written from the
paper.  It exists to check the GPU library; nothing in the product path may import
it.  It shares no code with the GPU library and never receives values from it.

What follows the paper directly
  * message passing layer h_v = U(h_v, AGG_{u in N(v)} M(h_u))            (Sec. 2, Eq. 1)
  * precomputed embeddings p_u^(l), l = 1..k-1, replace the layer
    embeddings of nodes that are not recomputed                           (Sec. 5)
  * candidates R = direct neighbours of the query nodes; a candidate is
    either recomputed (its query edges are taken into account) or reused  (Sec. 5.2.1)
  * budget: at most gamma * |R| candidates are recomputed                 (Sec. 5.2.1, Eq. 2)
  * policy: recompute the candidates with the largest |N_Q(u)| / |N(u)|   (Sec. 5.2.2)
  * last layer = edges whose destination is a query node; every other
    layer additionally holds all edges ending at a recompute target;
    layer outputs are joined with the stored embeddings to form the next
    layer's input                                                         (Sec. 6.1)

Readings where the paper is silent (each is listed in the design notes)
  * query edges are undirected: u->q is used for q's rows, q->u only if u is recomputed
  * |N(u)| = base in-degree + number of query edges at u
  * |T| = floor(gamma_ppm * |R| / 10^6); ties in the ratio go to the smaller node id
  * a recomputed node used as a source takes its recomputed value, not the stored one
  * layer math is the textbook form of each cited model (SAGE-mean, GCN with
    self loops and symmetric normalisation over degrees in the graph that includes the
    batch's query edges, GAT with LeakyReLU(0.2) scores and no implicit self loop)
  * duplicate query edges count with multiplicity
  * SAGE-style layers may use the other aggregation functions Sec. 6.2 names (sum, max, power mean,
    normalised moments) in place of the mean; the power mean takes positive messages max(h, 0) + eps

Canonical exported graph (what "bit-exact graph construction" compares)
  rows    : queries 0..B-1, then the targets in ascending node id
  columns : query row  -> its neighbours in ascending node id
            target row -> base in-neighbours in base-CSR order, then its query
                          neighbours in ascending query index
  tag     : col >= 0 reads row `col` of the stored table; col < 0 reads row ~col of
            the buffer of freshly computed rows (queries first, then targets)
  cdeg    : for every column, in-degree of the source in the graph that includes the
            batch (base in-degree + query edges at it; for a query source, its edge count)

Parity pins live in tests/test_oracle_pins.py.  Unpinned: nothing in this file.
(The paper's accuracy results need its datasets and trained weights and are not
reproduced anywhere here.)
"""
from __future__ import annotations

from dataclasses import dataclass
from functools import cmp_to_key
from typing import List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- storage decode

def decode_table(data: np.ndarray, dtype: str, dim: int) -> np.ndarray:
    """Stored table -> fp64 values (n_rows, dim).  bf16 is the upper half of an fp32."""
    if dtype in ("f32", "f64"):
        return np.asarray(data[:, :dim], dtype=np.float64)
    if dtype == "bf16":
        bits = np.ascontiguousarray(data[:, :dim]).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(dtype)


class LazyTable:
    """Row access into a stored table with fp64 decode of only the rows asked for."""

    def __init__(self, data: np.ndarray, dtype: str, dim: int):
        self.data, self.dtype, self.dim = data, dtype, dim

    def rows(self, idx: np.ndarray) -> np.ndarray:
        return decode_table(self.data[idx], self.dtype, self.dim)


# --------------------------------------------------------------------------- graph construction

@dataclass
class OracleGraph:
    n_query: int
    R: np.ndarray        # int64, candidates, ascending
    qdeg: np.ndarray     # int64, query edges at each candidate
    T: np.ndarray        # int64, recompute targets, ascending
    indptr: np.ndarray   # int64 [rows_in + 1]
    cols: np.ndarray     # int32 [nnz_in], tagged
    cdeg: np.ndarray     # int32 [nnz_in]

    @property
    def rows_in(self) -> int:
        return self.n_query + int(self.T.shape[0])

    @property
    def nnz_in(self) -> int:
        return int(self.indptr[-1])


def candidates(qe_node: np.ndarray):
    """Candidates = distinct training endpoints of the query edges, with the number of
    query edges at each (Sec. 5.2.1)."""
    R, qdeg = np.unique(np.asarray(qe_node, dtype=np.int64), return_counts=True)
    return R, qdeg.astype(np.int64)


def select_targets(R: np.ndarray, qdeg: np.ndarray, deg_base: np.ndarray, gamma_ppm: int) -> np.ndarray:
    """Top-query-edges-ratio policy (Sec. 5.2.2) under the budget of Eq. 2.

    score(u) = qdeg(u) / (deg_base(u) + qdeg(u)), compared exactly as fractions;
    equal scores go to the smaller node id.  Returns the targets in ascending id."""
    n_take = (int(gamma_ppm) * int(R.shape[0])) // 1_000_000
    if n_take == 0:
        return np.empty(0, dtype=np.int64)
    cand = [(int(q), int(q) + int(d), int(u)) for u, q, d in zip(R, qdeg, deg_base)]

    def better_first(a, b):
        lhs, rhs = a[0] * b[1], b[0] * a[1]          # a0/a1 vs b0/b1 by cross-multiplication
        if lhs != rhs:
            return -1 if lhs > rhs else 1
        return -1 if a[2] < b[2] else (1 if a[2] > b[2] else 0)

    cand.sort(key=cmp_to_key(better_first))
    return np.array(sorted(c[2] for c in cand[:n_take]), dtype=np.int64)


_M64 = (1 << 64) - 1


def random_policy_key(seed: int, node: int) -> int:
    """Key of the RANDOM policy: the top 39 bits of the splitmix64 finaliser of seed * C + node.  A
    counter-based generator, so that every implementation draws the same numbers."""
    z = (int(node) + int(seed) * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    z = z ^ (z >> 31)
    return z >> 25


def select_targets_alt(R: np.ndarray, gamma_ppm: int, policy: str, seed: int = 0,
                       node_scores: Optional[np.ndarray] = None) -> np.ndarray:
    """The alternative policies the paper compares with (Sec. 5.2.2), under the same budget:
      "random"  targets drawn at random: the candidates with the largest random keys
      "score"   the candidates with the largest per-node score (fp32, finite), e.g. the node importance
                IS(v) or the measured approximation error (AE)
    Equal keys / scores go to the smaller node id.  Returns the targets in ascending id."""
    n_take = (int(gamma_ppm) * int(R.shape[0])) // 1_000_000
    if n_take == 0:
        return np.empty(0, dtype=np.int64)
    if policy == "random":
        keyed = [(-random_policy_key(seed, int(u)), int(u)) for u in R]
    elif policy == "score":
        sc = np.asarray(node_scores, dtype=np.float32)
        if not np.all(np.isfinite(sc[R])):
            raise ValueError("scores must be finite")
        keyed = [(-float(sc[int(u)]), int(u)) for u in R]      # -0.0 and 0.0 compare equal, as floats do
    else:
        raise ValueError(policy)
    keyed.sort()
    return np.array(sorted(u for _, u in keyed[:n_take]), dtype=np.int64)


def importance_scores(base_indptr: np.ndarray, base_indices: np.ndarray) -> np.ndarray:
    """IS(v) = (1 / deg(v)) sum_{u in N(v)} 1 / deg(u) (Sec. 5.2.2), fp64; 0 for isolated nodes and for
    neighbours without in-edges."""
    deg = np.diff(base_indptr).astype(np.float64)
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1.0), 0.0)
    out = np.zeros(deg.shape[0])
    for v in range(deg.shape[0]):
        nb = base_indices[base_indptr[v]:base_indptr[v + 1]]
        if nb.size:
            out[v] = inv[nb].sum() / deg[v]
    return out


def approximation_errors(full_embeddings: List[np.ndarray], tables: List["LazyTable"], R: np.ndarray) -> np.ndarray:
    """Per candidate u: sum_{l=1}^{k-1} || f_u^(l) - p_u^(l) ||_2 (Sec. 5.1), f = embeddings on the graph that
    includes the batch (full_embeddings[l], all nodes), p = the stored tables."""
    err = np.zeros(R.shape[0])
    for l in range(1, len(tables)):
        p = tables[l].rows(R)
        err += np.linalg.norm(full_embeddings[l][R, :p.shape[1]] - p, axis=1)
    return err


def build_computation_graph(base_indptr: np.ndarray, base_indices: np.ndarray, n_query: int,
                            qe_query: np.ndarray, qe_node: np.ndarray, gamma_ppm: int,
                            recompute_set: Optional[Sequence[int]] = None, policy: str = "ratio", seed: int = 0,
                            node_scores: Optional[np.ndarray] = None) -> OracleGraph:
    """Computation graph of one batch in the canonical form described in the header
    (Sec. 6.1: last layer from the query-destination edges; the other layers add every
    edge that ends at a recompute target, from the base graph and from the request)."""
    n = base_indptr.shape[0] - 1
    qe_query = np.asarray(qe_query, dtype=np.int64)
    qe_node = np.asarray(qe_node, dtype=np.int64)
    if qe_query.shape != qe_node.shape:
        raise ValueError("edge arrays differ in length")
    if qe_query.size and (qe_query.min() < 0 or qe_query.max() >= n_query):
        raise ValueError("query index out of range")
    if qe_node.size and (qe_node.min() < 0 or qe_node.max() >= n):
        raise ValueError("node id out of range")

    R, qdeg = candidates(qe_node)
    deg_base = (base_indptr[R + 1] - base_indptr[R]).astype(np.int64)
    if recompute_set is None:
        T = (select_targets(R, qdeg, deg_base, gamma_ppm) if policy == "ratio"
             else select_targets_alt(R, gamma_ppm, policy, seed, node_scores))
    else:
        T = np.asarray(recompute_set, dtype=np.int64)
        if np.any(np.diff(T) <= 0) or not np.all(np.isin(T, R)):
            raise ValueError("recompute set must be ascending, unique and within the candidates")

    qdeg_of = dict(zip(R.tolist(), qdeg.tolist()))
    buf_row_of = {int(u): n_query + i for i, u in enumerate(T.tolist())}
    nodes_of_query = [[] for _ in range(n_query)]              # request edges, grouped both ways
    queries_of_node = {int(u): [] for u in R.tolist()}
    for q, u in zip(qe_query.tolist(), qe_node.tolist()):
        nodes_of_query[q].append(u)
        queries_of_node[u].append(q)

    def tag(u: int) -> int:
        return ~buf_row_of[u] if u in buf_row_of else u

    def deg_with_batch(u: int) -> int:
        return int(base_indptr[u + 1] - base_indptr[u]) + qdeg_of.get(u, 0)

    indptr, cols, cdeg = [0], [], []
    for q in range(n_query):                                   # query rows
        for u in sorted(nodes_of_query[q]):
            cols.append(tag(u))
            cdeg.append(deg_with_batch(u))
        indptr.append(len(cols))
    for u in T.tolist():                                       # target rows
        for w in base_indices[base_indptr[u]:base_indptr[u + 1]].tolist():
            cols.append(tag(w))
            cdeg.append(deg_with_batch(w))
        for q in sorted(queries_of_node[u]):
            cols.append(~q)
            cdeg.append(len(nodes_of_query[q]))
        indptr.append(len(cols))
    return OracleGraph(n_query, R, qdeg, T, np.array(indptr, dtype=np.int64),
                       np.array(cols, dtype=np.int32), np.array(cdeg, dtype=np.int32))


# --------------------------------------------------------------------------- layer math, one row

def _act(x: np.ndarray, kind: str) -> np.ndarray:
    if kind == "none":
        return x
    if kind == "relu":
        return np.maximum(x, 0.0)
    if kind == "elu":
        return np.where(x > 0.0, x, np.expm1(np.minimum(x, 0.0)))
    raise ValueError(kind)


def aggregate(p, h_src: np.ndarray) -> np.ndarray:
    """Neighbourhood aggregation of a SAGE-style layer over the rows of h_src (deg, d): the mean, or one
    of the other forms Sec. 6.2 names.  An empty neighbourhood gives zeros.
      sum     sum_u h_u
      max     element-wise maximum
      power   ((1/deg) sum_u m_u^p)^(1/p), messages m_u = max(h_u, 0) + eps (the cited model's positive messages)
      moment  ((1/deg) sum_u (h_u - mean)^n)^(1/n), n an integer >= 2; for odd n the root keeps the sign"""
    deg = h_src.shape[0]
    kind = getattr(p, "aggregator", "mean")
    if deg == 0:
        return np.zeros(h_src.shape[1])
    if kind == "mean":
        return h_src.sum(axis=0) / deg
    if kind == "sum":
        return h_src.sum(axis=0)
    if kind == "max":
        return h_src.max(axis=0)
    if kind == "power":
        m = np.maximum(h_src, 0.0) + float(p.agg_eps)
        return ((m ** float(p.agg_p)).sum(axis=0) / deg) ** (1.0 / float(p.agg_p))
    if kind == "moment":
        n = int(p.agg_p)
        mean = h_src.sum(axis=0) / deg
        c = ((h_src - mean[None, :]) ** n).sum(axis=0) / deg
        return np.sign(c) * np.abs(c) ** (1.0 / n)
    raise ValueError(kind)


def layer_row(p, h_self: np.ndarray, h_src: np.ndarray, deg_src: np.ndarray,
              h0_self: Optional[np.ndarray] = None) -> np.ndarray:
    """One destination of one layer (Eq. 1).  h_self (d_in,), h_src (deg, d_in) in neighbour
    order, deg_src (deg,) = in-degree of each source in the graph that includes the batch;
    h0_self: the row's layer-0 value (only the deep GCNII convolution reads it)."""
    W = np.asarray(p.W_nb, dtype=np.float64)
    b = np.asarray(p.bias, dtype=np.float64)
    deg = h_src.shape[0]
    if p.model == "sage":
        return _act(h_self @ np.asarray(p.W_self, dtype=np.float64) + aggregate(p, h_src) @ W + b, p.act)
    if p.model == "gcn":
        dv = deg + 1.0
        coef = 1.0 / np.sqrt((np.asarray(deg_src, dtype=np.float64) + 1.0) * dv)
        agg = h_self / dv + (coef[:, None] * h_src).sum(axis=0)
        return _act(agg @ W + b, p.act)
    if p.model == "gcnii":
        # the deep model of the paper's appendix on the number of layers: GCN's normalised sum (self loop
        # included), mixed with the row's layer-0 value, times the identity-mapped weight held in W_nb
        dv = deg + 1.0
        coef = 1.0 / np.sqrt((np.asarray(deg_src, dtype=np.float64) + 1.0) * dv)
        agg = h_self / dv + (coef[:, None] * h_src).sum(axis=0)
        mixed = (1.0 - float(p.alpha)) * agg + float(p.alpha) * np.asarray(h0_self, dtype=np.float64)
        return _act(mixed @ W + b, p.act)
    if p.model == "gat":
        H = p.heads
        dh = p.d_out // H
        a_s = np.asarray(p.a_src, dtype=np.float64)
        a_d = np.asarray(p.a_dst, dtype=np.float64)
        z_self = (h_self @ W).reshape(H, dh)
        out = np.zeros((H, dh))
        if deg:
            z = (h_src @ W).reshape(deg, H, dh)
            e = (z * a_s[None]).sum(-1) + (z_self * a_d).sum(-1)[None]      # (deg, H)
            e = np.where(e > 0.0, e, p.leaky_slope * e)
            e = e - e.max(axis=0, keepdims=True)
            alpha = np.exp(e)
            alpha = alpha / alpha.sum(axis=0, keepdims=True)
            out = (alpha[:, :, None] * z).sum(axis=0)
        out = out + b.reshape(H, dh)
        if p.head_mean:
            return _act(out.mean(axis=0), p.act)
        return _act(out.reshape(-1), p.act)
    raise ValueError(p.model)


# --------------------------------------------------------------------------- SRPE execution

def initial_buffer(g: OracleGraph, feat_table: LazyTable, query_feats: np.ndarray) -> np.ndarray:
    """Layer-0 values of the freshly computed rows: the queries' own features, then the
    stored features of the targets (features are exact for every node, Sec. 2)."""
    d = feat_table.dim
    return np.concatenate([np.asarray(query_feats[:, :d], dtype=np.float64), feat_table.rows(g.T)], axis=0)


def run_layer(g: OracleGraph, p, table_prev: LazyTable, buf_prev: np.ndarray, is_last: bool,
              rows: Optional[Sequence[int]] = None, buf0: Optional[np.ndarray] = None) -> np.ndarray:
    """Layer l over the batch's computation graph: sources are read from the stored table of
    layer l-1 unless they are freshly computed rows (Sec. 5, Sec. 6.1).  The last layer only
    has the query rows."""
    n_rows = g.n_query if is_last else g.rows_in
    todo = range(n_rows) if rows is None else rows
    out = np.zeros((len(todo), p.out_width))
    for i, v in enumerate(todo):
        c = g.cols[g.indptr[v]:g.indptr[v + 1]].astype(np.int64)
        h_src = np.empty((c.shape[0], p.d_in))
        stored = c >= 0
        if stored.any():
            h_src[stored] = table_prev.rows(c[stored])
        if (~stored).any():
            h_src[~stored] = buf_prev[~c[~stored], :p.d_in]
        out[i] = layer_row(p, buf_prev[v, :p.d_in], h_src, g.cdeg[g.indptr[v]:g.indptr[v + 1]],
                           None if buf0 is None else buf0[v, :p.d_in])
    return out


def srpe_reference(g: OracleGraph, tables: List[LazyTable], layers, query_feats: np.ndarray,
                   return_all: bool = False):
    """k layers over the batch's computation graph; returns h_q^(k) for the B queries."""
    k = len(layers)
    buf = initial_buffer(g, tables[0], query_feats)
    bufs = [buf]
    for l in range(1, k + 1):
        buf = run_layer(g, layers[l - 1], tables[l - 1], buf, is_last=(l == k), buf0=bufs[0])
        bufs.append(buf)
    return bufs if return_all else buf


def srpe_reference_rows(g: OracleGraph, tables: List[LazyTable], layers, query_feats: np.ndarray,
                        sample: Sequence[int]) -> np.ndarray:
    """h_q^(k) of the sampled query rows only (for batches too large to evaluate whole): the same layers over
    the same computation graph, evaluated only for the rows the sampled outputs depend on - the sample after
    layer k, those rows plus the freshly computed rows they read after layer k-1, and so on down (Sec. 6.1:
    a row of layer l reads stored embeddings and the rows of layer l-1).  Every value that was not computed is
    NaN, so reading one cannot go unnoticed.  Rows come back in ascending order of `sample`."""
    k = len(layers)
    sample = np.array(sorted(set(int(v) for v in sample)), dtype=np.int64)
    if sample.size and (sample[0] < 0 or sample[-1] >= g.n_query):
        raise ValueError("sampled rows must be query rows")
    need = [set(sample.tolist())]                         # need[j]: rows whose value after layer k-j is needed
    for _ in range(k - 1):
        cur = set(need[-1])
        for v in need[-1]:
            c = g.cols[g.indptr[v]:g.indptr[v + 1]]
            cur.update((~c[c < 0]).tolist())
        need.append(cur)
    need = need[::-1]                                     # need[l-1]: rows needed after layer l
    buf0 = buf = initial_buffer(g, tables[0], query_feats)
    for l in range(1, k + 1):
        last = l == k
        rows = np.array(sorted(need[l - 1]), dtype=np.int64)
        p = layers[l - 1]
        out = run_layer(g, p, tables[l - 1], buf, is_last=last, rows=rows, buf0=buf0)
        if last:
            return out
        buf = np.full((g.rows_in, p.out_width), np.nan)
        buf[rows] = out
    raise AssertionError("unreachable")


def serve_batch(base_indptr, base_indices, tables: List[LazyTable], layers, query_feats,
                n_query, qe_query, qe_node, gamma_ppm):
    g = build_computation_graph(base_indptr, base_indices, n_query, qe_query, qe_node, gamma_ppm)
    return srpe_reference(g, tables, layers, query_feats)
