"""Exact GNN inference in fp64.  TEST INFRASTRUCTURE ONLY.

Three functions, all written as whole-graph matrix algebra so that they share no code
with the row-by-row SRPE oracle they are used to pin:

  exact_full_inference  the k-layer model of Sec. 2, Eq. 1 evaluated on the graph G' that
                        holds the training graph plus the batch's query nodes and query
                        edges (both directions).  This is what serving with the full
                        k-hop computation graph returns (the "full computation graph"
                        method of Sec. 3.1, Table 1) and what SRPE approximates (Sec. 5).
                        Dense adjacency: small graphs only.
  exact_full_inference_sparse
                        the same quantity with a sparse adjacency (graphs of 10^4-10^5 nodes);
                        pinned to the dense form on small graphs.
  base_inference        the same model on the training graph alone, for every node: the
                        layer embeddings that are snapshotted as precomputed embeddings
                        p_u^(l), l = 1..k-1 (Sec. 5).  Sparse adjacency.

Layer forms (the paper names the models only; these are their textbook forms):
  SAGE-mean  act(H W_self + D^-1 A H W_nb + b), empty neighbourhood -> zero mean; the mean may be replaced
             by one of the other aggregation functions of Sec. 6.2 (sum, max, power mean of positive
             messages, normalised central moment)
  GCN        act(D~^-1/2 (A + I) D~^-1/2 H W + b), D~ = in-degree + 1
  GCNII      act(((1 - alpha) D~^-1/2 (A + I) D~^-1/2 H + alpha H^(0)) W_eff), W_eff = (1 - beta) I + beta W held
             as one matrix, H^(0) the layer-0 values (the deep model of the paper's appendix on depth)
  GAT        Z = H W per head; e_vu = LeakyReLU(a_src.z_u + a_dst.z_v); softmax over the
             in-neighbours u of v (each parallel edge is its own term); concat heads + b,
             or mean of heads on the output layer; no implicit self loop
A[v, u] is the number of edges u -> v.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import scipy.sparse as sp


def _act(x, kind):
    if kind == "none":
        return x
    if kind == "relu":
        return np.maximum(x, 0.0)
    if kind == "elu":
        return np.where(x > 0.0, x, np.expm1(np.minimum(x, 0.0)))
    raise ValueError(kind)


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _root(c: np.ndarray, n: int) -> np.ndarray:
    return np.sign(c) * np.abs(c) ** (1.0 / n)


def _aggregate_matrix(A, H: np.ndarray, p, deg: np.ndarray) -> np.ndarray:
    """Aggregation of a SAGE-style layer for all rows at once (A dense or sparse, A[v, u] = number of
    edges u -> v): matrix products where the form allows it, per-edge arrays otherwise."""
    kind = getattr(p, "aggregator", "mean")
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1.0), 0.0)[:, None]
    if kind == "mean":
        return inv * (A @ H)
    if kind == "sum":
        return A @ H
    if kind == "power":
        pw = float(p.agg_p)
        m = (np.maximum(H, 0.0) + float(p.agg_eps)) ** pw
        return np.where(deg[:, None] > 0, (inv * (A @ m)) ** (1.0 / pw), 0.0)
    C = sp.coo_matrix(A)                                         # one entry per distinct (v, u), data = multiplicity
    if kind == "moment":
        n = int(p.agg_p)
        mean = inv * (A @ H)
        c = np.zeros_like(mean)
        S = sp.csr_matrix((C.data, (C.row, np.arange(C.nnz))), shape=(H.shape[0], C.nnz))   # sums entries by destination
        for c0 in range(0, H.shape[1], 32):                      # a block of columns at a time: the per-edge array is large
            d = H[C.col, c0:c0 + 32] - mean[C.row, c0:c0 + 32]
            c[:, c0:c0 + 32] = S @ (d ** n)
        return np.where(deg[:, None] > 0, _root(inv * c, n), 0.0)
    if kind == "max":
        R = C.tocsr()
        out = np.zeros_like(H)
        for v in range(H.shape[0]):
            nb = R.indices[R.indptr[v]:R.indptr[v + 1]]
            if nb.size:
                out[v] = H[nb].max(axis=0)
        return out
    raise ValueError(kind)


def _dense_layer(A: np.ndarray, H: np.ndarray, p, H0: Optional[np.ndarray] = None) -> np.ndarray:
    deg = A.sum(axis=1)
    W, b = _f64(p.W_nb), _f64(p.bias)
    if p.model == "gcnii":
        s = 1.0 / np.sqrt(deg + 1.0)
        A_hat = s[:, None] * (A + np.eye(A.shape[0])) * s[None, :]
        return _act(((1.0 - float(p.alpha)) * (A_hat @ H) + float(p.alpha) * H0[:, :p.d_in]) @ W + b, p.act)
    if p.model == "sage":
        return _act(H @ _f64(p.W_self) + _aggregate_matrix(A, H, p, deg) @ W + b, p.act)
    if p.model == "gcn":
        s = 1.0 / np.sqrt(deg + 1.0)
        A_hat = s[:, None] * (A + np.eye(A.shape[0])) * s[None, :]
        return _act(A_hat @ H @ W + b, p.act)
    if p.model == "gat":
        n, nh = H.shape[0], p.heads
        dh = p.d_out // nh
        Z = (H @ W).reshape(n, nh, dh)
        s_src = (Z * _f64(p.a_src)[None]).sum(-1)            # (n, heads)
        s_dst = (Z * _f64(p.a_dst)[None]).sum(-1)
        out = np.zeros((n, nh, dh))
        for h in range(nh):
            E = s_dst[:, h][:, None] + s_src[:, h][None, :]   # E[v, u]
            E = np.where(E > 0.0, E, p.leaky_slope * E)
            E = np.where(A > 0, E, -np.inf)
            m = E.max(axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)
            P = A * np.exp(E - m)                             # multiplicity-weighted
            den = P.sum(axis=1, keepdims=True)
            P = np.where(den > 0, P / np.where(den > 0, den, 1.0), 0.0)
            out[:, h, :] = P @ Z[:, h, :]
        out = out + b.reshape(nh, dh)[None]
        if p.head_mean:
            return _act(out.mean(axis=1), p.act)
        return _act(out.reshape(n, nh * dh), p.act)
    raise ValueError(p.model)


def exact_full_inference(base_indptr, base_indices, X, query_feats, qe_query, qe_node, layers) -> np.ndarray:
    """h_q^(k) of every query node on G' (Eq. 1 applied k times to all N + B nodes)."""
    n = base_indptr.shape[0] - 1
    B = query_feats.shape[0]
    A = np.zeros((n + B, n + B))
    rows = np.repeat(np.arange(n), np.diff(base_indptr))
    np.add.at(A, (rows, np.asarray(base_indices, dtype=np.int64)), 1.0)
    qi = n + np.asarray(qe_query, dtype=np.int64)
    ui = np.asarray(qe_node, dtype=np.int64)
    np.add.at(A, (qi, ui), 1.0)          # u -> q
    np.add.at(A, (ui, qi), 1.0)          # q -> u
    H = H0 = np.concatenate([_f64(X), _f64(query_feats)], axis=0)
    for p in layers:
        H = _dense_layer(A, H[:, :p.d_in], p, H0)
    return H[n:]


def exact_layer_embeddings(base_indptr, base_indices, X, query_feats, qe_query, qe_node, layers) -> List[np.ndarray]:
    """All layer embeddings f^(l), l = 0..k, of all N + B nodes on G' (the "full embeddings" of Sec. 5.1)."""
    n = base_indptr.shape[0] - 1
    B = query_feats.shape[0]
    A = np.zeros((n + B, n + B))
    rows = np.repeat(np.arange(n), np.diff(base_indptr))
    np.add.at(A, (rows, np.asarray(base_indices, dtype=np.int64)), 1.0)
    qi = n + np.asarray(qe_query, dtype=np.int64)
    ui = np.asarray(qe_node, dtype=np.int64)
    np.add.at(A, (qi, ui), 1.0)
    np.add.at(A, (ui, qi), 1.0)
    H = np.concatenate([_f64(X), _f64(query_feats)], axis=0)
    out = [H]
    H0 = H
    for p in layers:
        H = _dense_layer(A, H[:, :p.d_in], p, H0)
        out.append(H)
    return out


def _sparse_layer(A: sp.csr_matrix, H: np.ndarray, p, H0: Optional[np.ndarray] = None) -> np.ndarray:
    deg = np.asarray(A.sum(axis=1)).ravel()
    W, b = _f64(p.W_nb), _f64(p.bias)
    if p.model == "gcnii":
        s = 1.0 / np.sqrt(deg + 1.0)
        A_hat = sp.diags(s) @ (A + sp.identity(A.shape[0], format="csr")) @ sp.diags(s)
        return _act(((1.0 - float(p.alpha)) * (A_hat @ H) + float(p.alpha) * H0[:, :p.d_in]) @ W + b, p.act)
    if p.model == "sage":
        return _act(H @ _f64(p.W_self) + _aggregate_matrix(A, H, p, deg) @ W + b, p.act)
    if p.model == "gcn":
        s = 1.0 / np.sqrt(deg + 1.0)
        A_hat = sp.diags(s) @ (A + sp.identity(A.shape[0], format="csr")) @ sp.diags(s)
        return _act((A_hat @ H) @ W + b, p.act)
    if p.model == "gat":
        n, nh = H.shape[0], p.heads
        dh = p.d_out // nh
        Z = (H @ W).reshape(n, nh, dh)
        s_src = (Z * _f64(p.a_src)[None]).sum(-1)
        s_dst = (Z * _f64(p.a_dst)[None]).sum(-1)
        indptr, src = A.indptr, A.indices
        dst = np.repeat(np.arange(n), np.diff(indptr))
        mult = A.data
        out = np.zeros((n, nh, dh))
        nonempty = np.diff(indptr) > 0
        starts = indptr[:-1][nonempty]
        for h in range(nh):
            e = s_src[src, h] + s_dst[dst, h]
            e = np.where(e > 0.0, e, p.leaky_slope * e)
            m = np.zeros(n)
            m[nonempty] = np.maximum.reduceat(e, starts)
            w = mult * np.exp(e - m[dst])
            den = np.zeros(n)
            den[nonempty] = np.add.reduceat(w, starts)
            alpha = w / den[dst]
            out[:, h, :] = sp.csr_matrix((alpha, src, indptr), shape=A.shape) @ Z[:, h, :]
        out = out + b.reshape(nh, dh)[None]
        if p.head_mean:
            return _act(out.mean(axis=1), p.act)
        return _act(out.reshape(n, nh * dh), p.act)
    raise ValueError(p.model)


def base_inference(base_indptr, base_indices, X, layers) -> List[np.ndarray]:
    """Precomputed embeddings p^(1..k-1): layer embeddings of every training node on the
    training graph alone (Sec. 5)."""
    n = base_indptr.shape[0] - 1
    A = sp.csr_matrix((np.ones(base_indices.shape[0]), base_indices, base_indptr), shape=(n, n))
    A.sum_duplicates()
    H = H0 = _f64(X)
    out = []
    for p in layers[:-1]:
        H = _sparse_layer(A, H[:, :p.d_in], p, H0)
        out.append(H)
    return out


def exact_full_inference_sparse(base_indptr, base_indices, X, query_feats, qe_query, qe_node, layers) -> np.ndarray:
    """h_q^(k) of every query node on G' (Sec. 2, Eq. 1 on all N + B nodes), sparse adjacency."""
    n = base_indptr.shape[0] - 1
    B = query_feats.shape[0]
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(base_indptr))
    qi = n + np.asarray(qe_query, dtype=np.int64)
    ui = np.asarray(qe_node, dtype=np.int64)
    dst = np.concatenate([rows, qi, ui])                   # training edges, u -> q, q -> u
    src = np.concatenate([np.asarray(base_indices, dtype=np.int64), ui, qi])
    A = sp.coo_matrix((np.ones(dst.shape[0]), (dst, src)), shape=(n + B, n + B)).tocsr()   # duplicates add up
    H = H0 = np.concatenate([_f64(X), _f64(query_feats)], axis=0)
    for p in layers:
        H = _sparse_layer(A, H[:, :p.d_in], p, H0)
    return H[n:]
