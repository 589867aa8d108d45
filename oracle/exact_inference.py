"""Exact GNN inference in fp64.  TEST INFRASTRUCTURE ONLY.

Whole-graph matrix algebra, sharing no code with the row-by-row SRPE oracle it is used to pin:

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

  exact_inference_rows  h_q^(k) on G' for a sample of the queries of a batch on a graph too large for the
                        whole-graph forms: Eq. 1 applied level by level to the nodes within k - l hops of
                        the sample (the memoised recursion of Sec. 2 from the sampled queries down to the
                        features), rectangular adjacency blocks.  Pinned to exact_full_inference_sparse.

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


# --------------------------------------------------------------------------- exact inference for a few queries

def _ranges(starts: np.ndarray, lens: np.ndarray) -> np.ndarray:
    """Concatenation of the integer ranges [starts[i], starts[i] + lens[i])."""
    total = int(lens.sum())
    if total == 0:
        return np.empty(0, dtype=np.int64)
    first = np.cumsum(lens) - lens                           # where range i starts in the output
    return np.arange(total, dtype=np.int64) - np.repeat(first, lens) + np.repeat(starts, lens)


def exact_inference_rows(base_indptr, base_indices, feature_rows, query_feats, qe_query, qe_node, layers,
                         sample) -> np.ndarray:
    """h_q^(k) on G' (training graph + the batch's query nodes + both directions of every query edge) of the
    sampled queries, in ascending order of `sample`.  Eq. 1 unrolled from the sample: S_k = the sample,
    S_{l-1} = S_l and every in-neighbour in G' of a node of S_l; H^(0) on S_0 are features, and layer l maps
    H^(l-1) on S_{l-1} to H^(l) on S_l through the |S_l| x |S_{l-1}| block of the adjacency.  Degrees are the
    full in-degrees in G'.  feature_rows(ids) -> fp64 (len(ids), d_0) for training-node ids.
    Node numbering inside: training node u -> u, query q -> n + q."""
    n = int(base_indptr.shape[0] - 1)
    B = int(query_feats.shape[0])
    k = len(layers)
    qq = np.asarray(qe_query, dtype=np.int64)
    uu = np.asarray(qe_node, dtype=np.int64)
    by_q = np.argsort(qq, kind="stable")                      # request grouped by query, and by node
    q_nodes = uu[by_q]
    q_ptr = np.concatenate([[0], np.cumsum(np.bincount(qq, minlength=B))]).astype(np.int64)
    by_u = np.argsort(uu, kind="stable")
    u_ids, u_cnt = np.unique(uu, return_counts=True)
    u_ptr = np.concatenate([[0], np.cumsum(u_cnt)]).astype(np.int64)
    u_queries = qq[by_u]
    base_indptr = np.asarray(base_indptr, dtype=np.int64)

    def attached(v):                                          # per training node: (first, count) in u_queries
        pos = np.searchsorted(u_ids, v)
        pos_c = np.minimum(pos, max(u_ids.shape[0] - 1, 0))
        hit = (pos < u_ids.shape[0]) & (u_ids[pos_c] == v) if u_ids.size else np.zeros(v.shape, bool)
        return np.where(hit, u_ptr[pos_c], 0), np.where(hit, u_cnt[pos_c] if u_ids.size else 0, 0)

    def in_degree(x):                                         # full in-degree in G'
        x = np.asarray(x, dtype=np.int64)
        out = np.empty(x.shape[0], dtype=np.int64)
        tr = x < n
        v = x[tr]
        out[tr] = base_indptr[v + 1] - base_indptr[v] + attached(v)[1]
        out[~tr] = q_ptr[x[~tr] - n + 1] - q_ptr[x[~tr] - n]
        return out

    def in_edges(S):
        """All edges of G' that end in S, grouped by destination in the order of S: (dst position, source id)."""
        lens = in_degree(S)
        src = np.empty(int(lens.sum()), dtype=np.int64)
        off = np.cumsum(lens) - lens
        tr = S < n
        v = S[tr]
        b_len = base_indptr[v + 1] - base_indptr[v]
        a_first, a_len = attached(v)
        # training destinations: base in-neighbours, then the queries attached to them
        src[_ranges(off[tr], b_len)] = np.asarray(base_indices[_ranges(base_indptr[v], b_len)], dtype=np.int64) \
            if b_len.sum() else np.empty(0, np.int64)
        src[_ranges(off[tr] + b_len, a_len)] = n + u_queries[_ranges(a_first, a_len)]
        q = S[~tr] - n
        q_len = q_ptr[q + 1] - q_ptr[q]
        src[_ranges(off[~tr], q_len)] = q_nodes[_ranges(q_ptr[q], q_len)]
        return np.repeat(np.arange(S.shape[0], dtype=np.int64), lens), src

    S = [None] * (k + 1)
    E = [None] * (k + 1)
    S[k] = n + np.array(sorted(set(int(q) for q in sample)), dtype=np.int64)
    for l in range(k, 0, -1):
        E[l] = in_edges(S[l])
        S[l - 1] = np.union1d(S[l], E[l][1])
    ids0 = S[0]
    H = np.empty((ids0.shape[0], int(layers[0].d_in)))
    tr0 = ids0 < n
    H[tr0] = feature_rows(ids0[tr0])[:, :layers[0].d_in]
    H[~tr0] = _f64(query_feats)[ids0[~tr0] - n, :layers[0].d_in]
    H0 = H
    for l in range(1, k + 1):
        p = layers[l - 1]
        dst, src = E[l]
        m, m_prev = S[l].shape[0], S[l - 1].shape[0]
        col = np.searchsorted(S[l - 1], src)
        own = np.searchsorted(S[l - 1], S[l])                 # every node of S_l is in S_{l-1}
        A = sp.csr_matrix((np.ones(dst.shape[0]), (dst, col)), shape=(m, m_prev))    # duplicates add up
        deg = in_degree(S[l]).astype(np.float64)
        W, b = _f64(p.W_nb), _f64(p.bias)
        Hp = H[:, :p.d_in]
        if p.model == "sage":
            kind = getattr(p, "aggregator", "mean")
            agg = A @ Hp
            if kind == "mean":
                agg = np.where(deg[:, None] > 0, agg / np.maximum(deg, 1.0)[:, None], 0.0)
            elif kind != "sum":
                raise NotImplementedError(kind)
            nxt = _act(Hp[own] @ _f64(p.W_self) + agg @ W + b, p.act)
        elif p.model in ("gcn", "gcnii"):
            s_src = 1.0 / np.sqrt(in_degree(S[l - 1]).astype(np.float64) + 1.0)
            s_dst = 1.0 / np.sqrt(deg + 1.0)
            agg = s_dst[:, None] * (A @ (s_src[:, None] * Hp)) + Hp[own] / (deg + 1.0)[:, None]
            if p.model == "gcnii":
                h0 = H0[np.searchsorted(ids0, S[l]), :p.d_in]
                agg = (1.0 - float(p.alpha)) * agg + float(p.alpha) * h0
            nxt = _act(agg @ W + b, p.act)
        elif p.model == "gat":
            nh = p.heads
            dh = p.d_out // nh
            Z = (Hp @ W).reshape(m_prev, nh, dh)
            s_s = (Z * _f64(p.a_src)[None]).sum(-1)
            s_d = (Z * _f64(p.a_dst)[None]).sum(-1)[own]
            out = np.zeros((m, nh, dh))
            lens = np.bincount(dst, minlength=m)
            nonempty = lens > 0
            starts = (np.cumsum(lens) - lens)[nonempty]
            for h in range(nh):
                e = s_s[col, h] + s_d[dst, h]
                e = np.where(e > 0.0, e, p.leaky_slope * e)
                mx = np.zeros(m)
                mx[nonempty] = np.maximum.reduceat(e, starts)
                w = np.exp(e - mx[dst])
                den = np.zeros(m)
                den[nonempty] = np.add.reduceat(w, starts)
                out[:, h, :] = sp.csr_matrix((w / den[dst], (dst, col)), shape=(m, m_prev)) @ Z[:, h, :]
            out = out + b.reshape(nh, dh)[None]
            nxt = _act(out.mean(axis=1), p.act) if p.head_mean else _act(out.reshape(m, nh * dh), p.act)
        else:
            raise ValueError(p.model)
        H = nxt
    return H
