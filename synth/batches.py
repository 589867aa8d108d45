"""Seeded serving requests: query-node features and query<->training edges.

A request is what the serving system receives for one batch: B new nodes, each
with a feature vector and a list of distinct existing nodes it is connected to.
Edges are handed over as an unordered list of (query index, node id) pairs.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

from .graphs import BaseGraph
from .tables import padded_ld


@dataclass
class QueryBatch:
    n_query: int
    qe_query: np.ndarray   # int32 [E_q], query index of each edge
    qe_node: np.ndarray    # int32 [E_q], training-node endpoint of each edge
    feats: np.ndarray      # fp32 (n_query, ld), padded like a table

    @property
    def n_edges(self) -> int:
        return int(self.qe_query.shape[0])


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _distinct(draw, want: int, limit: int) -> np.ndarray:
    """First `want` distinct values produced by draw(count), in draw order."""
    want = min(want, limit)
    got = np.empty(0, dtype=np.int64)
    for _ in range(32):
        more = draw(int(1.3 * (want - got.shape[0])) + 16)
        got = np.concatenate([got, more.astype(np.int64)])
        _, first = np.unique(got, return_index=True)
        got = got[np.sort(first)]
        if got.shape[0] >= want:
            break
    return got[:want]


def make_batch(g: BaseGraph, n_query: int, feat_dim: int, seed: int,
               degree: Tuple = ("uniform", 5, 20), endpoints: str = "uniform",
               intra: float = 0.8) -> QueryBatch:
    """degree: ("uniform", lo, hi) or ("graph",) = degree of a uniformly drawn existing node.
    endpoints: "uniform" | "degree" (probability proportional to degree) |
               "block" (a share `intra` of them inside one community per query)."""
    rng = _rng(seed)
    nnz = g.nnz
    if degree[0] == "uniform":
        qdeg = rng.integers(degree[1], degree[2] + 1, size=n_query)
    elif degree[0] == "graph":
        pick = rng.integers(0, g.n, size=n_query)
        qdeg = np.maximum(np.diff(g.indptr)[pick], 1)
    else:
        raise ValueError(degree)

    if endpoints == "block":
        order = np.argsort(g.block, kind="stable")
        blk_cnt = np.bincount(g.block, minlength=int(g.block.max()) + 1)
        blk_off = np.concatenate([[0], np.cumsum(blk_cnt)])

    qs, us = [], []
    for q in range(n_query):
        d = int(qdeg[q])
        if endpoints == "uniform":
            ep = _distinct(lambda c: rng.integers(0, g.n, size=c), d, g.n)
        elif endpoints == "degree":
            ep = _distinct(lambda c: g.indices[rng.integers(0, nnz, size=c)], d, g.n)
        elif endpoints == "block":
            b = int(rng.integers(0, blk_cnt.shape[0]))

            def draw(c, b=b):
                glob = g.indices[rng.integers(0, nnz, size=c)].astype(np.int64)
                loc = order[blk_off[b] + rng.integers(0, blk_cnt[b], size=c)]
                return np.where(rng.random(c) < intra, loc, glob)
            ep = _distinct(draw, d, g.n)
        else:
            raise ValueError(endpoints)
        qs.append(np.full(ep.shape[0], q, dtype=np.int32))
        us.append(ep.astype(np.int32))
    qe_query = np.concatenate(qs) if qs else np.empty(0, np.int32)
    qe_node = np.concatenate(us) if us else np.empty(0, np.int32)
    shuffle = rng.permutation(qe_query.shape[0])
    ld = padded_ld(feat_dim, 4)
    feats = np.zeros((n_query, ld), dtype=np.float32)
    feats[:, :feat_dim] = rng.standard_normal((n_query, feat_dim), dtype=np.float32)
    return QueryBatch(n_query, np.ascontiguousarray(qe_query[shuffle]),
                      np.ascontiguousarray(qe_node[shuffle]), feats)
