"""Seeded power-law base graphs (the "training graph" a serving system holds).

The graphs are Chung-Lu style: node i gets an expected degree w_i drawn from a
capped power law, and undirected edges are formed by pairing endpoints picked
with probability proportional to w.  Optionally nodes belong to communities and
a fixed share of edges stays inside the community of its first endpoint
(a stochastic-block-model flavour).  The result is symmetric, has no self loops
and no parallel edges, and is stored as a CSR of in-neighbours with ascending
neighbour ids per row.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class BaseGraph:
    n: int
    indptr: np.ndarray            # int64 [n+1]
    indices: np.ndarray           # int32 [nnz]
    block: Optional[np.ndarray]   # int32 [n] community of each node, or None

    @property
    def nnz(self) -> int:
        return int(self.indptr[-1])

    def degrees(self) -> np.ndarray:
        return np.diff(self.indptr)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _expected_degrees(n: int, avg_deg: float, exponent: float, max_deg: float) -> np.ndarray:
    """Capped power-law expected degrees with the requested mean, by rank."""
    alpha = 1.0 / (exponent - 1.0)
    w = (np.arange(n, dtype=np.float64) + 1.0) ** (-alpha)
    w *= (n * avg_deg) / w.sum()
    for _ in range(64):                       # clip the head, give the mass back to the tail
        over = w > max_deg
        if not over.any():
            break
        w[over] = max_deg
        free = ~over
        w[free] *= (n * avg_deg - max_deg * over.sum()) / w[free].sum()
    return np.maximum(w, 0.25)


def power_law_graph(n: int, avg_deg: float, exponent: float = 2.1, max_deg: Optional[float] = None,
                    seed: int = 1001, n_blocks: int = 1, intra: float = 0.0) -> BaseGraph:
    """Symmetric power-law graph on n nodes with mean degree close to avg_deg."""
    rng = _rng(seed)
    if max_deg is None:
        max_deg = max(4.0 * avg_deg, np.sqrt(n * avg_deg))
    w_rank = _expected_degrees(n, avg_deg, exponent, max_deg)
    perm = rng.permutation(n)                 # rank -> node id, so ids carry no degree information
    w = np.empty(n, dtype=np.float64)
    w[perm] = w_rank

    # integer stub counts with the fractional part resolved at random
    cnt = np.floor(w).astype(np.int64)
    cnt += (rng.random(n) < (w - cnt)).astype(np.int64)
    cnt = np.maximum(cnt, 1)

    if n_blocks > 1:
        block = rng.integers(0, n_blocks, size=n, dtype=np.int32)
        order = np.argsort(block, kind="stable").astype(np.int32)
    else:
        block = None
        order = np.arange(n, dtype=np.int32)
    stubs = np.repeat(order, cnt[order])      # node ids, grouped by community
    total = stubs.shape[0]
    m = total // 2

    u = stubs[rng.integers(0, total, size=m)]
    if n_blocks > 1 and intra > 0.0:
        blk_stub_cnt = np.bincount(block, weights=cnt, minlength=n_blocks).astype(np.int64)
        blk_off = np.concatenate([[0], np.cumsum(blk_stub_cnt)])
        stay = rng.random(m) < intra
        bu = block[u]
        pos_in = blk_off[bu] + (rng.random(m) * blk_stub_cnt[bu]).astype(np.int64)
        pos_out = rng.integers(0, total, size=m)
        v = stubs[np.where(stay, pos_in, pos_out)]
        del stay, bu, pos_in, pos_out
    else:
        v = stubs[rng.integers(0, total, size=m)]
    del stubs

    lo = np.minimum(u, v).astype(np.int64)
    hi = np.maximum(u, v).astype(np.int64)
    del u, v
    keep = lo != hi
    key = lo[keep] * n + hi[keep]
    del lo, hi, keep
    key = np.unique(key)                      # sorted by (lo, hi), duplicates dropped
    lo = (key // n).astype(np.int32)
    hi = (key - lo.astype(np.int64) * n).astype(np.int32)
    del key

    # Row i of the symmetric CSR = {lo : hi == i} (all < i) followed by {hi : lo == i} (all > i).
    cnt_dn = np.bincount(hi, minlength=n).astype(np.int64)   # neighbours with a smaller id
    cnt_up = np.bincount(lo, minlength=n).astype(np.int64)   # neighbours with a larger id
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(cnt_dn + cnt_up, out=indptr[1:])
    indices = np.empty(int(indptr[-1]), dtype=np.int32)

    # upper part: (lo, hi) is already sorted by lo then hi
    e = lo.shape[0]
    start_up = np.concatenate([[0], np.cumsum(cnt_up)])[:-1]
    rank_up = np.arange(e, dtype=np.int64) - start_up[lo]
    indices[indptr[:-1][lo] + cnt_dn[lo] + rank_up] = hi
    del rank_up
    # lower part: sort pairs by (hi, lo)
    o = np.argsort(hi.astype(np.int64) * n + lo, kind="stable")
    hi_s = hi[o]
    lo_s = lo[o]
    del o
    start_dn = np.concatenate([[0], np.cumsum(cnt_dn)])[:-1]
    rank_dn = np.arange(e, dtype=np.int64) - start_dn[hi_s]
    indices[indptr[:-1][hi_s] + rank_dn] = lo_s
    return BaseGraph(n=n, indptr=indptr, indices=indices, block=block)
