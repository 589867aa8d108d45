"""Hash-defined inputs for graphs too large to generate or hold on the host.

Everything is a pure function of (seed, index) in 64-bit integer arithmetic, written twice with the
same operations: once in numpy (any slice, on the host: what the CPU oracle reads) and once in
torch (whole arrays, on the device: what the GPU library reads).  No floating-point function is
evaluated on either side, so the two agree bit for bit.

  degree(i)      heavy-tailed: (2 + two hash bits) << floor(10 z / 11), z = leading zeros of a 32-bit
                 hash (a geometric variable), capped; P(degree > x) falls like x^-1.1
  neighbour(p)   hash of the edge slot p, reduced modulo the node count (in-neighbour CSR; not
                 symmetric, repeated neighbours possible and kept)
  table(t, r, c) 16 hash bits v -> (v - 32768) / 32768 in [-1, 1), rounded to bf16
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from .batches import QueryBatch
from .tables import LayerParams, make_layers, padded_ld, to_bf16_bits

_C1, _C2, _C3 = 0x9E3779B97F4A7C15, 0xBF58476D1CE4E5B9, 0x94D049BB133111EB
_M64 = (1 << 64) - 1


def _signed(c: int) -> int:
    return c - (1 << 64) if c >= (1 << 63) else c


# ---------------------------------------------------------------------------------- numpy side
def mix_np(x: np.ndarray, seed: int) -> np.ndarray:
    """splitmix64 finaliser of x + seed * C1 (uint64 in, uint64 out)."""
    with np.errstate(over="ignore"):
        z = x.astype(np.uint64) + np.uint64((seed * _C1) & _M64)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_C2)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C3)
        return z ^ (z >> np.uint64(31))


def _degree_from_hash_np(h: np.ndarray, max_shift: int) -> np.ndarray:
    h32 = (h >> np.uint64(32)).astype(np.int64)
    z = np.zeros(h32.shape, dtype=np.int64)
    for k in range(1, 33):
        z += (h32 < (1 << (32 - k))).astype(np.int64)          # leading zeros of the 32-bit value
    shift = np.minimum((z * 10) // 11, max_shift)
    return ((2 + (h.astype(np.int64) & 3)) << shift).astype(np.int64)


# ---------------------------------------------------------------------------------- torch side
def mix_torch(x, seed: int):
    """Same function on an int64 torch tensor (two's complement wrap-around = uint64 arithmetic)."""
    def lsr(v, s):
        return (v >> s) & ((1 << (64 - s)) - 1)
    z = x + _signed((seed * _C1) & _M64)
    z = (z ^ lsr(z, 30)) * _signed(_C2)
    z = (z ^ lsr(z, 27)) * _signed(_C3)
    return z ^ lsr(z, 31)


def _degree_from_hash_torch(h, max_shift: int):
    import torch
    h32 = (h >> 32) & 0xFFFFFFFF
    z = torch.zeros_like(h32)
    for k in range(1, 33):
        z += (h32 < (1 << (32 - k))).to(torch.int64)
    shift = torch.clamp((z * 10) // 11, max=max_shift)
    return (2 + (h & 3)) << shift


@dataclass
class ScaleSpec:
    n_nodes: int = 111_000_000
    feat_dim: int = 128
    dims: tuple = (128, 128, 128, 128)       # 3-layer SAGE
    max_shift: int = 16                      # degree cap (5 << 16), before deg_mult
    deg_mult: int = 1                        # every degree is multiplied by this (denser graphs)
    q_deg: tuple = (10, 50)                  # a query's number of distinct endpoints, uniform in this range
    seed_graph: int = 1001
    seed_table: int = 1002
    seed_weights: int = 1003

    @property
    def k(self) -> int:
        return len(self.dims) - 1


class HashIndices:
    """base_indices[a:b] for the oracle: neighbours are computed when a slice is asked for."""

    def __init__(self, n_nodes: int, nnz: int, seed: int):
        self.n_nodes, self.nnz, self.seed = n_nodes, nnz, seed
        self.shape = (nnz,)

    def __getitem__(self, key) -> np.ndarray:
        if isinstance(key, slice):
            p = np.arange(key.start or 0, self.nnz if key.stop is None else key.stop, dtype=np.uint64)
        else:
            p = np.asarray(key, dtype=np.uint64)
        return (mix_np(p, self.seed + 1) % np.uint64(self.n_nodes)).astype(np.int32)


class HashTable:
    """Stored bf16 table for the oracle: rows are computed when asked for (uint16 bit patterns)."""

    def __init__(self, n_rows: int, dim: int, seed: int, table_index: int):
        self.n_rows, self.dim, self.seed, self.t = n_rows, dim, seed, table_index
        self.ld = padded_ld(dim, 2)
        self.shape = (n_rows, self.ld)

    def __getitem__(self, rows) -> np.ndarray:
        rows = np.asarray(rows, dtype=np.uint64).reshape(-1)
        idx = rows[:, None] * np.uint64(self.dim) + np.arange(self.dim, dtype=np.uint64)[None, :]
        v = (mix_np(idx, self.seed + 16 * self.t) & np.uint64(0xFFFF)).astype(np.int64)
        x = ((v - 32768).astype(np.float32) / np.float32(32768.0)).astype(np.float32)
        out = np.zeros((rows.shape[0], self.ld), dtype=np.uint16)
        out[:, :self.dim] = to_bf16_bits(x)
        return out


def degrees_np(spec: ScaleSpec, lo: int, hi: int) -> np.ndarray:
    return _degree_from_hash_np(mix_np(np.arange(lo, hi, dtype=np.uint64), spec.seed_graph), spec.max_shift) * spec.deg_mult


def fb10b_spec() -> ScaleSpec:
    """The shape of the paper's largest dataset (Sec. 8.1, dataset table: 30 M nodes, 10 B edges, mean degree
    333, 1,024 features, hidden width 128), 3-layer SAGE: about 117 GB of graph and bf16 tables on the device."""
    return ScaleSpec(n_nodes=30_000_000, feat_dim=1024, dims=(1024, 128, 128, 128), max_shift=12, deg_mult=25,
                     q_deg=(100, 500))


def indptr_np(spec: ScaleSpec) -> np.ndarray:
    """Row pointers of the whole graph (int64 [n + 1]); chunked so that temporaries stay small."""
    out = np.zeros(spec.n_nodes + 1, dtype=np.int64)
    step = 1 << 22
    for lo in range(0, spec.n_nodes, step):
        hi = min(spec.n_nodes, lo + step)
        out[lo + 1:hi + 1] = degrees_np(spec, lo, hi)
    np.cumsum(out, out=out)
    return out


def device_arrays(spec: ScaleSpec, indptr_host: np.ndarray, device="cuda:0"):
    """(indptr, indices, [tables as int16 bit patterns]) generated on `device` with torch."""
    import torch
    dev = torch.device(device)
    n, nnz = spec.n_nodes, int(indptr_host[-1])
    indptr = torch.from_numpy(indptr_host).to(dev)
    indices = torch.empty(nnz, dtype=torch.int32, device=dev)
    step = 1 << 26
    for lo in range(0, nnz, step):
        hi = min(nnz, lo + step)
        p = torch.arange(lo, hi, dtype=torch.int64, device=dev)
        h = mix_torch(p, spec.seed_graph + 1)
        # unsigned remainder of a 64-bit pattern held in a signed tensor: split off the top bit
        r = ((h & 0x7FFFFFFFFFFFFFFF) % n + ((h >> 63) & 1) * ((1 << 63) % n)) % n
        indices[lo:hi] = r.to(torch.int32)
    tables = []
    for t, dim in enumerate(spec.dims[:-1]):
        ld = padded_ld(dim, 2)
        tab = torch.zeros((n, ld), dtype=torch.int16, device=dev)
        rows_step = max(1, (1 << 26) // dim)
        for lo in range(0, n, rows_step):
            hi = min(n, lo + rows_step)
            idx = (torch.arange(lo, hi, dtype=torch.int64, device=dev)[:, None] * dim
                   + torch.arange(dim, dtype=torch.int64, device=dev)[None, :])
            v = mix_torch(idx, spec.seed_table + 16 * t) & 0xFFFF
            x = (v - 32768).to(torch.float32) / 32768.0
            b = x.view(torch.int32)
            rounded = (b + 0x7FFF + ((b >> 16) & 1)) >> 16           # nearest-even on the fp32 bit pattern
            tab[lo:hi, :dim] = rounded.to(torch.int16)
        tables.append(tab)
    return indptr, indices, tables


def make_scale_batch(spec: ScaleSpec, indptr_host: np.ndarray, n_query: int, seed: int,
                     lo_deg: Optional[int] = None, hi_deg: Optional[int] = None) -> QueryBatch:
    """n_query queries with spec.q_deg (10-50) distinct endpoints each, drawn with probability proportional to degree."""
    lo_deg = spec.q_deg[0] if lo_deg is None else lo_deg
    hi_deg = spec.q_deg[1] if hi_deg is None else hi_deg
    rng = np.random.Generator(np.random.Philox(key=[seed, 7]))
    nnz = int(indptr_host[-1])
    qs, us = [], []
    for q in range(n_query):
        d = int(rng.integers(lo_deg, hi_deg + 1))
        got = np.empty(0, dtype=np.int64)
        while got.shape[0] < d:
            slots = rng.integers(0, nnz, size=2 * d + 8)
            nodes = np.searchsorted(indptr_host, slots, side="right") - 1
            got = np.concatenate([got, nodes])
            _, first = np.unique(got, return_index=True)
            got = got[np.sort(first)]
        qs.append(np.full(d, q, dtype=np.int32))
        us.append(got[:d].astype(np.int32))
    qq, uu = np.concatenate(qs), np.concatenate(us)
    perm = rng.permutation(qq.shape[0])
    ld = padded_ld(spec.feat_dim, 4)
    feats = np.zeros((n_query, ld), dtype=np.float32)
    feats[:, :spec.feat_dim] = rng.uniform(-1.0, 1.0, size=(n_query, spec.feat_dim)).astype(np.float32)
    return QueryBatch(n_query, np.ascontiguousarray(qq[perm]), np.ascontiguousarray(uu[perm]), feats)


def scale_layers(spec: ScaleSpec) -> List[LayerParams]:
    return make_layers("sage", list(spec.dims), spec.seed_weights)
