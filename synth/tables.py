"""Seeded feature / embedding tables and model weights.

Only random draws and storage-format conversion live here.  A table is a
row-major fp32 array whose leading dimension is padded so that every row
starts on a 16-byte boundary; padding columns hold zeros.  bf16 tables are
produced once, by rounding the fp32 values to nearest-even, and handed to both
sides as raw 16-bit patterns.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def padded_ld(dim: int, elem_bytes: int) -> int:
    """Smallest leading dimension >= dim whose row size is a multiple of 16 bytes."""
    per = 16 // elem_bytes
    return (dim + per - 1) // per * per


_CHUNK_ROWS = 1 << 15


def _for_row_chunks(n_rows: int, fn) -> None:
    """fn(chunk index, first row, end row) over fixed-size row chunks, on a few threads.  The
    chunking is fixed, so the result does not depend on how many threads run."""
    chunks = [(c, r0, min(n_rows, r0 + _CHUNK_ROWS)) for c, r0 in enumerate(range(0, n_rows, _CHUNK_ROWS))]
    if len(chunks) <= 1:
        for c in chunks:
            fn(*c)
        return
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        list(ex.map(lambda c: fn(*c), chunks))


def normal_table(n_rows: int, dim: int, seed: int, stream: int = 0, ld: Optional[int] = None,
                 relu: bool = False) -> np.ndarray:
    """fp32 N(0,1) table, shape (n_rows, ld) with columns dim..ld-1 zero.  Each chunk of rows has
    its own counter-based stream (seed, stream, chunk)."""
    ld = padded_ld(dim, 4) if ld is None else ld
    out = np.zeros((n_rows, ld), dtype=np.float32)

    def fill(c, r0, r1):
        rng = np.random.Generator(np.random.Philox(key=[seed, (stream << 32) | c]))
        blk = rng.standard_normal((r1 - r0, dim), dtype=np.float32)
        if relu:
            np.maximum(blk, 0.0, out=blk)
        out[r0:r1, :dim] = blk

    _for_row_chunks(n_rows, fill)
    return out


def relu_normal_table(n_rows: int, dim: int, seed: int, stream: int = 0, ld: Optional[int] = None) -> np.ndarray:
    """Stand-in for a hidden-layer embedding table: max(N(0,1), 0), i.e. what a
    ReLU layer leaves behind (about half the entries exactly zero)."""
    return normal_table(n_rows, dim, seed, stream, ld, relu=True)


def _bf16_block(x: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    x = np.asarray(x)
    if x.ndim != 2 or x.shape[0] <= _CHUNK_ROWS:
        return _bf16_block(x)
    out = np.empty(x.shape, dtype=np.uint16)

    def conv(c, r0, r1):
        out[r0:r1] = _bf16_block(x[r0:r1])

    _for_row_chunks(x.shape[0], conv)
    return out


def glorot(fan_in: int, fan_out: int, rng: np.random.Generator, shape=None) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    shape = (fan_in, fan_out) if shape is None else shape
    return rng.uniform(-lim, lim, size=shape).astype(np.float32)


@dataclass
class LayerParams:
    model: str                 # "sage" | "gcn" | "gat" | "gcnii"
    d_in: int
    d_out: int                 # width of the projection (heads * per-head width for gat)
    act: str                   # "none" | "relu" | "elu"
    W_nb: np.ndarray           # (d_in, d_out) fp32, applied to the aggregated neighbours
    bias: np.ndarray           # (d_out,) fp32
    W_self: Optional[np.ndarray] = None    # (d_in, d_out), sage only
    heads: int = 1
    a_src: Optional[np.ndarray] = None     # (heads, d_out // heads), gat only
    a_dst: Optional[np.ndarray] = None
    leaky_slope: float = 0.2
    head_mean: bool = False    # gat output layer: average the heads instead of concatenating
    aggregator: str = "mean"   # sage only: "mean" | "sum" | "max" | "power" | "moment"
    agg_p: float = 1.0         # exponent of the power mean, or order (integer >= 2) of the moment
    agg_eps: float = 1e-7      # power mean: messages are max(h, 0) + agg_eps
    alpha: float = 0.0         # gcnii: weight of the initial residual; W_nb then holds (1 - beta) I + beta W

    @property
    def out_width(self) -> int:
        return self.d_out // self.heads if self.head_mean else self.d_out


def make_layers(model: str, dims: List[int], seed: int = 1003, heads: int = 1, aggregator: str = "mean",
                agg_p: float = 1.0) -> List[LayerParams]:
    """Glorot-uniform weights, biases U(-0.1, 0.1) (non-zero on purpose).

    dims = [d_0, d_1, ..., d_k] are the widths of h^(0..k).  For gat every hidden
    width must be a multiple of `heads`; the last layer projects to heads * d_k
    and averages the heads.
    """
    rng = _rng(seed)
    layers: List[LayerParams] = []
    k = len(dims) - 1
    for l in range(k):
        d_in, d_out, last = dims[l], dims[l + 1], l == k - 1
        if model == "sage":
            layers.append(LayerParams("sage", d_in, d_out, "none" if last else "relu",
                                      W_nb=glorot(2 * d_in, d_out, rng, (d_in, d_out)),
                                      W_self=glorot(2 * d_in, d_out, rng, (d_in, d_out)),
                                      bias=rng.uniform(-0.1, 0.1, d_out).astype(np.float32),
                                      aggregator=aggregator, agg_p=agg_p))
        elif model == "gcn":
            layers.append(LayerParams("gcn", d_in, d_out, "none" if last else "relu",
                                      W_nb=glorot(d_in, d_out, rng),
                                      bias=rng.uniform(-0.1, 0.1, d_out).astype(np.float32)))
        elif model == "gcnii":
            # deep GCN with initial residual and identity mapping: out = act(((1 - alpha) P h + alpha h0) W_eff),
            # W_eff = (1 - beta_l) I + beta_l W_l, beta_l = log(lambda / l + 1), lambda = 0.5; all widths equal
            if d_in != d_out:
                raise ValueError("gcnii layers keep the width")
            beta = float(np.log(0.5 / (l + 1) + 1.0))
            W = glorot(d_in, d_out, rng)
            W_eff = ((1.0 - beta) * np.eye(d_in, dtype=np.float64) + beta * W.astype(np.float64)).astype(np.float32)
            layers.append(LayerParams("gcnii", d_in, d_out, "relu", W_nb=W_eff,
                                      bias=np.zeros(d_out, dtype=np.float32), alpha=0.1))
        elif model == "gat":
            proj = d_out * heads if last else d_out
            dh = proj // heads
            layers.append(LayerParams("gat", d_in, proj, "none" if last else "elu",
                                      W_nb=glorot(d_in, proj, rng),
                                      bias=rng.uniform(-0.1, 0.1, proj).astype(np.float32),
                                      heads=heads,
                                      a_src=glorot(dh, 1, rng, (heads, dh)),
                                      a_dst=glorot(dh, 1, rng, (heads, dh)),
                                      head_mean=last))
        else:
            raise ValueError(model)
    return layers
