"""Named workloads: the benchmark configurations and scaled-down copies for tests.

Each workload fixes a base graph recipe, table widths and storage types, a model
and a query-batch recipe.  `build_workload` draws everything from fixed seeds
(graph 1001, features 1002, weights 1003, embeddings 1004 + layer, batch r ->
2000 + r).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

from .graphs import BaseGraph, power_law_graph
from .tables import (LayerParams, make_layers, normal_table, padded_ld,
                     relu_normal_table, to_bf16_bits)
from .batches import QueryBatch, make_batch


@dataclass(frozen=True)
class Workload:
    name: str
    n_nodes: int
    avg_deg: float
    max_deg: Optional[float]
    model: str                       # "sage" | "gcn" | "gat"
    dims: Tuple[int, ...]            # widths of h^(0..k)
    batch: int
    gamma_ppm: int
    exponent: float = 2.1
    n_blocks: int = 1
    intra: float = 0.0
    heads: int = 1
    pe_dtype: str = "f32"            # storage of the precomputed-embedding tables
    feat_dtype: str = "f32"
    q_degree: Tuple = ("graph",)
    q_endpoints: str = "degree"
    aggregator: str = "mean"         # sage only
    agg_p: float = 1.0

    @property
    def k(self) -> int:
        return len(self.dims) - 1


CONFIGS: Dict[str, Workload] = {
    # 2,000 nodes, mean degree 10, 2-layer SAGE 64-64-16, 32 queries with 5-20 uniform edges, 10 %
    "tiny": Workload("tiny", 2_000, 10, None, "sage", (64, 64, 16), 32, 100_000,
                     q_degree=("uniform", 5, 20), q_endpoints="uniform"),
    # Reddit-shaped: 230 k nodes, mean degree ~500, tail capped near 20 k, 2-layer GCN 602-256-41
    "mid": Workload("mid", 230_000, 500, 20_000, "gcn", (602, 256, 41), 1024, 50_000),
    # Products-shaped: 2.4 M nodes, mean degree 50, 47 communities, 3-layer SAGE 100-256-256-47, bf16 PEs
    "large": Workload("large", 2_400_000, 50, 20_000, "sage", (100, 256, 256, 47), 4096, 50_000,
                      n_blocks=47, intra=0.8, pe_dtype="bf16", q_endpoints="block"),
    # same graph, 3-layer GAT with 4 heads x 64
    "attention": Workload("attention", 2_400_000, 50, 20_000, "gat", (100, 256, 256, 47), 4096, 100_000,
                          n_blocks=47, intra=0.8, heads=4, pe_dtype="bf16", q_endpoints="block"),
}
# scaled-down copies with the same structure, small enough for a CPU oracle to finish in seconds
CONFIGS["mid_s"] = replace(CONFIGS["mid"], name="mid_s", n_nodes=12_000, avg_deg=80, max_deg=3_000, batch=96)
CONFIGS["large_s"] = replace(CONFIGS["large"], name="large_s", n_nodes=60_000, avg_deg=30, max_deg=2_000, batch=256)
CONFIGS["attention_s"] = replace(CONFIGS["attention"], name="attention_s", n_nodes=60_000, avg_deg=30,
                                 max_deg=2_000, batch=256)
# `mid` with a feature table that fits the 256 MB memory-side cache (diagnostic: the same kernels in the regime
# where every re-read of a row is a cache hit)
CONFIGS["mid_fit"] = replace(CONFIGS["mid"], name="mid_fit", n_nodes=50_000, max_deg=10_000, gamma_ppm=120_000)
CONFIGS["tiny_gcn"] = replace(CONFIGS["tiny"], name="tiny_gcn", model="gcn")
CONFIGS["tiny_gat"] = replace(CONFIGS["tiny"], name="tiny_gat", model="gat", heads=4, dims=(64, 64, 16))
CONFIGS["tiny_gat8"] = replace(CONFIGS["tiny"], name="tiny_gat8", model="gat", heads=8, dims=(64, 64, 64, 10))
CONFIGS["tiny_sage3"] = replace(CONFIGS["tiny"], name="tiny_sage3", dims=(64, 64, 64, 16))
# SAGE-style layers with the other aggregation functions of Sec. 6.2
CONFIGS["tiny_sum"] = replace(CONFIGS["tiny"], name="tiny_sum", aggregator="sum")
CONFIGS["tiny_max"] = replace(CONFIGS["tiny"], name="tiny_max", aggregator="max")
CONFIGS["tiny_power"] = replace(CONFIGS["tiny"], name="tiny_power", aggregator="power", agg_p=3.0)
CONFIGS["tiny_moment"] = replace(CONFIGS["tiny"], name="tiny_moment", aggregator="moment", agg_p=2.0)
# GCNII convolutions (initial residual + identity mapping), 2 and 6 layers deep, all widths equal
CONFIGS["tiny_gcnii"] = replace(CONFIGS["tiny"], name="tiny_gcnii", model="gcnii", dims=(64, 64, 64))
CONFIGS["tiny_gcnii6"] = replace(CONFIGS["tiny"], name="tiny_gcnii6", model="gcnii", dims=(64,) * 7)
CONFIGS["mid_s_gcnii"] = replace(CONFIGS["mid_s"], name="mid_s_gcnii", model="gcnii", dims=(128,) * 5)
for _agg, _p in (("max", 1.0), ("power", 2.5), ("moment", 2.0)):       # long rows (cut into parts), bf16 tables
    CONFIGS[f"large_s_{_agg}"] = replace(CONFIGS["large_s"], name=f"large_s_{_agg}", aggregator=_agg, agg_p=_p)
CONFIGS["tiny_moment4"] = replace(CONFIGS["tiny"], name="tiny_moment4", aggregator="moment", agg_p=4.0,
                                  dims=(64, 64, 64, 16))


@dataclass
class Table:
    data: np.ndarray      # (n_rows, ld): float32 values, or uint16 bf16 bit patterns
    dtype: str            # "f32" | "bf16"
    dim: int

    @property
    def ld(self) -> int:
        return int(self.data.shape[1])


@dataclass
class Built:
    cfg: Workload
    graph: BaseGraph
    tables: List[Table]              # [features, PE^(1), ..., PE^(k-1)]
    layers: List[LayerParams]

    def batch(self, r: int = 0, n_query: Optional[int] = None) -> QueryBatch:
        c = self.cfg
        return make_batch(self.graph, c.batch if n_query is None else n_query, c.dims[0], 2000 + r,
                          degree=c.q_degree, endpoints=c.q_endpoints, intra=c.intra or 0.8)


def _store(x: np.ndarray, dim: int, dtype: str) -> Table:
    if dtype == "f32":
        return Table(x, "f32", dim)
    ld = padded_ld(dim, 2)
    bits = np.zeros((x.shape[0], ld), dtype=np.uint16)
    bits[:, :dim] = to_bf16_bits(x[:, :dim])
    return Table(bits, "bf16", dim)


def build_workload(cfg: Workload, graph: Optional[BaseGraph] = None,
                   pe_fn: Optional[Callable] = None) -> Built:
    """pe_fn(graph, features fp32 (n, d_0), layers) -> list of k-1 fp32 arrays (n, d_l): real
    precomputed embeddings.  Without it the tables are filled with seeded stand-in values."""
    g = graph if graph is not None else power_law_graph(
        cfg.n_nodes, cfg.avg_deg, cfg.exponent, cfg.max_deg, 1001, cfg.n_blocks, cfg.intra)
    layers = make_layers(cfg.model, list(cfg.dims), 1003, cfg.heads, cfg.aggregator, cfg.agg_p)
    x = normal_table(g.n, cfg.dims[0], 1002)
    tables = [_store(x, cfg.dims[0], cfg.feat_dtype)]
    if pe_fn is not None:
        # real embeddings are computed from the values as stored (after any bf16 rounding)
        pes = pe_fn(g, tables[0], layers)
        for l in range(1, cfg.k):
            d = layers[l].d_in
            p = np.zeros((g.n, padded_ld(d, 4)), dtype=np.float32)
            p[:, :d] = pes[l - 1]
            tables.append(_store(p, d, cfg.pe_dtype))
    else:
        for l in range(1, cfg.k):
            d = layers[l].d_in
            tables.append(_store(relu_normal_table(g.n, d, 1004 + l), d, cfg.pe_dtype))
    return Built(cfg, g, tables, layers)
