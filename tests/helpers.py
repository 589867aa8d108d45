"""Shared test scaffolding: small workloads with real precomputed embeddings."""
from __future__ import annotations

from dataclasses import replace

import numpy as np

from oracle import exact_inference as ex
from oracle import srpe_oracle as orc
from synth import CONFIGS, build_workload
from synth.configs import Built, Table


def pe_from_oracle(graph, feat_table: Table, layers):
    """Real precomputed embeddings: exact inference on the base graph from the features as stored."""
    x = orc.decode_table(feat_table.data, feat_table.dtype, feat_table.dim)
    return ex.base_inference(graph.indptr, graph.indices, x, layers)


def small_workload(name: str, n_nodes=None, batch=None, real_pe=True, **over) -> Built:
    cfg = CONFIGS[name]
    if n_nodes is not None:
        over["n_nodes"] = n_nodes
    if batch is not None:
        over["batch"] = batch
    if over:
        cfg = replace(cfg, **over)
    return build_workload(cfg, pe_fn=pe_from_oracle if real_pe else None)


def lazy_tables(built: Built):
    return [orc.LazyTable(t.data, t.dtype, t.dim) for t in built.tables]


def f64_tables(built: Built):
    """Tables for pins that must hold to 1e-12: features as stored, embeddings recomputed in fp64
    (not rounded to the storage type)."""
    x = orc.decode_table(built.tables[0].data, built.tables[0].dtype, built.tables[0].dim)
    pes = ex.base_inference(built.graph.indptr, built.graph.indices, x, built.layers)
    return [orc.LazyTable(x, "f64", x.shape[1])] + [orc.LazyTable(p, "f64", p.shape[1]) for p in pes]


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of ||g - r||_inf / ||r||_inf (rows whose reference is all zero compare absolutely)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    return float(np.max(np.where(den > 0, num / np.where(den > 0, den, 1.0), num))) if ref.size else 0.0
