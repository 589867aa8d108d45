"""Host-side checks: the seeded generators produce what they promise, and the oracle and the
product path stay separate (neither imports the other)."""
from __future__ import annotations

import os
import re

import numpy as np
import scipy.sparse as sp

from synth import CONFIGS, build_workload, make_layers, power_law_graph
from synth.batches import make_batch
from synth.tables import normal_table, padded_ld, relu_normal_table, to_bf16_bits

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_graph_is_symmetric_simple_and_heavy_tailed():
    g = power_law_graph(5_000, 20, max_deg=600, seed=3)
    A = sp.csr_matrix((np.ones(g.nnz), g.indices, g.indptr), shape=(g.n, g.n))
    assert (A != A.T).nnz == 0
    assert A.diagonal().sum() == 0 and A.max() == 1
    for v in (0, 17, g.n - 1):
        row = g.indices[g.indptr[v]:g.indptr[v + 1]]
        assert np.all(np.diff(row) > 0)
    deg = g.degrees()
    assert 12 < deg.mean() < 22 and deg.max() > 8 * deg.mean()
    g2 = power_law_graph(5_000, 20, max_deg=600, seed=3)
    assert np.array_equal(g.indptr, g2.indptr) and np.array_equal(g.indices, g2.indices)
    assert not np.array_equal(power_law_graph(5_000, 20, max_deg=600, seed=4).indices[:100], g.indices[:100])


def test_block_graph_keeps_most_edges_inside_communities():
    g = power_law_graph(20_000, 20, max_deg=500, seed=5, n_blocks=10, intra=0.8)
    dst = np.repeat(np.arange(g.n), np.diff(g.indptr))
    same = (g.block[dst] == g.block[g.indices]).mean()
    assert 0.75 < same < 0.9


def test_batches_have_distinct_in_range_endpoints_and_are_seeded():
    g = power_law_graph(3_000, 12, seed=7, n_blocks=5, intra=0.8)
    for mode in ("uniform", "degree", "block"):
        qb = make_batch(g, 24, 10, seed=11, degree=("graph",) if mode != "uniform" else ("uniform", 3, 9), endpoints=mode)
        assert qb.qe_query.dtype == np.int32 and qb.qe_node.dtype == np.int32
        assert qb.qe_query.min() >= 0 and qb.qe_query.max() < 24
        assert qb.qe_node.min() >= 0 and qb.qe_node.max() < g.n
        pairs = qb.qe_query.astype(np.int64) * g.n + qb.qe_node
        assert np.unique(pairs).size == pairs.size
        assert qb.feats.shape == (24, padded_ld(10, 4)) and np.all(qb.feats[:, 10:] == 0)
        qb2 = make_batch(g, 24, 10, seed=11, degree=("graph",) if mode != "uniform" else ("uniform", 3, 9), endpoints=mode)
        assert np.array_equal(qb.qe_node, qb2.qe_node) and np.array_equal(qb.feats, qb2.feats)


def test_tables_padding_chunk_independence_and_bf16():
    t = normal_table(70_000, 10, seed=2)                       # more than one generation chunk
    assert t.shape == (70_000, 12) and np.all(t[:, 10:] == 0)
    assert np.array_equal(t[:1000], normal_table(1000, 10, seed=2))
    assert abs(float(t[:, :10].mean())) < 0.01 and abs(float(t[:, :10].std()) - 1.0) < 0.01
    r = relu_normal_table(1000, 8, seed=3)
    assert r.min() == 0.0 and 0.4 < (r[:, :8] == 0).mean() < 0.6
    bits = to_bf16_bits(t)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.all(np.abs(back - t) <= np.abs(t) * 2.0 ** -8 + 1e-38)


def test_workload_shapes_follow_the_config():
    built = build_workload(CONFIGS["large_s"])
    c = built.cfg
    assert [t.dtype for t in built.tables] == ["f32", "bf16", "bf16"]
    assert [t.dim for t in built.tables] == [100, 256, 256]
    assert all((t.ld * (4 if t.dtype == "f32" else 2)) % 16 == 0 for t in built.tables)
    assert [(p.d_in, p.d_out) for p in built.layers] == [(100, 256), (256, 256), (256, 47)]
    gat = make_layers("gat", [100, 256, 256, 47], heads=4)
    assert gat[-1].head_mean and gat[-1].d_out == 4 * 47 and gat[-1].out_width == 47
    assert gat[0].a_src.shape == (4, 64)
    assert built.batch(0).n_query == c.batch


def _imports(path):
    text = open(path).read()
    return set(re.findall(r"^\s*(?:from|import)\s+([A-Za-z_][\w\.]*)", text, flags=re.M))


def test_oracle_and_product_do_not_import_each_other():
    pkg = os.path.join(ROOT, "paper_2501_08547_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            mods = _imports(os.path.join(pkg, name))
            assert not any(m == "oracle" or m.startswith("oracle.") for m in mods), name
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            mods = _imports(os.path.join(ROOT, "oracle", name))
            assert not any(m.startswith("paper_2501_08547_amd") or m == "torch" for m in mods), name
    for name in os.listdir(os.path.join(ROOT, "synth")):
        if name.endswith(".py"):
            mods = _imports(os.path.join(ROOT, "synth", name))
            assert not any(m.startswith("paper_2501_08547_amd") or m.startswith("oracle") for m in mods), name
    # the kernels' sources never mention the oracle either
    for name in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", name)).read().lower(), name
