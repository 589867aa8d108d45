"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Each pin names the passage it rests on.
"""
from __future__ import annotations

import os
from dataclasses import replace
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.special

from oracle import exact_inference as ex
from oracle import srpe_oracle as orc
from synth import make_layers, power_law_graph, to_bf16_bits
from synth.batches import make_batch
from tests.helpers import f64_tables, small_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MODELS = ["tiny", "tiny_gcn", "tiny_gat"]


def _x64(built):
    t = built.tables[0]
    return orc.decode_table(t.data, t.dtype, t.dim)


def _exact(built, qb):
    return ex.exact_full_inference(built.graph.indptr, built.graph.indices, _x64(built),
                                   qb.feats[:, :built.cfg.dims[0]], qb.qe_query, qb.qe_node, built.layers)


def _srpe(built, qb, gamma_ppm, tables=None, recompute_set=None, return_all=False):
    g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query,
                                    qb.qe_query, qb.qe_node, gamma_ppm, recompute_set)
    tabs = f64_tables(built) if tables is None else tables
    return g, orc.srpe_reference(g, tabs, built.layers, qb.feats, return_all=return_all)


# ---- P1: recomputing every candidate reproduces exact inference (Sec. 5.2.1: recomputation
#      takes the query edges into account; Sec. 6.1: all edges ending at a target are added).
#      Holds for k <= 3: a node's layer-l embedding depends on the batch only within l hops.
@pytest.mark.parametrize("name", MODELS + ["tiny_sage3"])
def test_full_budget_equals_exact_inference(name):
    built = small_workload(name, n_nodes=600)
    qb = built.batch(0, n_query=12)
    _, out = _srpe(built, qb, 1_000_000)
    ref = _exact(built, qb)
    assert out.shape == ref.shape
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-11)


@pytest.mark.parametrize("name", MODELS + ["tiny_sage3"])
def test_sparse_exact_inference_equals_dense(name):
    """The sparse form used at 10^4-10^5 nodes is the dense one, with a repeated request edge too."""
    built = small_workload(name, n_nodes=500)
    qb = built.batch(2, n_query=9)
    q = np.concatenate([qb.qe_query, qb.qe_query[:2]])
    u = np.concatenate([qb.qe_node, qb.qe_node[:2]])
    args = (built.graph.indptr, built.graph.indices, _x64(built), qb.feats[:, :built.cfg.dims[0]], q, u, built.layers)
    np.testing.assert_allclose(ex.exact_full_inference_sparse(*args), ex.exact_full_inference(*args), rtol=0, atol=1e-11)


# ---- the two restricted evaluations used at full size: exact inference for a few queries (Eq. 1 unrolled
#      from them) and the SRPE reference for a few rows, each against the whole-graph / whole-batch form
@pytest.mark.parametrize("name,over", [("tiny_sage3", {}), ("tiny_gcn", {}), ("tiny_gat", dict(dims=(64, 32, 32, 8))),
                                       ("tiny_gcnii", {}), ("tiny_sum", dict(dims=(64, 32, 32, 8))), ("large_s", dict(n_nodes=5000))])
def test_exact_inference_of_sampled_queries_equals_the_whole_graph_form(name, over):
    built = small_workload(name, n_nodes=over.pop("n_nodes", 700), real_pe=False, **over)
    qb = built.batch(4, n_query=14)
    q = np.concatenate([qb.qe_query, qb.qe_query[:3]])             # a repeated request edge counts twice
    u = np.concatenate([qb.qe_node, qb.qe_node[:3]])
    x = _x64(built)
    d0 = built.cfg.dims[0]
    whole = ex.exact_full_inference_sparse(built.graph.indptr, built.graph.indices, x, qb.feats[:, :d0], q, u, built.layers)
    touched = []

    def rows(ids):
        touched.append(ids)
        return x[ids]
    sample = [11, 0, 5, 13]
    got = ex.exact_inference_rows(built.graph.indptr, built.graph.indices, rows, qb.feats[:, :d0], q, u, built.layers, sample)
    np.testing.assert_allclose(got, whole[sorted(sample)], rtol=0, atol=1e-11)
    # it is a restriction: far fewer than all nodes are read on a sparse graph with few sampled queries
    if name == "large_s":
        assert np.unique(np.concatenate(touched)).size < built.graph.n
    # an isolated query (no edges) sees only itself
    got1 = ex.exact_inference_rows(built.graph.indptr, built.graph.indices, rows, qb.feats[:, :d0],
                                   q[q != 5], u[q != 5], built.layers, [5])
    whole1 = ex.exact_full_inference_sparse(built.graph.indptr, built.graph.indices, x, qb.feats[:, :d0],
                                            q[q != 5], u[q != 5], built.layers)
    np.testing.assert_allclose(got1, whole1[[5]], rtol=0, atol=1e-11)


@pytest.mark.parametrize("name", ["tiny_sage3", "tiny_gat", "tiny_gcnii6", "tiny_moment4"])
def test_reference_of_sampled_rows_equals_the_whole_batch(name):
    built = small_workload(name, n_nodes=600)
    qb = built.batch(1, n_query=16)
    tabs = f64_tables(built)
    g, whole = _srpe(built, qb, 400_000, tables=tabs)
    sample = [9, 2, 15]
    got = orc.srpe_reference_rows(g, tabs, built.layers, qb.feats, sample)
    np.testing.assert_array_equal(got, whole[sorted(sample)])
    with pytest.raises(ValueError):
        orc.srpe_reference_rows(g, tabs, built.layers, qb.feats, [16])


def test_full_budget_three_layer_gat():
    built = small_workload("tiny", n_nodes=400, model="gat", heads=2, dims=(64, 32, 32, 8))
    qb = built.batch(1, n_query=8)
    _, out = _srpe(built, qb, 1_000_000)
    np.testing.assert_allclose(out, _exact(built, qb), rtol=0, atol=1e-11)


def test_full_budget_three_layer_gcn_is_not_exact():
    """Scope of P1 for GCN: the symmetric normalisation makes a node's layer-1 embedding depend on
    the degrees of its neighbours, so a stored embedding two hops from the batch is already stale.
    Full budget is exact for GCN only up to k = 2 (the depth the paper uses for GCN, Sec. 8.1)."""
    built = small_workload("tiny", n_nodes=400, model="gcn", dims=(64, 32, 32, 8))
    qb = built.batch(1, n_query=8)
    _, out = _srpe(built, qb, 1_000_000)
    ref = _exact(built, qb)
    err = np.abs(out - ref).max()
    assert 1e-9 < err < 0.05 * np.abs(ref).max()


def test_partial_budget_differs_from_exact():
    """The approximation is real: with no recomputation the result is not the exact one
    (otherwise P1 could pass with a builder that ignores the budget)."""
    built = small_workload("tiny", n_nodes=600)
    qb = built.batch(0, n_query=12)
    _, out = _srpe(built, qb, 0)
    assert np.abs(out - _exact(built, qb)).max() > 1e-6


# ---- P11: at full budget every freshly computed row equals the full embedding f_u^(l) (Sec. 5.1)
def test_full_budget_intermediate_rows_equal_full_embeddings():
    built = small_workload("tiny_sage3", n_nodes=500)
    qb = built.batch(2, n_query=10)
    g, bufs = _srpe(built, qb, 1_000_000, return_all=True)
    full = ex.exact_layer_embeddings(built.graph.indptr, built.graph.indices, _x64(built),
                                     qb.feats[:, :64], qb.qe_query, qb.qe_node, built.layers)
    n = built.graph.n
    ids = np.concatenate([n + np.arange(qb.n_query), g.T])
    for l in range(0, built.cfg.k):
        np.testing.assert_allclose(bufs[l], full[l][ids], rtol=0, atol=1e-11)


# ---- P2: zero budget = serving from historical embeddings (Sec. 3.2, Sec. 5): per layer a dense
#      product with the B x N query adjacency, checked with library matmuls.
@pytest.mark.parametrize("name", ["tiny", "tiny_gcn", "tiny_sage3"])
def test_zero_budget_closed_form(name):
    built = small_workload(name, n_nodes=500)
    qb = built.batch(3, n_query=16)
    tabs = f64_tables(built)
    g, out = _srpe(built, qb, 0, tables=tabs)
    assert g.T.size == 0 and g.rows_in == qb.n_query
    n, B = built.graph.n, qb.n_query
    Aq = np.zeros((B, n))
    np.add.at(Aq, (qb.qe_query, qb.qe_node), 1.0)
    H = qb.feats[:, :built.cfg.dims[0]].astype(np.float64)
    deg_q = Aq.sum(1)
    deg_u = np.diff(built.graph.indptr) + Aq.sum(0)
    for l, p in enumerate(built.layers):
        P = tabs[l].rows(np.arange(n))
        W, b = p.W_nb.astype(np.float64), p.bias.astype(np.float64)
        if p.model == "sage":
            pre = H @ p.W_self.astype(np.float64) + ((Aq / deg_q[:, None]) @ P) @ W + b
        else:
            A_hat = Aq / np.sqrt((deg_q[:, None] + 1.0) * (deg_u[None, :] + 1.0))
            pre = (A_hat @ P + H / (deg_q[:, None] + 1.0)) @ W + b
        H = np.maximum(pre, 0.0) if p.act == "relu" else pre
    np.testing.assert_allclose(out, H, rtol=0, atol=1e-11)


# ---- P3: aggregation is commutative / associative (Sec. 6.2), so neither the order of the
#      request's edge list nor the numbering of the queries matters.
def test_edge_order_and_query_numbering_invariance():
    built = small_workload("tiny_gat", n_nodes=500)
    qb = built.batch(4, n_query=10)
    tabs = f64_tables(built)
    g0, out0 = _srpe(built, qb, 300_000, tables=tabs)
    rng = np.random.default_rng(7)
    perm = rng.permutation(qb.n_edges)
    qb1 = replace(qb, qe_query=qb.qe_query[perm], qe_node=qb.qe_node[perm])
    g1, out1 = _srpe(built, qb1, 300_000, tables=tabs)
    for a, b in ((g0.R, g1.R), (g0.T, g1.T), (g0.indptr, g1.indptr), (g0.cols, g1.cols), (g0.cdeg, g1.cdeg)):
        assert np.array_equal(a, b)
    np.testing.assert_array_equal(out0, out1)
    qperm = rng.permutation(qb.n_query)              # new index of query q is qperm[q]
    feats2 = np.empty_like(qb.feats)
    feats2[qperm] = qb.feats
    qb2 = replace(qb, qe_query=qperm[qb.qe_query].astype(np.int32), feats=feats2)
    g2, out2 = _srpe(built, qb2, 300_000, tables=tabs)
    assert np.array_equal(g2.T, g0.T)
    np.testing.assert_allclose(out2[qperm], out0, rtol=0, atol=1e-12)


def test_neighbour_order_invariance_of_a_row():
    rng = np.random.default_rng(3)
    for model, heads in (("sage", 1), ("gcn", 1), ("gat", 4)):
        p = make_layers(model, [24, 16, 8], heads=heads)[0]
        h_self, h_src = rng.standard_normal(24), rng.standard_normal((9, 24))
        deg = rng.integers(1, 50, size=9)
        a = orc.layer_row(p, h_self, h_src, deg)
        o = rng.permutation(9)
        np.testing.assert_allclose(orc.layer_row(p, h_self, h_src[o], deg[o]), a, rtol=0, atol=1e-12)


# ---- P4: mean aggregation of a constant is the constant; the mean's denominator counts the
#      query edges too (Sec. 5.2.1: |N(u)| is the whole neighbourhood).
def test_constant_features_mean_returns_constant():
    built = small_workload("tiny", n_nodes=400, real_pe=False)
    qb = built.batch(5, n_query=8)
    d = 64
    layers = make_layers("sage", [d, d, d])
    for p in layers:
        p.W_self[:] = 0.0
        p.W_nb[:] = np.eye(d, dtype=np.float32)
        p.bias[:] = 0.0
        p.act = "none"
    c = np.linspace(-1.0, 2.0, d)
    const = np.tile(c, (built.graph.n, 1))
    tabs = [orc.LazyTable(const, "f64", d), orc.LazyTable(const, "f64", d)]
    qb = replace(qb, feats=np.tile(c, (qb.n_query, 1)).astype(np.float64))
    g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query,
                                    qb.qe_query, qb.qe_node, 400_000)
    assert g.T.size > 0
    bufs = orc.srpe_reference(g, tabs, layers, qb.feats, return_all=True)
    for buf in bufs[1:]:
        np.testing.assert_allclose(buf, np.tile(c, (buf.shape[0], 1)), rtol=0, atol=1e-12)


# ---- P5 / P6: attention weights are a softmax over the row (Sec. 6.2, softmax-based aggregation)
def test_gat_zero_attention_vectors_give_mean_of_projected_neighbours():
    rng = np.random.default_rng(11)
    p = make_layers("gat", [20, 12, 6], heads=3)[0]
    p.a_src[:] = 0.0
    p.a_dst[:] = 0.0
    h_self, h_src = rng.standard_normal(20), rng.standard_normal((7, 20))
    got = orc.layer_row(p, h_self, h_src, np.ones(7))
    pre = (h_src.mean(0) @ p.W_nb.astype(np.float64)) + p.bias
    want = np.where(pre > 0, pre, np.expm1(pre))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_gat_row_matches_library_softmax_and_survives_large_logits():
    rng = np.random.default_rng(12)
    for scale in (1.0, 400.0):
        p = make_layers("gat", [20, 12, 6], heads=3)[0]
        p.a_src *= scale
        p.a_dst *= scale
        p.act = "none"
        h_self, h_src = rng.standard_normal(20), rng.standard_normal((11, 20))
        got = orc.layer_row(p, h_self, h_src, np.ones(11))
        assert np.all(np.isfinite(got))
        W = p.W_nb.astype(np.float64)
        z = (h_src @ W).reshape(11, 3, 4)
        zv = (h_self @ W).reshape(3, 4)
        e = np.einsum("uhd,hd->uh", z, p.a_src.astype(np.float64)) + np.einsum("hd,hd->h", zv, p.a_dst.astype(np.float64))
        e = np.where(e > 0, e, 0.2 * e)
        if scale > 1:
            assert np.abs(e).max() > 100.0
        alpha = scipy.special.softmax(e, axis=0)
        np.testing.assert_allclose(alpha.sum(0), 1.0, atol=1e-12)
        want = np.einsum("uh,uhd->hd", alpha, z).reshape(-1) + p.bias
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-10)


def test_gat_output_layer_averages_heads():
    rng = np.random.default_rng(13)
    p = make_layers("gat", [10, 8, 5], heads=4)[1]
    assert p.head_mean and p.d_out == 20 and p.out_width == 5
    h_self, h_src = rng.standard_normal(8), rng.standard_normal((6, 8))
    got = orc.layer_row(p, h_self, h_src, np.ones(6))
    q = replace(p, head_mean=False)
    full = orc.layer_row(q, h_self, h_src, np.ones(6)).reshape(4, 5)
    np.testing.assert_allclose(got, full.mean(0), rtol=0, atol=1e-12)


# ---- P7: a linear GCN is a matrix power (Eq. 1 with linear update) - pins the exact-inference code itself
def test_linear_gcn_is_matrix_power():
    g = power_law_graph(150, 6, seed=5)
    layers = make_layers("gcn", [10, 7, 7, 4])
    for p in layers:
        p.act = "none"
        p.bias[:] = 0.0
    rng = np.random.default_rng(1)
    X = rng.standard_normal((150, 10))
    qb = make_batch(g, 5, 10, seed=9, degree=("uniform", 2, 6))
    out = ex.exact_full_inference(g.indptr, g.indices, X, qb.feats[:, :10], qb.qe_query, qb.qe_node, layers)
    n = 155
    A = np.zeros((n, n))
    for v in range(150):
        for u in g.indices[g.indptr[v]:g.indptr[v + 1]]:
            A[v, u] += 1
    for q, u in zip(qb.qe_query, qb.qe_node):
        A[150 + q, u] += 1
        A[u, 150 + q] += 1
    A += np.eye(n)
    d = A.sum(1)
    A_hat = A / np.sqrt(np.outer(d, d))
    H = np.concatenate([X, qb.feats[:, :10].astype(np.float64)])
    W = layers[0].W_nb.astype(np.float64) @ layers[1].W_nb.astype(np.float64) @ layers[2].W_nb.astype(np.float64)
    want = (np.linalg.matrix_power(A_hat, 3) @ H @ W)[150:]
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-12)


def test_exact_sage_single_node_by_hand():
    """Two-layer SAGE on a 3-node path plus one query, written out term by term."""
    indptr = np.array([0, 1, 3, 4], dtype=np.int64)          # 0-1, 1-2
    indices = np.array([1, 0, 2, 1], dtype=np.int32)
    layers = make_layers("sage", [2, 2, 2], seed=4)
    X = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -1.0]])
    xq = np.array([[0.5, 0.5]])
    out = ex.exact_full_inference(indptr, indices, X, xq, np.array([0]), np.array([2]), layers)
    f = lambda p, hs, hn: np.maximum(hs @ p.W_self.astype(np.float64) + hn @ p.W_nb.astype(np.float64) + p.bias, 0) \
        if p.act == "relu" else hs @ p.W_self.astype(np.float64) + hn @ p.W_nb.astype(np.float64) + p.bias
    p1, p2 = layers
    h2 = f(p1, X[2], (X[1] + xq[0]) / 2)      # node 2 now has neighbours {1, q}
    hq = f(p1, xq[0], X[2])
    want = f(p2, hq, h2)
    np.testing.assert_allclose(out[0], want, rtol=0, atol=1e-14)


# ---- P8: counting identities of the computation graph (Eq. 2 budget; Sec. 6.1 edge sets)
@pytest.mark.parametrize("gamma_ppm", [0, 1, 49_999, 100_000, 333_333, 999_999, 1_000_000])
def test_graph_counting_identities(gamma_ppm):
    built = small_workload("tiny", real_pe=False)
    qb = built.batch(6)
    g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query,
                                    qb.qe_query, qb.qe_node, gamma_ppm)
    deg = np.diff(built.graph.indptr)
    assert g.T.size == (gamma_ppm * g.R.size) // 1_000_000
    assert g.T.size <= gamma_ppm / 1e6 * g.R.size + 1e-9
    assert np.all(np.isin(g.T, g.R)) and np.all(np.diff(g.T) > 0)
    assert g.qdeg.sum() == qb.n_edges and np.all(g.qdeg >= 1)
    qd = dict(zip(g.R.tolist(), g.qdeg.tolist()))
    assert g.nnz_in == qb.n_edges + sum(int(deg[u]) + qd[u] for u in g.T.tolist())
    assert g.indptr.shape[0] == g.rows_in + 1 and g.cols.shape[0] == g.nnz_in == g.cdeg.shape[0]
    score = lambda u: Fraction(qd[u], qd[u] + int(deg[u]))
    rest = [u for u in g.R.tolist() if u not in set(g.T.tolist())]
    if g.T.size and rest:
        assert min(score(u) for u in g.T.tolist()) >= max(score(u) for u in rest)
    # tags: buffer columns point at existing rows; table columns are never targets
    buf = g.cols[g.cols < 0]
    assert np.all(~buf < g.rows_in)
    assert not np.any(np.isin(g.cols[g.cols >= 0], g.T))
    # query rows list each neighbour once per request edge, ascending
    for q in range(qb.n_query):
        c = g.cols[g.indptr[q]:g.indptr[q + 1]].astype(np.int64)
        ids = np.where(c >= 0, c, g.T[np.maximum(~c - qb.n_query, 0)] if g.T.size else c)
        assert np.array_equal(ids, np.sort(qb.qe_node[qb.qe_query == q]))


def test_selection_matches_brute_force_with_ties():
    rng = np.random.default_rng(21)
    for _ in range(50):
        m = int(rng.integers(1, 40))
        R = np.sort(rng.choice(1000, size=m, replace=False)).astype(np.int64)
        qdeg = rng.integers(1, 4, size=m).astype(np.int64)
        deg = rng.integers(0, 5, size=m).astype(np.int64)           # few values -> many exact ties, some deg 0
        gamma = int(rng.integers(0, 1_000_001))
        want_n = gamma * m // 1_000_000
        order = sorted(range(m), key=lambda i: (-Fraction(int(qdeg[i]), int(qdeg[i] + deg[i])), int(R[i])))
        want = np.sort(R[order[:want_n]])
        assert np.array_equal(orc.select_targets(R, qdeg, deg, gamma), want)


def test_selection_uses_exact_fractions():
    """Two ratios that differ by less than double-precision resolution must still be ordered exactly."""
    a, b, c, d = 300_000_007, 900_000_011, 210_000_005, 630_000_008      # a*d - b*c = 1
    fa, fc = Fraction(a, b), Fraction(c, d)
    assert a / b == c / d and float(fa) == float(fc) and fa > fc
    R = np.array([5, 9], dtype=np.int64)
    qdeg = np.array([c, a], dtype=np.int64)                 # the larger ratio sits at the larger id
    deg = np.array([d - c, b - a], dtype=np.int64)
    assert orc.select_targets(R, qdeg, deg, 500_000).tolist() == [9]


# ---- P9: the worked example of Sec. 5.2 (candidates {2,3,4,7}, half of them recomputed -> {2,7})
def _read_fig7():
    vals = {}
    queries = []
    for line in open(os.path.join(GOLDEN, "fig7_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        if key == "query":
            qid, nb = rest.split(":")
            queries.append([int(x) for x in nb.split()])
        else:
            vals[key] = rest
    return vals, queries


def test_paper_worked_example():
    vals, queries = _read_fig7()
    n = int(vals["nodes"])
    nb = [[] for _ in range(n)]
    for e in vals["undirected_edges"].split():
        a, b = (int(x) for x in e.split("-"))
        nb[a].append(b)
        nb[b].append(a)
    assert sorted(nb[3]) == [0, 5, 7] and 1 in nb[2] and 4 in nb[2] and 6 in nb[7]      # facts from the text
    indptr = np.concatenate([[0], np.cumsum([len(x) for x in nb])]).astype(np.int64)
    indices = np.array([u for x in nb for u in sorted(x)], dtype=np.int32)
    qe_q = np.array([q for q, lst in enumerate(queries) for _ in lst], dtype=np.int32)
    qe_u = np.array([u for lst in queries for u in lst], dtype=np.int32)
    g = orc.build_computation_graph(indptr, indices, len(queries), qe_q, qe_u, int(vals["gamma_ppm"]))
    assert g.R.tolist() == [int(x) for x in vals["expect_candidates"].split()]
    assert g.qdeg.tolist() == [int(x) for x in vals["expect_qdeg"].split()]
    assert g.T.tolist() == [int(x) for x in vals["expect_targets"].split()]
    # Sec. 6.1: layer 1 of the example holds 4->2, 1->2, 8->2 (query 0), 9->2 and 6->7, 3->7, 9->7
    row2 = g.cols[g.indptr[2]:g.indptr[3]].tolist()
    row7 = g.cols[g.indptr[3]:g.indptr[4]].tolist()
    assert row2 == [1, 4, ~0, ~1] and row7 == [3, 6, ~1]
    # last layer: query 8 <- {2 (recomputed, buffer row 2), 3 (stored)}, query 9 <- {2, 4, 7 (buffer row 3)}
    assert g.cols[g.indptr[0]:g.indptr[1]].tolist() == [~2, 3]
    assert g.cols[g.indptr[1]:g.indptr[2]].tolist() == [~2, 4, ~3]
    assert g.cdeg[g.indptr[2]:g.indptr[3]].tolist() == [2, 3 + 1, 2, 3]


# ---- P10: a one-layer model uses no stored embedding, so it is exact for any budget (Sec. 5: l = 1..k-1)
@pytest.mark.parametrize("gamma_ppm", [0, 250_000, 1_000_000])
def test_one_layer_model_is_exact_for_any_budget(gamma_ppm):
    built = small_workload("tiny_gcn", n_nodes=300, dims=(64, 16))
    qb = built.batch(7, n_query=6)
    _, out = _srpe(built, qb, gamma_ppm)
    np.testing.assert_allclose(out, _exact(built, qb), rtol=0, atol=1e-12)


# ---- explicit recompute set, duplicates, degenerate inputs
def test_explicit_recompute_set_and_duplicate_edges():
    built = small_workload("tiny", n_nodes=300)
    qb = built.batch(8, n_query=6)
    dup_q = np.concatenate([qb.qe_query, qb.qe_query[:3]])
    dup_u = np.concatenate([qb.qe_node, qb.qe_node[:3]])
    qb2 = replace(qb, qe_query=dup_q, qe_node=dup_u)
    g, out = _srpe(built, qb2, 1_000_000)
    assert g.indptr[qb.n_query] == qb.n_edges + 3
    np.testing.assert_allclose(out, _exact(built, qb2), rtol=0, atol=1e-11)       # multiplicity on both sides
    R, _ = orc.candidates(qb.qe_node)
    g3, _ = _srpe(built, qb, 0, recompute_set=R[::2])
    assert np.array_equal(g3.T, R[::2])
    with pytest.raises(ValueError):
        _srpe(built, qb, 0, recompute_set=[built.graph.n - 1 if built.graph.n - 1 not in R else -5])


def test_empty_batch_edges_and_isolated_query():
    built = small_workload("tiny", n_nodes=300)
    qb = built.batch(9, n_query=4)
    keep = qb.qe_query != 2                       # query 2 has no edge at all
    qb = replace(qb, qe_query=qb.qe_query[keep], qe_node=qb.qe_node[keep])
    g, out = _srpe(built, qb, 500_000)
    assert g.indptr[3] == g.indptr[2]
    np.testing.assert_allclose(_srpe(built, qb, 1_000_000)[1], _exact(built, qb), rtol=0, atol=1e-11)
    none = replace(qb, qe_query=qb.qe_query[:0], qe_node=qb.qe_node[:0])
    g0, out0 = _srpe(built, none, 1_000_000)
    assert g0.nnz_in == 0 and g0.rows_in == 4 and out0.shape == (4, 16)
    np.testing.assert_allclose(out0, _exact(built, none), rtol=0, atol=1e-12)


def test_out_of_range_inputs_raise():
    built = small_workload("tiny", n_nodes=300, real_pe=False)
    ip, ix = built.graph.indptr, built.graph.indices
    with pytest.raises(ValueError):
        orc.build_computation_graph(ip, ix, 2, np.array([0, 2]), np.array([1, 1]), 0)
    with pytest.raises(ValueError):
        orc.build_computation_graph(ip, ix, 2, np.array([0, 1]), np.array([1, 300]), 0)


# ---- storage formats
def test_bf16_decode_and_rounding():
    bits = np.array([[0x3F80, 0xC000, 0x3FC0, 0x0000, 0x4049]], dtype=np.uint16)
    np.testing.assert_array_equal(orc.decode_table(bits, "bf16", 5)[0], [1.0, -2.0, 1.5, 0.0, 3.140625])
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.1], dtype=np.float32)
    got = orc.decode_table(to_bf16_bits(x)[None], "bf16", 4)[0]
    assert got[0] == 1.0                      # tie -> even mantissa
    assert got[1] == 1.0 + 2.0 ** -6          # tie -> even mantissa (up)
    assert got[2] == 1.0 + 2.0 ** -7          # above the tie -> up
    assert abs(got[3] + 0.1) <= 0.1 * 2.0 ** -8


# ---- other aggregation functions (Sec. 6.2): sum, max, power mean, normalised moments ----------------
# (moments of even order only in whole models: an odd central moment is exactly zero on every symmetric
# neighbourhood, e.g. any two neighbours, and the sign-keeping root has an unbounded derivative there, so
# rounding alone decides the result; the aggregation function itself is pinned for odd orders above)
AGG_MODELS = ["tiny_sum", "tiny_max", "tiny_power", "tiny_moment", "tiny_moment4"]


def _agg_params(kind, p=1.0, eps=1e-7):
    from types import SimpleNamespace
    return SimpleNamespace(aggregator=kind, agg_p=p, agg_eps=eps)


def test_aggregators_match_library_routines():
    import scipy.stats as st
    rng = np.random.default_rng(5)
    h = rng.normal(size=(9, 6))
    assert np.array_equal(orc.aggregate(_agg_params("max"), h), np.max(h, axis=0))
    np.testing.assert_allclose(orc.aggregate(_agg_params("sum"), h), 9 * np.mean(h, axis=0), rtol=1e-13)
    np.testing.assert_allclose(orc.aggregate(_agg_params("moment", 2), h), np.std(h, axis=0), rtol=1e-12)   # population
    m3 = st.moment(h, 3, axis=0)
    np.testing.assert_allclose(orc.aggregate(_agg_params("moment", 3), h), np.cbrt(m3), rtol=1e-12)          # keeps the sign
    assert (m3 < 0).any() and (m3 > 0).any()
    m4 = st.moment(h, 4, axis=0)
    np.testing.assert_allclose(orc.aggregate(_agg_params("moment", 4), h), m4 ** 0.25, rtol=1e-12)
    # power mean: p = 1 is the mean of the positive messages; p = -1 would be the harmonic mean (not used)
    pos = np.maximum(h, 0.0) + 1e-7
    np.testing.assert_allclose(orc.aggregate(_agg_params("power", 1.0), h), pos.mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(orc.aggregate(_agg_params("power", 2.0), h), np.sqrt((pos ** 2).mean(axis=0)), rtol=1e-13)
    # power mean inequality and its limit: M_1 <= M_2 <= M_8 <= max, and max * deg^(-1/p) <= M_p
    m1, m2, m8 = (orc.aggregate(_agg_params("power", q), h) for q in (1.0, 2.0, 8.0))
    assert np.all(m1 <= m2 + 1e-15) and np.all(m2 <= m8 + 1e-15) and np.all(m8 <= pos.max(axis=0) + 1e-15)
    assert np.all(pos.max(axis=0) * 9 ** (-1 / 8.0) <= m8 + 1e-15)
    # an empty neighbourhood gives zeros for every aggregator
    for kind in ("mean", "sum", "max", "power", "moment"):
        assert np.array_equal(orc.aggregate(_agg_params(kind, 2.0), np.zeros((0, 4))), np.zeros(4))


def test_local_aggregations_merge_to_the_global_one():
    """Sec. 6.2: per-partition aggregations and their merge functions give the aggregation of the whole
    neighbourhood: sums are added (then the root), maxima are maximised, the moment uses the global mean."""
    rng = np.random.default_rng(6)
    h = rng.normal(size=(11, 5))
    parts = [h[:4], h[4:5], h[5:]]
    assert np.array_equal(np.max([p.max(axis=0) for p in parts], axis=0), orc.aggregate(_agg_params("max"), h))
    pw = 3.0
    local = [((np.maximum(p, 0.0) + 1e-7) ** pw).sum(axis=0) for p in parts]
    np.testing.assert_allclose((np.sum(local, axis=0) / 11) ** (1 / pw), orc.aggregate(_agg_params("power", pw), h), rtol=1e-13)
    mean = np.sum([p.sum(axis=0) for p in parts], axis=0) / 11           # step 1: the mean, merged and broadcast
    local = [((p - mean) ** 3).sum(axis=0) for p in parts]              # step 2: as the power mean
    np.testing.assert_allclose(np.cbrt(np.sum(local, axis=0) / 11), orc.aggregate(_agg_params("moment", 3), h), rtol=1e-12)


@pytest.mark.parametrize("name", AGG_MODELS)
def test_full_budget_equals_exact_inference_other_aggregators(name):
    built = small_workload(name, n_nodes=600)
    qb = built.batch(0, n_query=12)
    _, out = _srpe(built, qb, 1_000_000)
    ref = _exact(built, qb)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-10)
    args = (built.graph.indptr, built.graph.indices, _x64(built), qb.feats[:, :built.cfg.dims[0]], qb.qe_query,
            qb.qe_node, built.layers)
    np.testing.assert_allclose(ex.exact_full_inference_sparse(*args), ref, rtol=0, atol=1e-10)


@pytest.mark.parametrize("name", ["tiny_max", "tiny_moment"])
def test_partial_budget_differs_and_isolated_query_sees_only_itself(name):
    built = small_workload(name, n_nodes=600)
    qb = built.batch(0, n_query=12)
    _, out = _srpe(built, qb, 100_000)
    assert np.abs(out - _exact(built, qb)).max() > 1e-6                  # an approximation, not a no-op
    # a query without edges: every aggregator returns zeros, the layer is act(W_self h + b)
    lone = orc.build_computation_graph(built.graph.indptr, built.graph.indices, 1, np.zeros(0, np.int32),
                                       np.zeros(0, np.int32), 100_000)
    got = orc.srpe_reference(lone, f64_tables(built), built.layers, qb.feats[:1])
    h = qb.feats[:1, :built.cfg.dims[0]].astype(np.float64)
    for p in built.layers:
        h = h @ p.W_self.astype(np.float64) + p.bias.astype(np.float64)
        if p.act == "relu":
            h = np.maximum(h, 0.0)
    np.testing.assert_allclose(got, h, rtol=0, atol=1e-12)


# ---- alternative recomputation policies (Sec. 5.2.2: RANDOM, IS; Sec. 5.1: the measured errors, AE) ----
def test_random_policy_is_seeded_unbiased_and_budgeted():
    g = power_law_graph(3000, 12, seed=21)
    qb = make_batch(g, 40, 8, seed=5, degree=("uniform", 10, 30), endpoints="uniform")
    a = orc.build_computation_graph(g.indptr, g.indices, 40, qb.qe_query, qb.qe_node, 250_000, policy="random", seed=3)
    b = orc.build_computation_graph(g.indptr, g.indices, 40, qb.qe_query, qb.qe_node, 250_000, policy="random", seed=3)
    c = orc.build_computation_graph(g.indptr, g.indices, 40, qb.qe_query, qb.qe_node, 250_000, policy="random", seed=4)
    assert np.array_equal(a.T, b.T) and not np.array_equal(a.T, c.T)
    assert a.T.size == (250_000 * a.R.size) // 1_000_000 and np.all(np.isin(a.T, a.R)) and np.all(np.diff(a.T) > 0)
    # brute force: sort the candidates by their key
    keys = np.array([orc.random_policy_key(3, int(u)) for u in a.R], dtype=np.uint64)
    order = np.lexsort((a.R, -keys.astype(np.float64)))           # 39-bit keys are exact in fp64
    assert np.array_equal(np.sort(a.R[order[:a.T.size]]), a.T)
    # over many seeds every candidate is chosen about a quarter of the time, whatever its degree
    hits = np.zeros(a.R.size)
    for seed in range(200):
        T = orc.select_targets_alt(a.R, 250_000, "random", seed)
        hits += np.isin(a.R, T)
    assert abs(hits.mean() / 200 - 0.25) < 0.01 and hits.min() > 20 and hits.max() < 85
    # the generator itself: a value computed by hand from the published splitmix64 constants
    z = (7 + 3 * 0x9E3779B97F4A7C15) % 2 ** 64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % 2 ** 64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % 2 ** 64
    assert orc.random_policy_key(3, 7) == (z ^ (z >> 31)) >> 25


def test_score_policy_takes_the_largest_scores_and_breaks_ties_by_id():
    R = np.array([2, 5, 7, 11, 13, 17, 19, 23], dtype=np.int64)
    scores = np.zeros(30, dtype=np.float32)
    scores[R] = [0.5, 0.25, 0.5, -1.0, 0.0, 0.5, -0.0, 3.0]
    T = orc.select_targets_alt(R, 500_000, "score", node_scores=scores)       # 4 of 8
    assert T.tolist() == [2, 7, 17, 23]                                       # 3.0, then the three 0.5 (all of them fit)
    T = orc.select_targets_alt(R, 375_000, "score", node_scores=scores)       # 3 of 8: 3.0, then 0.5 at the two smallest ids
    assert T.tolist() == [2, 7, 23]
    T = orc.select_targets_alt(R, 875_000, "score", node_scores=scores)       # 7 of 8: -0.0 ties with 0.0, smaller id first
    assert T.tolist() == [2, 5, 7, 13, 17, 19, 23]
    with pytest.raises(ValueError):
        orc.select_targets_alt(R, 500_000, "score", node_scores=np.full(30, np.nan, np.float32))


def test_importance_scores_closed_forms():
    # ring of n nodes (2-regular): IS = 1/2 * (1/2 + 1/2) = 1/2
    n = 12
    indptr = np.arange(0, 2 * n + 1, 2, dtype=np.int64)
    indices = np.array([[(v - 1) % n, (v + 1) % n] for v in range(n)], dtype=np.int32).reshape(-1)
    np.testing.assert_allclose(orc.importance_scores(indptr, indices), 0.5, rtol=1e-15)
    # star with m leaves: centre = (1/m) * m * 1 = 1, leaf = 1/m
    m = 7
    indptr = np.concatenate([[0, m], m + np.arange(1, m + 1)]).astype(np.int64)
    indices = np.concatenate([np.arange(1, m + 1), np.zeros(m)]).astype(np.int32)
    isc = orc.importance_scores(indptr, indices)
    np.testing.assert_allclose(isc, [1.0] + [1.0 / m] * m, rtol=1e-15)
    # against the matrix form D^-1 A D^-1 1 on a random graph
    g = power_law_graph(500, 8, seed=4)
    A = sp.csr_matrix((np.ones(g.nnz), g.indices, g.indptr), shape=(g.n, g.n))
    d = np.asarray(A.sum(axis=1)).ravel()
    inv = np.where(d > 0, 1 / np.maximum(d, 1), 0)
    np.testing.assert_allclose(orc.importance_scores(g.indptr, g.indices), inv * (A @ inv), rtol=1e-12)


def test_measured_errors_vanish_where_the_batch_does_not_reach_and_rank_the_ratio_policy_high():
    """AE of Sec. 5.1 on a small workload: zero for a table that IS the full embedding; with the real tables,
    recomputing the top-error candidates restores more of the exact output than recomputing random ones, and
    the ratio policy sits in between or better (the paper's Fig. 6 ordering, here on one synthetic batch)."""
    built = small_workload("tiny", n_nodes=600)
    qb = built.batch(0, n_query=12)
    tabs = f64_tables(built)
    full = ex.exact_layer_embeddings(built.graph.indptr, built.graph.indices, _x64(built),
                                     qb.feats[:, :built.cfg.dims[0]], qb.qe_query, qb.qe_node, built.layers)
    g0 = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, 0)
    ae = orc.approximation_errors(full, tabs, g0.R)
    assert ae.shape == g0.R.shape and np.all(ae > 0)                      # every candidate has a query edge: its embedding moved
    same = [tabs[0]] + [orc.LazyTable(full[l][:built.graph.n], "f64", full[l].shape[1]) for l in range(1, len(built.layers))]
    assert np.all(orc.approximation_errors(full, same, g0.R) == 0)
    exact = _exact(built, qb)
    scores = np.zeros(built.graph.n, dtype=np.float32)
    scores[g0.R] = ae.astype(np.float32)

    def loss(**kw):
        g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node,
                                        200_000, **kw)
        return np.abs(orc.srpe_reference(g, tabs, built.layers, qb.feats) - exact).mean()

    l_ae = loss(policy="score", node_scores=scores)
    l_ratio = loss()
    l_rand = np.mean([loss(policy="random", seed=s) for s in range(8)])
    l_none = np.abs(orc.srpe_reference(g0, tabs, built.layers, qb.feats) - exact).mean()
    assert l_ae < l_rand < l_none and l_ratio < l_rand


# ---- the deep convolution of the paper's appendix on depth (GCNII: initial residual + identity mapping) ----
def test_gcnii_row_reduces_to_gcn_and_to_the_initial_value():
    rng = np.random.default_rng(8)
    d = 6
    W = rng.normal(size=(d, d)).astype(np.float32)
    b = rng.normal(size=d).astype(np.float32)
    h_self, h0 = rng.normal(size=d), rng.normal(size=d)
    h_src, deg_src = rng.normal(size=(5, d)), rng.integers(1, 9, size=5)
    from synth.tables import LayerParams
    gcn = LayerParams("gcn", d, d, "relu", W_nb=W, bias=b)
    # alpha = 0: the pinned GCN layer with the same matrix
    np.testing.assert_allclose(orc.layer_row(LayerParams("gcnii", d, d, "relu", W_nb=W, bias=b, alpha=0.0), h_self, h_src, deg_src, h0),
                               orc.layer_row(gcn, h_self, h_src, deg_src), rtol=1e-14)
    # alpha = 1: only the row's own layer-0 value is left
    np.testing.assert_allclose(orc.layer_row(LayerParams("gcnii", d, d, "none", W_nb=W, bias=b, alpha=1.0), h_self, h_src, deg_src, h0),
                               h0 @ W.astype(np.float64) + b, rtol=1e-14)
    # in between: linear in alpha before the activation
    lo = orc.layer_row(LayerParams("gcnii", d, d, "none", W_nb=W, bias=b, alpha=0.0), h_self, h_src, deg_src, h0)
    hi = orc.layer_row(LayerParams("gcnii", d, d, "none", W_nb=W, bias=b, alpha=1.0), h_self, h_src, deg_src, h0)
    mid = orc.layer_row(LayerParams("gcnii", d, d, "none", W_nb=W, bias=b, alpha=0.3), h_self, h_src, deg_src, h0)
    np.testing.assert_allclose(mid, 0.7 * lo + 0.3 * hi, rtol=1e-13)


def test_gcnii_generator_holds_the_identity_mapped_weight():
    layers = make_layers("gcnii", [16] * 4, seed=9)
    first_raw = make_layers("gcn", [16, 16], seed=9)[0].W_nb.astype(np.float64)      # the same first draw
    lim = np.sqrt(6.0 / 32.0)                                                        # Glorot bound of the raw matrix
    for l, p in enumerate(layers, start=1):
        beta = np.log(0.5 / l + 1.0)
        raw = (p.W_nb.astype(np.float64) - (1 - beta) * np.eye(16)) / beta            # undo the identity mapping
        assert np.abs(raw).max() <= lim * (1 + 1e-5) and raw.std() > 0.5 * lim       # uniform on [-lim, lim]: std = 0.577 lim
        if l == 1:
            np.testing.assert_allclose(raw, first_raw, rtol=0, atol=1e-6)
        assert p.alpha == 0.1 and p.act == "relu" and np.all(p.bias == 0)


def test_gcnii_full_budget_exact_for_two_layers_and_sparse_equals_dense():
    built = small_workload("tiny_gcnii", n_nodes=600)
    qb = built.batch(0, n_query=12)
    _, out = _srpe(built, qb, 1_000_000)
    ref = _exact(built, qb)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-11)
    deep = small_workload("tiny_gcnii6", n_nodes=500)
    qd = deep.batch(1, n_query=10)
    args = (deep.graph.indptr, deep.graph.indices, _x64(deep), qd.feats[:, :64], qd.qe_query, qd.qe_node, deep.layers)
    exact6 = ex.exact_full_inference(*args)
    np.testing.assert_allclose(ex.exact_full_inference_sparse(*args), exact6, rtol=0, atol=1e-11)
    # six layers: an approximation at every budget (degrees leak one hop per layer, as for GCN), better with more budget
    tabs = f64_tables(deep)
    err = []
    for gamma in (0, 300_000, 1_000_000):
        g = orc.build_computation_graph(deep.graph.indptr, deep.graph.indices, qd.n_query, qd.qe_query, qd.qe_node, gamma)
        err.append(np.abs(orc.srpe_reference(g, tabs, deep.layers, qd.feats) - exact6).mean())
    assert err[0] > err[1] > err[2] > 0


# ---- computation graph parallelism (Sec. 6): local aggregations + merge functions
from oracle import cgp_oracle as cgp
from synth import block_partition, hash_partition

CGP_MODELS = ["tiny", "tiny_gcn", "tiny_gat", "tiny_gat8", "tiny_sage3", "tiny_sum", "tiny_max", "tiny_power", "tiny_moment",
              "tiny_moment4", "tiny_gcnii"]


@pytest.mark.parametrize("name", CGP_MODELS)
def test_cgp_merged_layers_equal_the_unpartitioned_model(name):
    """Eq. 3: for every model and aggregation the merge of the local aggregations is the aggregation over
    the whole neighbourhood, so the partitioned execution returns what the unpartitioned one returns (which
    the pins above tie to exact inference).  Checked for 1, 2, 3 and 8 partitions, hash and block placement."""
    built = small_workload(name, n_nodes=500)
    qb = built.batch(0, n_query=11)
    g, ref = _srpe(built, qb, 300_000)
    tabs = f64_tables(built)
    scale = np.abs(ref).max()
    for n_part, node_part in ((1, hash_partition(built.graph.n, 1)), (2, hash_partition(built.graph.n, 2)),
                              (3, block_partition(built.graph.n, 3)), (8, hash_partition(built.graph.n, 8, seed=5))):
        got = cgp.cgp_reference(g, node_part, n_part, tabs, built.layers, qb.feats)
        assert got.shape == ref.shape
        assert np.abs(got - ref).max() <= 1e-10 * max(scale, 1.0), (name, n_part)


def test_cgp_partitioned_graphs_split_every_row_by_source_partition():
    """Sec. 6.1: every edge goes to exactly one partition, that of its source; rows keep their order; a query
    source lives in partition q mod P, a recomputed target in its node's partition."""
    built = small_workload("tiny", n_nodes=500)
    qb = built.batch(1, n_query=9)
    g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, 400_000)
    P = 4
    node_part = hash_partition(built.graph.n, P, seed=3)
    parts = [cgp.partition_graph(g, node_part, P, p) for p in range(P)]
    assert sum(int(pg.indptr[-1]) for pg in parts) == g.nnz_in
    saw_query_source = saw_target_source = False
    for v in range(g.rows_in):
        full = list(zip(g.cols[g.indptr[v]:g.indptr[v + 1]].tolist(), g.cdeg[g.indptr[v]:g.indptr[v + 1]].tolist()))
        pieces = []
        for p, pg in enumerate(parts):
            mine = list(zip(pg.cols[pg.indptr[v]:pg.indptr[v + 1]].tolist(), pg.cdeg[pg.indptr[v]:pg.indptr[v + 1]].tolist()))
            # a subsequence of the whole row
            it = iter(full)
            assert all(any(x == y for y in it) for x in mine)
            for c, _ in mine:
                if c >= 0:
                    assert node_part[c] == p
                elif ~c < g.n_query:
                    assert (~c) % P == p
                    saw_query_source = True
                else:
                    assert node_part[g.T[~c - g.n_query]] == p
                    saw_target_source = True
            pieces += mine
        assert sorted(pieces) == sorted(full)
    assert saw_query_source and saw_target_source


def _gat_params(H, dh, d_in, W, a_src, a_dst):
    from synth.tables import LayerParams
    return LayerParams(model="gat", d_in=d_in, d_out=H * dh, heads=H, act="none", head_mean=False, leaky_slope=0.2,
                       W_self=None, W_nb=W, a_src=a_src, a_dst=a_dst, bias=np.zeros(H * dh))


def test_cgp_softmax_merge_closed_form_and_huge_scores():
    """Sec. 6.2, softmax-based aggregation: with scores 0, ln 2 in one partition and ln 3 in another the
    attention weights are 1/6, 2/6, 3/6; the record of a partition holds its own maximum and the sum of
    exponentials relative to it; scores of +-10^4 neither overflow nor lose the small partition."""
    W = np.eye(2)
    a_src = np.array([[1.0, 0.0]])            # score = first coordinate of the source (destination part is 0)
    layer = _gat_params(1, 2, 2, W, a_src, np.zeros((1, 2)))
    hA = np.array([[0.0, 1.0], [np.log(2.0), 10.0]])
    hB = np.array([[np.log(3.0), 100.0]])
    h_dst = np.zeros(2)
    rA = cgp.local_aggregation(layer, hA, np.zeros(2), h_dst)
    rB = cgp.local_aggregation(layer, hB, np.zeros(1), h_dst)
    rE = cgp.local_aggregation(layer, np.zeros((0, 2)), np.zeros(0), h_dst)
    assert rA["max"][0] == np.log(2.0) and abs(rA["expsum"][0] - 1.5) < 1e-15      # exp(0 - ln 2) + 1
    assert rB["max"][0] == np.log(3.0) and rB["expsum"][0] == 1.0
    assert rE["max"][0] == -np.inf and rE["expsum"][0] == 0.0
    out = cgp.merge(layer, [rA, rE, rB])
    want = (1 * hA[0] + 2 * hA[1] + 3 * hB[0]) / 6.0
    np.testing.assert_allclose(out[0], want, rtol=1e-14)
    # the same through the unpartitioned row
    np.testing.assert_allclose(orc.layer_row(layer, h_dst, np.vstack([hA, hB]), np.zeros(3)), want, rtol=1e-14)
    # huge scores: partition A dominates by e^20000, partition B must vanish without a NaN
    hA2 = np.array([[1e4, 1.0], [1e4, 3.0]])
    hB2 = np.array([[-1e4, 50.0]])
    out2 = cgp.merge(layer, [cgp.local_aggregation(layer, hA2, np.zeros(2), h_dst),
                             cgp.local_aggregation(layer, hB2, np.zeros(1), h_dst)])
    np.testing.assert_allclose(out2[0], [1e4, 2.0], rtol=1e-14)
    # a destination with no neighbour anywhere
    assert np.array_equal(cgp.merge(layer, [rE, rE]), np.zeros((1, 2)))


def test_cgp_gcn_factors_and_counts_by_hand():
    """GCN under CGP: sources carry 1 / sqrt(d_u + 1) locally, the merge knows d_v from the message counts and
    applies 1 / sqrt(d_v + 1); the update adds the self term h_v / (d_v + 1)."""
    from synth.tables import LayerParams
    layer = LayerParams(model="gcn", d_in=1, d_out=1, heads=1, act="none", head_mean=False, leaky_slope=0.2,
                        W_self=None, W_nb=np.array([[1.0]]), a_src=None, a_dst=None, bias=np.zeros(1))
    # destination value 8 with three neighbours: 4 (degree 3) in partition 0; 9 (degree 8) and 2 (degree 0) in partition 1
    r0 = cgp.local_aggregation(layer, np.array([[4.0]]), np.array([3]), np.array([8.0]))
    r1 = cgp.local_aggregation(layer, np.array([[9.0], [2.0]]), np.array([8, 0]), np.array([8.0]))
    assert r0["sum"][0] == 2.0 and r1["sum"][0] == 5.0 and r0["count"] == 1 and r1["count"] == 2
    merged = cgp.merge(layer, [r0, r1])
    assert merged[0] == 7.0 / 2.0                                  # d_v + 1 = 4
    assert cgp.update(layer, np.array([8.0]), merged, 3.0)[0] == 2.0 + 3.5


def test_cgp_partition_graph_is_the_masked_whole_graph():
    """The row-by-row construction equals its one-line definition: the whole graph's edge list filtered by
    source partition (rows are contiguous and keep their order), with row lengths counted per row."""
    built = small_workload("tiny_gcn", n_nodes=500)
    qb = built.batch(2, n_query=10)
    g = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, 500_000)
    P = 3
    node_part = block_partition(built.graph.n, P)
    sp = cgp.source_partitions(g, node_part, P)
    row_of_edge = np.repeat(np.arange(g.rows_in), np.diff(g.indptr))
    for p in range(P):
        pg = cgp.partition_graph(g, node_part, P, p)
        mine = sp == p
        assert np.array_equal(pg.cols, g.cols[mine]) and np.array_equal(pg.cdeg, g.cdeg[mine])
        assert np.array_equal(np.diff(pg.indptr), np.bincount(row_of_edge[mine], minlength=g.rows_in))
