"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Graph construction must match bit for bit; layer outputs within
max-over-rows ||g - r||_inf / ||r||_inf <= 1e-4 (fp32 tables) or 2e-2 (bf16 tables)."""
from __future__ import annotations

from dataclasses import replace

import numpy as np
import pytest

from oracle import exact_inference as ex
from oracle import srpe_oracle as orc
from tests.helpers import lazy_tables, row_rel_err, small_workload

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = {"f32": 1e-4, "bf16": 2e-2}
_cache = {}


def _model(name):
    """(built workload, device model), one per workload name for the whole session."""
    from paper_2501_08547_amd import device
    if name not in _cache:
        built = small_workload(name)
        _cache[name] = (built, device.upload(built))
    return _cache[name]


def _oracle_graph(built, qb, gamma_ppm, recompute_set=None):
    return orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query,
                                       qb.qe_node, gamma_ppm, recompute_set)


def _assert_same_graph(exp, og):
    assert np.array_equal(exp["cand"], og.R.astype(np.int32))
    assert np.array_equal(exp["qdeg"], og.qdeg.astype(np.int32))
    assert np.array_equal(exp["targets"], og.T.astype(np.int32))
    assert np.array_equal(exp["indptr"], og.indptr)
    assert np.array_equal(exp["cols"], og.cols)
    assert np.array_equal(exp["cdeg"], og.cdeg)


def _tol(built):
    return TOL["bf16"] if any(t.dtype == "bf16" for t in built.tables) else TOL["f32"]


GRAPH_CASES = [("tiny", 0), ("tiny", 100_000), ("tiny", 1_000_000), ("tiny_gcn", 333_333),
               ("mid_s", 50_000), ("mid_s", 1_000_000), ("large_s", 50_000), ("large_s", 200_000)]


@pytest.mark.parametrize("name,gamma_ppm", GRAPH_CASES)
def test_graph_construction_bit_exact(name, gamma_ppm):
    built, dm = _model(name)
    for r in range(2):
        qb = built.batch(r)
        print(f"case {name} gamma={gamma_ppm} batch={r} E_q={qb.n_edges}", flush=True)
        g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma_ppm)
        og = _oracle_graph(built, qb, gamma_ppm)
        s = g.sizes()
        assert (s["n_cand"], s["n_target"], s["rows_in"], s["nnz_in"]) == (og.R.size, og.T.size, og.rows_in, og.nnz_in)
        _assert_same_graph(g.export(), og)
        g.destroy()


@pytest.mark.parametrize("name,gamma_ppm", [("tiny", 300_000), ("mid_s", 1_000_000), ("large_s", 200_000)])
def test_graph_construction_with_prefix_totals_scanned_by_a_block_of_their_own(name, gamma_ppm):
    """The route the builder takes when there are more chunk / block totals than a consumer adds up by itself,
    forced on small requests by a limit of one total; then the default route again on the same context."""
    built, dm = _model(name)
    qb = built.batch(5)
    og = _oracle_graph(built, qb, gamma_ppm)
    R, _ = orc.candidates(qb.qe_node)
    chosen = R[::4].astype(np.int32)
    og_set = _oracle_graph(built, qb, 0, recompute_set=chosen)
    try:
        for limit in (1, 3, 4096):
            dm.ctx.debug_set_fused_sum_limit(limit)
            g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma_ppm)
            _assert_same_graph(g.export(), og)
            g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 0, recompute_set=chosen, graph=g)
            _assert_same_graph(g.export(), og_set)
            g.destroy()
    finally:
        dm.ctx.debug_set_fused_sum_limit(4096)


def test_small_requests_built_by_one_block_equal_the_general_route_and_the_oracle():
    """Requests of up to 2,048 edges and queries are built by one block (sorts in LDS); the same requests down the
    general route (counters, bitmap, per-row sorts) and through the oracle must give the same graph bit for bit:
    one edge, full size (2,048 edges on 2,048 queries, every candidate recomputed: 4,096 rows), duplicate edges,
    queries without edges, a hub that many queries attach to, every policy."""
    built, dm = _model("mid_s")
    n = built.graph.n
    rng = np.random.default_rng(41)
    cases = []
    for n_query, n_e, gamma in ((1, 1, 1_000_000), (1, 37, 50_000), (7, 64, 300_000), (64, 129, 500_000),
                                (300, 1000, 100_000), (2048, 2048, 1_000_000), (2048, 2048, 0), (5, 2048, 250_000),
                                (2000, 2047, 999_999)):
        q = rng.integers(0, n_query, size=n_e).astype(np.int32)
        u = rng.integers(0, n, size=n_e).astype(np.int32)
        if n_e >= 64:                                   # duplicate edges, and a hub with many queries attached
            q[:8], u[:8] = q[8:16], u[8:16]
            u[16:16 + n_e // 4] = u[16]
        if n_query >= 7:
            q[q == 3] = 4                               # query 3 has no edges
        cases.append((n_query, q, u, gamma))
    g = None
    try:
        for n_query, q, u, gamma in cases:
            print(f"  case B={n_query} E_q={q.size} gamma={gamma}", flush=True)
            og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, n_query, q, u, gamma)
            for small in (1, 2, 0):                     # one block / one block, then the general second half / general
                dm.ctx.debug_set_small_path(small)
                g = dm.ctx.build_computation_graph(n_query, q, u, gamma, graph=g)
                s = g.sizes()
                assert (s["n_cand"], s["n_target"], s["rows_in"], s["nnz_in"]) == (og.R.size, og.T.size, og.rows_in, og.nnz_in)
                _assert_same_graph(g.export(), og)
        # the other policies share the route
        n_query, q, u, gamma = cases[4]
        scores = np.random.default_rng(3).standard_normal(n).astype(np.float32)
        sc_dev = torch.from_numpy(scores).cuda()
        for policy, kw, okw in (("random", dict(seed=99), dict(policy="random", seed=99)),
                                ("score", dict(node_scores=sc_dev), dict(policy="score", node_scores=scores))):
            og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, n_query, q, u, gamma, **okw)
            for small in (True, False):
                dm.ctx.debug_set_small_path(small)
                dm.ctx.set_policy(policy, **kw)
                g = dm.ctx.build_computation_graph(n_query, q, u, gamma, graph=g)
                _assert_same_graph(g.export(), og)
        # a bad index is rejected by the one-block route too, and the context works afterwards
        from paper_2501_08547_amd import binding as B
        dm.ctx.set_policy("ratio")
        dm.ctx.debug_set_small_path(True)
        for bq, bu in ((np.array([0, 5], np.int32), np.array([1, 2], np.int32)), (np.array([0, 1], np.int32), np.array([1, n], np.int32))):
            with pytest.raises(B.OmegaError) as ei:
                dm.ctx.build_computation_graph(2, bq, bu, 500_000)
            assert ei.value.code == B.OMG_ERANGE
        n_query, q, u, gamma = cases[3]
        g = dm.ctx.build_computation_graph(n_query, q, u, gamma, graph=g)
        _assert_same_graph(g.export(), orc.build_computation_graph(built.graph.indptr, built.graph.indices, n_query, q, u, gamma))
    finally:
        dm.ctx.set_policy("ratio")
        dm.ctx.debug_set_small_path(True)
        if g is not None:
            g.destroy()


def test_graph_device_inputs_rebuild_in_place_and_explicit_set():
    built, dm = _model("tiny")
    g = None
    for r, nq in ((0, 32), (1, 7), (2, 32)):                       # larger, smaller, larger again, same object
        qb = built.batch(r, n_query=nq)
        q_dev = torch.from_numpy(qb.qe_query).cuda()
        u_dev = torch.from_numpy(qb.qe_node).cuda()
        g = dm.ctx.build_computation_graph(qb.n_query, q_dev, u_dev, 250_000, graph=g)
        _assert_same_graph(g.export(), _oracle_graph(built, qb, 250_000))
    qb = built.batch(3)
    R, _ = orc.candidates(qb.qe_node)
    chosen = R[1::3].astype(np.int32)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 0, recompute_set=chosen, graph=g)
    _assert_same_graph(g.export(), _oracle_graph(built, qb, 0, recompute_set=chosen))
    g.destroy()


def test_graph_ties_duplicates_and_degenerate_requests():
    built, dm = _model("tiny")
    qb = built.batch(4)
    # duplicate edges count with multiplicity
    dq = np.concatenate([qb.qe_query, qb.qe_query[:9]])
    du = np.concatenate([qb.qe_node, qb.qe_node[:9]])
    g = dm.ctx.build_computation_graph(qb.n_query, dq, du, 400_000)
    _assert_same_graph(g.export(), _oracle_graph(built, replace(qb, qe_query=dq, qe_node=du), 400_000))
    # many exact ties: every query attached to nodes of few distinct degrees
    deg = np.diff(built.graph.indptr)
    pool = np.flatnonzero((deg >= 2) & (deg <= 4))[:200].astype(np.int32)
    rng = np.random.default_rng(5)
    tq = np.repeat(np.arange(16, dtype=np.int32), 12)
    tu = np.concatenate([rng.choice(pool, 12, replace=False) for _ in range(16)]).astype(np.int32)
    for gamma in (100_000, 500_000, 900_000):
        g = dm.ctx.build_computation_graph(16, tq, tu, gamma, graph=g)
        _assert_same_graph(g.export(), _oracle_graph(built, replace(qb, n_query=16, qe_query=tq, qe_node=tu), gamma))
    # isolated nodes (base degree 0) rank first; no edges at all; a single edge
    iso = np.flatnonzero(deg == 0)[:3].astype(np.int32)
    if iso.size:
        iq = np.arange(iso.size + 2, dtype=np.int32) % 2
        iu = np.concatenate([iso, pool[:2]])
        g = dm.ctx.build_computation_graph(2, iq, iu, 600_000, graph=g)
        og = _oracle_graph(built, replace(qb, n_query=2, qe_query=iq, qe_node=iu), 600_000)
        assert set(iso.tolist()) <= set(og.T.tolist())
        _assert_same_graph(g.export(), og)
    e = np.empty(0, np.int32)
    g = dm.ctx.build_computation_graph(5, e, e, 1_000_000, graph=g)
    assert g.sizes() == dict(n_cand=0, n_target=0, rows_in=5, nnz_in=0)
    assert np.array_equal(g.export()["indptr"], np.zeros(6, np.int64))
    one_q, one_u = np.array([3], np.int32), np.array([17], np.int32)
    g = dm.ctx.build_computation_graph(5, one_q, one_u, 1_000_000, graph=g)
    _assert_same_graph(g.export(), _oracle_graph(built, replace(qb, n_query=5, qe_query=one_q, qe_node=one_u), 1_000_000))
    g.destroy()


def test_graph_long_rows_and_popular_targets():
    """Rows of every sorting class: a query with 5,000 edges and one with 300; nodes that 3,000 /
    150 / 40 queries attach to, all recomputed."""
    built, dm = _model("mid_s")
    n = built.graph.n
    rng = np.random.default_rng(23)
    B = 3_000
    hubs = rng.choice(n, size=3, replace=False).astype(np.int32)
    q_list = [np.arange(B, dtype=np.int32), rng.choice(B, 150, replace=False).astype(np.int32),
              rng.choice(B, 40, replace=False).astype(np.int32)]
    u_list = [np.full(B, hubs[0], np.int32), np.full(150, hubs[1], np.int32), np.full(40, hubs[2], np.int32)]
    rest = np.setdiff1d(np.arange(n, dtype=np.int32), hubs)
    q_list += [np.full(5_000, 7, np.int32), np.full(300, 11, np.int32)]
    u_list += [rng.choice(rest, 5_000, replace=False).astype(np.int32), rng.choice(rest, 300, replace=False).astype(np.int32)]
    qq, uu = np.concatenate(q_list), np.concatenate(u_list)
    perm = rng.permutation(qq.size)
    qq, uu = qq[perm], uu[perm]
    for kw in (dict(gamma_ppm=300_000), dict(gamma_ppm=0, recompute_set=np.sort(hubs))):
        g = dm.ctx.build_computation_graph(B, qq, uu, kw["gamma_ppm"], recompute_set=kw.get("recompute_set"))
        og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, B, qq, uu, kw["gamma_ppm"],
                                         kw.get("recompute_set"))
        if "recompute_set" in kw:
            assert og.T.tolist() == np.sort(hubs).tolist()
        _assert_same_graph(g.export(), og)
        g.destroy()


def test_graph_rows_longer_than_the_sorts_hold_in_registers():
    """One query with 120,000 edges (a row whose sixteen top-bit pieces are themselves beyond 4,096 keys, so both
    block sorts reload their keys on every pass) and one node that 20,000 queries attach to, recomputed."""
    from paper_2501_08547_amd import device
    from synth import CONFIGS, build_workload
    built = build_workload(replace(CONFIGS["tiny"], name="longrows", n_nodes=150_000, avg_deg=4.0, dims=(4, 4, 2)))
    dm = device.upload(built)
    n = built.graph.n
    rng = np.random.default_rng(77)
    B = 20_000
    hub = np.int32(rng.integers(0, n))
    rest = np.setdiff1d(np.arange(n, dtype=np.int32), [hub])
    q_list = [np.arange(B, dtype=np.int32), np.full(120_000, 5, np.int32)]
    u_list = [np.full(B, hub, np.int32), rng.choice(rest, 120_000, replace=False).astype(np.int32)]
    qq, uu = np.concatenate(q_list), np.concatenate(u_list)
    perm = rng.permutation(qq.size)
    qq, uu = qq[perm], uu[perm]
    for kw in (dict(gamma_ppm=0, recompute_set=np.array([hub], np.int32)), dict(gamma_ppm=20_000)):
        print(f"case long rows {kw}", flush=True)
        g = dm.ctx.build_computation_graph(B, qq, uu, kw["gamma_ppm"], recompute_set=kw.get("recompute_set"))
        og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, B, qq, uu, kw["gamma_ppm"],
                                         kw.get("recompute_set"))
        lens = np.diff(og.indptr)
        assert lens.max() >= 120_000 and (lens[B:] >= B).any() if "recompute_set" in kw else lens.max() >= 120_000
        _assert_same_graph(g.export(), og)
        g.destroy()


def test_bad_requests_are_rejected():
    from paper_2501_08547_amd import binding as B
    built, dm = _model("tiny")
    n = built.graph.n
    ok_q, ok_u = np.array([0, 1], np.int32), np.array([5, 6], np.int32)
    for q, u in ((np.array([0, 2], np.int32), ok_u), (ok_q, np.array([5, n], np.int32)),
                 (ok_q, np.array([-1, 6], np.int32))):
        with pytest.raises(B.OmegaError) as ei:
            dm.ctx.build_computation_graph(2, q, u, 0)
        assert ei.value.code == B.OMG_ERANGE
    with pytest.raises(B.OmegaError) as ei:
        dm.ctx.build_computation_graph(2, ok_q, ok_u, 1_000_001)
    assert ei.value.code == B.OMG_EINVAL
    with pytest.raises(B.OmegaError) as ei:                        # recompute set outside the candidates
        dm.ctx.build_computation_graph(2, ok_q, ok_u, 0, recompute_set=np.array([7], np.int32))
    assert ei.value.code == B.OMG_ERANGE
    # the context still works afterwards
    qb = built.batch(0)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 100_000)
    _assert_same_graph(g.export(), _oracle_graph(built, qb, 100_000))
    g.destroy()


def test_a_failed_allocation_leaves_the_context_usable():
    """Every growing allocation of a graph construction is made to fail in turn (fault injection inside the
    library); the call must report OMG_ENOMEM and the next construction on the same context must still be
    bit-exact: a build that stops after the candidates were emitted has to return the node-to-slot map to its
    idle state."""
    from paper_2501_08547_amd import binding as B
    from paper_2501_08547_amd import device
    built, dm = _model("tiny")
    L = B.lib()
    qa, qb = built.batch(0), built.batch(1)
    oa, ob = _oracle_graph(built, qa, 300_000), _oracle_graph(built, qb, 300_000)
    failed = 0
    for nth in range(200):
        # a fresh context and a fresh graph object each time: every buffer of the build still has to grow
        ctx = B.Context(dm.indptr, dm.indices, torch.cuda.current_stream().cuda_stream)
        g = None
        L.omg_debug_fail_allocation(nth)
        try:
            g = ctx.build_computation_graph(qa.n_query, qa.qe_query, qa.qe_node, 300_000)
        except B.OmegaError as e:
            assert e.code == B.OMG_ENOMEM
            failed += 1
        finally:
            L.omg_debug_fail_allocation(-1)
        if g is not None:
            _assert_same_graph(g.export(), oa)
            g.destroy()
        g2 = ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 300_000)
        _assert_same_graph(g2.export(), ob)
        g2.destroy()
        ctx.close()
        if g is not None:
            break                                               # nth is beyond the last allocation of a build
    print(f"  {failed} allocations failed in turn", flush=True)
    assert failed >= 30 and g is not None
    # the whole path afterwards
    feats = torch.from_numpy(qa.feats).cuda()
    out = torch.empty((qa.n_query, dm.out_width()), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qa.n_query, qa.qe_query, qa.qe_node, 300_000, out)
    torch.cuda.synchronize()
    ref = orc.srpe_reference(oa, lazy_tables(built), built.layers, qa.feats)
    assert row_rel_err(out.cpu().numpy(), ref) <= 1e-4
    # a budget beyond 100 % is an argument error, reported before anything is sized from it
    with pytest.raises(B.OmegaError) as ei:
        dm.ctx.serve_batch(dm.tables, dm.layers, feats, qa.n_query, qa.qe_query, qa.qe_node, 4_000_000_000, out)
    assert ei.value.code == B.OMG_EINVAL


SERVE_CASES = [("tiny", 100_000), ("tiny", 0), ("tiny", 1_000_000), ("tiny_gcn", 100_000), ("tiny_gcn", 1_000_000),
               ("tiny_sage3", 300_000), ("tiny_gat", 100_000), ("tiny_gat", 1_000_000), ("tiny_gat8", 100_000),
               ("mid_s", 50_000), ("mid_s", 1_000_000),
               ("large_s", 0), ("large_s", 50_000), ("large_s", 200_000), ("large_s", 1_000_000),
               ("attention_s", 100_000), ("attention_s", 1_000_000),
               # the other aggregation functions of SAGE-type layers
               ("tiny_sum", 100_000), ("tiny_max", 100_000), ("tiny_max", 0), ("tiny_power", 100_000),
               ("tiny_moment", 100_000), ("tiny_moment4", 300_000), ("tiny_moment4", 1_000_000),
               ("large_s_max", 50_000), ("large_s_power", 50_000), ("large_s_moment", 50_000),
               ("large_s_moment", 1_000_000),
               # the deep convolution with initial residual, 2 / 6 / 4 layers
               ("tiny_gcnii", 100_000), ("tiny_gcnii", 1_000_000), ("tiny_gcnii6", 300_000), ("tiny_gcnii6", 0),
               ("mid_s_gcnii", 50_000), ("mid_s_gcnii", 1_000_000)]


@pytest.mark.parametrize("name,gamma_ppm", SERVE_CASES)
def test_serve_batch_matches_oracle(name, gamma_ppm):
    built, dm = _model(name)
    qb = built.batch(0)
    print(f"case {name} gamma={gamma_ppm} B={qb.n_query} E_q={qb.n_edges}", flush=True)
    feats = torch.from_numpy(qb.feats).cuda()
    out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, gamma_ppm, out)
    torch.cuda.synchronize()
    og = _oracle_graph(built, qb, gamma_ppm)
    ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    err = row_rel_err(got, ref)
    print(f"  rows_in={og.rows_in} nnz_in={og.nnz_in} max row rel err={err:.3e}", flush=True)
    assert err <= _tol(built)
    s = dm.ctx.last_graph_sizes()
    assert (s["n_target"], s["nnz_in"]) == (og.T.size, og.nnz_in)


@pytest.mark.parametrize("name", ["tiny", "tiny_gcn", "tiny_gat", "tiny_gat8", "tiny_sage3", "mid_s", "large_s", "attention_s",
                                  "tiny_max", "tiny_power", "tiny_moment4", "large_s_max", "large_s_moment", "tiny_gcnii"])
def test_full_budget_equals_exact_full_inference(name):
    """Recompute fraction 100 %: the library's output against exact inference on the whole graph plus
    the batch (not against the SRPE oracle).  Holds for SAGE / GAT up to 3 layers and GCN up to 2;
    bf16 tables add their storage rounding, which the bf16 tolerance covers."""
    built, dm = _model(name)
    qb = built.batch(3)
    feats = torch.from_numpy(qb.feats).cuda()
    out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, 1_000_000, out)
    torch.cuda.synchronize()
    t0 = built.tables[0]
    x = orc.decode_table(t0.data, t0.dtype, t0.dim)
    ref = ex.exact_full_inference_sparse(built.graph.indptr, built.graph.indices, x, qb.feats[:, :built.cfg.dims[0]],
                                         qb.qe_query, qb.qe_node, built.layers)
    err = row_rel_err(out.cpu().numpy(), ref)
    print(f"  {name}: B={qb.n_query} max row rel err vs exact inference={err:.3e}", flush=True)
    assert err <= _tol(built)


@pytest.mark.parametrize("name", ["tiny_sage3", "tiny_gcn", "tiny_gat", "large_s", "tiny_moment4", "large_s_power"])
def test_layers_step_by_step(name):
    """omg_init_buffer + omg_run_layer, every intermediate buffer against the oracle's."""
    built, dm = _model(name)
    qb = built.batch(1)
    gamma = 200_000
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma)
    og = _oracle_graph(built, qb, gamma)
    ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats, return_all=True)
    rows_in = g.sizes()["rows_in"]
    feats = torch.from_numpy(qb.feats).cuda()
    d0 = built.cfg.dims[0]
    ld0 = (d0 + 7) // 8 * 8
    buf = torch.zeros((rows_in, ld0), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(buf.cpu().numpy()[:, :d0], ref[0].astype(np.float32))
    k = len(dm.layers)
    for l in range(1, k + 1):
        last = l == k
        w = built.layers[l - 1].out_width
        nxt = torch.zeros((qb.n_query if last else rows_in, (w + 7) // 8 * 8), dtype=torch.float32, device="cuda")
        dm.ctx.run_layer(g, last, dm.tables[l - 1], buf, dm.layers[l - 1], nxt)
        torch.cuda.synchronize()
        err = row_rel_err(nxt.cpu().numpy()[:, :w], ref[l])
        print(f"  {name} layer {l}: max row rel err {err:.3e}", flush=True)
        assert err <= _tol(built)
        buf = nxt
    g.destroy()


def test_long_rows_are_split_and_recombined():
    """A query attached to thousands of nodes spans many work items; mean, GCN and attention
    rows must come out the same as the oracle's single pass."""
    for name in ("mid_s", "attention_s"):
        built, dm = _model(name)
        qb = built.batch(2, n_query=4)
        rng = np.random.default_rng(17)
        big = rng.choice(built.graph.n, size=3_000, replace=False).astype(np.int32)
        qq = np.concatenate([qb.qe_query, np.zeros(big.size, np.int32)])
        uu = np.concatenate([qb.qe_node, big])
        feats = torch.from_numpy(qb.feats).cuda()
        out = torch.empty((4, dm.out_width()), dtype=torch.float32, device="cuda")
        dm.ctx.serve_batch(dm.tables, dm.layers, feats, 4, qq, uu, 20_000, out)
        torch.cuda.synchronize()
        og = _oracle_graph(built, replace(qb, qe_query=qq, qe_node=uu), 20_000)
        ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
        err = row_rel_err(out.cpu().numpy(), ref)
        print(f"  {name}: long row, max row rel err {err:.3e}", flush=True)
        assert err <= _tol(built)


@pytest.mark.parametrize("name", ["tiny_sage3", "tiny_gcn", "tiny_gat", "tiny_gat8", "tiny_moment4", "tiny_gcnii6", "large_s", "attention_s"])
def test_batches_of_one_to_a_few_queries(name):
    """A handful of rows takes the update's row-streaming kernel instead of the matrix-core tiles, and the request
    is built by one block: one, two and five queries, each model, against the oracle."""
    built, dm = _model(name)
    for nq, gamma in ((1, 1_000_000), (1, 0), (2, 500_000), (5, 300_000)):
        qb = built.batch(7, n_query=nq)
        feats = torch.from_numpy(qb.feats).cuda()
        out = torch.full((nq, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
        dm.ctx.serve_batch(dm.tables, dm.layers, feats, nq, qb.qe_query, qb.qe_node, gamma, out)
        torch.cuda.synchronize()
        og = _oracle_graph(built, qb, gamma)
        ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
        err = row_rel_err(out.cpu().numpy(), ref)
        print(f"  {name} B={nq} gamma={gamma}: rows_in={og.rows_in} max row rel err {err:.3e}", flush=True)
        assert err <= _tol(built)


@pytest.mark.parametrize("name", ["tiny_sage3", "tiny_gcn", "tiny_max", "tiny_power", "tiny_moment4", "tiny_gcnii6", "large_s"])
def test_short_work_items_several_per_wavefront_or_one(name):
    """Rows of a few edges are aggregated several work items per wavefront; the same batch with that switched off
    (one work item per wavefront) must agree with it to rounding and both with the oracle; a zero budget (query
    rows only, the shortest) and a mixed one."""
    built, dm = _model(name)
    try:
        for gamma, nq in ((0, None), (300_000, None), (500_000, 3)):
            qb = built.batch(6, n_query=nq)
            feats = torch.from_numpy(qb.feats).cuda()
            og = _oracle_graph(built, qb, gamma)
            ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
            outs = []
            for multi in (2, 0):                        # 2: also for launches of few work items, as these are
                dm.ctx.debug_set_gather_multi(multi)
                out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
                dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, gamma, out)
                torch.cuda.synchronize()
                outs.append(out.cpu().numpy())
                assert row_rel_err(outs[-1], ref) <= _tol(built)
            assert row_rel_err(outs[0], outs[1]) <= 1e-5
    finally:
        dm.ctx.debug_set_gather_multi(1)


def test_gat_without_side_table_and_results_are_repeatable():
    from paper_2501_08547_amd import device
    built, dm = _model("tiny_gat")
    dm2 = device.upload(built, gat_side_tables=False)
    qb = built.batch(3)
    feats = torch.from_numpy(qb.feats).cuda()
    outs = []
    for m in (dm, dm2, dm):
        out = torch.empty((qb.n_query, m.out_width()), dtype=torch.float32, device="cuda")
        m.ctx.serve_batch(m.tables, m.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, 300_000, out)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    np.testing.assert_array_equal(outs[0], outs[2])                 # no atomics: bit-identical reruns
    np.testing.assert_allclose(outs[0], outs[1], rtol=1e-5, atol=1e-6)
    dm2.close()


def test_empty_and_edgeless_batches():
    built, dm = _model("tiny")
    e = np.empty(0, np.int32)
    qb = built.batch(0, n_query=3)
    feats = torch.from_numpy(qb.feats).cuda()
    out = torch.empty((3, dm.out_width()), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, 3, e, e, 500_000, out)
    torch.cuda.synchronize()
    og = _oracle_graph(built, replace(qb, qe_query=e, qe_node=e), 500_000)
    ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
    assert row_rel_err(out.cpu().numpy(), ref) <= 1e-4
    dm.ctx.serve_batch(dm.tables, dm.layers, feats[:0], 0, e, e, 500_000, out[:0])   # nothing to do, no error
    torch.cuda.synchronize()


def test_two_contexts_on_two_streams_overlap_and_agree():
    """Consecutive batches served through two contexts on streams of their own (they overlap on the
    device) give bit for bit what one context gives one batch at a time."""
    from paper_2501_08547_amd import device
    built, dm = _model("mid_s")
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    models = [device.second_context(dm, st.cuda_stream) for st in streams]
    batches = [built.batch(r) for r in range(6)]
    feats = [torch.from_numpy(b.feats).cuda() for b in batches]
    qs = [torch.from_numpy(b.qe_query).cuda() for b in batches]
    us = [torch.from_numpy(b.qe_node).cuda() for b in batches]
    outs = [torch.full((b.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda") for b in batches]
    torch.cuda.synchronize()                           # inputs and outputs were made on the default stream
    for i, b in enumerate(batches):                    # nothing waits between the calls
        m = models[i % 2]
        m.ctx.serve_batch(m.tables, m.layers, feats[i], b.n_query, qs[i], us[i], 50_000, outs[i])
    torch.cuda.synchronize()
    for i, b in enumerate(batches):
        ref = torch.empty_like(outs[i])
        dm.ctx.serve_batch(dm.tables, dm.layers, feats[i], b.n_query, qs[i], us[i], 50_000, ref)
        torch.cuda.synchronize()
        assert torch.equal(outs[i].cpu(), ref.cpu()), i
    for m in models:
        m.close()


def test_aggregator_arguments_are_checked():
    from paper_2501_08547_amd import binding as B
    built, dm = _model("tiny_moment")
    qb = built.batch(0)
    feats = torch.from_numpy(qb.feats).cuda()
    out = torch.empty((qb.n_query, dm.out_width()), dtype=torch.float32, device="cuda")

    def serve(layers):
        dm.ctx.serve_batch(dm.tables, layers, feats, qb.n_query, qb.qe_query, qb.qe_node, 100_000, out)

    def variant(**kw):
        p = replace(built.layers[0], **kw)
        return [B.make_layer(p, dm.weights[0])] + dm.layers[1:]

    for kw, code in ((dict(agg_p=3.0), B.OMG_EUNSUPPORTED),            # odd order
                     (dict(agg_p=2.5), B.OMG_EINVAL),                  # not an integer
                     (dict(agg_p=10.0), B.OMG_EINVAL),                 # beyond the supported orders
                     (dict(aggregator="power", agg_p=0.0), B.OMG_EINVAL)):
        with pytest.raises(B.OmegaError) as ei:
            serve(variant(**kw))
        assert ei.value.code == code, kw
    built_g, dm_g = _model("tiny_gcn")
    bad = B.make_layer(replace(built_g.layers[0], aggregator="max"), dm_g.weights[0])
    with pytest.raises(B.OmegaError) as ei:
        dm_g.ctx.serve_batch(dm_g.tables, [bad] + dm_g.layers[1:], feats, qb.n_query, qb.qe_query, qb.qe_node, 100_000, out)
    assert ei.value.code == B.OMG_EINVAL
    serve(dm.layers)                                                    # the context still works
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["tiny", "mid_s"])
def test_alternative_policies_bit_exact_and_served(name):
    """RANDOM (two seeds) and per-node scores (node importance; scores with many ties and signed zeros):
    same targets, same graph, same outputs as the oracle under the same policy."""
    built, dm = _model(name)
    qb = built.batch(2)
    g = built.graph
    imp = orc.importance_scores(g.indptr, g.indices).astype(np.float32)
    rng = np.random.default_rng(17)
    coarse = rng.integers(-2, 3, size=g.n).astype(np.float32) * np.float32(0.5)      # five levels, many ties
    coarse[coarse == 0] = np.where(rng.random(int((coarse == 0).sum())) < 0.5, np.float32(-0.0), np.float32(0.0))
    cases = [("random", 3, None), ("random", 4, None), ("score", 0, imp), ("score", 0, coarse)]
    feats = torch.from_numpy(qb.feats).cuda()
    try:
        for policy, seed, scores in cases:
            dev_scores = None if scores is None else torch.from_numpy(scores).cuda()
            dm.ctx.set_policy(policy, seed, dev_scores)
            for gamma in (100_000, 500_000):
                og = orc.build_computation_graph(g.indptr, g.indices, qb.n_query, qb.qe_query, qb.qe_node, gamma,
                                                 policy=policy, seed=seed, node_scores=scores)
                gg = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma)
                _assert_same_graph(gg.export(), og)
                gg.destroy()
            out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
            dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, 500_000, out)
            torch.cuda.synchronize()
            ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats)
            assert row_rel_err(out.cpu().numpy(), ref) <= _tol(built)
        from paper_2501_08547_amd import binding as B
        with pytest.raises(B.OmegaError):
            dm.ctx.set_policy("score", 0, None)
    finally:
        dm.ctx.set_policy("ratio")
    # back to the paper's policy
    og = _oracle_graph(built, qb, 100_000)
    gg = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 100_000)
    _assert_same_graph(gg.export(), og)
    gg.destroy()


@pytest.mark.parametrize("name", ["tiny_sage3", "large_s", "attention_s"])
def test_phase_timing_levels_leave_the_result_alone(name):
    """Events around the phases (every phase / fewer events from the second layer on / none) change nothing in the
    output, and the reported phases are those the level promises."""
    built, dm = _model(name)
    qb = built.batch(0)
    feats = torch.from_numpy(qb.feats).cuda()
    k = len(built.layers)
    outs, times = [], []
    for level in (0, 1, 2):
        dm.ctx.set_profiling(level)
        out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
        dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, 100_000, out)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        times.append(dm.ctx.get_timing() if level else None)
    dm.ctx.set_profiling(0)
    np.testing.assert_array_equal(outs[0], outs[1])
    np.testing.assert_array_equal(outs[0], outs[2])
    for t in times[1:]:
        assert t.build_ms > 0
        for l in range(k):
            assert t.gather_ms[l] > 0 and t.update_ms[l] > 0 and t.combine_ms[l] >= 0
        parts = t.build_ms + sum(t.gather_ms[l] + t.combine_ms[l] + t.update_ms[l] for l in range(k))
        assert abs(t.total_ms - parts) <= 1e-3 * parts
    assert all(times[2].combine_ms[l] == 0 for l in range(1, k))       # timed together with the gather


@pytest.mark.parametrize("name", ["tiny", "tiny_gcnii", "tiny_gat"])
def test_back_to_back_batches_of_changing_size_and_budget(name):
    """One context, batches served one after the other without a synchronisation in between, with the number of
    queries and the budget jumping up and down: the buffers of freshly computed rows are sized before each
    graph is built (from what the budget allows at most) and grow while earlier batches may still be running."""
    built, dm = _model(name)
    plan = [(32, 100_000), (8, 1_000_000), (32, 0), (1, 500_000), (32, 1_000_000), (5, 50_000), (32, 1_000_000)]
    feats, outs, refs = [], [], []
    for r, (n_query, gamma) in enumerate(plan):
        qb = built.batch(10 + r, n_query=n_query)
        f = torch.from_numpy(qb.feats).cuda()
        out = torch.full((n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
        dm.ctx.serve_batch(dm.tables, dm.layers, f, n_query, qb.qe_query, qb.qe_node, gamma, out)
        feats.append(f)
        outs.append(out)
        og = _oracle_graph(built, qb, gamma)
        refs.append(orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats))
    torch.cuda.synchronize()
    for (n_query, gamma), out, ref in zip(plan, outs, refs):
        err = row_rel_err(out.cpu().numpy(), ref)
        assert err <= _tol(built), (n_query, gamma, err)
