"""GPU parity for computation graph parallelism (Sec. 6) as one GPU shows it: every partition's graph bit for
bit, its local aggregations, and the merged layer outputs against the CPU oracle on the same seeded inputs
(tolerances as in test_gpu_parity)."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest

from oracle import cgp_oracle as cgp
from oracle import srpe_oracle as orc
from synth import block_partition, hash_partition
from tests.helpers import lazy_tables, row_rel_err, small_workload

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = {"f32": 1e-4, "bf16": 2e-2}
_cache = {}


def _model(name):
    from paper_2501_08547_amd import device
    if name not in _cache:
        built = small_workload(name)
        _cache[name] = (built, device.upload(built))
    return _cache[name]


def _tol(built):
    return TOL["bf16"] if any(t.dtype == "bf16" for t in built.tables) else TOL["f32"]


def _pad8(w):
    return (w + 7) // 8 * 8


def _check_records(layer, wire_p, recs_p, n_rows, tol, what):
    """One partition's records against the oracle's: counts exactly, sums / maxima / softmax statistics within
    the tolerance (GAT's weighted sums are compared after the merge: the library sums unprojected rows)."""
    from paper_2501_08547_amd import binding as B
    w = _pad8(layer.d_in)
    d = layer.d_in
    a = wire_p.cpu().numpy()
    if layer.model == "gat":
        H = layer.heads
        cnt = a[:, H * w + 16].view(np.int32)
        assert np.array_equal(cnt, np.array([int(r["count"]) for r in recs_p], dtype=np.int32)), what
        mx = np.array([r["max"] for r in recs_p])
        es = np.array([r["expsum"] for r in recs_p])
        got_mx, got_es = a[:, H * w:H * w + H].astype(np.float64), a[:, H * w + 8:H * w + 8 + H].astype(np.float64)
        has = np.isfinite(mx)
        assert np.array_equal(np.isfinite(got_mx), has), what
        scale = max(1.0, float(np.abs(mx[has]).max()) if has.any() else 1.0)
        assert np.abs(got_mx[has] - mx[has]).max(initial=0.0) <= tol * scale, what
        assert np.abs(got_es - es).max(initial=0.0) <= 10 * tol * max(1.0, float(es.max(initial=0.0))), what
        return
    cnt = a[:, w].view(np.int32)
    assert np.array_equal(cnt, np.array([int(r["count"]) for r in recs_p], dtype=np.int32)), what
    key = "max" if "max" in recs_p[0] else "sum"
    ref = np.array([r[key] for r in recs_p])
    got = a[:, :d].astype(np.float64)
    if key == "max":
        empty = ~np.isfinite(ref)
        assert np.array_equal(np.isneginf(got), empty), what
        ref, got = np.where(empty, 0.0, ref), np.where(empty, 0.0, got)
    assert row_rel_err(got, ref) <= tol, what


def _run(name, n_part, node_part, batch_r=1, gamma=200_000, check_graphs=True):
    from paper_2501_08547_amd import binding as B
    built, dm = _model(name)
    qb = built.batch(batch_r)
    tol = _tol(built)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma)
    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, gamma)
    oparts = [cgp.partition_graph(og, node_part, n_part, p) for p in range(n_part)]
    np_dev = torch.from_numpy(node_part.astype(np.int32)).cuda()
    parts = []
    for p in range(n_part):
        pg = dm.ctx.cgp_partition_graph(g, np_dev, n_part, p)
        parts.append(pg)
        if check_graphs:
            e = pg.export()
            assert np.array_equal(e["indptr"], oparts[p].indptr), (name, p)
            assert np.array_equal(e["cols"], oparts[p].cols), (name, p)
            assert np.array_equal(e["cdeg"], oparts[p].cdeg), (name, p)
            assert np.array_equal(e["targets"], og.T.astype(np.int32))
    rows_in = g.sizes()["rows_in"]
    tabs = lazy_tables(built)
    ref0 = orc.initial_buffer(og, tabs[0], qb.feats)
    feats = torch.from_numpy(qb.feats).cuda()
    d0 = built.cfg.dims[0]
    buf0 = torch.zeros((rows_in, _pad8(d0)), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf0)
    buf, ref = buf0, ref0
    k = len(dm.layers)
    for l in range(1, k + 1):
        last = l == k
        p_l = built.layers[l - 1]
        n_rows = qb.n_query if last else rows_in
        lay = dm.layers[l - 1]
        if p_l.model == "gcnii":
            lay = B.make_layer(p_l, dm.weights[l - 1], init_rows=buf0)
        ldw = B.cgp_wire_width(lay)
        assert ldw == (p_l.heads * _pad8(p_l.d_in) + 20 if p_l.model == "gat" else _pad8(p_l.d_in) + 4)
        oref, owire = cgp.run_layer_cgp(og, oparts, p_l, tabs[l - 1], ref, last, buf0=ref0, return_wire=True)
        wire = torch.full((n_part, n_rows, ldw), float("nan"), dtype=torch.float32, device="cuda")
        row_mean = None
        if p_l.model == "sage" and p_l.aggregator == "moment":
            for p in range(n_part):
                dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p])
            row_mean = torch.full((n_rows, _pad8(p_l.d_in)), float("nan"), dtype=torch.float32, device="cuda")
            dm.ctx.cgp_merge_mean(wire, lay, row_mean)
            wire = torch.full((n_part, n_rows, ldw), float("nan"), dtype=torch.float32, device="cuda")
        for p in range(n_part):
            dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p], row_mean=row_mean)
        torch.cuda.synchronize()
        for p in range(n_part):
            _check_records(p_l, wire[p], [owire[v][p] for v in range(n_rows)], n_rows, tol, (name, l, p))
        w = p_l.out_width
        nxt = torch.zeros((n_rows, _pad8(w)), dtype=torch.float32, device="cuda")
        dm.ctx.cgp_merge_update(wire, lay, buf, nxt)
        whole = torch.zeros_like(nxt)
        dm.ctx.run_layer(g, last, dm.tables[l - 1], buf, lay, whole)
        torch.cuda.synchronize()
        got = nxt.cpu().numpy()[:, :w]
        err = row_rel_err(got, oref)
        err_whole = row_rel_err(got, whole.cpu().numpy()[:, :w])
        print(f"  {name} P={n_part} layer {l}: vs oracle {err:.3e}, vs the unpartitioned layer on the GPU {err_whole:.3e}", flush=True)
        assert err <= tol
        assert err_whole <= 1e-4
        buf, ref = nxt, oref
    for pg in parts:
        pg.destroy()
    g.destroy()


CASES = [("tiny", 2), ("tiny_sage3", 3), ("tiny_gcn", 4), ("tiny_gat", 3), ("tiny_gat8", 4), ("tiny_sum", 2), ("tiny_max", 5),
         ("tiny_power", 2), ("tiny_moment4", 3), ("tiny_gcnii", 2), ("large_s", 4), ("mid_s", 8), ("attention_s", 4),
         ("large_s_max", 3), ("large_s_moment", 2)]


@pytest.mark.parametrize("name,n_part", CASES)
def test_partitioned_layers_match_oracle(name, n_part):
    built, _ = _model(name)
    _run(name, n_part, hash_partition(built.graph.n, n_part, seed=40 + n_part))


def test_one_partition_many_partitions_and_empty_partitions():
    built, _ = _model("tiny_gat")
    _run("tiny_gat", 1, np.zeros(built.graph.n, dtype=np.int32))
    _run("tiny_gcn", 64, hash_partition(built.graph.n, 64, seed=9), check_graphs=False)
    # every existing node in partition 2 of 3: the other partitions hold only query rows as sources
    _run("tiny_max", 3, np.full(built.graph.n, 2, dtype=np.int32))
    _run("tiny", 4, block_partition(built.graph.n, 4), batch_r=2, gamma=1_000_000)
    _run("tiny_sage3", 2, block_partition(built.graph.n, 2), batch_r=3, gamma=0)


def test_arguments_are_checked_and_handles_are_refilled():
    from paper_2501_08547_amd import binding as B
    built, dm = _model("tiny")
    qb = built.batch(0)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 300_000)
    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, 300_000)
    node_part = hash_partition(built.graph.n, 3, seed=1)
    npd = torch.from_numpy(node_part).cuda()
    L = B.lib()
    h = C.c_void_p(None)
    assert L.omg_cgp_partition_graph(dm.ctx.handle, g.handle, npd.data_ptr(), 65, 0, C.byref(h)) == B.OMG_EINVAL
    assert L.omg_cgp_partition_graph(dm.ctx.handle, g.handle, npd.data_ptr(), 3, 3, C.byref(h)) == B.OMG_EINVAL
    assert L.omg_cgp_partition_graph(dm.ctx.handle, g.handle, None, 3, 0, C.byref(h)) == B.OMG_EINVAL
    assert not h
    # a node whose partition is out of range
    bad = node_part.copy(); bad[17] = 3
    assert L.omg_cgp_partition_graph(dm.ctx.handle, g.handle, torch.from_numpy(bad).cuda().data_ptr(), 3, 0,
                                     C.byref(h)) == B.OMG_ERANGE
    assert not h
    # one handle filled for partition 0, then again for partition 2
    pg = dm.ctx.cgp_partition_graph(g, npd, 3, 0)
    assert np.array_equal(pg.export()["cols"], cgp.partition_graph(og, node_part, 3, 0).cols)
    dm.ctx.cgp_partition_graph(g, npd, 3, 2, part_graph=pg)
    e = pg.export()
    o2 = cgp.partition_graph(og, node_part, 3, 2)
    assert np.array_equal(e["indptr"], o2.indptr) and np.array_equal(e["cols"], o2.cols) and np.array_equal(e["cdeg"], o2.cdeg)
    # records narrower than the layer needs, a mean handed to a layer that has no second step
    lay = dm.layers[0]
    rows = g.sizes()["rows_in"]
    buf = torch.zeros((rows, _pad8(built.cfg.dims[0])), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], torch.from_numpy(qb.feats).cuda(), buf)
    ldw = B.cgp_wire_width(lay)
    narrow = torch.zeros((rows, ldw - 4), dtype=torch.float32, device="cuda")
    with pytest.raises(B.OmegaError):
        dm.ctx.cgp_local_aggregate(pg, False, dm.tables[0], buf, lay, narrow)
    wire = torch.zeros((rows, ldw), dtype=torch.float32, device="cuda")
    with pytest.raises(B.OmegaError):
        dm.ctx.cgp_local_aggregate(pg, False, dm.tables[0], buf, lay, wire, row_mean=buf)
    with pytest.raises(B.OmegaError):
        dm.ctx.cgp_merge_mean(wire[None], lay, buf)
    pg.destroy()
    g.destroy()
