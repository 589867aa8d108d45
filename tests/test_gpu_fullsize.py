"""GPU parity at the benchmark's full sizes, through the same call bench.py times
(omg_serve_batch with the request in device memory).  The whole computation graph is compared
bit for bit with the oracle's; outputs are compared on a sample of query rows that the oracle
computes one by one (it evaluates only the layer-1 rows those queries read)."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import cgp_oracle as cgp
from oracle import srpe_oracle as orc
from synth import CONFIGS, build_workload, hash_partition
from tests.helpers import lazy_tables, row_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _oracle_rows(built, og, qb, sample):
    """Oracle outputs of the sampled query rows; inner layers are evaluated only where needed."""
    tabs = lazy_tables(built)
    k = len(built.layers)
    B = qb.n_query
    need = [set(sample.tolist())]                         # rows whose layer-l value is needed, from the top down
    for _ in range(k - 1):
        cur = set(need[-1])
        for v in need[-1]:
            c = og.cols[og.indptr[v]:og.indptr[v + 1]]
            cur.update((~c[c < 0]).tolist())
        need.append(cur)
    need = need[::-1]                                     # need[l - 1] = rows needed after layer l, need[k-1] = sample
    buf = orc.initial_buffer(og, tabs[0], qb.feats)
    for l in range(1, k + 1):
        last = l == k
        rows = np.array(sorted(need[l - 1] if not last else sample.tolist()), dtype=np.int64)
        p = built.layers[l - 1]
        out = orc.run_layer(og, p, tabs[l - 1], buf, is_last=last, rows=rows)
        if last:
            return out
        nxt = np.full((og.rows_in, p.out_width), np.nan)  # anything not computed must not be read
        nxt[rows] = out
        buf = nxt


def _check_batch(name, built, dm, qb, q_dev, u_dev, feats, gamma_ppm, n_sample):
    out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, q_dev, u_dev, gamma_ppm, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    out2 = torch.empty_like(out)
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, q_dev, u_dev, gamma_ppm, out2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got, out2.cpu().numpy())          # run-to-run bit identical

    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query,
                                     qb.qe_node, gamma_ppm)
    g = dm.ctx.build_computation_graph(qb.n_query, q_dev, u_dev, gamma_ppm)
    exp = g.export()
    assert np.array_equal(exp["cand"], og.R.astype(np.int32))
    assert np.array_equal(exp["qdeg"], og.qdeg.astype(np.int32))
    assert np.array_equal(exp["targets"], og.T.astype(np.int32))
    assert np.array_equal(exp["indptr"], og.indptr)
    assert np.array_equal(exp["cols"], og.cols)
    assert np.array_equal(exp["cdeg"], og.cdeg)
    g.destroy()

    rng = np.random.default_rng(99)
    deg = np.diff(og.indptr[:qb.n_query + 1])
    sample = np.unique(np.concatenate([rng.choice(qb.n_query, size=n_sample, replace=False),
                                       [int(np.argmax(deg)), int(np.argmin(deg))]]))
    ref = _oracle_rows(built, og, qb, sample)
    err = row_rel_err(got[sample], ref)
    tol = 2e-2 if any(t.dtype == "bf16" for t in built.tables) else 1e-4
    print(f"{name} gamma={gamma_ppm / 1e4:.0f}%: rows_in={og.rows_in} nnz_in={og.nnz_in} sampled rows {sample.size} "
          f"(degrees {deg[sample].min()}..{deg[sample].max()}), max row rel err {err:.3e}", flush=True)
    assert err <= tol
    return og, sample, ref, got


def _pad8(w):
    return (w + 7) // 8 * 8


def _check_cgp(name, built, dm, qb, q_dev, u_dev, feats, gamma_ppm, n_part, og, sample, ref, got_whole):
    """The same batch executed as n_part partitions' shares and merged (Sec. 6): every partition's graph bit for
    bit against the oracle's definition (the whole graph's edges whose source the partition holds, in order), the
    merged outputs against the oracle on the sampled rows and against the unpartitioned run on all rows."""
    from paper_2501_08547_amd import binding as B
    node_part = hash_partition(built.graph.n, n_part, seed=77)
    np_dev = torch.from_numpy(node_part).cuda()
    g = dm.ctx.build_computation_graph(qb.n_query, q_dev, u_dev, gamma_ppm)
    sp = cgp.source_partitions(og, node_part, n_part)
    row_of_edge = np.repeat(np.arange(og.rows_in), np.diff(og.indptr))
    parts, t_build = [], []
    for p in range(n_part):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        pg = dm.ctx.cgp_partition_graph(g, np_dev, n_part, p)
        e1.record()
        torch.cuda.synchronize()
        t_build.append(e0.elapsed_time(e1))
        parts.append(pg)
        e = pg.export()
        mine = sp == p
        indptr_p = np.concatenate([[0], np.cumsum(np.bincount(row_of_edge[mine], minlength=og.rows_in))])
        assert np.array_equal(e["indptr"], indptr_p)
        assert np.array_equal(e["cols"], og.cols[mine])
        assert np.array_equal(e["cdeg"], og.cdeg[mine])
    # a handle that is filled again allocates nothing: the time of the construction itself
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dm.ctx.cgp_partition_graph(g, np_dev, n_part, 0, part_graph=parts[0])
    e1.record()
    torch.cuda.synchronize()
    t_refill = e0.elapsed_time(e1)
    assert np.array_equal(parts[0].export()["cols"], og.cols[sp == 0])
    rows_in = og.rows_in
    d0 = built.cfg.dims[0]
    buf0 = torch.zeros((rows_in, _pad8(d0)), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf0)
    buf = buf0
    k = len(dm.layers)
    for l in range(1, k + 1):
        last = l == k
        p_l = built.layers[l - 1]
        lay = dm.layers[l - 1]
        n_rows = qb.n_query if last else rows_in
        wire = torch.full((n_part, n_rows, B.cgp_wire_width(lay)), float("nan"), dtype=torch.float32, device="cuda")
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_part + 2)]
        for p in range(n_part):
            ev[p].record()
            dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p])
        ev[n_part].record()
        nxt = torch.zeros((n_rows, _pad8(p_l.out_width)), dtype=torch.float32, device="cuda")
        dm.ctx.cgp_merge_update(wire, lay, buf, nxt)
        ev[n_part + 1].record()
        torch.cuda.synchronize()
        loc = [ev[p].elapsed_time(ev[p + 1]) for p in range(n_part)]
        print(f"{name} P={n_part} layer {l}: local aggregation per partition {min(loc):.3f}..{max(loc):.3f} ms, "
              f"merge + update {ev[n_part].elapsed_time(ev[n_part + 1]):.3f} ms "
              f"(records {wire[0].numel() * 4 / 1e6:.1f} MB per partition)", flush=True)
        buf = nxt
    got = buf.cpu().numpy()[:, :built.layers[-1].out_width]
    tol = 2e-2 if any(t.dtype == "bf16" for t in built.tables) else 1e-4
    err = row_rel_err(got[sample], ref)
    err_whole = row_rel_err(got, got_whole)
    print(f"{name} P={n_part}: partition graphs built in {min(t_build):.3f}..{max(t_build):.3f} ms each with new handles, "
          f"{t_refill:.3f} ms into an existing one, "
          f"max row rel err vs oracle {err:.3e} (sampled rows), vs the unpartitioned run {err_whole:.3e} (all rows)", flush=True)
    assert err <= tol
    assert err_whole <= 1e-4
    for pg in parts:
        pg.destroy()
    g.destroy()


@pytest.mark.parametrize("name", ["mid", "large", "attention"])
def test_full_size_workload(name):
    from paper_2501_08547_amd import device
    cfg = CONFIGS[name]
    print(f"generating {name}", flush=True)
    built = build_workload(cfg)
    dm = device.upload(built)
    qb = built.batch(0)
    print(f"{name}: {built.graph.n} nodes {built.graph.nnz} edges, batch E_q={qb.n_edges}", flush=True)
    feats = torch.from_numpy(qb.feats).cuda()
    q_dev = torch.from_numpy(qb.qe_query).cuda()
    u_dev = torch.from_numpy(qb.qe_node).cuda()
    og, sample, ref, got = _check_batch(name, built, dm, qb, q_dev, u_dev, feats, cfg.gamma_ppm, 12)
    _check_cgp(name, built, dm, qb, q_dev, u_dev, feats, cfg.gamma_ppm, 4, og, sample, ref, got)
    if name == "large":                                   # the recompute fraction swept at full size: none, a fifth
        for gamma in (0, 200_000):
            _check_batch(name, built, dm, qb, q_dev, u_dev, feats, gamma, 6)
    dm.close()
