"""GPU parity on seeded random configurations: model, depth, widths that are no multiple of anything, storage
types, graph density, batch size and budget are all drawn per case.  Graph construction bit for bit, outputs
within the usual tolerance, and the same batch once more as a random number of partitions' shares."""
from __future__ import annotations

from dataclasses import replace

import numpy as np
import pytest

from oracle import cgp_oracle as cgp
from oracle import srpe_oracle as orc
from synth import CONFIGS, build_workload, hash_partition
from tests.helpers import lazy_tables, row_rel_err

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _draw(seed: int):
    rng = np.random.default_rng([seed, 4242])
    model = ["sage", "gcn", "gat", "gcnii", "sage"][int(rng.integers(0, 5))]
    k = int(rng.integers(1, 5))
    heads = int([1, 2, 4][int(rng.integers(0, 3))]) if model == "gat" else 1
    if model == "gat" and seed % 2 == 1:
        heads = 8
    def width(lo, hi):
        w = int(rng.integers(lo, hi))
        return max(heads, w // heads * heads) if model == "gat" else w
    if model == "gcnii":
        d = int(rng.integers(3, 90))
        dims = (d,) * (k + 1)
    else:
        d0 = int(rng.integers(1, 300))
        dims = (d0,) + tuple(width(heads, 140) for _ in range(k - 1)) + (int(rng.integers(1, 50)),)
        if model == "gat":
            # hidden GAT layers concatenate heads x d_head; the output layer averages heads x classes
            dims = dims[:-1] + (dims[-1],)
    agg = ["mean", "sum", "max", "power", "moment"][int(rng.integers(0, 5))] if model == "sage" else "mean"
    agg_p = {"power": float(rng.choice([0.5, 2.0, 3.0])), "moment": float(rng.choice([2, 4]))}.get(agg, 1.0)
    store = ["f32", "bf16"][int(rng.integers(0, 2))]
    cfg = replace(CONFIGS["tiny"], name=f"rnd{seed}", model=model, dims=dims, heads=heads, aggregator=agg, agg_p=agg_p,
                  n_nodes=int(rng.integers(40, 1500)), avg_deg=float(rng.choice([1.5, 4, 10, 30])),
                  batch=int(rng.integers(1, 30)), feat_dtype=store, pe_dtype=["f32", "bf16"][int(rng.integers(0, 2))],
                  q_degree=("uniform", 1, int(rng.integers(2, 40))))
    gamma = int(rng.choice([0, 1_000_000, int(rng.integers(1, 1_000_000))]))
    return cfg, gamma, int(rng.integers(1, 7))


@pytest.mark.parametrize("seed", list(range(64)))
def test_random_configuration(seed):
    from paper_2501_08547_amd import binding as B
    from paper_2501_08547_amd import device
    cfg, gamma, n_part = _draw(seed)
    print(f"case {seed}: {cfg.model} dims={cfg.dims} heads={cfg.heads} agg={cfg.aggregator}/{cfg.agg_p} n={cfg.n_nodes} "
          f"deg={cfg.avg_deg} B={cfg.batch} store={cfg.feat_dtype}/{cfg.pe_dtype} gamma={gamma} P={n_part}", flush=True)
    built = build_workload(cfg)
    dm = device.upload(built)
    qb = built.batch(seed)
    tol = 2e-2 if "bf16" in (cfg.feat_dtype, cfg.pe_dtype) else 1e-4
    feats = torch.from_numpy(qb.feats).cuda()
    out = torch.full((qb.n_query, dm.out_width()), float("nan"), dtype=torch.float32, device="cuda")
    dm.ctx.serve_batch(dm.tables, dm.layers, feats, qb.n_query, qb.qe_query, qb.qe_node, gamma, out)
    torch.cuda.synchronize()
    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node, gamma)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma)
    e = g.export()
    assert np.array_equal(e["cand"], og.R.astype(np.int32)) and np.array_equal(e["qdeg"], og.qdeg.astype(np.int32))
    assert np.array_equal(e["targets"], og.T.astype(np.int32)) and np.array_equal(e["indptr"], og.indptr)
    assert np.array_equal(e["cols"], og.cols) and np.array_equal(e["cdeg"], og.cdeg)
    tabs = lazy_tables(built)
    ref = orc.srpe_reference(og, tabs, built.layers, qb.feats)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    err = row_rel_err(got, ref)
    assert err <= tol, err

    # the same batch as n_part partitions' shares
    node_part = hash_partition(built.graph.n, n_part, seed=seed)
    np_dev = torch.from_numpy(node_part).cuda()
    parts = [dm.ctx.cgp_partition_graph(g, np_dev, n_part, p) for p in range(n_part)]
    oparts = [cgp.partition_graph(og, node_part, n_part, p) for p in range(n_part)]
    for pg, opg in zip(parts, oparts):
        ep = pg.export()
        assert np.array_equal(ep["indptr"], opg.indptr) and np.array_equal(ep["cols"], opg.cols)
        assert np.array_equal(ep["cdeg"], opg.cdeg)
    pad8 = lambda w: (w + 7) // 8 * 8
    rows_in = og.rows_in
    buf0 = torch.zeros((rows_in, pad8(cfg.dims[0])), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf0)
    buf = buf0
    k = len(dm.layers)
    for l in range(1, k + 1):
        last = l == k
        p_l = built.layers[l - 1]
        lay = B.make_layer(p_l, dm.weights[l - 1], src_logits=dm.side[l - 1], init_rows=buf0 if p_l.model == "gcnii" else None)
        n_rows = qb.n_query if last else rows_in
        wire = torch.full((n_part, n_rows, B.cgp_wire_width(lay)), float("nan"), dtype=torch.float32, device="cuda")
        row_mean = None
        if p_l.model == "sage" and p_l.aggregator == "moment":
            for p in range(n_part):
                dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p])
            row_mean = torch.full((n_rows, pad8(p_l.d_in)), float("nan"), dtype=torch.float32, device="cuda")
            dm.ctx.cgp_merge_mean(wire, lay, row_mean)
            wire = torch.full_like(wire, float("nan"))
        for p in range(n_part):
            dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p], row_mean=row_mean)
        nxt = torch.zeros((n_rows, pad8(p_l.out_width)), dtype=torch.float32, device="cuda")
        dm.ctx.cgp_merge_update(wire, lay, buf, nxt)
        buf = nxt
    torch.cuda.synchronize()
    got_p = buf.cpu().numpy()[:, :built.layers[-1].out_width]
    ref_p = cgp.cgp_reference(og, node_part, n_part, tabs, built.layers, qb.feats)
    err_p = row_rel_err(got_p, ref_p)
    print(f"  rows_in={og.rows_in} nnz_in={og.nnz_in} err={err:.2e} partitioned err={err_p:.2e}", flush=True)
    assert err_p <= tol, err_p
    for pg in parts:
        pg.destroy()
    g.destroy()
    dm.close()
