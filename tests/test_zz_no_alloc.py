"""omg_run_layer_static (the entry point that allocates nothing: its scratch is a device array inside the
library's image) against omg_run_layer on the same graph and buffers, layer by layer, through the C ABI:
bit-identical outputs (same kernels), and both within the stated tolerance of the CPU oracle.  Two calls
in a row on one context, the second on a smaller batch, so that whatever the first call left in the shared
array is still there when the second runs."""
from __future__ import annotations

from dataclasses import replace

import numpy as np
import pytest

from oracle import srpe_oracle as orc
from tests.helpers import lazy_tables, row_rel_err, small_workload

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _pad8(w):
    return (w + 7) // 8 * 8


def _layers_both_ways(built, dm, qb, gamma_ppm, tag):
    from paper_2501_08547_amd import binding as B
    tol = TOL["bf16"] if any(t.dtype == "bf16" for t in built.tables) else TOL["f32"]
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, gamma_ppm)
    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node,
                                     gamma_ppm)
    ref = orc.srpe_reference(og, lazy_tables(built), built.layers, qb.feats, return_all=True)
    rows_in = g.sizes()["rows_in"]
    assert rows_in == og.rows_in
    feats = torch.from_numpy(qb.feats).cuda()
    buf0 = torch.zeros((rows_in, _pad8(built.cfg.dims[0])), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf0)
    buf = buf0
    k = len(dm.layers)
    for l in range(1, k + 1):
        last = l == k
        p = built.layers[l - 1]
        lay = dm.layers[l - 1]
        if p.model == "gcnii":
            lay = B.make_layer(p, dm.weights[l - 1], init_rows=buf0)
        shape = (qb.n_query if last else rows_in, _pad8(p.out_width))
        a = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        b = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        print(f"  {tag} layer {l}: omg_run_layer, then omg_run_layer_static, rows={shape[0]}", flush=True)
        dm.ctx.run_layer(g, last, dm.tables[l - 1], buf, lay, a)
        torch.cuda.synchronize()
        dm.ctx.run_layer_static(g, last, dm.tables[l - 1], buf, lay, b)
        torch.cuda.synchronize()
        w = p.out_width
        an, bn = a.cpu().numpy()[:, :w], b.cpu().numpy()[:, :w]
        assert np.all(np.isfinite(bn))
        np.testing.assert_array_equal(an, bn)
        err = row_rel_err(bn, ref[l])
        print(f"  {tag} layer {l}: identical to omg_run_layer; max row rel err vs oracle {err:.3e}", flush=True)
        assert err <= tol
        buf = b                                        # the next layer reads what the static call wrote
    g.destroy()


@pytest.mark.parametrize("name", ["tiny_sage3", "tiny_gcn", "tiny_gat", "tiny_moment4", "tiny_gcnii6", "large_s", "attention_s"])
def test_run_layer_static_matches_run_layer_on_two_calls_in_a_row(name):
    from paper_2501_08547_amd import device
    built = small_workload(name)
    dm = device.upload(built)
    n0 = built.cfg.batch
    # a batch, then a smaller one: the second call finds the first call's contents in the shared array
    for r, nq, gamma in ((1, n0, 200_000), (2, max(3, n0 // 5), 350_000)):
        _layers_both_ways(built, dm, built.batch(r, n_query=nq), gamma, f"{name} B={nq}")
    dm.close()


def test_a_layer_beyond_the_static_buffer_is_refused_and_the_next_call_works():
    from paper_2501_08547_amd import binding as B
    from paper_2501_08547_amd import device
    from synth import CONFIGS, build_workload
    limit = B.lib().omg_static_scratch_bytes()
    assert limit == 32 << 20
    # 9,000 query rows of 1,024 aggregated values = 36.9 MB of aggregated rows alone
    built = build_workload(replace(CONFIGS["tiny"], name="wide", dims=(1024, 8, 2), batch=9000))
    dm = device.upload(built)
    qb = built.batch(0)
    g = dm.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 0)
    rows_in = g.sizes()["rows_in"]
    assert rows_in * 1024 * 4 > limit
    feats = torch.from_numpy(qb.feats).cuda()
    buf0 = torch.zeros((rows_in, 1024), dtype=torch.float32, device="cuda")
    dm.ctx.init_buffer(g, dm.tables[0], feats, buf0)
    out = torch.full((rows_in, 8), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.OmegaError) as ei:
        dm.ctx.run_layer_static(g, False, dm.tables[0], buf0, dm.layers[0], out)
    assert ei.value.code == B.OMG_ESCRATCH
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(out.max()) == 7.0           # nothing was launched
    # the growable path takes the same layer, and a smaller batch fits the static buffer again
    dm.ctx.run_layer(g, False, dm.tables[0], buf0, dm.layers[0], out)
    torch.cuda.synchronize()
    whole = out.cpu().numpy().copy()
    g.destroy()
    qb2 = built.batch(0, n_query=512)
    _layers_both_ways(built, dm, qb2, 100_000, "wide B=512")
    assert np.all(np.isfinite(whole))
    # a GAT layer without its side table would have to allocate one: refused
    built_g = small_workload("tiny_gat")
    dm_g = device.upload(built_g, gat_side_tables=False)
    qb = built_g.batch(0)
    g = dm_g.ctx.build_computation_graph(qb.n_query, qb.qe_query, qb.qe_node, 100_000)
    rows_in = g.sizes()["rows_in"]
    buf0 = torch.zeros((rows_in, 64), dtype=torch.float32, device="cuda")
    dm_g.ctx.init_buffer(g, dm_g.tables[0], torch.from_numpy(qb.feats).cuda(), buf0)
    out = torch.zeros((rows_in, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(B.OmegaError) as ei:
        dm_g.ctx.run_layer_static(g, False, dm_g.tables[0], buf0, dm_g.layers[0], out)
    assert ei.value.code == B.OMG_EINVAL
    g.destroy()
    dm_g.close()
    dm.close()
