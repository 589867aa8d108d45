#!/usr/bin/env python3
"""Benchmark of the single-GPU SRPE serving path.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mid] [--configs all|headline]

One step = omg_serve_batch on one query batch: computation-graph construction plus every GNN layer.  The base
graph, the tables, the weights and the batches (features and edge lists) are in device memory before the timed
region starts.  Prints ONE JSON line.  The headline figures are those of the workload the metric is quoted on
(`mid`); with `--configs all` (the default of a plain run) the same line also carries, in the object `configs`,
every other configuration of the baseline file measured the same way: Tiny, Large at recompute fractions 0 / 5 /
20 / 100 %, Attention, Scale at 1 / 64 / 1,024 / 16,384 queries, and the layer-1 gather of an FB10B-shaped
graph, whose table is far larger than any cache and is read once (the reuse-free reference for the HBM roofline).

The CPU oracle is timed first, before the GPU is touched (one thread, then one batch per process on all cores
of this machine's share), on the first batches of the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
N_BATCHES = 200              # distinct seeded batches cycled through the steps (--distinct-batches)
T_START = time.perf_counter()


def log(msg: str):
    print(f"[bench {time.perf_counter() - T_START:6.1f}s] {msg}", file=sys.stderr, flush=True)


def algorithmic_gather_bytes(model: str, d_in: int, elem_bytes: int, nnz: int, rows: int, heads: int = 1) -> int:
    """Bytes the aggregation of one layer has to move: per edge the source row, its column id and
    (GCN) the source degree or (GAT) the per-head source score; per row the two row pointers and
    (GCN) its own previous embedding."""
    per_edge = d_in * elem_bytes + 4
    per_row = 8
    if model in ("gcn", "gcnii"):
        per_edge += 4
        per_row += d_in * 4
    if model == "gat":
        per_edge += 4 * heads
        per_row += 4 * heads
    return nnz * per_edge + rows * per_row


# ------------------------------------------------------------------------------------------ CPU oracle legs
def _host_cores() -> int:
    """Cores this process may use: its affinity mask, capped by the share the environment announces."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, n)


def _oracle_batch(built, qb, gamma_ppm):
    """One batch through the CPU oracle: (reference output, oracle graph, edges aggregated, seconds)."""
    from oracle import srpe_oracle as orc
    k = len(built.layers)
    t0 = time.perf_counter()
    og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node,
                                     gamma_ppm)
    tabs = [orc.LazyTable(t.data, t.dtype, t.dim) for t in built.tables]
    ref = orc.srpe_reference(og, tabs, built.layers, qb.feats)
    dt = time.perf_counter() - t0
    return ref, og, (k - 1) * og.nnz_in + int(og.indptr[qb.n_query]), dt


_POOL_STATE = {}


def _pool_job(i):
    from threadpoolctl import threadpool_limits
    with threadpool_limits(limits=1):
        built, batches, gamma_ppm = _POOL_STATE["args"]
        _, _, edges, dt = _oracle_batch(built, batches[i], gamma_ppm)
    return edges, dt


def cpu_baseline(built, batches, gamma_ppm, min_seconds=10.0):
    """The CPU oracle as it stands on the first batches of the workload: whole batches, one thread, until at
    least min_seconds are on the clock; then one batch per worker process on every core at once (the processes
    are forked, so the graph and the tables are shared, not copied).  Must run before the GPU is initialised.
    Returns the first batch's reference output and graph, and the baseline object."""
    import multiprocessing as mp
    from threadpoolctl import threadpool_limits
    k = len(built.layers)
    edges, spent, used, first = 0, 0.0, 0, None
    with threadpool_limits(limits=1):
        for qb in batches:
            ref, og, e, dt = _oracle_batch(built, qb, gamma_ppm)
            edges += e
            spent += dt
            used += 1
            if first is None:
                first = (ref, og)
            if spent >= min_seconds:
                break
    qb = batches[0]
    shape = f"{qb.n_query} queries and about {qb.n_edges} query edges each"
    base = {"value": edges / spent, "unit": "edges/s", "cores": 1, "kind": "oracle", "seconds": round(spent, 2),
            "sample": f"the first {used} of the workload's batches ({shape}), graph construction + {k} layers per "
                      f"batch, numpy fp64, 1 thread"}
    cores = _host_cores()
    if cores > 1:
        n_jobs = min(len(batches), 2 * cores)
        _POOL_STATE["args"] = (built, batches, gamma_ppm)
        t0 = time.perf_counter()
        with mp.get_context("fork").Pool(cores) as pool:
            res = pool.map(_pool_job, range(n_jobs), chunksize=1)
        wall = time.perf_counter() - t0
        _POOL_STATE.clear()
        base["all_cores"] = {"value": sum(e for e, _ in res) / wall, "unit": "edges/s", "cores": cores,
                             "kind": "oracle", "seconds": round(wall, 2),
                             "cpu_seconds": round(sum(d for _, d in res), 2),
                             "sample": f"the first {n_jobs} of the workload's batches ({shape}), one batch per "
                                       f"process, {cores} processes of one thread each, wall-clock time incl. "
                                       f"starting the processes"}
    base["host_cpus_visible"] = os.cpu_count()
    return first[0], first[1], base


# ------------------------------------------------------------------------------------------ workloads
def host_synth(name, args):
    """Host side of a generated workload (graph, tables, weights): nothing here touches the GPU."""
    from dataclasses import replace
    from synth import CONFIGS, build_workload
    cfg = CONFIGS[name]
    if args.batch:
        cfg = replace(cfg, batch=args.batch)
    if args.gamma_ppm >= 0:
        cfg = replace(cfg, gamma_ppm=args.gamma_ppm)
    if args.layers:
        d = cfg.dims
        cfg = replace(cfg, dims=(d[0],) + (d[1],) * (args.layers - 1) + (d[-1],))
    return cfg, build_workload(cfg)


def hash_workload(name, n_batch, gamma_ppm):
    """scale: 111 M nodes / 1.67 G edges / three 28 GB bf16 tables; fb10b: 30 M nodes / 9.8 G edges / 1,024
    features (61 GB bf16) + two 7.7 GB tables; hash-defined, generated on the device, the oracle evaluates the
    same integer hash for the rows it touches."""
    from types import SimpleNamespace
    from paper_2501_08547_amd import device
    from synth import scale as S
    spec = S.ScaleSpec() if name == "scale" else S.fb10b_spec()
    ip = S.indptr_np(spec)
    nnz = int(ip[-1])
    indptr, indices, tabs = S.device_arrays(spec, ip, "cuda:0")
    layers = S.scale_layers(spec)
    dm = device.assemble(indptr, indices, [(t, "bf16", d) for t, d in zip(tabs, spec.dims[:-1])], layers)
    cfg = SimpleNamespace(name=name, model="sage", dims=spec.dims, k=spec.k, batch=n_batch, gamma_ppm=gamma_ppm,
                          feat_dtype="bf16", pe_dtype="bf16", heads=1)
    built = SimpleNamespace(cfg=cfg, layers=layers,
                            graph=SimpleNamespace(n=spec.n_nodes, nnz=nnz, indptr=ip,
                                                  indices=S.HashIndices(spec.n_nodes, nnz, spec.seed_graph)),
                            tables=[SimpleNamespace(data=S.HashTable(spec.n_nodes, d, spec.seed_table, t),
                                                    dtype="bf16", dim=d) for t, d in enumerate(spec.dims[:-1])])
    return spec, ip, cfg, built, dm


def workload_text(cfg, built, gamma_ppm=None, batch=None):
    g = cfg.gamma_ppm if gamma_ppm is None else gamma_ppm
    return (f"{cfg.name}: {built.graph.n} nodes, {built.graph.nnz} directed edges, {cfg.model} "
            f"{'-'.join(map(str, cfg.dims))}, tables {cfg.feat_dtype}/{cfg.pe_dtype}, batch {batch or cfg.batch}, "
            f"gamma {g / 1e4:.2f}%")


# ------------------------------------------------------------------------------------------ measurement
def to_device(torch, batches):
    return [(torch.from_numpy(b.feats).cuda(), torch.from_numpy(b.qe_query).cuda(), torch.from_numpy(b.qe_node).cuda())
            for b in batches]


def timed_steps(torch, np, dm, batches, dev_batches, gamma_ppm, outs, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` timed ones, each ending when its output is ready."""
    nb = len(batches)

    def step(i):
        f, q, u = dev_batches[i % nb]
        dm.ctx.serve_batch(dm.tables, dm.layers, f, batches[i % nb].n_query, q, u, gamma_ppm, outs)

    dm.ctx.set_profiling(False)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    dm.ctx.set_profiling(2)              # phases, and the first layer's gather apart from its combine
    lat, tim, sizes = [], [], []
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(steps):
        t1 = time.perf_counter()
        step(i)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t1)
        tim.append(dm.ctx.get_timing())             # event times of this step (stream already idle)
        sizes.append(dm.ctx.last_graph_sizes())
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin
    dm.ctx.set_profiling(False)
    return step, np.array(lat) * 1e3, tim, sizes, t_total


def events_off_p50(torch, np, dm, batches, dev_batches, gamma_ppm, outs, n):
    """p50 of the same steps without the HIP events that time the phases (each record costs the host a few
    microseconds, which shows in batches that take 0.1-0.2 ms)."""
    nb = len(batches)
    lat = []
    for i in range(n + 2):
        f, q, u = dev_batches[i % nb]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dm.ctx.serve_batch(dm.tables, dm.layers, f, batches[i % nb].n_query, q, u, gamma_ppm, outs)
        torch.cuda.synchronize()
        if i >= 2:
            lat.append(time.perf_counter() - t1)
    return float(np.percentile(np.array(lat) * 1e3, 50))


def pinned_request_p50(torch, np, dm, batches, dev_batches, gamma_ppm, outs, n):
    """The same steps with the request handed over in pinned host memory (the copy over PCIe is then part of
    the call): context for the latency figure, never the headline value."""
    nb = len(batches)
    pinned = [(torch.from_numpy(b.qe_query).pin_memory(), torch.from_numpy(b.qe_node).pin_memory())
              for b in batches[:min(nb, n + 2)]]
    lat = []
    for i in range(n + 2):
        b = batches[i % len(pinned)]
        f = dev_batches[i % len(pinned)][0]
        qh, uh = pinned[i % len(pinned)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dm.ctx.serve_batch(dm.tables, dm.layers, f, b.n_query, qh.numpy(), uh.numpy(), gamma_ppm, outs)
        torch.cuda.synchronize()
        if i >= 2:
            lat.append(time.perf_counter() - t1)
    return float(np.percentile(np.array(lat) * 1e3, 50))


def summarise(np, layers, table_dtypes, n_query, batches, steps, lat_ms, tim, sizes, t_total, traffic=None):
    """Figures of one measured configuration from the per-step latencies, HIP-event phase times and graph sizes."""
    k = len(layers)
    nb = len(batches)
    e_q = np.array([batches[i % nb].n_edges for i in range(steps)], dtype=np.float64)
    nnz = np.array([s["nnz_in"] for s in sizes], dtype=np.float64)
    rows = np.array([s["rows_in"] for s in sizes], dtype=np.float64)
    edges_per_step = (k - 1) * nnz + e_q
    # dominant kernel: the aggregation of layer 1 (inner layers have the most edges; k = 1: the only layer)
    p0 = layers[0]
    es = 4 if table_dtypes[0] == "f32" else 2
    g_ms = np.array([t.gather_ms[0] for t in tim], dtype=np.float64)
    g_bytes = np.array([algorithmic_gather_bytes(p0.model, p0.d_in, es, int(n), int(r), p0.heads)
                        for n, r in zip(nnz if k > 1 else e_q, rows if k > 1 else np.full_like(rows, n_query))])
    alg_rate = float(g_bytes.mean() / 1e9 / (g_ms.mean() / 1e3))
    # bytes that can have come from HBM: never more than the memory fabric delivered (rows re-read within a launch
    # are partly L2 hits), never more than the algorithm asks for
    moved = float(g_bytes.mean()) if traffic is None else min(float(g_bytes.mean()), float(traffic["hbm_bytes_per_launch"]))
    achieved = moved / 1e9 / (g_ms.mean() / 1e3)
    upd_flops = np.zeros(steps)
    for l, p in enumerate(layers):
        r_l = rows if l < k - 1 else np.full_like(rows, n_query)
        upd_flops += r_l * 2.0 * p.d_in * p.d_out * (2 if p.model == "sage" else 1)
    upd_ms = np.array([sum(t.update_ms[l] for l in range(k)) for t in tim])
    gather_ms = np.array([sum(t.gather_ms[l] + t.combine_ms[l] for l in range(k)) for t in tim])
    build_ms = np.array([t.build_ms for t in tim])
    upd_tflops = float(upd_flops.mean() / (upd_ms.mean() / 1e3) / 1e12)
    kernel = "k_gat" if p0.model == "gat" else "k_gather"
    roof = {"bound": "hbm", "kernel": f"{kernel} (layer 1)", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": None if traffic is None else float(traffic["hbm_bytes_per_launch"]),
            "algorithmic_bytes_per_launch": float(g_bytes.mean()), "algorithmic_rate": alg_rate,
            "avg_launch_ms": float(g_ms.mean())}
    if traffic is not None:
        roof["traffic_source"] = {k2: traffic[k2] for k2 in ("file", "command", "batches", "scale_factor") if k2 in traffic}
        roof["note"] = ("achieved = min(algorithmic bytes, bytes the memory fabric delivered by counters) per launch / "
                        "average launch time; algorithmic_rate counts every row read and can exceed the peak when a "
                        "launch re-reads rows that it finds in L2; traffic is a citation of the named profile, not a "
                        "measurement of this run")
    return {
        "value": float(edges_per_step.sum() / t_total), "ms_per_step": t_total * 1e3 / steps,
        "p50_latency_ms": float(np.percentile(lat_ms, 50)), "p10_latency_ms": float(np.percentile(lat_ms, 10)),
        "p90_latency_ms": float(np.percentile(lat_ms, 90)),
        "phase_ms": {"build": float(build_ms.mean()), "gather": float(gather_ms.mean()), "update": float(upd_ms.mean())},
        "gather_edges_per_s": float(edges_per_step.mean() / (gather_ms.mean() / 1e3)),
        "sizes": {"mean_query_edges": float(e_q.mean()), "mean_rows_in": float(rows.mean()), "mean_nnz_in": float(nnz.mean())},
        "roofline": roof,
        "update_roofline": {"bound": "mfma", "kernel": "k_update (all layers)", "achieved": upd_tflops,
                            "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": upd_tflops / MFMA_F32_PEAK_TFLOPS,
                            "flops_per_step": float(upd_flops.mean()), "ms_per_step": float(upd_ms.mean())},
    }


def row_rel_err(np, got, ref) -> float:
    num = np.abs(got - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), 1e-30)
    return float(np.max(num / den)) if ref.size else 0.0


def oracle_check(torch, np, dm, built, qb, dev, gamma_ppm, outs, sample=None):
    """One batch on the GPU against the CPU oracle: all query rows, or a sample of them for the batches whose
    whole evaluation would take the oracle minutes.  Also the oracle's own speed on that batch (one thread)."""
    from oracle import srpe_oracle as orc
    from threadpoolctl import threadpool_limits
    f, q, u = dev
    dm.ctx.serve_batch(dm.tables, dm.layers, f, qb.n_query, q, u, gamma_ppm, outs)
    torch.cuda.synchronize()
    got = outs[:qb.n_query].cpu().numpy().astype(np.float64)
    k = len(built.layers)
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query, qb.qe_node,
                                         gamma_ppm)
        tabs = [orc.LazyTable(t.data, t.dtype, t.dim) for t in built.tables]
        if sample is None:
            ref = orc.srpe_reference(og, tabs, built.layers, qb.feats)
            rows = np.arange(qb.n_query)
        else:
            rows = np.sort(np.asarray(sample))
            ref = orc.srpe_reference_rows(og, tabs, built.layers, qb.feats, rows)
        dt = time.perf_counter() - t0
    out = {"max_row_rel_err_vs_oracle": row_rel_err(np, got[rows], ref), "oracle_rows_compared": int(rows.size),
           "oracle_seconds": round(dt, 2)}
    if sample is None:
        out["oracle_edges_per_s_1_thread"] = ((k - 1) * og.nnz_in + int(og.indptr[qb.n_query])) / dt
    return out


def measure_config(torch, np, dm, built, cfg_text, batches, gamma_ppm, steps, warmup, sample=None, host_steps=8):
    """One entry of the `configs` object."""
    n_query = batches[0].n_query
    dev = to_device(torch, batches)
    outs = torch.empty((n_query, dm.out_width()), dtype=torch.float32, device="cuda:0")
    _, lat_ms, tim, sizes, t_total = timed_steps(torch, np, dm, batches, dev, gamma_ppm, outs, steps, warmup)
    r = summarise(np, built.layers, [t.dtype for t in built.tables], n_query, batches, steps, lat_ms, tim, sizes, t_total)
    r = {"workload": cfg_text, "unit": "edges/s", "steps": steps, "warmup": warmup, "distinct_batches": len(batches), **r}
    r["p50_latency_ms_phase_events_off"] = events_off_p50(torch, np, dm, batches, dev, gamma_ppm, outs, min(steps, 40))
    r["p50_latency_ms_request_in_pinned_host_memory"] = pinned_request_p50(torch, np, dm, batches, dev, gamma_ppm, outs,
                                                                           host_steps)
    r.update(oracle_check(torch, np, dm, built, batches[0], dev[0], gamma_ppm, outs, sample))
    return r


def other_configs(args, torch, np, budget_s):
    """Every configuration of the baseline file besides the headline one, each measured like the headline."""
    from paper_2501_08547_amd import device
    from synth import CONFIGS, build_workload
    out = {}

    def over_budget(name):
        if time.perf_counter() - T_START > budget_s:
            out[name] = {"skipped": f"time budget of {budget_s:.0f} s for the whole run was used up"}
            log(f"{name}: skipped (time budget)")
            return True
        return False

    def guarded(name, fn):
        """A configuration that fails is reported as failed; the line with the others is still printed."""
        try:
            fn()
        except Exception as e:                              # noqa: BLE001 - reported in the output, not swallowed
            out[name + "_error"] = f"{type(e).__name__}: {e}"
            log(f"{name}: FAILED {type(e).__name__}: {e}")
        torch.cuda.empty_cache()

    # Tiny, with precomputed embeddings from exact inference on the base graph
    def run_tiny():
        from oracle import exact_inference as ex
        from oracle import srpe_oracle as orc
        built = build_workload(CONFIGS["tiny"], pe_fn=lambda g, ft, ly: ex.base_inference(
            g.indptr, g.indices, orc.decode_table(ft.data, ft.dtype, ft.dim), ly))
        dm = device.upload(built, "cuda:0")
        batches = [built.batch(r) for r in range(32)]
        out["tiny"] = measure_config(torch, np, dm, built, workload_text(built.cfg, built), batches, built.cfg.gamma_ppm, 100, 10)
        dm.close()
        log(f"tiny: p50 {out['tiny']['p50_latency_ms']:.3f} ms")
    if not over_budget("tiny"):
        guarded("tiny", run_tiny)

    # Large (sweep of the recompute fraction) and Attention share one graph
    shared = {}

    def run_large():
        built = build_workload(CONFIGS["large"])
        shared["graph"] = built.graph
        log("large: generated")
        dm = device.upload(built, "cuda:0")
        batches = [built.batch(r) for r in range(16)]
        rng = np.random.default_rng(7)
        for gamma in (0, 50_000, 200_000, 1_000_000):
            key = f"large_gamma_{gamma // 10_000}pct"
            if over_budget(key):
                continue
            full = gamma == 1_000_000       # 27 M edges per inner layer: the oracle takes two sampled rows, not the batch
            out[key] = measure_config(torch, np, dm, built, workload_text(built.cfg, built, gamma), batches[:4] if full else batches,
                                      gamma, 12 if full else 60, 3 if full else 10,
                                      sample=rng.choice(built.cfg.batch, 2, replace=False) if full else None,
                                      host_steps=4 if full else 8)
            log(f"{key}: p50 {out[key]['p50_latency_ms']:.3f} ms, err {out[key]['max_row_rel_err_vs_oracle']:.2e}")
        dm.close()
    if not over_budget("large"):
        guarded("large", run_large)

    def run_attention():
        built = build_workload(CONFIGS["attention"], graph=shared.get("graph"))
        shared.clear()
        dm = device.upload(built, "cuda:0")
        batches = [built.batch(r) for r in range(16)]
        out["attention"] = measure_config(torch, np, dm, built, workload_text(built.cfg, built), batches,
                                          built.cfg.gamma_ppm, 60, 10)
        log(f"attention: p50 {out['attention']['p50_latency_ms']:.3f} ms, err {out['attention']['max_row_rel_err_vs_oracle']:.2e}")
        dm.close()
    if not over_budget("attention"):
        guarded("attention", run_attention)
    shared.clear()

    # Scale: batch sizes 1 .. 16,384 on the 111 M-node graph
    def run_scale():
        from synth import scale as S
        spec, ip, cfg, built, dm = hash_workload("scale", 1024, 50_000)
        log("scale: generated")
        for nq in (1, 64, 1024, 16384):
            key = f"scale_batch_{nq}"
            if over_budget(key):
                continue
            batches = [S.make_scale_batch(spec, ip, nq, 2000 + r) for r in range(8 if nq < 16384 else 4)]
            out[key] = measure_config(torch, np, dm, built, workload_text(cfg, built, batch=nq), batches, cfg.gamma_ppm, 60, 10,
                                      sample=None if nq <= 1024 else np.random.default_rng(5).choice(nq, 64, replace=False))
            log(f"{key}: p50 {out[key]['p50_latency_ms']:.3f} ms, err {out[key]['max_row_rel_err_vs_oracle']:.2e}")
        dm.close()
    if not over_budget("scale"):
        guarded("scale", run_scale)

    # FB10B-shaped: 2 KB rows scattered over a 61 GB table, each read once: the gather with no reuse to find in a cache
    def run_fb10b():
        from synth import scale as S
        spec, ip, cfg, built, dm = hash_workload("fb10b", 1024, 50_000)
        log("fb10b: generated")
        batches = [S.make_scale_batch(spec, ip, 1024, 2000 + r) for r in range(6)]
        key = "fb10b_batch_1024"
        out[key] = measure_config(torch, np, dm, built, workload_text(cfg, built), batches, cfg.gamma_ppm, 40, 6,
                                  sample=np.random.default_rng(6).choice(1024, 4, replace=False), host_steps=4)
        out[key]["note"] = ("HBM-bound reference: the layer-1 gather reads 2 KB rows scattered over a 61 GB table, nearly "
                            "every row once; nothing of it can come from a cache")
        log(f"fb10b: p50 {out[key]['p50_latency_ms']:.3f} ms, gather frac {out[key]['roofline']['frac']:.3f}")
        dm.close()
    if not over_budget("fb10b_batch_1024"):
        guarded("fb10b", run_fb10b)
    return out


def partitioned_share(args, torch, np, dm, built, cfg, batches, dev_batches, outs_ref):
    """The batches once more as P partitions' shares (Sec. 6): per step the whole graph, then for every
    partition its graph and, layer by layer, its local aggregations, then the merge and update of all rows.
    Times are HIP-event times on the library's stream (torch's current stream), averaged over the steps; a
    partition's share is its graph + its local aggregations + 1 / P of the merges (a GPU merges the rows it owns)."""
    from paper_2501_08547_amd import binding as B
    from synth import hash_partition
    P = args.partitions
    k = cfg.k
    pad8 = lambda w: (w + 7) // 8 * 8
    node_part = torch.from_numpy(hash_partition(built.graph.n, P, seed=77)).cuda()
    parts = [None] * P
    g = None
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_graph, t_local, t_merge, rec_bytes = [], [[] for _ in range(k)], [[] for _ in range(k)], [0] * k
    err = 0.0
    steps = max(4, min(args.steps, 20))
    for i in range(-2, steps):                                         # two untimed rounds first
        b = batches[i % N_BATCHES]
        f, q, u = dev_batches[i % N_BATCHES]
        g = dm.ctx.build_computation_graph(b.n_query, q, u, cfg.gamma_ppm, graph=g)
        rows_in = g.sizes()["rows_in"]
        marks = []
        for p in range(P):
            e0, e1 = ev(), ev()
            e0.record()
            parts[p] = dm.ctx.cgp_partition_graph(g, node_part, P, p, part_graph=parts[p])
            e1.record()
            marks.append((e0, e1))
        buf0 = torch.zeros((rows_in, pad8(cfg.dims[0])), dtype=torch.float32, device="cuda:0")
        dm.ctx.init_buffer(g, dm.tables[0], f, buf0)
        buf = buf0
        lmarks = []
        for l in range(1, k + 1):
            last = l == k
            p_l = built.layers[l - 1]
            lay = dm.layers[l - 1] if p_l.model != "gcnii" else B.make_layer(p_l, dm.weights[l - 1], init_rows=buf0)
            n_rows = b.n_query if last else rows_in
            wire = torch.empty((P, n_rows, B.cgp_wire_width(lay)), dtype=torch.float32, device="cuda:0")
            rec_bytes[l - 1] = wire[0].numel() * 4
            row_mean = None
            es = [ev() for _ in range(P + 2)]
            if p_l.model == "sage" and p_l.aggregator == "moment":
                for p in range(P):
                    dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p])
                row_mean = torch.empty((n_rows, pad8(p_l.d_in)), dtype=torch.float32, device="cuda:0")
                dm.ctx.cgp_merge_mean(wire, lay, row_mean)
            for p in range(P):
                es[p].record()
                dm.ctx.cgp_local_aggregate(parts[p], last, dm.tables[l - 1], buf, lay, wire[p], row_mean=row_mean)
            es[P].record()
            nxt = torch.empty((n_rows, pad8(p_l.out_width)), dtype=torch.float32, device="cuda:0")
            dm.ctx.cgp_merge_update(wire, lay, buf, nxt)
            es[P + 1].record()
            lmarks.append(es)
            buf = nxt
        torch.cuda.synchronize()
        if i < 0:
            continue
        t_graph.append(np.mean([a.elapsed_time(c) for a, c in marks]))
        for l in range(k):
            es = lmarks[l]
            t_local[l].append(np.mean([es[p].elapsed_time(es[p + 1]) for p in range(P)]))
            t_merge[l].append(es[P].elapsed_time(es[P + 1]))
        if i == 0:
            # against the unpartitioned library on the same batch (both against the oracle in the tests)
            dm.ctx.serve_batch(dm.tables, dm.layers, f, b.n_query, q, u, cfg.gamma_ppm, outs_ref)
            torch.cuda.synchronize()
            w = built.layers[-1].out_width
            a, c = buf[:, :w].double(), outs_ref[:, :w].double()
            err = float(((a - c).abs().amax(dim=1) / c.abs().amax(dim=1).clamp_min(1e-30)).max())
    for pg in parts:
        pg.destroy()
    g.destroy()
    local = [float(np.mean(t)) for t in t_local]
    merge = [float(np.mean(t)) for t in t_merge]
    share = float(np.mean(t_graph)) + sum(local) + sum(merge) / P
    return {"partitions": P, "placement": "hash", "steps": steps,
            "partition_graph_ms": float(np.mean(t_graph)),
            "local_aggregation_ms_per_layer": local, "merge_update_ms_per_layer_all_rows": merge,
            "record_bytes_per_partition_per_layer": rec_bytes,
            "one_partition_share_ms": share,
            "note": "graph of one partition + its local aggregations + 1/P of the merges; excludes the whole graph's "
                    "construction and the exchange of the records between GPUs",
            "max_row_rel_err_vs_unpartitioned": err}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mid", help="mid (default) | large | attention | scale | fb10b | tiny ...")
    ap.add_argument("--configs", default="", choices=["", "all", "headline"],
                    help="all: besides the headline workload, measure every other configuration of the baseline file "
                         "(object `configs`); headline: only --workload.  Default: all for a plain run of `mid`, "
                         "headline as soon as the workload or its shape is overridden")
    ap.add_argument("--time-budget", type=float, default=420.0,
                    help="seconds after which no further configuration of --configs all is started (it is then "
                         "reported as skipped)")
    ap.add_argument("--batch", type=int, default=0, help="override the number of queries per batch")
    ap.add_argument("--distinct-batches", type=int, default=200,
                    help="number of distinct seeded batches the steps cycle through (generated on the host before the "
                         "timed region; 200 of workload mid take about ten seconds to generate)")
    ap.add_argument("--gamma-ppm", type=int, default=-1,
                    help="override the recomputation budget (parts per million of the candidates; the paper's gamma)")
    ap.add_argument("--layers", type=int, default=0,
                    help="override the number of layers k (hidden width repeated): latency against depth, App. 'Impact of "
                         "Number of Layers'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--core-only", action="store_true",
                    help="only the warm-up and the timed steps of --workload (no CPU baseline, no host-memory request "
                         "timing, no second stream, no other configuration): what the profiler runs, so that every "
                         "dispatch belongs to a counted step")
    ap.add_argument("--streams", type=int, default=2,
                    help="> 1: after the standard measurement, also serve the same batches through this many contexts "
                         "on streams of their own, so that consecutive batches overlap (request-stream throughput, "
                         "reported as an extra object; the headline value stays one batch at a time)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB a few times (reference for HBM counters)")
    ap.add_argument("--poisson", default="", metavar="LOADS",
                    help="with --streams S > 1: also serve requests that arrive as a Poisson process (seeded), at each of "
                         "these fractions of the measured request-stream throughput, e.g. 0.25,0.5,0.75,0.9, and report "
                         "the latency from arrival to completion (extra object `poisson`)")
    ap.add_argument("--partitions", type=int, default=0, metavar="P",
                    help="> 1: after the standard measurement, also execute the batches as the shares of P hash-placed "
                         "partitions, one after the other on this GPU (computation graph parallelism, Sec. 6), and "
                         "report what ONE partition's share costs, as the extra object `partitioned`; the exchange "
                         "of the records between GPUs is not part of it")
    ap.add_argument("--read-calibration", action="store_true",
                    help="only measure the rate of a plain read sweep over buffers that fit the memory-side cache and "
                         "over ones that do not (the delivery ceiling the gather is set against)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box; nothing here uses a second). "
              "Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    global N_BATCHES
    N_BATCHES = max(1, args.distinct_batches)
    if args.core_only:
        args.no_cpu_baseline = True
        args.streams = 1
    plain = (args.workload == "mid" and not args.batch and args.gamma_ppm < 0 and not args.layers and not args.poisson
             and not args.partitions)
    if not args.configs:
        args.configs = "all" if plain and not args.core_only else "headline"

    if args.copy_calibration > 0:
        import torch
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": args.copy_calibration, "reads_MiB": args.copy_calibration,
                          "writes_MiB": args.copy_calibration, "launches": 5}))
        return 0
    if args.read_calibration:
        import torch
        from paper_2501_08547_amd import binding
        tiny = torch.zeros(2, dtype=torch.int64, device="cuda:0")
        ctx = binding.Context(tiny, torch.zeros(1, dtype=torch.int32, device="cuda:0"))
        rows = []
        for mib in (64, 128, 256, 512, 2048):
            buf = torch.zeros(mib << 18, dtype=torch.float32, device="cuda:0")
            for blocks in (2048, 4096):
                nbytes, ms = ctx.measure_read_rate(buf, 16 if mib <= 256 else 4, blocks)
                rows.append({"MiB": mib, "blocks": blocks, "ms": round(ms, 4), "TB_per_s": round(nbytes / ms / 1e9, 3)})
            del buf
        ctx.close()
        print(json.dumps({"read_calibration": rows}))
        return 0

    # ---- host side of the headline workload, and the CPU oracle on it, before the GPU is touched
    hashed = args.workload in ("scale", "fb10b")
    ref = og = cpu = None
    if not hashed:
        cfg, built = host_synth(args.workload, args)
        log(f"workload {cfg.name}: {built.graph.n} nodes, {built.graph.nnz} directed edges generated")
        batches = [built.batch(r) for r in range(N_BATCHES)]
        log(f"{N_BATCHES} batches generated")
        if not args.no_cpu_baseline:
            ref, og, cpu = cpu_baseline(built, batches, cfg.gamma_ppm)
            log(f"CPU oracle: {cpu['value']:.3g} edges/s on 1 thread"
                + (f", {cpu['all_cores']['value']:.3g} on {cpu['all_cores']['cores']} cores" if "all_cores" in cpu else ""))

    import torch
    from paper_2501_08547_amd import device
    if hashed:
        from synth import scale as S
        spec, ip, cfg, built, dm = hash_workload(args.workload, args.batch or 1024,
                                                 args.gamma_ppm if args.gamma_ppm >= 0 else 50_000)
        batches = [S.make_scale_batch(spec, ip, cfg.batch, 2000 + r) for r in range(N_BATCHES)]
        if not args.no_cpu_baseline:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):            # (the GPU is initialised already: one thread, no processes)
                edges = spent = used = 0
                for qb in batches:
                    r_, og_, e, dt = _oracle_batch(built, qb, cfg.gamma_ppm)
                    if ref is None:
                        ref, og = r_, og_
                    edges, spent, used = edges + e, spent + dt, used + 1
                    if spent >= 10.0:
                        break
            cpu = {"value": edges / spent, "unit": "edges/s", "cores": 1, "kind": "oracle", "seconds": round(spent, 2),
                   "sample": f"the first {used} of the workload's batches, graph construction + {cfg.k} layers per batch, "
                             f"numpy fp64 with hash-defined table rows, 1 thread", "host_cpus_visible": os.cpu_count()}
    else:
        dm = device.upload(built, "cuda:0")
    log("uploaded")
    dev_batches = to_device(torch, batches)
    outs = torch.empty((cfg.batch, dm.out_width()), dtype=torch.float32, device="cuda:0")
    k = cfg.k

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"gather_{cfg.name}_traffic.json")
    if os.path.exists(tpath) and plain:
        traffic = json.load(open(tpath))

    # ---- timed region: exactly `steps` steps; each ends when its output is ready
    step, lat_ms, tim, sizes, t_total = timed_steps(torch, np, dm, batches, dev_batches, cfg.gamma_ppm, outs,
                                                    args.steps, args.warmup)
    s = summarise(np, built.layers, [t.dtype for t in built.tables], cfg.batch, batches, args.steps, lat_ms, tim, sizes,
                  t_total, traffic)
    total_edges = s["value"] * t_total
    result = {
        "metric": "aggregated edges/sec over the whole query-batch path (p50 latency and gather GB/s alongside)",
        "value": s["value"],
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": s["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",          # arithmetic type of the path (tables may be stored as bf16)
        "data": "synthetic",
        "config": {"workload": workload_text(cfg, built), "distinct_batches": N_BATCHES, **s["sizes"]},
        "p50_latency_ms": s["p50_latency_ms"],
        "p10_latency_ms": s["p10_latency_ms"],
        "p90_latency_ms": s["p90_latency_ms"],
        "phase_ms": s["phase_ms"],
        "gather_edges_per_s": s["gather_edges_per_s"],
        "roofline": s["roofline"],
        "update_roofline": s["update_roofline"],
    }
    log(f"{cfg.name}: p50 {s['p50_latency_ms']:.3f} ms")

    if not args.core_only:
        result["p50_latency_ms_phase_events_off"] = events_off_p50(torch, np, dm, batches, dev_batches, cfg.gamma_ppm, outs,
                                                                   min(args.steps, 50))
        result["p50_latency_ms_request_in_pinned_host_memory"] = pinned_request_p50(
            torch, np, dm, batches, dev_batches, cfg.gamma_ppm, outs, max(8, args.steps // 4))

    if args.streams > 1:
        # Request-stream throughput (the paper's Sec. 8.4 serves a stream of requests): consecutive batches go
        # to different contexts, each on its own stream, so the graph construction of one batch runs while the
        # previous batch aggregates.  One host thread; a call returns once its layers are queued.
        streams = [torch.cuda.Stream(device="cuda:0") for _ in range(args.streams)]
        models = [device.second_context(dm, st.cuda_stream) for st in streams]
        outs_s = [torch.empty_like(outs) for _ in streams]

        def step_s(i):
            j = i % args.streams
            b = batches[i % N_BATCHES]
            f, q, u = dev_batches[i % N_BATCHES]
            models[j].ctx.serve_batch(models[j].tables, models[j].layers, f, b.n_query, q, u, cfg.gamma_ppm, outs_s[j])

        for i in range(max(args.warmup, 2 * args.streams)):
            step_s(i)
        torch.cuda.synchronize()
        t_b = time.perf_counter()
        for i in range(args.steps):
            step_s(i)
        torch.cuda.synchronize()
        t_s = time.perf_counter() - t_b
        step(args.steps - 1)
        torch.cuda.synchronize()
        same = bool(torch.equal(outs_s[(args.steps - 1) % args.streams].cpu(), outs.cpu()))
        result["overlapped"] = {"streams": args.streams, "value": total_edges / t_s, "unit": "edges/s",
                                "ms_per_step": t_s * 1e3 / args.steps, "steps": args.steps,
                                "speedup_vs_one_stream": t_total / t_s, "last_output_identical": same}
        if args.poisson:
            # Open-loop arrivals (the paper's throughput experiment models request arrivals as a Poisson process):
            # one host thread hands each request to the next context when it arrives, or as soon as the thread is
            # free again; latency runs from the arrival to the completion of the request's last kernel.
            max_rate = args.steps / t_s
            rows_p = []
            for load in [float(x) for x in args.poisson.split(",") if x]:
                rate = load * max_rate
                n_req = 400
                rng = np.random.Generator(np.random.PCG64([int(load * 1000), 31]))
                arr = np.cumsum(rng.exponential(1.0 / rate, size=n_req))
                done = [torch.cuda.Event(enable_timing=True) for _ in range(n_req)]
                base_ev = torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                base_ev.record()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for i in range(n_req):
                    while time.perf_counter() - t0 < arr[i]:
                        pass
                    step_s(i)
                    done[i].record(streams[i % args.streams])
                torch.cuda.synchronize()
                t_end = time.perf_counter() - t0
                lat = np.array([base_ev.elapsed_time(done[i]) / 1e3 - arr[i] for i in range(n_req)]) * 1e3
                rows_p.append({"load": load, "rate_per_s": rate, "achieved_rate_per_s": n_req / t_end, "requests": n_req,
                               "p50_ms": float(np.percentile(lat, 50)), "p90_ms": float(np.percentile(lat, 90)),
                               "p99_ms": float(np.percentile(lat, 99))})
            result["poisson"] = {"streams": args.streams, "max_rate_per_s": max_rate, "loads": rows_p,
                                 "note": "latency = completion of the request's last kernel minus its arrival time; the "
                                         "two clocks are aligned by one synchronisation (some 10 us of slack)"}
        for m in models:
            m.close()

    if args.partitions > 1 and not hashed:
        result["partitioned"] = partitioned_share(args, torch, np, dm, built, cfg, batches, dev_batches, outs)

    if cpu is not None:
        result["cpu_baseline"] = cpu
        # the batch the oracle computed first, once more on the GPU: the benchmark's own parity check
        f, q, u = dev_batches[0]
        dm.ctx.serve_batch(dm.tables, dm.layers, f, batches[0].n_query, q, u, cfg.gamma_ppm, outs)
        torch.cuda.synchronize()
        result["max_row_rel_err_vs_oracle"] = row_rel_err(np, outs.cpu().numpy().astype(np.float64), ref)
    dm.close()
    del dm, dev_batches, outs
    if args.configs == "all":
        built = batches = None
        torch.cuda.empty_cache()
        result["configs"] = other_configs(args, torch, np, args.time_budget)
    result["bench_wall_seconds"] = round(time.perf_counter() - T_START, 1)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
