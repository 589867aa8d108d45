#!/usr/bin/env python3
"""Benchmark of the single-GPU SRPE serving path.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mid]

One step = omg_serve_batch on one query batch: computation-graph construction plus every
GNN layer.  The base graph, the tables, the weights and the batches (features and edge
lists) are in device memory before the timed region starts.  Prints ONE JSON line.
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

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3 # MI355X dense fp32 matrix peak
N_BATCHES = 200             # distinct seeded batches cycled through the steps (--distinct-batches)


def algorithmic_gather_bytes(model: str, d_in: int, elem_bytes: int, nnz: int, rows: int, heads: int = 1) -> int:
    """Bytes the aggregation of one layer has to move: per edge the source row, its column id and
    (GCN) the source degree or (GAT) the per-head source score; per row the two row pointers and
    (GCN) its own previous embedding."""
    per_edge = d_in * elem_bytes + 4
    per_row = 8
    if model == "gcn":
        per_edge += 4
        per_row += d_in * 4
    if model == "gat":
        per_edge += 4 * heads
        per_row += 4 * heads
    return nnz * per_edge + rows * per_row


def cpu_baseline(built, batches, gamma_ppm, min_seconds=10.0):
    """The CPU oracle as it stands, timed on the first batches of the same workload (one thread): whole
    batches until at least min_seconds of oracle work are on the clock.  Returns the first batch's reference
    output and graph, and the baseline object."""
    from threadpoolctl import threadpool_limits
    from oracle import srpe_oracle as orc
    k = len(built.layers)
    tabs = [orc.LazyTable(t.data, t.dtype, t.dim) for t in built.tables]
    edges, spent, used, first = 0, 0.0, 0, None
    with threadpool_limits(limits=1):
        for qb in batches:
            t0 = time.perf_counter()
            og = orc.build_computation_graph(built.graph.indptr, built.graph.indices, qb.n_query, qb.qe_query,
                                             qb.qe_node, gamma_ppm)
            ref = orc.srpe_reference(og, tabs, built.layers, qb.feats)
            spent += time.perf_counter() - t0
            edges += (k - 1) * og.nnz_in + int(og.indptr[qb.n_query])
            used += 1
            if first is None:
                first = (ref, og)
            if spent >= min_seconds:
                break
    qb = batches[0]
    return first[0], first[1], {"value": edges / spent, "unit": "edges/s", "cores": 1, "kind": "oracle",
                                "seconds": round(spent, 2),
                                "sample": f"the first {used} of the workload's batches ({qb.n_query} queries and about "
                                          f"{qb.n_edges} query edges each), graph construction + {k} layers per batch, "
                                          f"numpy fp64, 1 thread"}


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


def _last_out(step, i, outs, torch):
    """Output of step i served the ordinary way (one context), for comparison."""
    step(i)
    torch.cuda.synchronize()
    return outs.cpu()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mid", help="mid (default) | large | attention | scale | fb10b | tiny ...")
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
                    help="only the warm-up and the timed steps (no CPU baseline, no host-memory request timing, no "
                         "second stream): what the profiler runs, so that every dispatch belongs to a counted step")
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
    import torch
    global N_BATCHES
    N_BATCHES = max(1, args.distinct_batches)
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": args.copy_calibration, "reads_MiB": args.copy_calibration,
                          "writes_MiB": args.copy_calibration, "launches": 5}))
        return 0
    from paper_2501_08547_amd import device
    from synth import CONFIGS, build_workload
    if args.read_calibration:
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

    t0 = time.perf_counter()
    if args.workload in ("scale", "fb10b"):
        # scale: 111 M nodes / 1.67 G edges / three 28 GB bf16 tables; fb10b: 30 M nodes / 9.8 G edges / 1,024
        # features (61 GB bf16) + two 7.7 GB tables; hash-defined and generated on the device
        from types import SimpleNamespace
        from synth import scale as S
        spec = S.ScaleSpec() if args.workload == "scale" else S.fb10b_spec()
        ip = S.indptr_np(spec)
        nnz = int(ip[-1])
        indptr, indices, tabs = S.device_arrays(spec, ip, "cuda:0")
        layers = S.scale_layers(spec)
        dm = device.assemble(indptr, indices, [(t, "bf16", d) for t, d in zip(tabs, spec.dims[:-1])], layers)
        n_batch = args.batch or 1024
        cfg = SimpleNamespace(name=args.workload, model="sage", dims=spec.dims, k=spec.k, batch=n_batch,
                              gamma_ppm=args.gamma_ppm if args.gamma_ppm >= 0 else 50_000,
                              feat_dtype="bf16", pe_dtype="bf16")
        built = SimpleNamespace(cfg=cfg, layers=layers,
                                graph=SimpleNamespace(n=spec.n_nodes, nnz=nnz, indptr=ip,
                                                      indices=S.HashIndices(spec.n_nodes, nnz, spec.seed_graph)),
                                tables=[SimpleNamespace(data=S.HashTable(spec.n_nodes, d, spec.seed_table, t),
                                                        dtype="bf16", dim=d) for t, d in enumerate(spec.dims[:-1])])
        batches = [S.make_scale_batch(spec, ip, n_batch, 2000 + r) for r in range(N_BATCHES)]
    else:
        cfg = CONFIGS[args.workload]
        from dataclasses import replace
        if args.batch:
            cfg = replace(cfg, batch=args.batch)
        if args.gamma_ppm >= 0:
            cfg = replace(cfg, gamma_ppm=args.gamma_ppm)
        if args.layers:
            d = cfg.dims
            cfg = replace(cfg, dims=(d[0],) + (d[1],) * (args.layers - 1) + (d[-1],))
        built = build_workload(cfg)
        dm = device.upload(built, "cuda:0")
        batches = [built.batch(r) for r in range(N_BATCHES)]
    print(f"[bench] workload {cfg.name}: {built.graph.n} nodes, {built.graph.nnz} directed edges "
          f"({time.perf_counter() - t0:.1f}s to generate and upload)", file=sys.stderr, flush=True)
    dev_batches = [(torch.from_numpy(b.feats).cuda(), torch.from_numpy(b.qe_query).cuda(),
                    torch.from_numpy(b.qe_node).cuda()) for b in batches]
    outs = torch.empty((cfg.batch, dm.out_width()), dtype=torch.float32, device="cuda:0")
    k = cfg.k

    def step(i):
        b = batches[i % N_BATCHES]
        f, q, u = dev_batches[i % N_BATCHES]
        dm.ctx.serve_batch(dm.tables, dm.layers, f, b.n_query, q, u, cfg.gamma_ppm, outs)

    dm.ctx.set_profiling(False)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps; each ends when its output is ready
    dm.ctx.set_profiling(True)
    lat, tim, sizes = [], [], []
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        t1 = time.perf_counter()
        step(i)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t1)
        tim.append(dm.ctx.get_timing())             # event times of this step (stream already idle)
        sizes.append(dm.ctx.last_graph_sizes())
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin

    lat_ms = np.array(lat) * 1e3
    e_q = np.array([batches[i % N_BATCHES].n_edges for i in range(args.steps)], dtype=np.float64)
    nnz = np.array([s["nnz_in"] for s in sizes], dtype=np.float64)
    rows = np.array([s["rows_in"] for s in sizes], dtype=np.float64)
    edges_per_step = (k - 1) * nnz + e_q
    total_edges = float(edges_per_step.sum())

    # dominant kernel: the gather-reduce of layer 1 (inner layers have the most edges)
    p0 = built.layers[0]
    es = 4 if built.tables[0].dtype == "f32" else 2
    g_ms = np.array([t.gather_ms[0] for t in tim], dtype=np.float64)
    g_bytes = np.array([algorithmic_gather_bytes(p0.model, p0.d_in, es, int(n), int(r), p0.heads)
                        for n, r in zip(nnz if k > 1 else e_q, rows if k > 1 else np.full_like(rows, cfg.batch))])
    achieved = float(g_bytes.mean() / 1e9 / (g_ms.mean() / 1e3))
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"gather_{cfg.name}_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
    # update phase: flops of the dense products against the fp32 matrix-core peak
    upd_flops = np.zeros(args.steps)
    for l, p in enumerate(built.layers):
        r_l = rows if l < k - 1 else np.full_like(rows, cfg.batch)
        upd_flops += r_l * 2.0 * p.d_in * p.d_out * (2 if p.model == "sage" else 1)
    upd_s = np.array([sum(t.update_ms[l] for l in range(k)) for t in tim]) / 1e3
    upd_tflops = float(upd_flops.mean() / upd_s.mean() / 1e12)
    gather_all_ms = np.array([sum(t.gather_ms[l] + t.combine_ms[l] for l in range(k)) for t in tim])
    update_all_ms = np.array([sum(t.update_ms[l] for l in range(k)) for t in tim])
    build_ms = np.array([t.build_ms for t in tim])

    result = {
        "metric": "aggregated edges/sec over the whole query-batch path (p50 latency and gather GB/s alongside)",
        "value": total_edges / t_total,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_total * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",          # arithmetic type of the path (tables may be stored as bf16)
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {built.graph.n} nodes, {built.graph.nnz} directed edges, "
                               f"{cfg.model} {'-'.join(map(str, cfg.dims))}, tables {cfg.feat_dtype}/{cfg.pe_dtype}, "
                               f"batch {cfg.batch}, gamma {cfg.gamma_ppm / 1e4:.2f}%",
                   "distinct_batches": N_BATCHES,
                   "mean_query_edges": float(e_q.mean()), "mean_rows_in": float(rows.mean()),
                   "mean_nnz_in": float(nnz.mean())},
        "p50_latency_ms": float(np.percentile(lat_ms, 50)),
        "p10_latency_ms": float(np.percentile(lat_ms, 10)),
        "p90_latency_ms": float(np.percentile(lat_ms, 90)),
        "phase_ms": {"build": float(build_ms.mean()), "gather": float(gather_all_ms.mean()),
                     "update": float(update_all_ms.mean())},
        "gather_edges_per_s": float(edges_per_step.mean() / (gather_all_ms.mean() / 1e3)),
        "roofline": {"bound": "hbm", "kernel": "k_gather (layer 1)", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": float(g_bytes.mean()), "avg_launch_ms": float(g_ms.mean()),
                     "note": "algorithmic bytes over the HBM peak; a batch that reads the rows of a table several times over "
                             "in table-region order finds part of them in the L2 caches (`traffic`, the bytes the "
                             "memory fabric delivered, is below the algorithmic bytes), so this can exceed 1; a plain "
                             "read sweep on the same GPU is delivered 7.0-7.3 TB/s (--read-calibration)"},
        "update_roofline": {"bound": "mfma", "kernel": "k_update (all layers)", "achieved": upd_tflops,
                            "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": upd_tflops / MFMA_F32_PEAK_TFLOPS,
                            "flops_per_step": float(upd_flops.mean()), "ms_per_step": float(upd_s.mean() * 1e3)},
    }

    # the same steps with the request handed over in pinned host memory (the copy over PCIe is then part of
    # the call): context for the latency figure, never the headline value
    if args.core_only:
        args.no_cpu_baseline = True
        args.streams = 1
    n_host = 0 if args.core_only else max(8, args.steps // 4)
    pinned = [(torch.from_numpy(b.qe_query).pin_memory(), torch.from_numpy(b.qe_node).pin_memory()) for b in batches]
    lat_h = []
    dm.ctx.set_profiling(False)
    for i in range(n_host + 2 if n_host else 0):
        b = batches[i % N_BATCHES]
        f = dev_batches[i % N_BATCHES][0]
        qh, uh = pinned[i % N_BATCHES]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        dm.ctx.serve_batch(dm.tables, dm.layers, f, b.n_query, qh.numpy(), uh.numpy(), cfg.gamma_ppm, outs)
        torch.cuda.synchronize()
        if i >= 2:
            lat_h.append(time.perf_counter() - t1)
    if lat_h:
        result["p50_latency_ms_request_in_pinned_host_memory"] = float(np.percentile(np.array(lat_h) * 1e3, 50))

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
        same = bool(torch.equal(outs_s[(args.steps - 1) % args.streams].cpu(), _last_out(step, args.steps - 1, outs, torch)))
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

    if args.partitions > 1 and args.workload not in ("scale", "fb10b"):
        result["partitioned"] = partitioned_share(args, torch, np, dm, built, cfg, batches, dev_batches, outs)

    if not args.no_cpu_baseline:
        ref, og, cb = cpu_baseline(built, batches, cfg.gamma_ppm)
        result["cpu_baseline"] = cb
        # the batch the oracle just computed, once more on the GPU: the benchmark's own parity check
        f, q, u = dev_batches[0]
        dm.ctx.serve_batch(dm.tables, dm.layers, f, batches[0].n_query, q, u, cfg.gamma_ppm, outs)
        torch.cuda.synchronize()
        got = outs.cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)))
        result["max_row_rel_err_vs_oracle"] = err
    print(json.dumps(result), flush=True)
    dm.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
