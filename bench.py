#!/usr/bin/env python3
"""Benchmark of the broadcast layer step on one MI355X.

One "step" is one whole layer of the large GraphSAGE-mean workload (R-MAT
scale 26, edge factor 32, bf16 features of width 128, degree-ordered ids,
16 chunks of 2^22 sources): layer init (pending counts, zeroed accumulators),
all chunk broadcasts (scatter-aggregate + pending decrement + ready
compaction), a flush (MFMA update) after every chunk, and the exactly-once
check.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is aggregated edges per second of the layer;
`roofline` describes the scatter-aggregate kernel (HIP-event time summed over
its launches inside the timed steps); `cpu_baseline` is the CPU oracle timed on
a bounded sample of the same layer.
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


def cpu_model() -> str:
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.lower().startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", choices=["config2", "config3", "config4", "config5", "wide"], default="config5",
                    help="config5 (default) is the workload the metric is quoted on; the others are the smaller "
                         "parity workloads, timed for the record")
    ap.add_argument("--layer-type", choices=["sage", "gin"], default="sage",
                    help="config5 only: run the same graph and widths through GIN layers instead of SAGE-mean")
    ap.add_argument("--plan-block-log2", type=int, default=-1,
                    help="source-blocked plan: log2 of the sources per block (0: plain destination order; default: "
                         "blocks of 2 MiB of rows for config5, plain order for the other workloads)")
    ap.add_argument("--plan-hot-min", type=int, default=0,
                    help="source-blocked plan: destinations with at least this many messages from a chunk are blocked "
                         "(default: 32 per block of the chunk)")
    ap.add_argument("--d-in", type=int, default=512, help="workload wide: input feature width (up to 1024 with "
                                                          "--transform-first, 512 without)")
    ap.add_argument("--store", choices=["bf16", "f16"], default="bf16",
                    help="config5 / wide: 16-bit storage format of features, weights and outputs (f16 = IEEE half, "
                         "half-precision MFMA in the update)")
    ap.add_argument("--transform-first", action="store_true",
                    help="apply W to each chunk before it is pushed (d_out-wide messages and accumulators)")
    ap.add_argument("--hot-slots-frac", type=float, default=0.0,
                    help="bounded accumulator store: slots = this fraction of the vertices with an in-edge "
                         "(0: one accumulator row per vertex); needs chunks small enough to fit")
    ap.add_argument("--evict-policy", choices=["min", "max"], default="min",
                    help="bounded store: evict fewest (the paper's policy) or most pending messages first")
    ap.add_argument("--scale", type=int, default=None, help="R-MAT scale (default: the workload's own)")
    ap.add_argument("--edge-factor", type=int, default=32)
    ap.add_argument("--no-plan", action="store_true", help="push straight from the CSR (atomic path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--side-stream", action="store_true", help="run on a non-default stream")
    ap.add_argument("--sync-chunks", action="store_true",
                    help="wait for the device after every chunk (no copy / compute overlap): times the stages alone")
    ap.add_argument("--no-e2e", action="store_true", help="skip the three-layer end-to-end run")
    ap.add_argument("--sample-dst", type=int, default=1 << 16, help="destinations in the oracle sample")
    ap.add_argument("--residency", choices=["device", "pinned"], default="device",
                    help="pinned: graph and features stay in pinned host memory and are streamed per chunk "
                         "(host-link bound; reported for the record, never the headline value)")
    ap.add_argument("--order", choices=["indegree", "score", "original"], default="indegree",
                    help="vertex ids: in-degree descending (the workload's), the paper's greedy Score order, "
                         "or the generator's raw ids")
    ap.add_argument("--chunk-log2", type=int, default=None, help="chunk size in sources (default N/16)")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run a plain 4 GiB device copy three times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only; --gpus must be 1 (no collectives or sharding here)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2605_09402_amd as atlas
    from gen import in_edges_of, workloads

    atlas.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()

    # ---- inputs (outside the timed region) ----
    def reorder(off, col):
        n = off.numel() - 1
        indeg = torch.empty(n, dtype=torch.int32, device=dev)
        atlas.atlas_in_degree(atlas.make_graph(n, col.numel(), off, col), indeg)
        new_of_old = torch.empty(n, dtype=torch.int32, device=dev)
        old_of_new = torch.empty(n, dtype=torch.int32, device=dev)
        g = atlas.make_graph(n, col.numel(), off, col, indeg)
        if args.order == "score":
            atlas.atlas_reorder_score_desc(g, new_of_old, old_of_new)
        else:
            atlas.atlas_reorder_indegree_desc(g, new_of_old, old_of_new)
        return new_of_old

    t0 = time.time()
    ck = None if args.chunk_log2 is None else 1 << args.chunk_log2
    ro = None if args.order == "original" else reorder
    store = torch.float16 if args.store == "f16" else torch.bfloat16
    if args.workload == "config5":
        if args.scale is None:
            args.scale = 26
        wl = workloads.config5(dev, scale=args.scale, reorder=ro, edge_factor=args.edge_factor, chunk=ck,
                               model=args.layer_type, store=store)
    elif args.workload == "config2":
        wl = workloads.config2(dev, scale=args.scale or 20, reorder=ro, chunk=ck)
    elif args.workload == "wide":
        wl = workloads.wide(dev, scale=args.scale or 22, d_in=args.d_in, reorder=ro, chunk=ck, store=store)
    elif args.workload == "config3":
        wl = workloads.config3(dev, scale=args.scale or 22, chunk=ck)
    else:
        wl = workloads.config4(dev, scale=args.scale or 22, chunk=ck)
    is_headline = (args.workload == "config5" and args.scale == 26 and args.edge_factor == 32 and ck is None
                   and args.layer_type == "sage" and args.store == "bf16")
    torch.cuda.synchronize()
    n, e, chunk = wl.n, wl.e, wl.chunk
    log("generated %s: N=%d E=%d chunk=%d in %.1f s" % (wl.name, n, e, chunk, time.time() - t0))
    indeg = torch.empty(n, dtype=torch.int32, device=dev)
    atlas.atlas_in_degree(atlas.make_graph(n, e, wl.off, wl.col), indeg)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()

    plan = None
    plan_ms = None
    if not args.no_plan and args.residency == "device":
        t0 = time.time()
        pg = atlas.make_graph(n, e, wl.off, wl.col)
        if args.plan_block_log2 < 0:   # default: 2 MiB of source rows per block on the large workload
            row_bytes = wl.dims[0] * (2 if wl.store != torch.float32 else 4)
            args.plan_block_log2 = max(6, ((2 << 20) // row_bytes).bit_length() - 1) if args.workload == "config5" else 0
        if args.plan_block_log2 > 0 and args.plan_hot_min <= 0:
            args.plan_hot_min = 32 * max(1, chunk >> args.plan_block_log2)
        if args.plan_block_log2 > 0 and chunk <= (1 << args.plan_block_log2):
            args.plan_block_log2 = 0   # a chunk of one block: nothing to reorder
        if args.plan_block_log2 > 0:
            plan = atlas.atlas_plan_create_blocked(pg, chunk, 1 << args.plan_block_log2, args.plan_hot_min)
        else:
            plan = atlas.atlas_plan_create(pg, chunk)
        plan_ms = (time.time() - t0) * 1e3
        log("plan built in %.1f ms" % plan_ms)
    graph = atlas.make_graph(n, e, wl.off, wl.col, indeg, atlas.RESIDENT_DEVICE, plan)
    x_layer0 = wl.X
    if args.residency == "pinned":
        t0 = time.time()
        off_h = torch.empty(wl.off.shape, dtype=wl.off.dtype, pin_memory=True).copy_(wl.off)
        col_h = torch.empty(wl.col.shape, dtype=wl.col.dtype, pin_memory=True).copy_(wl.col)
        x_layer0 = torch.empty(wl.X.shape, dtype=wl.X.dtype, pin_memory=True).copy_(wl.X)
        if not args.no_plan:
            t1 = time.time()
            plan = atlas.atlas_plan_create(atlas.make_graph(n, e, off_h, col_h, None, atlas.RESIDENT_PINNED_HOST), chunk)
            plan_ms = (time.time() - t1) * 1e3
        graph = atlas.make_graph(n, e, off_h, col_h, indeg, atlas.RESIDENT_PINNED_HOST, plan)
        log("pinned host copies made in %.1f s" % (time.time() - t0))

    params = []
    for p in wl.layers:
        params.append((p.W.to(wl.store).to(dev).contiguous(), p.bias.to(wl.store).to(dev).contiguous()))
    outs = [torch.empty((n, wl.dims[li + 1]), dtype=wl.store, device=dev) for li in range(len(wl.layers))]

    model_id = {"sage": atlas.MODEL_SAGE_MEAN, "gcn": atlas.MODEL_GCN_SYM, "gat": atlas.MODEL_GAT,
                "gin": atlas.MODEL_GIN}[wl.model]
    sdt = {torch.bfloat16: atlas.DTYPE_BF16, torch.float16: atlas.DTYPE_F16}.get(wl.store, atlas.DTYPE_F32)
    between = atlas.ACT_ELU if wl.act == "elu" else atlas.ACT_RELU
    attn = [(None if p.attn_src is None else p.attn_src.to(wl.store).to(dev).contiguous(),
             None if p.attn_dst is None else p.attn_dst.to(wl.store).to(dev).contiguous()) for p in wl.layers]

    bounds = list(range(0, n, chunk)) + [n]
    per_chunk = (wl.off[bounds[1:]] - wl.off[bounds[:-1]]).tolist()
    log("edges per chunk (millions): " + " ".join("%.1f" % (x / 1e6) for x in per_chunk[:16]) +
        (" ..." if len(per_chunk) > 16 else ""))
    hot_slots = 0
    if args.hot_slots_frac > 0:
        hot_slots = max(1, int(args.hot_slots_frac * int((indeg > 0).sum().item())))
        log("bounded store: %d slots (%.0f%% of the vertices with an in-edge)" % (hot_slots, 100 * args.hot_slots_frac))

    chunk_wall_ms = []   # --sync-chunks: wall time of every chunk (copy + kernels), all layers run so far

    def run_layer(li: int, x: torch.Tensor, timing: bool) -> dict:
        d_in, d_out = wl.dims[li], wl.dims[li + 1]
        act = atlas.ACT_NONE if li + 1 == len(wl.layers) else between
        dims = atlas.make_dims(model_id, d_in, d_out, sdt, sdt, act, chunk, heads=wl.heads,
                               flags=(atlas.FLAG_TIMING if timing else 0) | atlas.FLAG_EMB_RESIDENT |
                               (atlas.FLAG_PLANNED_ONLY if plan is not None else 0) |
                               (atlas.FLAG_TRANSFORM_FIRST if args.transform_first else 0),
                               hot_slots=hot_slots, evict_policy=1 if args.evict_policy == "max" else 0)
        W, b = params[li]
        h = atlas.atlas_layer_init(graph, dims, atlas.make_weights(W, b, sdt, attn[li][0], attn[li][1]), stream)
        out = outs[li]
        if wl.model == "gat":
            for b0 in range(0, n, chunk):
                atlas.atlas_attention_prepass(h, b0, min(n, b0 + chunk), x[b0:b0 + chunk], stream)
        atlas.atlas_flush_ready(h, out, stream)
        for b0 in range(0, n, chunk):
            b1 = min(n, b0 + chunk)
            tc = time.perf_counter()
            atlas.atlas_broadcast_chunk(h, b0, b1, x[b0:b1], stream)
            atlas.atlas_flush_ready(h, out, stream)
            if args.sync_chunks:
                torch.cuda.synchronize()
                chunk_wall_ms.append((time.perf_counter() - tc) * 1e3)
        return atlas.atlas_layer_finish(h)

    if args.traffic_calibration:
        # a plain copy of known size: 4 GiB read + 4 GiB written per launch
        ca = torch.empty(1 << 30, dtype=torch.int32, device=dev)
        cb = torch.empty_like(ca)
        for _ in range(3):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    if args.side_stream:
        # The layers run on a stream of their own.  Only from here on: the set-up above calls the
        # library's synchronous helpers (plan, ordering), which work on the default stream and do not
        # wait for work queued on other non-blocking streams.
        torch.cuda.synchronize()
        stream = torch.cuda.Stream()
        torch.cuda.set_stream(stream)

    # ---- warm-up, then exactly K timed steps ----
    for _ in range(args.warmup):
        run_layer(0, x_layer0, True)
    torch.cuda.synchronize()
    agg_ms = upd_ms = self_ms = init_ms = copy_ms = 0.0
    h2d_bytes = 0
    step_ms = []          # per step: atlas_layer_finish waits for the layer, so each step ends synchronised
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ts = time.perf_counter()
        st = run_layer(0, x_layer0, True)
        step_ms.append((time.perf_counter() - ts) * 1e3)
        agg_ms += st["ms_aggregate"]
        copy_ms += st["ms_copy"]
        h2d_bytes = st["bytes_copied_h2d"]
        upd_ms += st["ms_update"]
        self_ms += st["ms_self"]
        init_ms += st["ms_init"]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    nchunks = (n + chunk - 1) // chunk
    launches = nchunks * args.steps
    log("layer: %.2f ms/step; aggregate %.2f, update %.2f, self %.2f, init %.2f ms per step"
        % (ms_per_step, agg_ms / args.steps, upd_ms / args.steps, self_ms / args.steps, init_ms / args.steps))
    if args.sync_chunks:
        log("last layer, ms per chunk (copy + kernels, no overlap): " + " ".join("%.1f" % v for v in chunk_wall_ms[-nchunks:]))
    if copy_ms > 0:
        log("chunk loader: %.1f GB per layer in %.1f ms on the copy stream = %.1f GB/s"
            % (h2d_bytes / 1e9, copy_ms / args.steps, h2d_bytes / (copy_ms / args.steps) / 1e6))

    # ---- end-to-end: all three layers once ----
    e2e_ms = None
    layer_ms = []
    if not args.no_e2e:
        # pinned residency: layer 1 streams features and edges from the host, the later layers read the
        # previous layer's output in HBM and stream the edges only
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        x = x_layer0
        for li in range(len(wl.layers)):
            t1 = time.perf_counter()
            run_layer(li, x, False)
            layer_ms.append((time.perf_counter() - t1) * 1e3)
            x = outs[li]
        torch.cuda.synchronize()
        e2e_ms = (time.perf_counter() - t0) * 1e3
        log("end-to-end all layers: %.1f ms (%s)" % (e2e_ms, ", ".join("%.1f" % v for v in layer_ms)))

    # ---- roofline of the scatter-aggregate kernel ----
    d = wl.dims[1] if wl.model == "gat" else wl.dims[0]   # width of the accumulated row
    s_in = 4 if wl.model == "gat" or wl.store == torch.float32 else 2
    bytes_per_edge = 4 + 2 * 4 * d + 8          # destination id, fp32 row read + write, pending RMW
    bytes_per_source = d * s_in + 8             # source row, row offset
    algo_bytes_layer = e * bytes_per_edge + n * bytes_per_source
    agg_s_per_layer = agg_ms / args.steps / 1e3
    achieved = algo_bytes_layer / agg_s_per_layer / 1e9
    peak = 8000.0
    # bytes the regrouped kernel itself must move (source id + bf16 source row per edge)
    kernel_bytes_per_edge = 4 + d * s_in
    # HBM bytes per launch from the committed counter summary; null when the
    # kernels changed after the counters were taken (or for another workload)
    traffic = None
    kname = "k_aggregate_grouped" if plan else "k_aggregate"
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_config5_rmat26.json")
    if os.path.exists(tpath) and is_headline and args.order == "indegree" and args.residency == "device":
        from paper_2605_09402_amd.profile_summary import kernel_source_hash
        doc = json.load(open(tpath))
        if doc.get("kernel_source_hash") == kernel_source_hash() and kname in doc["kernels"]:
            traffic = doc["kernels"][kname]["bytes_per_launch"]
    roofline = {
        "bound": "hbm", "kernel": kname,
        "achieved": round(achieved, 1), "peak": peak, "unit": "GB/s", "frac": round(achieved / peak, 4),
        "traffic": traffic,
        "traffic_GBps": None if traffic is None else round(traffic * nchunks / agg_s_per_layer / 1e9, 1),
        # measured HBM bytes per second over the peak: what the kernel really draws from memory
        "traffic_frac_of_peak": None if traffic is None else round(traffic * nchunks / agg_s_per_layer / 1e9 / peak, 4),
        "launches": launches, "avg_launch_ms": round(agg_ms / launches, 4),
        "algorithmic_bytes_per_edge": bytes_per_edge, "algorithmic_bytes_per_source": bytes_per_source,
        "edges_per_s_in_kernel": round(e / agg_s_per_layer, 1),
        "per_edge_reads_only_GBps": round(e * kernel_bytes_per_edge / agg_s_per_layer / 1e9, 1),
    }
    K = 2 * wl.dims[0] if wl.model == "sage" else wl.dims[0]
    n_with_in = int((indeg > 0).sum().item())
    upd_flops = 2.0 * n * K * wl.dims[1]      # SAGE / GCN: the flush GEMM; GAT: the per-chunk transform (in ms_self)
    upd_s = upd_ms / args.steps / 1e3
    upd_bytes = n_with_in * 4 * d + n * ((s_in * d if wl.model in ("sage", "gin") else 0) + s_in * wl.dims[1])
    mfma_peak = 2.5e15 if sdt in (atlas.DTYPE_BF16, atlas.DTYPE_F16) else 157.3e12
    # the contraction's ceiling at this shape: the MFMA peak, or its flops in the time its bytes need at the HBM peak
    upd_ceiling = min(mfma_peak, upd_flops / (upd_bytes / 8e12))
    update = {
        "kernel": "k_update", "tflops": round(upd_flops / upd_s / 1e12, 2),
        "mfma_peak_tflops": mfma_peak / 1e12,
        "frac_of_mfma_peak": round(upd_flops / upd_s / mfma_peak, 4),
        # accumulator rows are read only for vertices that received something
        "hbm_GBps": round(upd_bytes / upd_s / 1e9, 1),
        "ceiling_tflops": round(upd_ceiling / 1e12, 1),
        "frac_of_ceiling": round(upd_flops / upd_s / upd_ceiling, 4),
        "rows_with_in_edges": n_with_in,
        "ms_per_layer": round(upd_ms / args.steps, 3),
    }

    # ---- CPU oracle on a bounded sample of the same layer ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        gsel = torch.Generator().manual_seed(12345)
        pick = torch.randperm(n, generator=gsel)[: args.sample_dst]
        pick = torch.unique(torch.cat([pick, torch.topk(indeg.to(torch.int64), min(1024, n)).indices.cpu()]))
        in_off, in_src = in_edges_of(wl.off, wl.col, pick.to(dev))
        need = torch.unique(torch.cat([in_src.to(torch.int64), pick.to(dev)]))
        remap = torch.full((n,), -1, dtype=torch.int64, device=dev)
        remap[need] = torch.arange(need.numel(), device=dev)
        Xs = wl.X[need].float().cpu().numpy()
        il = oracle.InLists(in_off.cpu().numpy(), remap[in_src.to(torch.int64)].to(torch.int32).cpu().numpy(),
                            remap[pick.to(dev)].cpu().numpy())
        p0 = wl.layers[0]
        indeg_s = indeg[need].cpu().numpy().astype(np.int64)
        t1 = time.perf_counter()
        Y = oracle.run_layer(wl.model, il, indeg_s, Xs, p0, {"relu": oracle.ACT_RELU, "elu": oracle.ACT_ELU}[wl.act],
                             {torch.bfloat16: oracle.FMT_BF16, torch.float16: oracle.FMT_F16}.get(wl.store, oracle.FMT_F32))
        t_or = time.perf_counter() - t1
        sample_edges = int(in_src.numel())
        # sampled parity of the timed configuration, on the way
        run_layer(0, x_layer0, False)
        got = outs[0][pick.to(dev)].float().cpu().numpy().astype(np.float64)
        rn = np.maximum(np.abs(Y).max(axis=1), 1e-6 * np.abs(Y).max())
        err = float((np.abs(got - Y).max(axis=1) / rn).max())
        log("oracle sample: %d destinations, %d edges, %.2f s; sampled parity error %.3e" %
            (pick.numel(), sample_edges, t_or, err))
        cpu = {"value": round(sample_edges / t_or / 1e9, 6), "unit": "GTEPS", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "%d destinations (%d random + the 1,024 highest in-degree) with all %d of their in-edges, "
                         "layer 1 aggregate + update in fp64" % (pick.numel(), args.sample_dst, sample_edges),
               "seconds": round(t_or, 3), "sampled_parity_max_rel_err": err,
               "cpu_model": cpu_model(), "host_cpus": os.cpu_count()}

    if plan is not None:
        atlas.atlas_plan_destroy(plan)
    gteps = e / (ms_per_step / 1e3) / 1e9
    line = {
        "metric": "aggregated edges/s per layer (GTEPS)", "value": round(gteps, 4), "unit": "GTEPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "ms_per_step_median": round(sorted(step_ms)[len(step_ms) // 2], 3), "ms_per_step_min": round(min(step_ms), 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {atlas.DTYPE_BF16: "bf16 storage / f32 accumulate", atlas.DTYPE_F16: "f16 storage / f32 accumulate"}.get(sdt, "f32"),
        "data": "synthetic",
        "config": {"workload": wl.name, "layer_type": wl.model, "vertices": n, "edges": e, "d_in": wl.dims[0], "d_out": wl.dims[1],
                   "chunk_sources": chunk, "chunks": nchunks, "flush": "after every chunk",
                   "ids": {"indegree": "in-degree descending", "score": "greedy Score order (paper Sec. 3.8)",
                           "original": "generator's raw ids"}[args.order], "in_degree": "precomputed once per graph",
                   "residency": "HBM" if args.residency == "device" else
                   "pinned host, staged per chunk on a copy stream (%.2f GB, copies %.1f ms per layer)"
                   % (h2d_bytes / 1e9, copy_ms / args.steps),
                   "edge_order": "per-chunk destination-grouped plan" if plan else "CSR stream (atomics)",
                   "plan_build_ms": None if plan_ms is None else round(plan_ms, 1)},
        "transform_first": bool(args.transform_first),
        "plan_blocking": None if args.plan_block_log2 <= 0 else {"block_sources": 1 << args.plan_block_log2,
                                                                  "hot_min_edges": args.plan_hot_min},
        "hot_store": None if not hot_slots else {
            "slots": hot_slots, "policy": args.evict_policy + "-pending", "evictions_per_layer": st["hot_evictions"],
            "reloads_per_layer": st["hot_reloads"], "peak_slots": st["hot_peak_slots"]},
        "layer_ms": {"aggregate": round(agg_ms / args.steps, 3), "update": round(upd_ms / args.steps, 3),
                     "self": round(self_ms / args.steps, 3), "init": round(init_ms / args.steps, 3)},
        "end_to_end_ms": None if e2e_ms is None else round(e2e_ms, 2),
        "end_to_end_layer_ms": [round(v, 2) for v in layer_ms],
        "roofline": roofline, "update": update, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
