#!/usr/bin/env python3
"""Benchmark of the broadcast layer step on one MI355X.

One "step" is one whole layer of the large GraphSAGE-mean workload (R-MAT
scale 26, edge factor 32, bf16 features of width 128, degree-ordered ids,
16 chunks of 2^22 sources): layer init (pending counts), all chunk broadcasts
(scatter-aggregate + pending decrement + ready compaction), a flush (MFMA
update) after every chunk, and the exactly-once check.

The layer is timed in two executions, both in the one JSON line:

  * inputs resident in HBM before the timed region starts: `value`,
    `ms_per_step`, `roofline` (the scatter-aggregate kernel, HIP-event time
    summed over its launches inside the timed steps) and `update`;
  * as the workload's configuration states it -- CSR and features in pinned
    host memory, streamed chunk by chunk on the library's copy stream while the
    previous chunk's kernels run: `config5_as_stated` (host-link bound).

`prep_ms` is the one-time, per-graph preparation (in-degree, ordering, plan)
that every layer and every run on the graph reuses; `measured_peak` is what
bare kernels of the same access patterns reach on the box at hand;
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same layer.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def cpu_model() -> str:
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.lower().startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def kernel_source_hash() -> str:
    """Identifies the kernels the committed HBM counter summary was taken with."""
    h = hashlib.sha256()
    for name in ("k_aggregate.hip", "k_update.hip", "k_dense.hip"):
        with open(os.path.join(ROOT, "paper_2605_09402_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


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
    ap.add_argument("--dense-max-gb", type=float, default=-1.0,
                    help="plan with a dense part for the first chunk: byte limit of its cells in GB (0: none; "
                         "default: 32 for config5, none for the other workloads)")
    ap.add_argument("--dense-cells-per-edge", type=int, default=0,
                    help="dense part: most cells a block may spend per edge it holds (0: the library's default)")
    ap.add_argument("--no-dense", action="store_true",
                    help="push the plan's dense part as the planned chunk it also is (ATLAS_FLAG_NO_DENSE)")
    ap.add_argument("--no-handover", action="store_true",
                    help="switch the fused part of the flush off: every finished row takes the fp32 round trip")
    ap.add_argument("--no-narrow-first", action="store_true",
                    help="end-to-end runs: do not switch a layer whose output is narrower than its input (the last "
                         "layer, 128 -> 64) to the transform-first order")
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
    ap.add_argument("--no-e2e", action="store_true", help="skip the three-layer end-to-end runs")
    ap.add_argument("--sample-dst", type=int, default=1 << 16, help="destinations in the oracle sample")
    ap.add_argument("--residency", choices=["both", "device", "pinned"], default="both",
                    help="which executions to time: inputs resident in HBM, streamed from pinned host memory, or "
                         "both (default)")
    ap.add_argument("--no-measured-peak", action="store_true", help="skip the bare copy / gather / MFMA probes")
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
    from gen import sample_subgraph, workloads

    atlas.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()

    def timed_ms(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return r, (time.perf_counter() - t) * 1e3

    # ---- inputs (outside the timed region); the per-graph preparation is timed step by step ----
    prep = {"in_degree_raw_ids": None, "reorder": None, "in_degree": None, "plan": None, "plan_pinned_host": None}

    def warm_up_preparation():
        """The preparation calls once on a toy graph, untimed: the first call of a kernel in a process pays for
        loading its code (about 20 ms over the ordering sort and the plan's sorts and scans together), which is a
        cost of the process, not of the graph."""
        tn = 4096
        toff = torch.arange(0, (tn + 1) * 8, 8, dtype=torch.int64, device=dev)
        tcol = torch.randint(0, tn, (tn * 8,), dtype=torch.int32, device=dev)
        tin = torch.empty(tn, dtype=torch.int32, device=dev)
        tg = atlas.make_graph(tn, tn * 8, toff, tcol)
        atlas.atlas_in_degree(tg, tin)
        ta, tb = torch.empty(tn, dtype=torch.int32, device=dev), torch.empty(tn, dtype=torch.int32, device=dev)
        tgi = atlas.make_graph(tn, tn * 8, toff, tcol, tin)
        (atlas.atlas_reorder_score_desc if args.order == "score" else atlas.atlas_reorder_indegree_desc)(tgi, ta, tb)
        for tp in (atlas.atlas_plan_create_blocked(tg, 512, 64, 4), atlas.atlas_plan_create_dense(tg, 512, 0, 0, 1 << 24, 1 << 20)):
            atlas.atlas_plan_in_degree(tp, tin)
            atlas.atlas_plan_destroy(tp)
        torch.cuda.synchronize()

    warm_up_preparation()

    def reorder(off, col):
        n = off.numel() - 1
        indeg = torch.empty(n, dtype=torch.int32, device=dev)
        _, prep["in_degree_raw_ids"] = timed_ms(
            lambda: atlas.atlas_in_degree(atlas.make_graph(n, col.numel(), off, col), indeg))
        new_of_old = torch.empty(n, dtype=torch.int32, device=dev)
        old_of_new = torch.empty(n, dtype=torch.int32, device=dev)
        g = atlas.make_graph(n, col.numel(), off, col, indeg)
        if args.order == "score":
            _, prep["reorder"] = timed_ms(lambda: atlas.atlas_reorder_score_desc(g, new_of_old, old_of_new))
        else:
            _, prep["reorder"] = timed_ms(lambda: atlas.atlas_reorder_indegree_desc(g, new_of_old, old_of_new))
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
    # the run the committed counter summary was taken with: the default workload with the default plan and flags
    is_headline = (args.workload == "config5" and args.scale == 26 and args.edge_factor == 32 and ck is None
                   and args.layer_type == "sage" and args.store == "bf16" and args.dense_max_gb < 0
                   and args.dense_cells_per_edge == 0 and not args.no_dense and not args.no_handover
                   and not args.no_plan and args.plan_block_log2 < 0 and args.hot_slots_frac <= 0
                   and not args.transform_first)
    if args.dense_max_gb < 0:   # default: a dense part for the large workload's first chunk, up to 32 GB of cells
        args.dense_max_gb = 32.0 if args.workload == "config5" and args.hot_slots_frac <= 0 else 0.0
    torch.cuda.synchronize()
    n, e, chunk = wl.n, wl.e, wl.chunk
    log("generated %s: N=%d E=%d chunk=%d in %.1f s" % (wl.name, n, e, chunk, time.time() - t0))
    indeg = torch.empty(n, dtype=torch.int32, device=dev)
    torch.cuda.empty_cache()
    do_device = args.residency in ("both", "device")
    do_pinned = args.residency in ("both", "pinned")

    plan = None
    plan_info = None
    if not args.no_plan and do_device:
        pg = atlas.make_graph(n, e, wl.off, wl.col)
        if args.plan_block_log2 < 0:
            # default: plain destination order.  (Source blocks of 2 MiB of rows for the heavy destinations gained
            # 4 ms on the large workload before the plan had a dense part; with it they gain nothing and cost 58 ms
            # of plan construction.  The large workload without a dense part still gets them.)
            row_bytes = wl.dims[0] * (2 if wl.store != torch.float32 else 4)
            args.plan_block_log2 = (max(6, ((2 << 20) // row_bytes).bit_length() - 1)
                                    if args.workload == "config5" and args.dense_max_gb <= 0 else 0)
        if args.plan_block_log2 > 0 and args.plan_hot_min <= 0:
            args.plan_hot_min = 32 * max(1, chunk >> args.plan_block_log2)
        if args.plan_block_log2 > 0 and chunk <= (1 << args.plan_block_log2):
            args.plan_block_log2 = 0   # a chunk of one block: nothing to reorder
        if args.dense_max_gb > 0:
            plan, prep["plan"] = timed_ms(lambda: atlas.atlas_plan_create_dense(
                pg, chunk, (1 << args.plan_block_log2) if args.plan_block_log2 > 0 else 0,
                args.plan_hot_min if args.plan_block_log2 > 0 else 0, int(args.dense_max_gb * 1e9),
                args.dense_cells_per_edge))
        elif args.plan_block_log2 > 0:
            plan, prep["plan"] = timed_ms(
                lambda: atlas.atlas_plan_create_blocked(pg, chunk, 1 << args.plan_block_log2, args.plan_hot_min))
        else:
            plan, prep["plan"] = timed_ms(lambda: atlas.atlas_plan_create(pg, chunk))
        plan_info = atlas.atlas_plan_info(plan)
        log("plan built in %.1f ms: %d groups, %.2f GB" % (prep["plan"], plan_info["num_groups"],
                                                            plan_info["bytes_device"] / 1e9))
        if plan_info["dense_edges"]:
            log("dense part of chunk 0: %.1f M edges (%.1f%% of all) in %.2f G cells, %d destinations x up to %d sources"
                % (plan_info["dense_edges"] / 1e6, 100.0 * plan_info["dense_edges"] / max(e, 1),
                   plan_info["dense_cells"] / 1e9, plan_info["dense_rows"], plan_info["dense_max_sources"]))
        # the ordered graph's in-degrees are the plan's group sizes
        _, prep["in_degree"] = timed_ms(lambda: atlas.atlas_plan_in_degree(plan, indeg))
    else:
        _, prep["in_degree"] = timed_ms(lambda: atlas.atlas_in_degree(atlas.make_graph(n, e, wl.off, wl.col), indeg))
    graph_dev = atlas.make_graph(n, e, wl.off, wl.col, indeg, atlas.RESIDENT_DEVICE, plan)

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

    def run_layer(graph, planned: bool, li: int, x: torch.Tensor, timing: bool, narrow_first: bool = False) -> dict:
        d_in, d_out = wl.dims[li], wl.dims[li + 1]
        # the linear map commutes with the neighbour sum: a layer that narrows its rows pushes the narrow products
        tf = args.transform_first or (narrow_first and d_out < d_in and wl.model in ("sage", "gcn", "gin")
                                      and d_out % 64 == 0)
        act = atlas.ACT_NONE if li + 1 == len(wl.layers) else between
        dims = atlas.make_dims(model_id, d_in, d_out, sdt, sdt, act, chunk, heads=wl.heads,
                               flags=(atlas.FLAG_TIMING if timing else 0) | atlas.FLAG_EMB_RESIDENT |
                               (atlas.FLAG_PLANNED_ONLY if planned else 0) |
                               (atlas.FLAG_TRANSFORM_FIRST if tf else 0) |
                               (atlas.FLAG_NO_HANDOVER if args.no_handover else 0) |
                               (atlas.FLAG_NO_DENSE if args.no_dense else 0),
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
        st = atlas.atlas_layer_finish(h)
        assert st["chunks_planned"] == (st["num_chunks"] if planned else 0), "a chunk left the planned path"
        return st

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

    nchunks = (n + chunk - 1) // chunk

    def time_layers(graph, planned, x0):
        """W warm-up steps, then exactly K timed steps of layer 1; then all layers once."""
        for _ in range(args.warmup):
            run_layer(graph, planned, 0, x0, True)
        torch.cuda.synchronize()
        acc = {"ms_aggregate": 0.0, "ms_dense": 0.0, "ms_contract": 0.0, "ms_update": 0.0, "ms_self": 0.0, "ms_init": 0.0, "ms_copy": 0.0}
        step_ms = []   # atlas_layer_finish waits for the layer, so each step ends synchronised
        t0 = time.perf_counter()
        st = None
        for _ in range(args.steps):
            ts = time.perf_counter()
            st = run_layer(graph, planned, 0, x0, True)
            step_ms.append((time.perf_counter() - ts) * 1e3)
            for k in acc:
                acc[k] += st[k]
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        res = {"ms_per_step": wall * 1e3 / args.steps, "step_ms": step_ms, "last_stats": st,
               "per_step": {k: v / args.steps for k, v in acc.items()}, "e2e_ms": None, "layer_ms": []}
        if not args.no_e2e:
            # later layers read the previous layer's output where it lies in HBM (a pinned-host graph then
            # streams its edges only)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            x = x0
            for li in range(len(wl.layers)):
                t1 = time.perf_counter()
                run_layer(graph, planned, li, x, False, narrow_first=not args.no_narrow_first)
                res["layer_ms"].append((time.perf_counter() - t1) * 1e3)
                x = outs[li]
            torch.cuda.synchronize()
            res["e2e_ms"] = (time.perf_counter() - t0) * 1e3
        return res

    # ---- inputs resident in HBM ----
    dev_res = None
    if do_device:
        dev_res = time_layers(graph_dev, plan is not None, wl.X)
        ps = dev_res["per_step"]
        log("HBM-resident layer: %.2f ms/step; aggregate %.2f, dense part %.2f, update %.2f, self %.2f, init %.2f ms per step"
            % (dev_res["ms_per_step"], ps["ms_aggregate"], ps["ms_dense"], ps["ms_update"], ps["ms_self"], ps["ms_init"]))
        if args.sync_chunks:
            log("last layer, ms per chunk (kernels, no overlap): " + " ".join("%.1f" % v for v in chunk_wall_ms[-nchunks:]))
        if dev_res["e2e_ms"] is not None:
            log("end-to-end all layers: %.1f ms (%s)" % (dev_res["e2e_ms"], ", ".join("%.1f" % v for v in dev_res["layer_ms"])))

    # ---- as stated: CSR and features in pinned host memory, streamed per chunk ----
    pin_res = None
    plan_host = None
    plan_host_info = None
    if do_pinned:
        t0 = time.time()
        off_h = torch.empty(wl.off.shape, dtype=wl.off.dtype, pin_memory=True).copy_(wl.off)
        col_h = torch.empty(wl.col.shape, dtype=wl.col.dtype, pin_memory=True).copy_(wl.col)
        x_h = torch.empty(wl.X.shape, dtype=wl.X.dtype, pin_memory=True).copy_(wl.X)
        log("pinned host copies made in %.1f s" % (time.time() - t0))
        if not args.no_plan:
            pgh = atlas.make_graph(n, e, off_h, col_h, None, atlas.RESIDENT_PINNED_HOST)
            if args.dense_max_gb > 0:
                # the dense part of the first chunk stays in HBM: topology that does not cross the host link again
                plan_host, prep["plan_pinned_host"] = timed_ms(lambda: atlas.atlas_plan_create_dense(
                    pgh, chunk, 0, 0, int(args.dense_max_gb * 1e9), args.dense_cells_per_edge))
            else:
                plan_host, prep["plan_pinned_host"] = timed_ms(lambda: atlas.atlas_plan_create(pgh, chunk))
            plan_host_info = atlas.atlas_plan_info(plan_host)
        graph_pin = atlas.make_graph(n, e, off_h, col_h, indeg, atlas.RESIDENT_PINNED_HOST, plan_host)
        pin_res = time_layers(graph_pin, plan_host is not None, x_h)
        ps = pin_res["per_step"]
        h2d = pin_res["last_stats"]["bytes_copied_h2d"]
        log("pinned-host layer: %.2f ms/step; %.1f GB per layer in %.1f ms on the copy stream = %.1f GB/s"
            % (pin_res["ms_per_step"], h2d / 1e9, ps["ms_copy"], h2d / max(ps["ms_copy"], 1e-9) / 1e6))
        if pin_res["e2e_ms"] is not None:
            log("end-to-end all layers: %.1f ms (%s)" % (pin_res["e2e_ms"], ", ".join("%.1f" % v for v in pin_res["layer_ms"])))

    main_res = dev_res if dev_res is not None else pin_res
    ms_per_step = main_res["ms_per_step"]
    step_ms = main_res["step_ms"]
    ps = main_res["per_step"]

    # ---- roofline of the scatter-aggregate kernel ----
    d = wl.dims[1] if wl.model == "gat" or args.transform_first else wl.dims[0]   # width of the accumulated row
    s_in = 4 if wl.model == "gat" or wl.store == torch.float32 else 2
    agg_s_per_layer = ps["ms_aggregate"] / 1e3
    n_with_in = int((indeg > 0).sum().item())
    launches = nchunks * args.steps
    kname = "k_aggregate_grouped" if (plan or plan_host) else "k_aggregate"
    if plan_info is not None:
        # What the planned kernel itself must move: per edge its 4-byte edge word and one source row; per
        # (chunk, destination) group the group's destination word, a pending-count read-modify-write and the
        # accumulator row -- written only by a destination's first group, read and written by every later one;
        # per 64-edge tile its first-group index.
        G, G1 = plan_info["num_groups"], plan_info["num_first_groups"]
        e_list = e
        if main_res["last_stats"]["edges_contracted"]:
            # the dense part went through the contraction (timed apart, see `dense_part`): its edges and groups are
            # not the edge-list kernel's, and its destinations' first touch is the contraction's
            e_list = e - plan_info["dense_edges"]
            G -= plan_info["dense_groups"]
            G1 = max(0, G1 - plan_info["dense_groups"])
        algo_bytes_layer = e_list * (4 + d * s_in) + G * (4 + 8) + (2 * G - G1) * 4 * d + ((e_list + 63) // 64) * 4
        # a row handed over to the update leaves the kernel in the storage type, not as an fp32 row
        algo_bytes_layer -= main_res["last_stats"]["rows_handed_over"] * (4 - s_in) * d
        algo_note = ("edge word + source row per edge; destination word, pending RMW and fp32 row "
                     "(store for a first group, read + write otherwise; a row handed over to the update is written in "
                     "the storage type) per group; tile index per 64 edges")
    else:
        # CSR stream with atomics: destination id, fp32 row read-modify-write and pending RMW per edge
        algo_bytes_layer = e * (4 + 2 * 4 * d + 8) + n * (d * s_in + 8)
        algo_note = "streaming model: per edge destination id + fp32 row RMW + pending RMW, per source its row + offset"
    achieved = algo_bytes_layer / agg_s_per_layer / 1e9
    # Two reference figures beside it: the streaming model (a destination row RMW per edge, which the planned kernel
    # does not do: reported as an effective rate, never as a fraction) and the compulsory lower bound (every edge
    # word, source row and accumulator row crossing the memory interface once)
    streaming_bytes = e * (4 + 2 * 4 * d + 8) + n * (d * s_in + 8)
    compulsory_bytes = 4 * e + n * d * s_in + 2 * n * d * 4 + 8 * n
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_config5_rmat26.json")
    if os.path.exists(tpath) and is_headline and args.order == "indegree" and dev_res is not None:
        doc = json.load(open(tpath))
        if doc.get("kernel_source_hash") == kernel_source_hash() and kname in doc["kernels"]:
            traffic = doc["kernels"][kname]["bytes_per_launch"]
    roofline = {
        "bound": "hbm", "kernel": kname,
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_launch": int(algo_bytes_layer / nchunks), "algorithmic_bytes": algo_note,
        # HBM bytes per launch from the committed rocprofv3 counter summary; null once the kernels have changed
        "traffic": traffic,
        "traffic_GBps": None if traffic is None else round(traffic * nchunks / agg_s_per_layer / 1e9, 1),
        "traffic_frac_of_peak": None if traffic is None else round(traffic * nchunks / agg_s_per_layer / 1e9 / HBM_PEAK_GBPS, 4),
        "traffic_over_algorithmic": None if traffic is None else round(traffic * nchunks / algo_bytes_layer, 3),
        "compulsory_bytes_per_layer": compulsory_bytes,
        "traffic_over_compulsory": None if traffic is None else round(traffic * nchunks / compulsory_bytes, 2),
        "streaming_model_effective_GBps": round(streaming_bytes / agg_s_per_layer / 1e9, 1),
        "launches": launches, "avg_launch_ms": round(ps["ms_aggregate"] / nchunks, 4),
        "edges_per_s_in_kernel": round((e_list if plan_info is not None else e) / agg_s_per_layer, 1),
    }
    dense_part = None
    if plan_info is not None and plan_info["dense_edges"]:
        ms_d = ps["ms_dense"]
        contracted = bool(main_res["last_stats"]["edges_contracted"])
        dense_part = {"edges": plan_info["dense_edges"], "share_of_edges": round(plan_info["dense_edges"] / max(e, 1), 4),
                      "cells": plan_info["dense_cells"], "destinations": plan_info["dense_rows"],
                      "max_sources": plan_info["dense_max_sources"], "contracted": contracted,
                      "ms_per_layer": round(ms_d, 3),
                      "edges_per_s": round(plan_info["dense_edges"] / max(ms_d, 1e-9) * 1e3, 1)}
        if contracted:
            # the contraction kernel alone (ms_per_layer also clears the rows, repacks the chunk's rows and
            # lowers the pending counts): flops of the dense product over the region's cells
            fl = 2.0 * plan_info["dense_cells"] * d
            ms_c = ps["ms_contract"]
            dense_part.update({"kernel": "k_dense_contract", "kernel_ms": round(ms_c, 3),
                               "tflops": round(fl / (ms_c / 1e3) / 1e12, 1),
                               "frac_of_mfma_peak": round(fl / (ms_c / 1e3) / 2.5e15, 4),
                               "cell_stream_GBps": round(plan_info["dense_cells"] / 2 / (ms_c / 1e3) / 1e9, 1)})
    if roofline["frac"] > 1.0:
        log("note: the kernel's algorithmic bytes per second exceed the HBM peak (rows served from cache)")
    K = 2 * wl.dims[0] if wl.model == "sage" else wl.dims[0]
    upd_flops = 2.0 * n * K * wl.dims[1]      # SAGE / GCN: the flush GEMM; GAT: the per-chunk transform (in ms_self)
    upd_s = ps["ms_update"] / 1e3
    handed = main_res["last_stats"]["rows_handed_over"]   # their operand is read in the storage type, not as fp32 sums
    upd_bytes = ((n_with_in - handed) * 4 * d + handed * s_in * d +
                 n * ((s_in * d if wl.model in ("sage", "gin") else 0) + s_in * wl.dims[1]))
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
        "ms_per_layer": round(ps["ms_update"], 3),
    }

    # ---- measured peaks: bare kernels of the same access patterns on this machine ----
    measured = None
    if not args.no_measured_peak:
        def ev_ms(fn, reps):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps
        cbytes = 4 << 30
        ca = torch.empty(cbytes // 4, dtype=torch.int32, device=dev).fill_(1)
        cb = torch.empty_like(ca)
        copy_ms = ev_ms(lambda: atlas.atlas_probe_copy(cb, ca, cbytes), 5)
        cc = torch.empty_like(ca)
        mix_ms = ev_ms(lambda: atlas.atlas_probe_mix21(cc, ca, cb, cbytes), 5)   # 2 reads : 1 write, the flush's mix
        del cb, cc
        # 2^27 random rows of 256 bytes out of a 1 GiB table (the size of one chunk's bf16 rows)
        table_rows, n_ids = 1 << 22, 1 << 27
        ids = torch.randint(0, table_rows, (n_ids,), dtype=torch.int32, device=dev)
        sink = torch.empty(atlas.atlas_probe_gather_sink_bytes() // 4, dtype=torch.int32, device=dev)
        gather_ms = ev_ms(lambda: atlas.atlas_probe_row_gather(ca, table_rows, ids, n_ids, sink), 3)
        del ids, ca
        mf = {}
        if sdt != atlas.DTYPE_F32:
            # nothing but bf16 32x32x16 matrix instructions on register operands, 2 and 4 wavefronts per SIMD
            for wps in (2, 4):
                it_n = 1 << 15
                fl = atlas.atlas_probe_mfma(wps, 1 << 10, sink)
                t_ms = ev_ms(lambda: atlas.atlas_probe_mfma(wps, it_n, sink), 1)
                fl = atlas.atlas_probe_mfma(wps, it_n, sink)
                torch.cuda.synchronize()
                mf["bare_issue_%d_waves_per_simd" % wps] = {
                    "tflops": round(fl / (t_ms / 1e3) / 1e12, 1), "frac_of_mfma_peak": round(fl / (t_ms / 1e3) / mfma_peak, 4)}
            # the contraction on a block of rows small enough to stay in the memory-side cache, many passes:
            # the flush's shape (K = 2 d_in -> d_out) and the wide first-layer transform (K = 1024 -> 256)
            for label, rows_n, kk, dd in (("flush_shape", 1 << 16, K, wl.dims[1]), ("wide_transform", 1 << 15, 1024, 256)):
                if kk > 1024 or dd > 256 or dd % 32 or kk % 64:
                    continue
                rows = (torch.rand((rows_n, kk), device=dev) - 0.5).to(wl.store)
                Wp = (torch.rand((kk, dd), device=dev) - 0.5).to(wl.store)
                po = torch.empty((rows_n, dd), dtype=wl.store, device=dev)
                reps = 40
                atlas.atlas_probe_dense_rows(sdt, rows, rows_n, kk, dd, Wp, po, 2)
                t_ms = ev_ms(lambda: atlas.atlas_probe_dense_rows(sdt, rows, rows_n, kk, dd, Wp, po, reps), 1) / reps
                tf = 2.0 * rows_n * kk * dd / (t_ms / 1e3) / 1e12
                mf[label] = {"rows": rows_n, "K": kk, "d_out": dd, "tflops": round(tf, 1),
                             "frac_of_mfma_peak": round(tf * 1e12 / mfma_peak, 4)}
                del rows, Wp, po
        measured = {
            "copy_GBps": round(2 * cbytes / (copy_ms / 1e3) / 1e9, 1),   # 1 read : 1 write
            "copy_frac_of_peak": round(2 * cbytes / (copy_ms / 1e3) / 1e9 / HBM_PEAK_GBPS, 4),
            "mix_2r1w_GBps": round(3 * cbytes / (mix_ms / 1e3) / 1e9, 1),
            # the flush moves its bytes at this share of what a bare 2:1 stream reaches
            "update_frac_of_measured_mix": round(upd_bytes / upd_s / 1e9 / (3 * cbytes / (mix_ms / 1e3) / 1e9), 4),
            "gather_GBps": round(n_ids * 256 / (gather_ms / 1e3) / 1e9, 1),
            "gather": "2^27 random 256-byte rows of a 1 GiB table, one wave per row, 8 rows in flight per wave",
            "mfma": mf,
            # (the edges the edge-list kernel pushes: without those of a contracted dense part)
            "aggregate_frac_of_measured_gather": round((e_list if plan_info is not None else e) * (4 + d * s_in) /
                                                       agg_s_per_layer / 1e9 /
                                                       (n_ids * 256 / (gather_ms / 1e3) / 1e9), 4),
        }
        log("measured peaks: copy %.0f GB/s, row gather %.0f GB/s, MFMA %s" %
            (measured["copy_GBps"], measured["gather_GBps"], {k: v["tflops"] for k, v in mf.items()}))
        torch.cuda.empty_cache()

    # ---- CPU oracle on a bounded sample of the same layer ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        gsel = torch.Generator().manual_seed(12345)
        pick_random = torch.randperm(n, generator=gsel)[: args.sample_dst]
        pick = torch.unique(torch.cat([pick_random, torch.topk(indeg.to(torch.int64), min(1024, n)).indices.cpu()])).to(dev)
        in_off, in_src_local, need, pick_local = sample_subgraph(wl.off, wl.col, pick)
        Xs = wl.X[need].float().cpu().numpy()
        il = oracle.InLists(in_off.cpu().numpy(), in_src_local.cpu().numpy(), pick_local.cpu().numpy())
        # How many vertices does an edge message complete (the row then leaves the aggregation kernel and is read
        # back by the flush of the same call: what a flush fused into the aggregation could hand over directly),
        # and how many the vertex's own message, long after its last data arrived?  On the random part of the sample.
        is_random = torch.zeros(n, dtype=torch.bool, device=dev)
        is_random[pick_random.to(dev)] = True
        deg_s = in_off[1:] - in_off[:-1]
        has_in = deg_s > 0
        last_src = torch.zeros(pick.numel(), dtype=torch.int64, device=dev)
        last_pos = (in_off[1:] - 1).clamp(min=0)
        last_src[has_in] = need[in_src_local.to(torch.int64)[last_pos[has_in]]]     # lists ascend: the last is the largest
        by_edge = has_in & ((last_src // chunk) >= (pick // chunk))
        sel = is_random[pick]
        frac_with_in = float((has_in & sel).sum().item()) / max(1, int(sel.sum().item()))
        frac_by_edge = float((by_edge & sel).sum().item()) / max(1, int(sel.sum().item()))
        p0 = wl.layers[0]
        indeg_s = indeg[need].cpu().numpy().astype(np.int64)
        t1 = time.perf_counter()
        Y = oracle.run_layer(wl.model, il, indeg_s, Xs, p0, {"relu": oracle.ACT_RELU, "elu": oracle.ACT_ELU}[wl.act],
                             {torch.bfloat16: oracle.FMT_BF16, torch.float16: oracle.FMT_F16}.get(wl.store, oracle.FMT_F32))
        t_or = time.perf_counter() - t1
        sample_edges = int(in_src_local.numel())
        # sampled parity of the timed configurations, on the way
        errs = {}
        for label, graph, planned, x0 in (("hbm_resident", graph_dev if do_device else None, plan is not None, wl.X),
                                          ("pinned_host", graph_pin if do_pinned else None, plan_host is not None,
                                           x_h if do_pinned else None)):
            if graph is None:
                continue
            outs[0].fill_(float("nan"))
            run_layer(graph, planned, 0, x0, False)
            got = outs[0][pick].float().cpu().numpy().astype(np.float64)
            rn = np.maximum(np.abs(Y).max(axis=1), 1e-6 * np.abs(Y).max())
            errs[label] = float((np.abs(got - Y).max(axis=1) / rn).max())
        log("oracle sample: %d destinations, %d edges, %.2f s; sampled parity error %s" %
            (pick.numel(), sample_edges, t_or, errs))
        cpu = {"value": round(sample_edges / t_or / 1e9, 6), "unit": "GTEPS", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "%d destinations (%d random + the 1,024 highest in-degree) with all %d of their in-edges, "
                         "layer 1 aggregate + update in fp64" % (pick.numel(), args.sample_dst, sample_edges),
               "seconds": round(t_or, 3), "sampled_parity_max_rel_err": errs,
               "completion": {"vertices_with_in_edges": round(frac_with_in, 4),
                              "completed_by_an_edge_message": round(frac_by_edge, 4),
                              "note": "share of all vertices, estimated on the random part of the sample; only the "
                                      "second kind could be handed from the aggregation to the update without a "
                                      "round trip of its accumulator row"} if wl.model in ("sage", "gin") else None,
               "cpu_model": cpu_model(), "host_cpus": os.cpu_count()}

    # ---- teardown: nothing of the library's stays alive until the process exits ----
    for ph in (plan, plan_host):
        if ph is not None:
            atlas.atlas_plan_destroy(ph)
    torch.cuda.synchronize()
    atlas.atlas_release_cache()

    def r1(v):
        return None if v is None else round(v, 1)
    prep_total = sum(v for k, v in prep.items() if v is not None and k != "plan_pinned_host")
    prep_out = {k: r1(v) for k, v in prep.items()}
    prep_out["total_hbm_resident"] = r1(prep_total)
    prep_out["note"] = ("one-time per graph, reused by every layer and run: in-degree of the raw ids (for the ordering), "
                        "the ordering sort, the destination-grouped plan, in-degree of the ordered graph (read off "
                        "the plan); the "
                        "generator's own relabelling and CSR build are input production and are not in here")
    stated = None
    if pin_res is not None:
        h2d = pin_res["last_stats"]["bytes_copied_h2d"]
        cms = pin_res["per_step"]["ms_copy"]
        stated = {
            "execution": "CSR, features and plan in pinned host memory (of the plan, the first chunk's dense corner in "
                         "HBM); every chunk staged into HBM on the library's copy stream (long chunks in pieces) while "
                         "the previous chunk's kernels run; fp32 accumulators resident in HBM",
            "ms_per_step": round(pin_res["ms_per_step"], 3),
            "ms_per_step_min": round(min(pin_res["step_ms"]), 3),
            "gteps": round(e / (pin_res["ms_per_step"] / 1e3) / 1e9, 4),
            "h2d_GB_per_layer": round(h2d / 1e9, 2), "copy_stream_ms": round(cms, 1),
            "h2d_GBps": round(h2d / max(cms, 1e-9) / 1e6, 1),
            "copy_stream_busy_frac": round(cms / pin_res["ms_per_step"], 3),
            "kernels_ms": {k[3:]: round(v, 2) for k, v in pin_res["per_step"].items() if k != "ms_copy"},
            "end_to_end_ms": r1(pin_res["e2e_ms"]), "end_to_end_layer_ms": [round(v, 1) for v in pin_res["layer_ms"]],
            "plan_build_ms": r1(prep["plan_pinned_host"]),
            # the part of the plan that stays in HBM (cells of the first chunk's dense corner and its edge list):
            # those edges do not cross the host link in any layer
            "resident_dense_part": None if not plan_host_info or not plan_host_info["dense_edges"] else {
                "edges": plan_host_info["dense_edges"], "cells": plan_host_info["dense_cells"],
                "plan_bytes_device": plan_host_info["bytes_device"],
                "plan_bytes_pinned_host": plan_host_info["bytes_pinned_host"]},
        }
    gteps = e / (ms_per_step / 1e3) / 1e9
    st = main_res["last_stats"]
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
                           "original": "generator's raw ids"}[args.order],
                   "value_is": ("inputs resident in HBM when the timed region starts; the same layer in the "
                                "configuration's stated execution (streamed from pinned host memory) is "
                                "config5_as_stated") if dev_res is not None else
                               "streamed from pinned host memory (host-link inclusive)",
                   "edge_order": "per-chunk destination-grouped plan" if (plan or plan_host) else "CSR stream (atomics)"},
        "transform_first": bool(args.transform_first),
        "end_to_end_note": None if args.no_narrow_first else
        "layers whose output is narrower than their input run in the transform-first order (narrow messages)",
        "plan_blocking": None if args.plan_block_log2 <= 0 else {"block_sources": 1 << args.plan_block_log2,
                                                                  "hot_min_edges": args.plan_hot_min},
        "plan": plan_info,
        "hot_store": None if not hot_slots else {
            "slots": hot_slots, "policy": args.evict_policy + "-pending", "evictions_per_layer": st["hot_evictions"],
            "reloads_per_layer": st["hot_reloads"], "peak_slots": st["hot_peak_slots"]},
        "layer_ms": {"aggregate": round(ps["ms_aggregate"], 3), "dense_part": round(ps["ms_dense"], 3),
                     "update": round(ps["ms_update"], 3), "self": round(ps["ms_self"], 3), "init": round(ps["ms_init"], 3)},
        # the first chunk's dense corner, pushed as a contraction on the matrix cores (atlas_plan_create_dense)
        "dense_part": dense_part,
        # the fused part of the flush: rows that went from the aggregation to the update as its 16-bit operand
        "fused_flush": {"rows_handed_over_per_layer": st["rows_handed_over"],
                        "share_of_vertices": round(st["rows_handed_over"] / max(n, 1), 4)},
        "end_to_end_ms": r1(main_res["e2e_ms"]),
        "end_to_end_layer_ms": [round(v, 2) for v in main_res["layer_ms"]],
        "prep_ms": prep_out,
        "end_to_end_with_prep_ms": None if main_res["e2e_ms"] is None else r1(main_res["e2e_ms"] + prep_total),
        # the same layer in the execution the workload's configuration states (host-link inclusive), at top level too
        "value_as_stated": None if stated is None else stated["gteps"],
        "ms_per_step_as_stated": None if stated is None else stated["ms_per_step"],
        "config5_as_stated": stated,
        "roofline": roofline, "update": update, "measured_peak": measured, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
