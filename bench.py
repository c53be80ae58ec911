#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic workload:
  configs 1, 2 : one layer-wise GCN epoch (forward + backward) at full width: every
                 forward aggregation, backward aggregation, transform and transform gradient;
  configs 3, 4 : one worker's share of an epoch: the slice aggregations (forward and
                 backward) at F_slice = width / 8 on the full graph, and the transforms on
                 ceil(N / 8) vertices at full width.
  config 5     : the same share with the topology cut into chunks under the config's device
                 budget (ntp_chunked_aggregate).
Prints ONE JSON line.  `value` is aggregation GEPS over the whole step: stored entries of
A_hat (self loops included) x slice width, summed over the step's aggregation calls,
divided by the step time (transforms included in the time).

Without --config the line is that of config 3 (the power-law graph the bandwidth target is
stated on) and carries a `configs` object with the same measurements of config 4 (fp32 and
bf16 slices), config 2, config 5's shape at one eighth of its size, and config 5 itself when
the host has the memory for it (75 GB) and its projected time fits --time-budget - else a
`skipped` note with the reason.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix rate
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
# The transform forms every fp32 product from six bf16 piece products on the bf16 matrix
# instructions (narrow or short products stay on the fp32 instructions): its useful flops are
# priced against a sixth of the bf16 rate.
SPLIT_PEAK_TFLOPS = BF16_MFMA_PEAK_TFLOPS / 6.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def agg_bytes(n, nnz, f, elem=4):
    """algorithmic bytes of one aggregation call: entries (index + weight), row pointers,
    X read once, Y written once"""
    return 8 * nnz + 8 * (n + 1) + 2 * n * f * elem


def line_padded_ld(f, elem=4):
    """row stride (elements) for a slice of width f: rows at least one 128-byte line wide start
    on line boundaries, narrower ones on 16-byte vectors"""
    per_line, per_vec = 128 // elem, 16 // elem
    return -(-f // per_line) * per_line if f >= per_line else -(-f // per_vec) * per_vec


def copy_probe(torch, dev):
    """a plain 1 GiB device copy: what the memory system delivers to a streaming kernel (read +
    write), the practical ceiling beside the 8 TB/s nominal one"""
    a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    b = torch.empty_like(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b.copy_(a)
    e0.record()
    for _ in range(5):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    gbs = 5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    log("copy probe: 1 GiB read + 1 GiB written per copy, %.1f GB/s" % gbs)
    return gbs


def line_rate_probe():
    """random 128-byte lines per second the memory system delivers beyond the L2 (Infinity Cache / HBM), measured by
    the stand-alone probe paper_2412_20379_amd/line_rate_probe (its own process; run before this one touches the GPU).
    Returns GB/s at 128 MB and at 1 GB, or None when the executable is not built."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2412_20379_amd", "line_rate_probe")
    if not os.path.exists(exe):
        return None
    # under a profiler the GPU is initialised before this program starts, and a process that has
    # initialised the GPU must not start another program: no probe then
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", "").lower():
        log("line-rate probe skipped (profiler environment)")
        return None
    try:
        r = subprocess.run([exe, "--quick"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, timeout=120)
        w = [l for l in r.stdout.splitlines() if l.startswith("quick")][-1].split()
        out = {"infinity_cache_128mb_gbs": float(w[1]) * 128.0, "hbm_1gb_gbs": float(w[2]) * 128.0}
        log("line-rate probe: random 128-byte lines beyond the L2: %.0f GB/s (128 MB), %.0f GB/s (1 GB)" % (out["infinity_cache_128mb_gbs"], out["hbm_1gb_gbs"]))
        return out
    except Exception as e:
        log("line-rate probe failed: %r" % (e,))
        return None


LINE_RATE = None


def profile_traffic(key):
    """L2-boundary bytes per launch of the aggregation kernel as counted in an earlier rocprofv3
    run (profiles/traffic.json): not measured by this process, so it comes with the commit and
    the kernel it was counted at"""
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        t = json.load(open(tfile))
    except Exception:
        return None, None
    e = t.get(key)
    if isinstance(e, dict):
        return e.get("bytes"), {"from_profile": e.get("profile"), "counted_at_commit": e.get("commit"), "kernel": e.get("kernel")}
    return None, None


def step_bench(args, cfg, scale_down=1, agg_dtype="f32", copy_gbs=None, graph=None, cpu_seconds=20.0, context=True, cpu_baseline_from=None):
    """One config's step, timed: returns (the JSON object of that config, (n, src, dst) for reuse)."""
    import numpy as np
    import torch
    import ntp_inputs as gen
    import paper_2412_20379_amd as ntp
    from paper_2412_20379_amd.gcn import GcnEpoch
    from paper_2412_20379_amd.tp import TensorParallelEpoch

    dev = "cuda:0"
    spec = gen.CONFIGS[cfg]
    t0 = time.time()
    if graph is None:
        graph = gen.make_graph(cfg, args.seed, scale_down, permute=not args.unpermuted)
    n, src, dst = graph
    t_gen = time.time() - t0
    log("config %d%s: %d undirected edges on %d vertices (generated in %.1fs)"
        % (cfg, "" if scale_down == 1 else " / %d" % scale_down, src.size, n, t_gen))
    t0 = time.time()
    use_chunked = cfg == 5       # the config's device budget and chunk size apply
    if use_chunked:
        g = ntp.ntp_graph_build(n, src, dst, device_budget_bytes=spec.device_budget_bytes // scale_down,
                                chunk_edges=max(1024, spec.chunk_edges // scale_down))
    else:
        g = ntp.ntp_graph_build(n, src, dst)
    t_build = time.time() - t0
    info = ntp.ntp_graph_info(g)
    nnz = info["nnz"]
    log("config %d: n=%d nnz=%d max_degree=%d chunks=%d (graph build %.2fs)" % (cfg, n, nnz, info["max_degree"], info["n_chunks"], t_build))

    dims = spec.layers
    L = len(dims) - 1
    f32 = dict(dtype=torch.float32, device=dev)
    events = []
    full_model = cfg in (1, 2) or args.full_width
    share_bf16 = agg_dtype == "bf16" and not full_model
    X = Ws = labels = None

    if full_model:
        X = torch.from_numpy(gen.make_features(cfg, dims[0], args.seed, scale_down)).to(dev)
        Ws = [torch.from_numpy(gen.glorot_weight(dims[i], dims[i + 1], args.seed, i)).to(dev) for i in range(L)]
        labels = torch.from_numpy(gen.uniform_labels(n, dims[-1], args.seed).astype(np.int64)).to(dev)
        ep = GcnEpoch(g, n, dims, order=args.order)

        def step():
            ep.run(X, Ws, labels)

        def set_events(lst):
            ep.events = lst
        if args.order == "decoupled":
            edge_feats = nnz * dims[-1] * 2 * L
        else:       # per layer: aggregation at the input width, or at the output width when transform-first
            tf = ep.transform_first
            fwd_w = sum(dims[l + 1] if tf[l] else dims[l] for l in range(L))
            bwd_w = sum(dims[l + 1] if tf[l] else (dims[l] if l > 0 else 0) for l in range(L))
            edge_feats = nnz * (fwd_w + bwd_w)
        flops_nn = sum(2 * n * dims[i] * dims[i + 1] * (3 if i > 0 else 2) for i in range(L))
        workload = "%s: %s GCN epoch fwd+bwd, %s, full width" % (spec.name, args.order, "->".join(map(str, dims)))
    else:
        # one worker's share (1 of 8): slice aggregations on the full graph, transforms on N/8 rows
        W8 = spec.n_workers
        slices = [-(-dims[l] // W8) for l in range(L)]          # ceil(width / 8) per layer input
        n_share = -(-n // W8)
        edge_feats = nnz * (sum(slices) + sum(slices[1:]))
        flops_nn = sum(2 * n_share * dims[i] * dims[i + 1] * (3 if i > 0 else 2) for i in range(L))
        workload = ("%s%s: one worker's share (1/%d) of a %s epoch: slice aggregations F=%s fwd+bwd on the full graph, "
                    "transforms on %d rows" % (spec.name, "" if scale_down == 1 else " at 1/%d size" % scale_down, W8,
                                               "->".join(map(str, dims)), slices, n_share))
        if not share_bf16 and not use_chunked:
            # fp32 on a resident graph: all eight workers run once on seeded inputs (the full model's
            # epoch: the buffers then hold real activations and gradients), and the timed step is
            # worker 0's calls on them
            X = torch.empty(n, dims[0], **f32)
            tg = torch.Generator(device=dev)
            tg.manual_seed(args.seed)
            X.normal_(generator=tg)
            Ws = [torch.from_numpy(gen.glorot_weight(dims[l], dims[l + 1], args.seed, l)).to(dev) for l in range(L)]
            labels = torch.from_numpy(gen.uniform_labels(n, dims[-1], args.seed).astype(np.int64)).to(dev)
            tp = TensorParallelEpoch(g, n, dims, workers=W8, overlap_dw=args.overlap_dw)
            tp.run(X, Ws, labels)
            torch.cuda.synchronize()
            log("config %d: all %d workers ran once, loss %.5f; timing worker 0's calls" % (cfg, W8, float(tp.loss)))

            def step():
                tp.run_worker(0)

            def set_events(lst):
                tp.events = lst
            workload += "; operands: the activations and gradients of a full 8-worker epoch"
        else:
            # bf16 slices, and config 5 (whose full-width matrices do not fit beside the topology):
            # timing only, on seeded random operands of the share's shapes
            tg = torch.Generator(device=dev)
            tg.manual_seed(args.seed)
            code_s = ntp.NTP_BF16 if share_bf16 else ntp.NTP_F32
            tdt = torch.bfloat16 if share_bf16 else torch.float32
            lds = [line_padded_ld(s_, 2 if share_bf16 else 4) for s_ in slices]
            xs = [torch.randn(n, ld, generator=tg, **f32).to(tdt) for ld in lds]
            ys = [torch.empty_like(x) for x in xs]
            A = [torch.randn(n_share, dims[l], generator=tg, **f32).to(tdt) for l in range(L)]
            Ws = [torch.from_numpy(gen.glorot_weight(dims[l], dims[l + 1], args.seed, l)).to(dev).to(tdt) for l in range(L)]
            H = [torch.empty(n_share, dims[l + 1], dtype=tdt, device=dev) for l in range(L)]
            dH = [torch.randn(n_share, dims[l + 1], generator=tg, **f32).to(tdt) for l in range(L)]
            dA = [torch.empty(n_share, dims[l], dtype=tdt, device=dev) for l in range(L)]
            dW = [torch.empty(dims[l], dims[l + 1], **f32) for l in range(L)]
            wsb = max(ntp.ntp_nn_bwd_workspace_bytes(n_share, dims[l], dims[l + 1]) for l in range(L))
            ws = torch.empty(max(wsb, 4), dtype=torch.uint8, device=dev)
            holder = {"ev": None}
            copy_stream = torch.cuda.Stream() if use_chunked else None

            def agg_fwd(gr, xi, yo, s_, ldx, ldy, code, st):
                if use_chunked:
                    ntp.ntp_chunked_aggregate(gr, ntp.NTP_FWD, xi, yo, s_, ldx, ldy, code, st, copy_stream)
                else:
                    ntp.ntp_aggregate_fwd(gr, xi, yo, s_, ldx, ldy, code, st)

            def agg_bwd(gr, xi, yo, s_, ldx, ldy, code, st):
                if use_chunked:
                    ntp.ntp_chunked_aggregate(gr, ntp.NTP_BWD, xi, yo, s_, ldx, ldy, code, st, copy_stream)
                else:
                    ntp.ntp_aggregate_bwd(gr, xi, yo, s_, ldx, ldy, code, st)

            def timed(tag, fn, *a):
                if holder["ev"] is None:
                    return fn(*a)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn(*a)
                e1.record()
                holder["ev"].append((tag, e0, e1))

            def step():
                st = torch.cuda.current_stream()
                for l in range(L):
                    s_ = slices[l]
                    timed("agg_fwd f=%d" % s_, agg_fwd, g, xs[l], ys[l], s_, lds[l], lds[l], code_s, st)
                    act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
                    timed("nn_fwd %dx%d" % (dims[l], dims[l + 1]), ntp.ntp_nn_fwd, A[l], Ws[l], H[l], n_share, dims[l], dims[l + 1], act, code_s, st)
                for l in range(L - 1, -1, -1):
                    act = ntp.NTP_ACT_RELU if l < L - 1 else ntp.NTP_ACT_NONE
                    timed("nn_bwd %dx%d" % (dims[l], dims[l + 1]), ntp.ntp_nn_bwd, A[l], Ws[l], H[l], dH[l], dA[l] if l > 0 else None, dW[l],
                          n_share, dims[l], dims[l + 1], act, code_s, ws, wsb, st)
                    if l > 0:
                        s_ = slices[l]
                        timed("agg_bwd f=%d" % s_, agg_bwd, g, ys[l], xs[l], s_, lds[l], lds[l], code_s, st)

            def set_events(lst):
                holder["ev"] = lst
            workload += "; operands: seeded random matrices of the share's shapes"

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Every eighth step of the timed region records a pair of HIP events around each library call
    # (the per-call durations below); the pairs cost about 6 us per call, which over all steps
    # would be 5-6 % of a config-2 epoch.
    every = 8
    n_instrumented = 0
    t0 = time.perf_counter()
    for i in range(args.steps):
        instrument = i % every == 0
        set_events(events if instrument else None)
        n_instrumented += instrument
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    set_events(None)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    geps = edge_feats / (ms_per_step * 1e-3) / 1e9

    # per-call durations from the HIP events recorded inside the timed region
    per = {}
    for tag, e0, e1 in events:
        per.setdefault(tag, []).append(e0.elapsed_time(e1))
    calls = {k: dict(n=len(v), avg_ms=float(np.mean(v)), min_ms=float(np.min(v))) for k, v in per.items()}
    agg_ms = sum(np.sum(v) for k, v in per.items() if k.startswith("agg")) / n_instrumented
    nn_ms = sum(np.sum(v) for k, v in per.items() if k.startswith("nn")) / n_instrumented

    # roofline of the dominant aggregation kernel: the width with the largest share of step time
    # (timed on its forward launches: a backward launch may carry the ReLU mask of the layer below on
    # its way out, which reads one more matrix than the algorithmic bytes of a plain aggregation count)
    agg_tags = [k for k in per if k.startswith("agg")]
    by_width = {}
    for k in agg_tags:
        f = int(k.split("f=")[1])
        by_width.setdefault(f, []).extend(per[k])
    fdom = max(by_width, key=lambda f: np.sum(by_width[f]))
    dur_ms = float(np.mean(per.get("agg_fwd f=%d" % fdom, by_width[fdom])))
    dtype_label = "bf16" if share_bf16 else "f32"
    balg = agg_bytes(n, nnz, fdom, 2 if share_bf16 else 4)
    achieved = balg / (dur_ms * 1e-3) / 1e9
    traffic, traffic_source = (profile_traffic("cfg%d_f%d%s" % (cfg, fdom, "_bf16" if share_bf16 else ""))
                               if scale_down == 1 and not args.unpermuted else (None, None))
    roofline = dict(bound="hbm", kernel="agg_kernel (F_slice=%d, %s, forward launches)" % (fdom, "bf16" if share_bf16 else "fp32"), achieved=achieved, peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=achieved / HBM_PEAK_GBS, traffic=traffic,
                    # `traffic` is not counted by this run: it is the L2-boundary byte count (reads that
                    # miss the L2, Infinity-Cache hits included, plus writes) of an earlier rocprofv3 run
                    traffic_source=traffic_source,
                    algorithmic_bytes_per_launch=balg, avg_launch_ms=dur_ms,
                    traffic_gbs=(traffic / (dur_ms * 1e-3) / 1e9) if traffic else None,
                    overfetch=(traffic / balg) if traffic else None,
                    # what this chip delivers for random 128-byte lines that miss the L2 (stand-alone probe, same
                    # run), and the kernel's L2-boundary traffic against it: at 1.0 the kernel's time is its L2 misses
                    random_line_rate_gbs=LINE_RATE,
                    traffic_vs_random_line_rate=((traffic / (dur_ms * 1e-3) / 1e9) / LINE_RATE["hbm_1gb_gbs"]) if traffic and LINE_RATE else None,
                    # the algorithmic rate against a plain device copy measured in this run
                    copy_gbs=copy_gbs, frac_of_copy=(achieved / copy_gbs) if copy_gbs else None,
                    geps_kernel=nnz * fdom / (dur_ms * 1e-3) / 1e9)
    nn_tflops = flops_nn / (nn_ms * 1e-3) / 1e12 if nn_ms > 0 else None
    split_core = not os.environ.get("NTP_NN_CORE", "").startswith("f")
    nn_peak = SPLIT_PEAK_TFLOPS if split_core else FP32_MFMA_PEAK_TFLOPS
    if share_bf16:
        nn_peak = BF16_MFMA_PEAK_TFLOPS       # bf16 operands: one bf16 matrix instruction per product
    roofline_nn = dict(bound="mfma",
                       kernel=("gemm_split_kernel (fp32 products from bf16 pieces, 6 bf16 MFMA per product; "
                               "peak = 2500/6) + gemm_kernel (fp32 MFMA) for narrow products, all transform calls of a step"
                               if split_core else "gemm_kernel (fp32 MFMA, all transform calls of a step)"),
                       achieved=nn_tflops, peak=nn_peak, unit="TFLOP/s (useful fp32 flops)",
                       frac=(nn_tflops / nn_peak) if nn_tflops else None,
                       frac_of_fp32_mfma_peak=(nn_tflops / FP32_MFMA_PEAK_TFLOPS) if nn_tflops else None, traffic=None)

    # context, outside the timed region: the same model in the paper's decoupled order
    # (all transforms first, then L aggregations at the output width, Section 4.1)
    other_order_ms = None
    reordered_ms = None
    overlap_ms = None
    if context and cfg in (1, 2) and args.order == "layerwise" and not args.full_width and not args.no_context:
        def epoch_ms(**kw):
            e = GcnEpoch(g, n, dims, **kw)
            for _ in range(3):
                e.run(X, Ws, labels)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for _ in range(args.steps):
                e.run(X, Ws, labels)
            torch.cuda.synchronize()
            return (time.perf_counter() - t2) * 1e3 / args.steps
        other_order_ms = epoch_ms(order="decoupled")
        # the layer-wise epoch with its last layer evaluated as A_hat (H W)
        reordered_ms = epoch_ms(order="reordered")
        # and with every dW issued on a second stream beside dA and the backward aggregation that follows it
        overlap_ms = epoch_ms(order="layerwise", overlap_dw=True)

    cpu_baseline = None
    if cpu_baseline_from is not None and not args.no_cpu_baseline:
        # the oracle's rate measured on a smaller instance of the same generator (building sampled rows
        # of this one means a pass over all of its edges on the host, a minute at 1.6 G edges)
        cpu_baseline = dict(cpu_baseline_from)
        cpu_baseline["sample"] = "taken from the 1/8-size instance of the same graph: " + cpu_baseline_from["sample"]
    elif not args.no_cpu_baseline:
        import oracle
        t0 = time.time()
        fo = fdom
        # the oracle's rate on this graph is some 10 G edge-features/s on 16 cores: bound the sample
        # to about cpu_seconds / 3 per repetition (three repetitions, the best one counts)
        budget_ef = 3e9 * cpu_seconds / 20.0
        xo = gen.normal_features(n, fo, args.seed)
        if nnz * fo <= budget_ef and nnz <= 2e8:
            og = oracle.build_graph(n, src, dst)
            m = og.csr
            done = og.nnz * fo
            sample = "one forward aggregation of the whole graph at F_slice=%d" % fo
        else:
            # a uniform sample of rows, built one by one from the edge list
            og = None
            k = max(1000, int(n * budget_ef / (nnz * fo)))
            rows = np.sort(gen.stream_rng(args.seed, 99).choice(n, size=min(k, n), replace=False)).astype(np.int64)
            m = oracle.rows_from_undirected_edges(n, src, dst, rows)
            done = m.nnz * fo
            sample = "forward aggregation of %d uniformly sampled rows (%d entries) at F_slice=%d" % (rows.size, m.nnz, fo)
        best = None
        for _ in range(3):
            t1 = time.perf_counter()
            oracle.aggregate(m, xo)
            dt = time.perf_counter() - t1
            best = dt if best is None else min(best, dt)
        cpu_baseline = dict(value=done / best / 1e9, unit="GEPS", cores=oracle.num_threads(), kind="oracle",
                            sample=sample + ", fp64, best of 3 (%.3fs)" % best)
        if cfg <= 2 and og is not None:        # small enough to time on one core as well
            all_cores = oracle.num_threads()
            oracle.set_num_threads(1)
            t1 = time.perf_counter()
            oracle.aggregate(m, xo)
            cpu_baseline["single_core_value"] = done / (time.perf_counter() - t1) / 1e9
            oracle.set_num_threads(all_cores)
            if args.order == "layerwise" and not args.full_width and context:
                # the same step as `value` (one whole layer-wise epoch: every aggregation and every
                # transform, fp64) through the oracle, and its rate by the same definition
                Xo = gen.make_features(cfg, dims[0], args.seed, scale_down)
                Wo = [gen.glorot_weight(dims[i], dims[i + 1], args.seed, i) for i in range(L)]
                lo = gen.uniform_labels(n, dims[-1], args.seed).astype(np.int64)
                t1 = time.perf_counter()
                oracle.epoch_layerwise(og, Xo, Wo, lo)
                dt = time.perf_counter() - t1
                cpu_baseline["epoch_s"] = dt
                cpu_baseline["epoch_value"] = edge_feats / dt / 1e9
                cpu_baseline["sample"] += "; epoch_value: one whole layer-wise epoch of the same model (%.2fs)" % dt
        log("oracle baseline: %.2f GEPS on %d threads (%.1fs incl. building the rows)" % (cpu_baseline["value"], cpu_baseline["cores"], time.time() - t0))

    # arithmetic type of the step: fp32 storage and accumulation; the transforms form every fp32
    # product from three bf16 pieces per operand on the bf16 matrix instructions (as accurate as fp32
    # arithmetic; narrow products use the fp32 matrix instructions)
    dtype_full = "bf16 (fp32 accumulate)" if share_bf16 else ("f32 (transform: 3x bf16-split MFMA)" if split_core else "f32")
    out = {
        "metric": "aggregation GEPS (stored entries x F_slice / s) over the step; epoch ms in ms_per_step",
        "value": geps, "unit": "GEPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_full, "data": "synthetic",
        "config": {"workload": workload, "n_vertices": n, "nnz": nnz, "max_degree": info["max_degree"],
                   "seed": args.seed, "scale_down": scale_down,
                   "vertex_ids": "generator order" if args.unpermuted else "random relabelling"},
        "roofline": roofline, "roofline_nn": roofline_nn, "cpu_baseline": cpu_baseline,
        "agg_ms_per_step": float(agg_ms), "nn_ms_per_step": float(nn_ms),
        "agg_geps_calls_only": edge_feats / (agg_ms * 1e-3) / 1e9 if agg_ms > 0 else None,
        "calls": calls, "instrumented_steps": n_instrumented, "graph_build_s": t_build, "graph_generate_s": t_gen,
    }
    if other_order_ms is not None:
        out.update(epoch_ms_decoupled_order=other_order_ms, epoch_ms_dw_on_second_stream=overlap_ms, epoch_ms_last_layer_reordered=reordered_ms)
    if use_chunked:
        res = ntp.ntp_graph_chunks(g)["resident"]
        out["chunks"] = {"n": int(res.size), "resident": int(res.sum()), "device_budget_bytes": spec.device_budget_bytes // scale_down,
                         "chunk_edges": max(1024, spec.chunk_edges // scale_down), "streamed_bytes_per_pass": ntp.ntp_graph_stream_bytes(g)}
    log("config %d%s %s: %.3f ms per step, %.0f GEPS; dominant aggregation F=%d %.3f ms = %.0f GB/s algorithmic = %.3f of 8 TB/s"
        % (cfg, "" if scale_down == 1 else " / %d" % scale_down, dtype_label, ms_per_step, geps, fdom, dur_ms, achieved, achieved / HBM_PEAK_GBS))
    g.close()
    return out, graph


def host_mem_available_gb():
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable:"):
                return int(line.split()[1]) / 1e6
    except Exception:
        pass
    return None


def run_step_mode(args):
    global LINE_RATE
    LINE_RATE = None if args.no_line_probe else line_rate_probe()
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(3)
    t_start = time.time()
    copy_gbs = copy_probe(torch, "cuda:0")
    if args.config is not None:
        out, _ = step_bench(args, args.config, args.scale_down, args.agg_dtype, copy_gbs)
        print(json.dumps(out), flush=True)
        return
    # default: config 3 is the line; the other configs ride along as sub-entries, each with its own
    # roofline and oracle baseline.  A sub-entry that fails is reported, not fatal.
    head, _ = step_bench(args, 3, 1, "f32", copy_gbs, cpu_seconds=20.0)
    subs = {}

    def sub(key, fn):
        try:
            t0 = time.time()
            torch.cuda.empty_cache()
            subs[key] = fn()
            subs[key]["wall_s"] = time.time() - t0
        except Exception as e:          # never lose the headline to a sub-entry
            log("bench.py: %s failed: %r" % (key, e))
            subs[key] = {"failed": repr(e)[:300]}

    keep = {}

    def cfg4_f32():
        o, keep["g4"] = step_bench(args, 4, 1, "f32", copy_gbs, cpu_seconds=6.0)
        return o
    sub("cfg4_f32", cfg4_f32)
    sub("cfg4_bf16", lambda: step_bench(args, 4, 1, "bf16", copy_gbs, graph=keep.get("g4"), cpu_seconds=6.0)[0])
    keep.clear()
    sub("cfg2", lambda: step_bench(args, 2, 1, "f32", copy_gbs, cpu_seconds=6.0, context=False)[0])
    if not args.no_scaled_config5:
        sub("cfg5_at_one_eighth", lambda: step_bench(args, 5, 8, "f32", copy_gbs, cpu_seconds=6.0)[0])
    # config 5 at full size: 75 GB of host memory, and host work (generation, graph build) that is
    # eight times that of the 1/8 instance: only if memory and the time budget allow
    mem = host_mem_available_gb()
    eighth = subs.get("cfg5_at_one_eighth", {})
    projected = 8 * (eighth.get("graph_generate_s", 30.0) + eighth.get("graph_build_s", 30.0)) + 60.0
    elapsed = time.time() - t_start
    if args.no_config5:
        subs["cfg5"] = {"skipped": "--no-config5"}
    elif mem is not None and mem < 100:
        subs["cfg5"] = {"skipped": "%.0f GB of host memory available, config 5 needs 100" % mem}
    elif not args.with_config5 and elapsed + projected > args.time_budget:
        subs["cfg5"] = {"skipped": "projected %.0f s on top of %.0f s already spent exceeds the time budget of %.0f s (--with-config5 runs it anyway)"
                                   % (projected, elapsed, args.time_budget)}
    else:
        log("config 5 at full size: projected %.0f s, %.0f s spent so far" % (projected, elapsed))
        sub("cfg5", lambda: step_bench(args, 5, 1, "f32", copy_gbs, cpu_seconds=6.0, cpu_baseline_from=eighth.get("cpu_baseline"))[0])
    head["configs"] = subs
    head["bench_wall_s"] = time.time() - t_start
    print(json.dumps(head), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None, choices=[1, 2, 3, 4, 5],
                    help="one config only (default: config 3 as the headline plus the other configs as sub-entries)")
    ap.add_argument("--with-config5", action="store_true",
                    help="default run: time config 5 at full size whatever the time budget says")
    ap.add_argument("--no-config5", action="store_true", help="default run: leave out config 5 at full size")
    ap.add_argument("--time-budget", type=float, default=420.0,
                    help="default run: seconds the whole run may take; config 5 at full size (75 GB of host memory) runs only if "
                         "its projected time fits")
    ap.add_argument("--no-scaled-config5", action="store_true", help="default run: leave out config 5's shape at 1/8 size")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--scale-down", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the extra epochs in other evaluation orders (keeps a profile to the step's own kernels)")
    ap.add_argument("--order", default="layerwise", choices=["layerwise", "decoupled", "reordered", "auto"])
    ap.add_argument("--full-width", action="store_true",
                    help="configs 3, 4: the whole model at full width on this GPU instead of one worker's share")
    ap.add_argument("--mode", default="step", choices=["step", "agg", "chunk", "budget", "gat"],
                    help="agg: time only aggregation calls at --widths (kernel tuning / profiling); "
                         "chunk: chunk-streamed vs in-memory aggregation; "
                         "budget: the config's own device budget and chunk size (config 5), with a sampled parity check")
    ap.add_argument("--chunk-edges", type=int, default=0, help="entries per chunk for --mode chunk (default nnz/8)")
    ap.add_argument("--widths", default="", help="comma-separated slice widths for --mode agg")
    ap.add_argument("--agg-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--parity-rows", type=int, default=2000,
                    help="--mode gat: uniformly sampled destinations checked against the oracle (0: no check)")
    ap.add_argument("--overlap-dw", action="store_true",
                    help="worker-share steps (configs 3, 4 in fp32): issue every weight gradient on a second stream beside dA and "
                         "the backward aggregation that follows it")
    ap.add_argument("--unpermuted", action="store_true",
                    help="keep the generator's vertex numbering (hubs at the low ids) instead of the random relabelling "
                         "the configs ask for: the best case for locality, reported as context only")
    ap.add_argument("--no-line-probe", action="store_true",
                    help="do not run paper_2412_20379_amd/line_rate_probe (a child process, started before this one touches the GPU)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (the method's collectives are out of scope); "
            "use --gpus 1.  value is the one GPU's throughput.")
        sys.exit(2)

    if args.mode == "step":
        return run_step_mode(args)
    if args.config is None:
        args.config = 2

    import numpy as np
    import torch
    import ntp_inputs as gen
    import paper_2412_20379_amd as ntp

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(3)
    dev = "cuda:0"
    spec = gen.CONFIGS[args.config]
    if args.config == 5 and args.mode != "budget":
        log("bench.py: config 5 runs under its device budget: use --mode budget or --mode step")
        sys.exit(2)
    t0 = time.time()
    n, src, dst = gen.make_graph(args.config, args.seed, args.scale_down, permute=not args.unpermuted)
    t_gen = time.time() - t0
    log("config %d: generated %d undirected edges on %d vertices in %.1fs" % (args.config, src.size, n, t_gen))

    if args.mode == "budget":
        # the config's own budget and chunk size, scaled with --scale-down
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from helpers import rel_errors
        budget = (spec.device_budget_bytes or (64 << 30)) // args.scale_down
        ce = max(1024, (spec.chunk_edges or (256 << 20)) // args.scale_down)
        f = int(args.widths.split(",")[0]) if args.widths else spec.agg_slices[0]
        out = {"mode": "budget", "config": args.config, "scale_down": args.scale_down, "n_vertices": n,
               "width": f, "device_budget_bytes": budget, "chunk_edges": ce}
        x_np = gen.normal_features(n, f, args.seed)
        x = torch.from_numpy(x_np).to(dev)
        y = torch.empty_like(x)
        cs, xs = torch.cuda.Stream(), torch.cuda.Stream()

        def timeit(fn, reps):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        # 1. every chunk streamed from pinned host memory (cold)
        t0 = time.time()
        gc = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | ntp.NTP_FORCE_STREAM,
                                 device_budget_bytes=budget, chunk_edges=ce)
        out["build_cold_s"] = time.time() - t0
        info = ntp.ntp_graph_info(gc)
        nnz = info["nnz"]
        out.update(nnz=nnz, max_degree=info["max_degree"], n_chunks=info["n_chunks"])
        log("cold graph built in %.1fs: nnz=%d chunks=%d" % (out["build_cold_s"], nnz, info["n_chunks"]))
        ch = ntp.ntp_graph_chunks(gc)
        b_pcie = ntp.ntp_graph_stream_bytes(gc)
        out["t_cold_ms"] = timeit(lambda: ntp.ntp_chunked_aggregate(gc, ntp.NTP_FWD, x, y, f, f, f, ntp.NTP_F32, cs, xs), 2)
        out["cold_pcie_bytes"] = b_pcie
        out["cold_pcie_gbs"] = b_pcie / (out["t_cold_ms"] * 1e-3) / 1e9
        y_cold = y.clone()
        log("cold: %.1f ms per aggregation (%.1f GB/s over PCIe)" % (out["t_cold_ms"], out["cold_pcie_gbs"]))
        gc.close()
        # 2. the budget decides residency (everything that fits stays on the device)
        t0 = time.time()
        gw = ntp.ntp_graph_build(n, src, dst, device_budget_bytes=budget, chunk_edges=ce)
        out["build_s"] = time.time() - t0
        chw = ntp.ntp_graph_chunks(gw)
        out["resident_chunks"] = "%d of %d" % (int(chw["resident"].sum()), len(chw["resident"]))
        out["device_bytes"] = ntp.ntp_graph_device_bytes(gw)
        out["t_warm_ms"] = timeit(lambda: ntp.ntp_chunked_aggregate(gw, ntp.NTP_FWD, x, y, f, f, f, ntp.NTP_F32, cs, xs), args.steps)
        assert torch.equal(y, y_cold), "streamed and resident results differ"
        if chw["resident"].all():
            out["t_inmem_ms"] = timeit(lambda: ntp.ntp_aggregate_fwd(gw, x, y, f, f, f, ntp.NTP_F32, cs), args.steps)
            out["warm_over_inmem"] = out["t_warm_ms"] / out["t_inmem_ms"]
        out["geps_warm"] = nnz * f / (out["t_warm_ms"] * 1e-3) / 1e9
        out["alg_gbs_warm"] = agg_bytes(n, nnz, f) / (out["t_warm_ms"] * 1e-3) / 1e9
        out["geps_cold"] = nnz * f / (out["t_cold_ms"] * 1e-3) / 1e9
        log("resident: %s chunks, %.3f ms per aggregation, %.0f GEPS" % (out["resident_chunks"], out["t_warm_ms"], out["geps_warm"]))
        # 3. parity on sampled rows, recomputed by the oracle from the edge list
        rowptr, _, _ = (ntp.ntp_graph_export(gw) if nnz < (1 << 28) else (None, None, None))
        if rowptr is None:
            rp = np.empty(n + 1, dtype=np.int64)
            ntp.binding._check(ntp.lib().ntp_graph_export(gw.handle, ntp.NTP_CSR, ntp.binding._ptr(rp), None, None))
            rowptr = rp
        deg = np.diff(rowptr)
        top = np.argsort(deg)[-1000:]                  # the 1,000 highest-degree rows ...
        uni = gen.stream_rng(args.seed, 98).choice(n, size=min(n, 100000), replace=False)     # ... and 100,000 uniform ones
        rows = np.unique(np.concatenate([top, uni])).astype(np.int64)
        t0 = time.time()
        m = oracle.rows_from_undirected_edges(n, src, dst, rows)
        assert np.array_equal(np.diff(m.rowptr), deg[rows]), "row lengths differ from the oracle's"
        ref, ref_abs = oracle.aggregate(m, x_np, with_abs=True)
        got = y[torch.from_numpy(rows).to(dev)].cpu().numpy()
        nerr, cerr, zok = rel_errors(got, ref, ref_abs)
        out["parity"] = {"rows": int(rows.size), "normwise": nerr, "componentwise": cerr, "pass": bool(nerr <= 1e-5 and cerr <= 1e-5 and zok),
                         "oracle_s": time.time() - t0}
        log("parity on %d sampled rows: normwise %.2e componentwise %.2e" % (rows.size, nerr, cerr))
        gw.close()
        print(json.dumps(out), flush=True)
        if not out["parity"]["pass"]:
            sys.exit(1)
        return

    t0 = time.time()
    g = ntp.ntp_graph_build(n, src, dst)
    t_build = time.time() - t0
    info = ntp.ntp_graph_info(g)
    nnz = info["nnz"]
    log("config %d: n=%d nnz=%d max_degree=%d (generated in %.1fs, graph build %.2fs)"
        % (args.config, n, nnz, info["max_degree"], t_gen, t_build))
    if args.copy_probe:
        copy_probe(torch, dev)

    if args.mode == "chunk":
        # Section 4.2.1 schedule: in-memory call vs chunked call with every chunk resident, with
        # about half of the chunks resident (budget), and with every chunk streamed from pinned memory
        f = int(args.widths.split(",")[0]) if args.widths else spec.agg_slices[0]
        ce = args.chunk_edges or max(1024, nnz // 8)
        x = torch.from_numpy(gen.normal_features(n, f, args.seed)).to(dev)
        y = torch.empty_like(x)
        cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
        # PCIe probe: pinned host -> device copy of 256 MiB
        hp = torch.empty(1 << 26, dtype=torch.float32).pin_memory()
        dp = torch.empty(1 << 26, dtype=torch.float32, device=dev)
        dp.copy_(hp, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4):
            dp.copy_(hp, non_blocking=True)
        torch.cuda.synchronize()
        pcie_gbs = 4 * (1 << 28) / (time.perf_counter() - t0) / 1e9
        del hp, dp

        def timeit(graph, chunked):
            def call():
                if chunked:
                    ntp.ntp_chunked_aggregate(graph, ntp.NTP_FWD, x, y, f, f, f, ntp.NTP_F32, cs, xs)
                else:
                    ntp.ntp_aggregate_fwd(graph, x, y, f, f, f, ntp.NTP_F32, cs)
            for _ in range(args.warmup):
                call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                call()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps

        t_inmem = timeit(g, False)
        ref = y.clone()
        out = {"mode": "chunk", "config": args.config, "n_vertices": n, "nnz": nnz, "width": f, "chunk_edges": ce,
               "pcie_h2d_gbs": pcie_gbs, "t_inmem_ms": t_inmem}
        g_all = ntp.ntp_graph_build(n, src, dst, chunk_edges=ce)
        out["t_chunked_all_resident_ms"] = timeit(g_all, True)
        # the chunked plan cuts long rows into pieces sized for a chunk's launch, the in-memory plan for
        # the whole graph: the same sums in another order, equal to rounding; the streamed variants below
        # share the chunked plan and must reproduce its bits
        diff = float((y - ref).abs().max() / ref.abs().max())
        assert diff <= 1e-5, diff
        out["chunked_vs_inmem_max_rel_diff"] = diff
        ref = y.clone()
        g_all.close()
        total_bytes = nnz * 8 + n * 12
        g_half = ntp.ntp_graph_build(n, src, dst, device_budget_bytes=int(total_bytes * 0.62), chunk_edges=ce)
        chh = ntp.ntp_graph_chunks(g_half)
        streamed = ~chh["resident"].astype(bool)
        b_pcie_half = ntp.ntp_graph_stream_bytes(g_half)
        out["t_warm_ms"] = timeit(g_half, True)
        assert torch.equal(y, ref)
        out["warm_resident_chunks"] = "%d of %d" % (int(chh["resident"].sum()), len(streamed))
        out["warm_pcie_bytes"] = b_pcie_half
        out["warm_floor_ms"] = max(t_inmem, b_pcie_half / (pcie_gbs * 1e9) * 1e3)
        g_half.close()
        g_cold = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | ntp.NTP_FORCE_STREAM, chunk_edges=ce)
        chc = ntp.ntp_graph_chunks(g_cold)
        b_pcie = ntp.ntp_graph_stream_bytes(g_cold)
        out["t_cold_ms"] = timeit(g_cold, True)
        assert torch.equal(y, ref)
        out["cold_pcie_bytes"] = b_pcie
        out["cold_floor_ms"] = max(t_inmem, b_pcie / (pcie_gbs * 1e9) * 1e3)
        # four column slices against one streamed pass over the topology
        xs4 = [torch.randn_like(x) for _ in range(4)]
        ys4 = [torch.empty_like(x) for _ in range(4)]

        def four_separate():
            for a_, b_ in zip(xs4, ys4):
                ntp.ntp_chunked_aggregate(g_cold, ntp.NTP_FWD, a_, b_, f, f, f, ntp.NTP_F32, cs, xs)

        def four_multi():
            ntp.ntp_chunked_aggregate_multi(g_cold, ntp.NTP_FWD, xs4, ys4, f, f, f, ntp.NTP_F32, cs, xs)
        for fn, key in ((four_separate, "t_cold_4_slices_separate_ms"), (four_multi, "t_cold_4_slices_one_pass_ms")):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            out[key] = (time.perf_counter() - t0) * 1e3 / args.steps
        out["cold_over_floor"] = out["t_cold_ms"] / out["cold_floor_ms"]
        out["warm_over_floor"] = out["t_warm_ms"] / out["warm_floor_ms"]
        out["all_resident_over_inmem"] = out["t_chunked_all_resident_ms"] / t_inmem
        g_cold.close()
        log(json.dumps(out, indent=1))
        print(json.dumps(out), flush=True)
        g.close()
        return

    if args.mode == "gat":
        # GAT-style edge attention (Section 2.1): weights of all edges by ntp_edge_softmax, then the
        # aggregation with them as edge weights
        f = int(args.widths.split(",")[0]) if args.widths else spec.agg_slices[0]
        tg = torch.Generator(device=dev)
        tg.manual_seed(args.seed)
        p = torch.randn(n, generator=tg, device=dev)
        q = torch.randn(n, generator=tg, device=dev)
        a_in = torch.empty(nnz, device=dev)
        a_out = torch.empty(nnz, device=dev)
        ld = line_padded_ld(f, 4)
        x = torch.randn(n, ld, generator=tg, device=dev)
        y = torch.empty_like(x)
        st = torch.cuda.current_stream()

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        t_att = timed(lambda: ntp.ntp_edge_softmax(g, p, q, 0.2, a_in, a_out, st))
        t_att_in = timed(lambda: ntp.ntp_edge_softmax(g, p, q, 0.2, a_in, None, st))
        t_w = timed(lambda: ntp.ntp_aggregate_weighted(g, ntp.NTP_FWD, a_in, x, y, f, ld, ld, ntp.NTP_F32, st))
        t_s = timed(lambda: ntp.ntp_aggregate_fwd(g, x, y, f, ld, ld, ntp.NTP_F32, st))
        # gradient of the scores through the weights: two passes that each gather one feature row
        # per edge (as an aggregation of that width does) and form a dot product with it
        dp = torch.empty(n, device=dev)
        dq = torch.empty(n, device=dev)
        dy = torch.randn(n, ld, generator=tg, device=dev)
        f_sg = min(f, 1024)          # widest row the score gradient takes
        t_sg = timed(lambda: ntp.ntp_edge_softmax_bwd(g, p, q, 0.2, a_in, a_out, x, dy, f_sg, ld, ld, dp, dq, False, st))
        if f_sg != f:
            t_w = timed(lambda: ntp.ntp_aggregate_weighted(g, ntp.NTP_FWD, a_in, x, y, f_sg, ld, ld, ntp.NTP_F32, st))
        # parity at this size on sampled vertices, each built by the oracle from the edge list:
        # weights and dq of sampled destinations (uniform + the largest), dp of sampled sources
        # (all their neighbours' rows are needed for that)
        def gat_parity(tag):
            import oracle as orc          # the cpu-side check is the only user of the oracle here
            t0 = time.time()
            rng = gen.stream_rng(args.seed, 123)
            deg = np.bincount(src, minlength=n) + np.bincount(dst, minlength=n) + 1
            rowptr = np.zeros(n + 1, dtype=np.int64)
            np.cumsum(deg, out=rowptr[1:])
            order = np.argsort(deg)
            ph, qh = p.cpu().numpy(), q.cpu().numpy()
            Zh, dYh = x[:, :f_sg].cpu().numpy(), dy[:, :f_sg].cpu().numpy()
            a_h, dq_h, dp_h = a_in.cpu().numpy(), dq.cpu().numpy(), dp.cpu().numpy()

            def abs_scale(m, rows, o):
                sc = np.zeros(rows.size)
                per_entry = np.zeros(int(m.rowptr[-1]))
                for i, v in enumerate(rows):
                    b, e = int(m.rowptr[i]), int(m.rowptr[i + 1])
                    A = np.abs(Zh[m.colidx[b:e]]).astype(np.float64) @ np.abs(dYh[v]).astype(np.float64)
                    a = o["alpha"][b:e]
                    per_entry[b:e] = a * (A + float(a @ A))
                    sc[i] = per_entry[b:e].sum()
                return sc, per_entry

            vs = np.unique(np.concatenate([rng.choice(n, size=min(n, args.parity_rows), replace=False), order[-50:]])).astype(np.int64)
            mv = orc.rows_from_undirected_edges(n, src, dst, vs)
            ov = orc.edge_softmax_bwd_rows(mv, vs, ph, qh, Zh, dYh, 0.2)
            err_a = 0.0
            for i, v in enumerate(vs):
                got = a_h[rowptr[v]:rowptr[v + 1]].astype(np.float64)
                ref = ov["alpha"][mv.rowptr[i]:mv.rowptr[i + 1]]
                err_a = max(err_a, float((np.abs(got - ref) / ref).max()))
            sc_q, _ = abs_scale(mv, vs, ov)
            err_q = float((np.abs(dq_h[vs] - ov["dq"]) / np.maximum(sc_q, 1e-300)).max())
            us = np.unique(np.concatenate([rng.choice(n, size=min(n, 100), replace=False), order[-2:]])).astype(np.int64)
            mu = orc.rows_from_undirected_edges(n, src, dst, us)          # symmetric graph: a row lists the out-neighbours too
            allv = np.unique(mu.colidx).astype(np.int64)
            mn = orc.rows_from_undirected_edges(n, src, dst, allv)
            on = orc.edge_softmax_bwd_rows(mn, allv, ph, qh, Zh, dYh, 0.2)
            _, mag = abs_scale(mn, allv, on)
            where = {int(v): i for i, v in enumerate(allv)}
            err_p = 0.0
            for j, u in enumerate(us):
                tot = sc = 0.0
                for v in mu.colidx[mu.rowptr[j]:mu.rowptr[j + 1]]:
                    i = where[int(v)]
                    b, e = int(mn.rowptr[i]), int(mn.rowptr[i + 1])
                    k = b + int(np.searchsorted(mn.colidx[b:e], u))
                    tot += on["ds"][k]
                    sc += mag[k]
                err_p = max(err_p, abs(float(dp_h[u]) - tot) / max(sc, 1e-300))
            res = {"destinations": int(vs.size), "sources": int(us.size), "neighbour_rows_for_dp": int(allv.size),
                   "alpha_max_rel_err": err_a, "dq_max_err_over_sum_of_magnitudes": err_q,
                   "dp_max_err_over_sum_of_magnitudes": err_p, "seconds": time.time() - t0}
            log("GAT parity (%s) on %d destinations, %d sources (%d neighbour rows): alpha %.1e, dq %.1e, dp %.1e  (%.0fs)"
                % (tag, vs.size, us.size, allv.size, err_a, err_q, err_p, res["seconds"]))
            assert err_a <= 1e-5 and err_q <= 1e-5 and err_p <= 1e-5, "GAT parity failed (%s)" % tag
            return res

        parity = None
        if args.parity_rows > 0:
            ntp.ntp_edge_softmax_bwd(g, p, q, 0.2, a_in, a_out, x, dy, f_sg, ld, ld, dp, dq, False, st)
            torch.cuda.synchronize()
            parity = {"two_dot_product_passes": gat_parity("two dot-product passes")}
        # a whole decoupled GAT epoch (Section 4.1): MLP to the class width, attention weights, two
        # weighted aggregation rounds, loss, and the exact backward pass
        from paper_2412_20379_amd.gat import GatEpoch
        dims = spec.layers
        Xg = torch.randn(n, dims[0], generator=tg, device=dev)
        Wg = [torch.randn(dims[i], dims[i + 1], generator=tg, device=dev) * (2.0 / (dims[i] + dims[i + 1])) ** 0.5
              for i in range(len(dims) - 1)]
        a_s = torch.randn(dims[-1], generator=tg, device=dev)
        a_d = torch.randn(dims[-1], generator=tg, device=dev)
        lab = torch.randint(0, dims[-1], (n,), generator=tg, device=dev)
        gep = GatEpoch(g, n, nnz, dims, rounds=2)
        t_ep = timed(lambda: gep.run(Xg, Wg, a_s, a_d, lab))
        del gep
        # the same with the edge permutation stored (NTP_EDGE_PERM): one dot product per edge
        gp = ntp.ntp_graph_build(n, src, dst, flags=ntp.NTP_GCN_FLAGS | ntp.NTP_EDGE_PERM)
        ntp.ntp_edge_softmax(gp, p, q, 0.2, a_in, a_out, st)
        t_sg_perm = timed(lambda: ntp.ntp_edge_softmax_bwd(gp, p, q, 0.2, a_in, a_out, x, dy, f_sg, ld, ld, dp, dq, False, st))
        if parity is not None:
            ntp.ntp_edge_softmax_bwd(gp, p, q, 0.2, a_in, a_out, x, dy, f_sg, ld, ld, dp, dq, False, st)
            torch.cuda.synchronize()
            parity["with_edge_permutation"] = gat_parity("edge permutation")
        gep = GatEpoch(gp, n, nnz, dims, rounds=2)
        t_ep_perm = timed(lambda: gep.run(Xg, Wg, a_s, a_d, lab))
        del gep
        gp.close()
        # algorithmic bytes: by-destination pass reads indices, writes weights (8 B per entry) plus
        # per-vertex arrays (row pointers, p, q, the two statistics); the by-source pass the same
        # per entry plus reads of the statistics
        b_in = 8 * nnz + 8 * (n + 1) + 16 * n
        b_out = 8 * nnz + 8 * (n + 1) + 16 * n
        out = {"mode": "gat", "config": args.config, "n_vertices": n, "nnz": nnz, "width": f,
               "edge_softmax_both_orders_ms": t_att, "edge_softmax_by_destination_ms": t_att_in,
               "edge_softmax_gbs": (b_in + b_out) / (t_att * 1e-3) / 1e9,
               "edge_softmax_frac_hbm": (b_in + b_out) / (t_att * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "edges_per_s_both_orders": nnz / (t_att * 1e-3),
               "aggregate_weighted_fwd_ms": t_w, "aggregate_stored_weights_fwd_ms": t_s,
               "edge_softmax_bwd_ms": t_sg, "edge_softmax_bwd_vs_two_aggregations": t_sg / (2 * t_w),
               "edge_softmax_bwd_gathered_gbs": 2 * nnz * f_sg * 4 / (t_sg * 1e-3) / 1e9, "edge_softmax_bwd_width": f_sg,
               "gat_epoch_ms": t_ep, "gat_epoch_dims": list(dims), "gat_epoch_rounds": 2,
               "edge_softmax_bwd_with_edge_perm_ms": t_sg_perm, "gat_epoch_with_edge_perm_ms": t_ep_perm,
               "parity_sample": parity}
        log("edge softmax: %.3f ms both orders (%.0f GB/s algorithmic, %.1f%% of 8 TB/s), %.3f ms by destination only; "
            "weighted aggregation f=%d %.3f ms (stored weights %.3f ms); score gradient %.3f ms (%.2f x two aggregations)"
            % (t_att, out["edge_softmax_gbs"], 100 * out["edge_softmax_frac_hbm"], t_att_in, f, t_w, t_s, t_sg,
               out["edge_softmax_bwd_vs_two_aggregations"]))
        log("decoupled GAT epoch %s, 2 rounds: %.3f ms; with NTP_EDGE_PERM: score gradient %.3f ms, epoch %.3f ms"
            % ("-".join(str(x) for x in dims), t_ep, t_sg_perm, t_ep_perm))
        print(json.dumps(out), flush=True)
        g.close()
        return

    if args.mode == "agg":
        widths = [int(w) for w in args.widths.split(",")] if args.widths else list(spec.agg_slices)
        res = []
        scrub = None
        for f in widths:
            x0 = torch.from_numpy(gen.normal_features(n, f, args.seed)).to(dev)
            code, elem = ntp.NTP_F32, 4
            if args.agg_dtype == "bf16":
                x0 = torch.from_numpy(gen.to_bf16_bits(x0.cpu().numpy()).view(np.int16)).to(dev)
                code, elem = ntp.NTP_BF16, 2
            ld = line_padded_ld(f, elem)          # rows start on 128-byte lines
            x = torch.zeros(n, ld, dtype=x0.dtype, device=dev)
            x[:, :f] = x0
            del x0
            y = torch.empty_like(x)
            st = torch.cuda.current_stream()
            for direction, fn in (("fwd", ntp.ntp_aggregate_fwd), ("bwd", ntp.ntp_aggregate_bwd)):
                for _ in range(args.warmup):
                    fn(g, x, y, f, ld, ld, code, st)
                evs = []
                for _ in range(args.steps):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    fn(g, x, y, f, ld, ld, code, st)
                    e1.record()
                    evs.append((e0, e1))
                torch.cuda.synchronize()
                ms = np.array([a.elapsed_time(b) for a, b in evs])
                # the repetitions above start with whatever the previous one left in the caches;
                # one more call after 1 GiB of unrelated writes gives the cache-cold time
                if scrub is None:
                    scrub = torch.empty(1 << 28, dtype=torch.float32, device=dev)
                scrub.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn(g, x, y, f, ld, ld, code, st)
                e1.record()
                torch.cuda.synchronize()
                cold_ms = e0.elapsed_time(e1)
                balg = agg_bytes(n, nnz, f, elem)
                r = dict(width=f, row_stride=ld, direction=direction, dtype=args.agg_dtype, avg_ms=float(ms.mean()), min_ms=float(ms.min()),
                         median_ms=float(np.median(ms)), cache_cold_ms=float(cold_ms),
                         geps=nnz * f / (ms.mean() * 1e-3) / 1e9, alg_gbs=balg / (ms.mean() * 1e-3) / 1e9,
                         frac_hbm=balg / (ms.mean() * 1e-3) / 1e9 / HBM_PEAK_GBS)
                log("agg %s f=%d %s: %.3f ms (median %.3f, min %.3f, cache-cold %.3f)  %.0f GEPS  %.0f GB/s algorithmic (%.1f%% of 8 TB/s)"
                    % (direction, f, args.agg_dtype, r["avg_ms"], r["median_ms"], r["min_ms"], r["cache_cold_ms"], r["geps"], r["alg_gbs"],
                       100 * r["frac_hbm"]))
                res.append(r)
        print(json.dumps({"mode": "agg", "config": args.config, "n_vertices": n, "nnz": nnz,
                          "max_degree": info["max_degree"], "vertex_ids": "generator order" if args.unpermuted else "random relabelling",
                          "results": res}), flush=True)
        g.close()
        return


if __name__ == "__main__":
    main()
