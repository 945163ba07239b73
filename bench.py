#!/usr/bin/env python3
"""Throughput of one BSP Parameter-Server training iteration on one MI355X.

A step is the whole hot path on one fresh synthetic batch that is already resident in
HBM: set_batch + worker_step for all K shards + aggregate + apply_update (parameters are
really updated every step; distinct resident batches are rotated).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1|cfg2|cfg3|cfg4|cfg5]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0
VALU_FP32_PEAK_TFLOPS = 157.3  # fp32 vector arithmetic (the fp32 products of small models use no matrix cores)


# HBM bytes per step and kernel class of the config-2 workload, from rocprofv3 counter runs
# (FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy kernel's reading).  A class's entry
# is only reported while the code of the source file of its kernels and of the file that launches
# them (comments and white space aside) still has the fingerprint it had when the counters were taken.
MEASURED_TRAFFIC = {
    "cfg2": {
        "gemm_fwd": (73.7e6, "gemm.hip"), "gemm_bwd": (90.6e6, "gemm.hip"), "wgrad_adagrad": (183.9e6, "gemm.hip"),
        "pool": (92.3e6, "embed.hip"),
        "sparse_adagrad": (201.5e6, "coalesce.hip"), "seg_reduce_long": (2.5e6, "coalesce.hip"),
    },
    "cfg3": {"sparse_adagrad": (761.0e6, "coalesce.hip"), "wgrad_adagrad": (623.8e6, "gemm.hip"),
             "pool": (304.6e6, "embed.hip")},
    "cfg4": {"sparse_adagrad": (8871.4e6, "coalesce.hip"), "wgrad_adagrad": (2131.3e6, "gemm.hip"),
             "pool": (2245.4e6, "embed.hip")},
    "cfg5": {"adam": (15032.4e6, "optim.hip")},
    "sha1": {"gemm.hip": "67876aa8387e26f2bce5efd17e6ee8c9737eade0",
             "embed.hip": "2ab400f86171f3c0a2539f685328e0b9611bdaef",
             "coalesce.hip": "662ffdbbe53e42ee464a9896528c53d71366ee53",
             "optim.hip": "79090e5f4d378e258fa3538b8574f6e9a57c6998",
             "ctx.hip": "61eb7572c3832fd95dcb74b7e9b648c38227aa35"},
}


def _code_fingerprint(path):
    """sha1 of a source file's code: comments removed, white space collapsed."""
    import re
    try:
        text = open(path, encoding="utf-8").read()
    except OSError:
        return None
    text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
    text = re.sub(r"//[^\n]*", " ", text)
    return hashlib.sha1(" ".join(text.split()).encode()).hexdigest()


def _measured_traffic(workload, kernel_class, launches_per_step):
    entry = MEASURED_TRAFFIC.get(workload, {}).get(kernel_class)
    if entry is None:
        return None
    nbytes, src = entry
    # the kernel's own source file and the file that chooses its launch shape and the sizes of its work items
    for name in (src, "ctx.hip"):
        sha = _code_fingerprint(os.path.join(ROOT, "paper_2404_09679_amd", "csrc", name))
        if sha is None or sha != MEASURED_TRAFFIC["sha1"].get(name):
            return None
    return nbytes / max(launches_per_step, 1e-9)


def _bytes_and_flops(cfg, stats, model):
    """Algorithmic (compulsory) HBM bytes, or flops, of one step per kernel class."""
    F, D, B, K = cfg.num_fields, cfg.dim, stats["B"], stats["K"]
    nnz, U, P = stats["nnz"], stats["U"], cfg.num_params
    e = 2 if cfg.table_dtype == "bf16" else 4
    es = 2 if cfg.gemm_dtype == "bf16" else 4
    ldx = (cfg.input_width + 7) // 8 * 8
    state_row = 4 if cfg.adagrad_state == "rowwise" else 4 * D
    s = cfg.layer_sizes
    L = len(s) - 1
    fwd = sum(2 * B * s[l] * s[l + 1] for l in range(L - 1))
    dgrad = sum(2 * B * s[l + 1] * (s[l] if l > 0 else F * D) for l in range(L - 1))
    passes = model["sort_passes"]
    gemm = "mfma" if cfg.gemm_dtype == "bf16" else "alu"
    out = {
        # ids, offsets, every distinct row once, pooled inputs (+ transposed copy and the sample
        # index of every lookup for the sort)
        "pool": ("hbm", 4 * nnz + 4 * F * (B + 1) + U * D * e + B * ldx * es
                 + (B * ldx * 2 if cfg.gemm_dtype == "bf16" else 0) + 4 * nnz),
        "gemm_fwd": (gemm, fwd),
        "gemm_bwd": (gemm, dgrad),           # the data-gradient chain on the launch stream
        "gemm_dgrad": (gemm, dgrad),
        "gemm_wgrad": (gemm, fwd),
        "wgrad_adagrad": (gemm, fwd),    # weight gradients with the aggregation and dense Adagrad in the epilogue
        "sort_hist": ("hbm", passes * 4 * nnz),
        "sort_scatter": ("hbm", 4 * nnz + 8 * nnz + (passes - 1) * 16 * nnz),
        "seg_heads": ("hbm", 4 * nnz),
        "seg_emit": ("hbm", 4 * nnz + 8 * U),
        # one fused kernel: segmented sum of the per-lookup gradient rows + row-sparse Adagrad
        # (sample indices, run table, every pooled-gradient row once, touched rows and state
        # read and written); the long-run chunk kernels work on the same bytes
        "sparse_adagrad": ("hbm", 4 * nnz + 12 * U + B * F * D * 4 + U * (2 * D * e + 2 * state_row)),
        # the long runs' finish kernel: chunk sums read, rows and state of the hot rows (counted
        # with the fused kernel above, whose launch computes the chunk sums)
        "seg_reduce_long": ("hbm", 0),
        # K shard gradients read once, fp32 weights and state read and written, both bf16 copies
        "dense_adagrad": ("hbm", P * ((K + 4) * 4 + (4 if cfg.gemm_dtype == "bf16" else 0))),
        # last hidden activation read; its gradient written row-major and transposed; labels,
        # logits, per-sample loss and dz
        "head": ("hbm", B * (s[L - 1] * es * (3 if cfg.gemm_dtype == "bf16" else 2) + 16)),
        "head_reduce": ("hbm", B * (s[L - 1] * es + 8)),
        "bias_grad": ("hbm", sum(B * s[l + 1] * 4 for l in range(L - 1))),
        "sort_scan": ("hbm", 0),
        "seg_scan": ("hbm", 4 * B),
        "transpose": ("hbm", 0),
        # the views' kernels (not part of a bench step)
        "seg_reduce": ("hbm", 4 * nnz + 12 * U + B * F * D * 4 + U * D * 4),
        "dense_agg": ("hbm", P * (K + 1) * 4),
    }
    return out


def run_ranking(args, cfg_id):
    import numpy as np
    import torch

    import paper_2404_09679_amd as A
    import workload as wl

    cfg = wl.CONFIGS[cfg_id]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    F, R, D = cfg.num_fields, cfg.rows_per_field, cfg.dim
    tdtype = torch.bfloat16 if cfg.table_dtype == "bf16" else torch.float32
    tables = torch.empty((F * R, D), dtype=tdtype, device=dev)
    A.fill_tables(tables, F, R, D, 0.05)
    state = torch.zeros((F * R, D) if cfg.adagrad_state == "elementwise" else (F * R,), dtype=torch.float32,
                        device=dev)
    params = torch.from_numpy(wl.make_mlp_params(cfg)).to(dev)
    pstate = torch.zeros_like(params)
    nb = 8 if cfg.batch * cfg.num_fields < (1 << 20) else 2   # resident batches that are rotated
    batches = [wl.make_batch(cfg, i) for i in range(nb)]
    max_nnz = max(int(b.field_ptr[-1]) for b in batches)
    model = A.model_from_config(cfg, max_nnz=max_nnz)
    ctx = A.Context(model)
    ctx.bind(tables, state, params, pstate)
    if args.single_stream:   # no overlap: every kernel on the launch stream (stand-alone durations per class)
        ctx.set_library_streams(False)
    for i, b in enumerate(batches):   # fingerprints of the generated inputs, for the run log
        h = hashlib.sha256()
        for arr in (b.ids, b.offsets, b.dense, b.labels):
            h.update(np.ascontiguousarray(arr).tobytes())
        print(f"[inputs] {cfg.name} batch {i}: lookups {int(b.field_ptr[-1])}, sha256 {h.hexdigest()}",
              file=sys.stderr)
    dbatches = []
    for b in batches:
        dbatches.append((torch.from_numpy(b.ids).to(dev), b.field_ptr, torch.from_numpy(b.offsets).to(dev),
                         torch.from_numpy(b.dense).to(dev) if cfg.num_dense else None,
                         torch.from_numpy(b.labels).to(dev)))
    K, B = cfg.num_shards, cfg.batch
    loss = torch.zeros(K, dtype=torch.float32, device=dev)
    ctx.assign_shard(B, K, sizes=cfg.shard_sizes)

    def step(i):
        ids, fp, off, dense, labels = dbatches[i % nb]
        ctx.set_batch(ids, fp, off, dense, labels)
        ctx.worker_step_all(loss)
        ctx.aggregate()
        ctx.apply_update()

    names = A.kernel_names()
    # W untimed warm-up steps (first launches, code object loading, cold caches), then a short
    # classification pass on the warm library: every kernel class bracketed by HIP events on its
    # stream, read back after each step, so that the per-class figure is a median over steps
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    CLASSIFY_STEPS = 9
    samples = {}
    ctx.profile(1)
    for i in range(CLASSIFY_STEPS):
        step(args.warmup + i)
        torch.cuda.synchronize()
        for kid, name in enumerate(names):
            n, ms = ctx.profile_read(kid)
            if n:
                samples.setdefault(name, []).append((n, ms))
    ctx.profile(0)
    per_class = {k: (float(np.median([n for n, _ in v])), float(np.median([ms for _, ms in v])))
                 for k, v in samples.items()}   # launches per step, ms per step
    # the kernels that build the coalescing structure, the weight-gradient products and the dense
    # update run on side streams beside the launch stream: they are off the critical path
    side = {"sort_hist", "sort_scan", "sort_scatter", "seg_heads", "seg_scan", "seg_emit", "gemm_wgrad",
            "dense_adagrad", "wgrad_adagrad"}
    bits = max(1, int(np.ceil(np.log2(R))))
    stats = dict(B=B, K=K, nnz=float(np.mean([b.field_ptr[-1] for b in batches])),
                 U=float(np.mean([sum(len(np.unique(b.field_ids(f))) for f in range(F)) for b in batches])))
    table = _bytes_and_flops(cfg, stats, dict(sort_passes=(bits + 9) // 10))
    # candidates for the reported roofline: classes on the launch stream that have a byte (or flop) count
    critical = {k: v for k, v in per_class.items() if k not in side and table.get(k, ("", 0.0))[1] > 0}
    if not critical:
        raise SystemExit("bench.py: no kernel class of the launch stream was timed")
    # dominant kernel: the longest single launch on the critical path
    dominant = max(critical, key=lambda k: critical[k][1] / max(critical[k][0], 1e-9))
    # the longest class of the other kind (memory-bound beside a matrix-product class, or the
    # reverse) is timed as well
    kind = table[dominant][0]
    others = [k for k in critical if table[k][0] != kind]
    second = max(others, key=lambda k: per_class[k][1]) if others else None
    # timed region: events only around the dominant class and only in every fourth step (a pair
    # of event records costs the launch stream several microseconds); the second class is timed
    # in the pass after it
    dom_mask, stride, sampled = 1 << names.index(dominant), 4, 0
    first = args.warmup + CLASSIFY_STEPS
    # The classification pass synchronised after every step; before the clock starts the device
    # runs back-to-back steps again (the warm-up asked for, but at least MIN_UNTIMED untimed steps in
    # all), so that a short timed region sees the steady state a long one sees (clocks up, the
    # hot rows of all rotating batches in the memory-side cache).
    MIN_UNTIMED = 64
    spin = max(args.warmup, MIN_UNTIMED - first)
    for i in range(spin):
        step(first + i)
    first += spin
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % stride == 0:
            ctx.profile(3, dom_mask)
            sampled += 1
        elif i % stride == 1:
            ctx.profile(0)
        step(first + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    n_dom, ms_dom = ctx.profile_read(names.index(dominant))
    ctx.profile(3, 1 << names.index(second)) if second else ctx.profile(0)
    # spread of the step time, in a pass of its own: an event record on the launch stream costs
    # several microseconds of device time, which the timed region above should not carry
    nd = min(args.steps, 100)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(nd + 1)]
    marks[0].record()
    for i in range(nd):
        step(first + args.steps + i)
        marks[i + 1].record()   # a step ends on the launch stream (its side work is joined there)
    torch.cuda.synchronize()
    step_us = np.array([marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(nd)])
    ctx_second = ctx.profile_read(names.index(second)) if second else None
    ctx.profile(0)
    copy_gbs = measured_copy_gbs()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = B / (ms_per_step * 1e-3)


    # what a pair of timing events adds to the time it reports (pair with nothing inside it)
    empty_ms, tiny_ms = ctx.profile_overhead(200)

    def roofline_of(name, n_launch, ms_total, steps, launches_per_pair):
        launches_per_step = n_launch / steps
        pairs = n_launch / launches_per_pair
        bracket_ms = ms_total / max(pairs, 1)
        avg_ms = (bracket_ms - empty_ms) / launches_per_pair
        bound, per_step = table.get(name, ("hbm", 0.0))
        per_launch = per_step / max(launches_per_step, 1e-9)
        if bound == "hbm":
            achieved = per_launch / (avg_ms * 1e-3) / 1e9
            roof = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS)
        else:
            achieved = per_launch / (avg_ms * 1e-3) / 1e12
            peak = MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else VALU_FP32_PEAK_TFLOPS
            roof = dict(bound=bound, achieved=achieved, peak=peak, unit="TFLOP/s", frac=achieved / peak)
        if bound == "hbm":
            roof["frac_of_measured_copy"] = achieved / copy_gbs
        roof["traffic"] = _measured_traffic(f"cfg{cfg_id}", name, launches_per_step)
        roof.update(kernel=name, avg_launch_us=avg_ms * 1e3, launches_per_step=launches_per_step,
                    algorithmic_per_launch=per_launch, event_pair_us=bracket_ms * 1e3,
                    event_pair_overhead_us=empty_ms * 1e3, event_pair_around_smallest_kernel_us=tiny_ms * 1e3)
        return roof

    # (the matrix products of one pass share a pair of events; every other class has one per launch)
    per_pair = lambda k: (len(cfg.layer_sizes) - 2) if k in ("gemm_fwd", "gemm_bwd") else 1
    roof = roofline_of(dominant, n_dom, ms_dom, sampled, per_pair(dominant))
    roof["timed_steps_with_events"] = sampled
    if not roof["frac"] > 0.0:
        raise SystemExit(f"bench.py: roofline fraction of {dominant} is not positive: {roof}")
    roof_second = roofline_of(second, *ctx_second, nd, per_pair(second)) if second else None
    total_bytes = sum(v for k, (b, v) in table.items() if b == "hbm" and k in per_class)   # classes of a step
    breakdown = {k: round(v[1] * 1e3, 2) for k, v in sorted(per_class.items(), key=lambda kv: -kv[1][1])}
    out = {
        "metric": "training samples/sec per iteration (1 GPU)", "value": value, "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "untimed_steps_before_the_clock": first,   # warm-up + per-class timing pass + back-to-back steps
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.gemm_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"configs[{cfg_id - 1}] {cfg.name}: F={F} R={R} D={D} {cfg.table_dtype} tables, "
                               f"B={B} as {K} shards, MLP {'-'.join(map(str, cfg.layer_sizes))} "
                               f"{cfg.gemm_dtype} GEMM, Adagrad", "global_batch": B, "shards": K,
                   "lookups_per_step": stats["nnz"], "unique_rows_per_step": stats["U"]},
        "roofline": roof,
        "roofline_second": roof_second,   # the longest class bound by the other resource
        "hbm_composite": {"algorithmic_bytes_per_step": total_bytes,
                          "frac_of_peak": total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "frac_of_measured_copy": total_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbs},
        "measured_copy_gbs": copy_gbs,   # the library's plain copy kernel, 1 GiB read + 1 GiB written
        # device time between the ends of successive steps on the launch stream, from a separate
        # pass of up to 100 steps with one event record per step (each adds a few microseconds)
        "step_us": {"median": float(np.median(step_us)), "p10": float(np.percentile(step_us, 10)),
                    "p90": float(np.percentile(step_us, 90))},
        "kernel_us_per_step": breakdown,
        "streams": "caller's stream only" if args.single_stream else "launch stream + 2 library streams",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, batches[0])
    return out


def measured_copy_gbs(n=1 << 28, launches=20):
    """Bandwidth of the library's plain copy kernel (bytes read + written per second)."""
    import torch

    import paper_2404_09679_amd as A

    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        A.stream_copy(dst, src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        A.stream_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    return 2 * 4 * n * launches / (e0.elapsed_time(e1) * 1e-3) / 1e9


def cpu_baseline(cfg, batch):
    """The oracle, as it stands, on one iteration of the same workload (host cores).

    The tables are restricted to the rows the batch touches (ids relabelled in order), which
    changes no arithmetic and avoids materialising the full tables on the host."""
    import numpy as np

    import oracle
    import workload as wl
    from threadpoolctl import threadpool_info

    F, D = cfg.num_fields, cfg.dim
    uniq = [np.unique(batch.field_ids(f)) for f in range(F)]
    Rc = max(len(u) for u in uniq)
    ids = batch.ids.copy()
    for f in range(F):
        lo, hi = batch.field_ptr[f], batch.field_ptr[f + 1]
        ids[lo:hi] = np.searchsorted(uniq[f], batch.field_ids(f)).astype(np.int32)
    cb = wl.Batch(ids, batch.field_ptr, batch.offsets, batch.dense, batch.labels)
    tabs = []
    for f in range(F):
        t = np.zeros((Rc, D), np.float32)
        t[:len(uniq[f])] = wl.table_rows_f32(cfg, f, uniq[f])
        tabs.append(t)
    state = [np.zeros((Rc, D) if cfg.adagrad_state == "elementwise" else (Rc,), np.float32) for _ in range(F)]
    flat = wl.make_mlp_params(cfg)
    layers = wl.split_params(cfg, flat)
    lstate = wl.split_params(cfg, np.zeros_like(flat))
    model = oracle.Model(F, Rc, D, cfg.num_dense, tuple(cfg.layer_sizes), cfg.adagrad_state == "rowwise",
                         cfg.table_dtype == "bf16", cfg.gemm_dtype == "bf16", cfg.lr, cfg.eps)
    iters, t0 = 0, time.perf_counter()
    while True:  # whole iterations until about ten seconds of CPU work are done
        res = [oracle.worker_step(model, tabs, layers, cb, s, n) for s, n in wl.shard_slices(cfg.shard_sizes)]
        agg = oracle.aggregate(model, cb, res)
        oracle.apply_update(model, tabs, state, layers, lstate, agg)
        iters += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or iters >= 64:
            break
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": cfg.batch * iters / dt, "unit": "samples/s", "cores": threads, "kind": "oracle",
            "seconds": dt, "iterations": iters,
            "sample": f"{iters} full iterations of the same workload (B={cfg.batch}, {cfg.num_shards} shards, "
                      "same batch), numpy float64, tables restricted to the touched rows"}


def run_batch_sweep(args):
    """Batch processing time of one worker against its local batch size (the F(B_k) curve of
    Section VI-B): worker_step of a single shard of B_k samples of the config-2 workload, timed
    with events.  The saturation batch is the largest B_k whose time is within 10 % of the
    smallest batch's: below it a smaller batch no longer shortens the step."""
    import numpy as np
    import torch

    import paper_2404_09679_amd as A
    import workload as wl

    cfg = wl.CONFIGS[2]
    dev = "cuda:0"
    F, R, D = cfg.num_fields, cfg.rows_per_field, cfg.dim
    tables = torch.empty((F * R, D), dtype=torch.float32, device=dev)
    A.fill_tables(tables, F, R, D, 0.05)
    state = torch.zeros((F * R, D), dtype=torch.float32, device=dev)
    params = torch.from_numpy(wl.make_mlp_params(cfg)).to(dev)
    pstate = torch.zeros_like(params)
    b = wl.make_batch(cfg, 0)
    ctx = A.Context(A.model_from_config(cfg, max_nnz=int(b.field_ptr[-1])))
    ctx.bind(tables, state, params, pstate)
    ctx.set_eager_weight_gradients(True)   # a worker's batch time includes its weight gradients
    ctx.set_batch(torch.from_numpy(b.ids).to(dev), b.field_ptr, torch.from_numpy(b.offsets).to(dev),
                  torch.from_numpy(b.dense).to(dev), torch.from_numpy(b.labels).to(dev))
    B = cfg.batch
    curve = []
    bk = 8
    while bk <= B:
        ctx.assign_shard(B, 2, sizes=[bk, B - bk])
        for _ in range(args.warmup):
            ctx.worker_step(0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            ctx.worker_step(0)
        e1.record()
        torch.cuda.synchronize()
        curve.append([bk, e0.elapsed_time(e1) * 1e3 / args.steps])
        bk *= 2
    base = curve[0][1]
    sat = max(bk for bk, us in curve if us <= 1.1 * base)
    return {"metric": "worker batch processing time vs local batch size", "unit": "us", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "data": "synthetic",
            "dtype": "bf16", "config": {"workload": f"configs[1] {cfg.name}: worker_step of one shard of B_k samples"},
            "curve_us": curve, "saturation_batch": sat,
            "samples_per_s": [[bk, bk / (us * 1e-6)] for bk, us in curve]}


def run_adjust_bs(args):
    """ADJUST_BS on measured batch times (Section VI-A step 3, Eq. 2-3): the heterogeneous shards of
    configuration 3 are stepped one worker at a time, every worker's batch processing time T_k is
    measured with events (its weight gradients included), v_k = B_k / T_k goes into
    antdt_assign_shard's speed mode, and the workers are timed again on the split that comes
    back.  Reported: max_k T_k (what a bulk-synchronous iteration of K real workers would wait
    for) before and after.  On one device all workers run on the same hardware, so what the
    adjustment evens out here is the shard sizes; the batch time has a latency floor (see
    --workload batch-sweep), which Eq. 3's linear model F(B) = B / v leaves out."""
    import numpy as np
    import torch

    import paper_2404_09679_amd as A
    import workload as wl

    cfg = wl.CONFIGS[3]
    dev = "cuda:0"
    F, R, D = cfg.num_fields, cfg.rows_per_field, cfg.dim
    tables = torch.empty((F * R, D), dtype=torch.float32, device=dev)
    A.fill_tables(tables, F, R, D, 0.05)
    state = torch.zeros((F * R, D), dtype=torch.float32, device=dev)
    params = torch.from_numpy(wl.make_mlp_params(cfg)).to(dev)
    pstate = torch.zeros_like(params)
    b = wl.make_batch(cfg, 0)
    ctx = A.Context(A.model_from_config(cfg, max_nnz=int(b.field_ptr[-1])))
    ctx.bind(tables, state, params, pstate)
    ctx.set_eager_weight_gradients(True)
    ctx.set_batch(torch.from_numpy(b.ids).to(dev), b.field_ptr, torch.from_numpy(b.offsets).to(dev),
                  torch.from_numpy(b.dense).to(dev), torch.from_numpy(b.labels).to(dev))
    K, B = cfg.num_shards, cfg.batch

    def times(sizes):
        ctx.assign_shard(B, K, sizes=sizes)
        out = []
        for k in range(K):
            for _ in range(args.warmup):
                ctx.worker_step(k)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                ctx.worker_step(k)
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) * 1e-3 / args.steps)
        return out

    before = list(cfg.shard_sizes)
    t_before = times(before)
    v = [n / t for n, t in zip(before, t_before)]
    after = [n for _, n in ctx.assign_shard(B, K, speed=v)]
    t_after = times(after)
    equal = [n for _, n in ctx.assign_shard(B, K)]
    t_equal = times(equal)
    us = lambda ts: [round(t * 1e6, 1) for t in ts]
    return {"metric": "slowest worker's batch processing time before and after ADJUST_BS", "unit": "us", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "data": "synthetic", "dtype": "bf16",
            "config": {"workload": f"configs[2] {cfg.name}: worker_step of each of the {K} shards, one at a time"},
            "value": max(t_after) * 1e6,
            "before": {"sizes": before, "T_us": us(t_before), "max_T_us": max(t_before) * 1e6},
            "measured_speed_samples_per_s": [round(x) for x in v],
            "after_eq3": {"sizes": after, "T_us": us(t_after), "max_T_us": max(t_after) * 1e6,
                          "predicted_max_T_us": max(n / x for n, x in zip(after, v)) * 1e6},
            "equal_split": {"sizes": equal, "T_us": us(t_equal), "max_T_us": max(t_equal) * 1e6}}


def run_straggler_sim(args):
    """Job completion times under the injection pattern of Section VII-A.2, from the batch times
    measured on this GPU: ten workers whose batch time is the affine fit of the measured
    F(B_k) curve, the server term the measured aggregate + update time of a whole batch, and
    every duration of the pattern (sleep 1.5 s, bursts of 15 in 30 minutes, decisions every
    5 minutes, windows of 5 and 10 minutes, restart 2 minutes) scaled by (measured batch time
    of B/n samples) / 0.5 s, so that delays and batch times keep the proportions of the
    evaluation's CPU workers.  The host-side model is antdt_simulate_bsp."""
    import numpy as np

    import paper_2404_09679_amd as A

    sweep = run_batch_sweep(args)
    bk = np.array([p[0] for p in sweep["curve_us"]], float)
    us = np.array([p[1] for p in sweep["curve_us"]], float)
    slope, icpt = np.polyfit(bk, us, 1)                      # F(b) = icpt + slope * b, microseconds
    n, B = 10, 4096
    t0, v = max(icpt, 0.0) * 1e-6, 1.0 / (slope * 1e-6)
    base = t0 + (B / n) / v
    scale = base / 0.5
    common = dict(n=n, B=B, N=B * 20000, t0=[t0] * n, v=[v] * n, t_server=0.2 * base, period=1800.0 * scale,
                  duration=900.0 * scale, sleep_duration=1.5 * scale, decide_every=300.0 * scale,
                  L_trans=300.0 * scale, L_per=600.0 * scale, lam=1.5, restart_cost=120.0 * scale, seed=20240413)
    names = ["BSP", "ADJUST_BS", "BACKUP_WORKERS(b=3)", "AntDT-ND"]
    rows = []
    for intensity in (0.1, 0.2, 0.4, 0.8):
        jct = [A.simulate_bsp(policy=p, backup_b=3 if p == 2 else 0, prob=0.3, intensity=intensity, **common)[0].jct
               for p in range(4)]
        rows.append({"pattern": f"transient, intensity {intensity}", **{nm: j / jct[0] for nm, j in zip(names, jct)},
                     "BSP_seconds": jct[0]})
    pers = [0.0] * n
    pers[3] = 4.0 * scale
    jct = [A.simulate_bsp(policy=p, backup_b=3 if p == 2 else 0, prob=0.0, persistent_delay=pers, **common)[0].jct
           for p in range(4)]
    rows.append({"pattern": "one persistent straggler (4 s)", **{nm: j / jct[0] for nm, j in zip(names, jct)},
                 "BSP_seconds": jct[0]})
    return {"metric": "job completion time relative to BSP (host-side model on measured batch times)",
            "unit": "ratio", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False,
            "data": "synthetic", "dtype": "f64",
            "config": {"workload": "configs[1] batch times, 10 simulated workers, global batch 4096, 20000 iterations",
                       "batch_time_fit_us": {"floor": icpt, "per_sample": slope}, "time_scale": scale},
            "table": rows}


def run_copy_calibration(args):
    """A plain elementwise copy of known size (1 GiB read, 1 GiB written per launch): the
    reference against which the HBM byte counters of a profiler run are scaled."""
    import torch

    import paper_2404_09679_amd as A

    n = 1 << 28
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        A.stream_copy(dst, src)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    return {"metric": "plain copy", "value": 2 * 4 * n / (ms * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": 0, "ms_per_step": ms, "higher_is_better": True, "data": "synthetic",
            "dtype": "f32", "config": {"workload": "elementwise copy, 2^28 fp32 read and written per launch",
                                       "bytes_read_per_launch": 4 * n, "bytes_written_per_launch": 4 * n}}


def run_dense(args):
    import numpy as np
    import torch

    import paper_2404_09679_amd as A
    import workload as wl

    dc = wl.DENSE_CONFIG
    dev = "cuda:0"
    n, K = dc.n, dc.num_buffers
    gen = torch.Generator(device=dev)
    gen.manual_seed(dc.seed)
    p = torch.randn(n, device=dev, generator=gen) * dc.param_std
    m, v = torch.zeros_like(p), torch.zeros_like(p)
    grads = [torch.randn(n, device=dev, generator=gen) * dc.grad_std for _ in range(K)]
    w = [1.0 / K] * K
    step_no = 0
    for _ in range(args.warmup):
        step_no += 1
        A.dense_aggregate_adam(p, m, v, grads, w, dc.lr, dc.beta1, dc.beta2, dc.eps, step_no)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_no += 1
        ev[i][0].record()
        A.dense_aggregate_adam(p, m, v, grads, w, dc.lr, dc.beta1, dc.beta2, dc.eps, step_no)
        ev[i][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    avg_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    nbytes = (K + 3) * 4 * n + 3 * 4 * n
    achieved = nbytes / (avg_ms * 1e-3) / 1e9
    copy_gbs = measured_copy_gbs()
    return {
        "metric": "dense weighted-average + Adam steps/sec (1 GPU)", "value": 1e3 / ms_per_step, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[4] {dc.name}: {K} gradient buffers x 2^28 fp32, fused Adam"},
        "roofline": dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                         frac=achieved / HBM_PEAK_GBS, frac_of_measured_copy=achieved / copy_gbs,
                         traffic=_measured_traffic("cfg5", "adam", 1.0) if (K, n) == (8, 1 << 28) else None,
                         kernel="adam", avg_launch_us=avg_ms * 1e3, algorithmic_per_launch=nbytes),
        "measured_copy_gbs": copy_gbs,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "batch-sweep", "copy-calibration", "straggler-sim", "adjust-bs"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--single-stream", action="store_true",
                    help="ranking workloads: enqueue every kernel on one stream (per-kernel durations without overlap)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (the K workers are shards on that device); "
                 "use --gpus 1")
    if args.workload == "straggler-sim":
        out = run_straggler_sim(args)
    elif args.workload == "adjust-bs":
        out = run_adjust_bs(args)
    elif args.workload == "copy-calibration":
        out = run_copy_calibration(args)
    elif args.workload == "batch-sweep":
        out = run_batch_sweep(args)
    elif args.workload == "cfg5":
        out = run_dense(args)
    else:
        out = run_ranking(args, int(args.workload[3:]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
