#!/usr/bin/env python3
"""Benchmark of the GPT stage forward+backward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME|INDEX|all]

One "step" = the whole hot path over one batch of the workload: every
micro-batch's forward and backward (for the decoupled workload: all forwards on
a forward stream, then all backwards on a backward stream).  Inputs are seeded
synthetic tensors already resident in HBM.  Prints ONE JSON line (one per workload
with --workload all).

Other modes (each prints one JSON line):
    --op attention|layernorm|gemm   one operator alone through its gpt_stage_op_* entry point, at
                                    the shapes of the chosen workload (for rocprofv3 counter runs)
    --dpp CHUNKS                    traversal policies over model chunks
    --pmc-summary DIR               no GPU work: average the counters of a `rocprofv3 --pmc` output
                                    directory per kernel and print a table
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# Memory traffic of the matrix-product kernels on the default workload and schedule (one weight
# phase per step), from two rocprofv3 --pmc passes: FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 averaged
# over the 272 matrix-product launches of a step (the summary under profiles/ has the commands
# and the per-kernel figures).  Only reported while the kernel source is the one the counters
# were taken on.
GEMM_TRAFFIC = {"workload": "decoupled_bf16", "weight_phase": True, "bytes_per_launch": 1016.6 * 2**20,
                "source_sha256_16": "369e0b5450094d57"}
PEAK_FP32_TFLOPS = 157.3    # MI355X fp32 vector
DEFAULT_WORKLOAD = "decoupled_bf16"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prepare", action="store_true",
                    help="run the products on the raw weights instead of the prepared images")
    ap.add_argument("--force-prepare", action="store_true",
                    help="use prepared weight images also where they do not pay (fewer than 3 micro-batches per step)")
    ap.add_argument("--schedule", choices=["auto", "coupled", "decoupled"], default="auto")
    ap.add_argument("--wgrad", choices=["auto", "flush", "per-microbatch"], default="auto",
                    help="decoupled schedule: weight gradients in one weight phase after all backward data "
                         "phases (flush; auto picks it when there are several micro-batches) or inside every "
                         "micro-batch's backward call")
    ap.add_argument("--recompute", type=int, nargs="?", const=1, default=0, choices=[0, 1, 2],
                    help="activation recomputation: 1 = LayerNorm/GeLU outputs rebuilt in backward, "
                         "2 = only each layer's input is stashed and backward re-runs the layer's forward")
    ap.add_argument("--graph", action="store_true",
                    help="coupled schedule only: capture one step in a HIP graph and time its replays "
                         "(the stage calls only enqueue kernels; pays on launch-bound small stages)")
    ap.add_argument("--op", choices=["attention", "layernorm", "gemm"], default=None,
                    help="time one operator alone (gpt_stage_op_* entry points) at the workload's shapes")
    ap.add_argument("--pmc-summary", default=None, metavar="DIR",
                    help="summarise the counter_collection csv files of a rocprofv3 --pmc run under DIR")
    ap.add_argument("--dpp", type=int, default=0, metavar="CHUNKS",
                    help="instead of the stage benchmark: split the workload's layers into CHUNKS model "
                         "chunks and time the depth-first / breadth-first traversals of the "
                         "(micro-batch, chunk) task matrix")
    return ap.parse_args()


def pick_workload(arg):
    from paper_2507_19845_amd import synth
    if arg.isdigit():
        return synth.WORKLOADS[int(arg)]
    for w in synth.WORKLOADS:
        if w.name == arg:
            return w
    raise SystemExit(f"unknown workload {arg!r}; known: {[w.name for w in synth.WORKLOADS]}")


def cpu_baseline(shape):
    """Time the oracle, as it stands, on a bounded sample of the workload:
    one layer, one micro-batch, the first min(S, 4096) tokens of each sequence."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import gpt_stage_oracle as orc
    from paper_2507_19845_amd import binding as B
    from paper_2507_19845_amd import synth
    s = shape.with_(n_layers=1, seq=min(shape.seq, 4096), n_microbatches=1)
    params = [{k: v.astype(np.float64) for k, v in synth.make_layer_params(s, 0, 0).items()}]
    x, dy = synth.make_x(s, 0).astype(np.float64), synth.make_dy(s, 0).astype(np.float64)
    t0 = time.perf_counter()
    orc.stage_fwd_bwd(x, dy, params, s.n_heads, s.head_dim, s.ln_eps, s.gelu)
    dt = time.perf_counter() - t0
    flops = B.gpt_stage_model_flops(B.make_cfg(s), True)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "host_cores": os.cpu_count(), "cores_note": "cores = BLAS threads the oracle's matrix products used",
            "seconds": dt,
            "sample": f"1 layer, 1 micro-batch, first {s.seq} tokens x batch {s.batch} of {shape.name} "
                      f"(fp64 numpy oracle, {flops / 1e12:.3f} model TFLOP causal-aware)"}


def gemm_traffic(shape, weight_phase):
    """Measured HBM bytes per launch of the matrix-product kernel, or None when no counters
    exist for this workload or the kernel source has changed since they were taken."""
    import hashlib
    src = os.path.join(ROOT, "paper_2507_19845_amd", "csrc", "gemm_mfma.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if (shape.name != GEMM_TRAFFIC["workload"] or sha != GEMM_TRAFFIC["source_sha256_16"]
            or weight_phase != GEMM_TRAFFIC["weight_phase"]):
        return None
    return GEMM_TRAFFIC["bytes_per_launch"]


def traced_pass(step, bufs, shape, n_ops, steps, weight_phase):
    """Run `steps` more steps of the same workload with the library's operator tracer
    attached: a start/end hipEvent pair is recorded around every operator on the stream
    it is launched on.  Returns per-operator-class totals and the roofline object of
    the dominant kernel class (the matrix products)."""
    from paper_2507_19845_amd import binding as B
    tr = B.gpt_stage_trace_create(n_ops * steps)
    bufs.trace = tr
    try:
        for _ in range(steps):
            step()
        import torch
        torch.cuda.synchronize()
        recs, dropped = B.gpt_stage_trace_collect(tr, n_ops * steps)
    finally:
        bufs.trace = None
        B.gpt_stage_trace_destroy(tr)
    classes = {}
    for r in recs:
        c = classes.setdefault(r["op"], {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        c["launches"] += 1
        c["ms"] += r["dur_ms"]
        c["flops"] += r["flops"]
        c["bytes"] += r["bytes"]
    table = {}
    for k, c in classes.items():
        row = {"launches_per_step": c["launches"] // steps, "ms_per_step": c["ms"] / steps,
               "avg_launch_ms": c["ms"] / c["launches"]}
        if c["flops"] > 0:
            row["TFLOP/s"] = c["flops"] / c["ms"] / 1e9
        row["GB/s_algorithmic"] = c["bytes"] / c["ms"] / 1e6
        table[k] = row
    gemm = [classes[k] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad") if k in classes]
    n = sum(c["launches"] for c in gemm)
    ms = sum(c["ms"] for c in gemm)
    fl = sum(c["flops"] for c in gemm)
    peak = PEAK_BF16_TFLOPS if shape.dtype == "bf16" else PEAK_FP32_TFLOPS
    achieved = fl / ms / 1e9
    roof = {"bound": "mfma" if shape.dtype == "bf16" else "alu", "achieved": achieved, "peak": peak,
            "unit": "TFLOP/s", "frac": achieved / peak, "traffic": gemm_traffic(shape, weight_phase),
            "kernel": "the matrix products (gemm_mi16_kernel where the shape allows): the 12 of a layer, "
                      "forward, dgrad, wgrad, averaged",
            "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)",
            "algorithmic_bytes_per_launch": sum(c["bytes"] for c in gemm) / n,
            "launches": n, "launches_per_step": n // steps, "avg_launch_ms": ms / n, "flops_per_launch": fl / n,
            "avg_launch_ms_source": "hipEvent pairs recorded on the launch stream by the library's tracer (not rocprofv3)",
            "measured": f"hipEvent pairs around every launch, {steps} traced step(s) after the timed region",
            "dropped_records": dropped}
    return roof, table


def dpp_bench(args, shape):
    """Traversal policies over CHUNKS chunks x the workload's micro-batches: wall time per
    iteration, peak stash, and when each chunk's gradients are complete."""
    import torch
    from paper_2507_19845_amd import binding as B
    from paper_2507_19845_amd import synth
    C, M = args.dpp, shape.n_microbatches
    if shape.n_layers % C:
        raise SystemExit(f"--dpp {C}: the workload has {shape.n_layers} layers")
    Lc = shape.n_layers // C
    cs = shape.with_(n_layers=Lc)
    cfg = B.make_cfg(cs)
    n = B.gpt_stage_param_count(cfg)
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    ws = torch.empty(max(B.gpt_stage_workspace_bytes(cfg, 1), 256), dtype=torch.uint8, device="cuda")
    weights, prepared, dps, chunks = [], [], [], []
    for j in range(C):
        w = torch.empty(n, dtype=tdt, device="cuda")
        for l in range(Lc):
            p = synth.make_layer_params(shape, j * Lc + l, 0)
            for tid, name in enumerate(synth.TENSOR_NAMES):
                off, cnt = B.gpt_stage_param_offset(cfg, l, tid)
                w[off:off + cnt].copy_(B.to_device(p[name].reshape(-1), shape.dtype))
        weights.append(w)
        dps.append(torch.zeros(n, dtype=torch.float32, device="cuda"))
        pb = B.gpt_stage_prepared_bytes(cfg)
        prep = torch.empty(max(pb, 256), dtype=torch.uint8, device="cuda") if pb and not args.no_prepare else None
        prepared.append(prep)
        chunks.append(B.gpt_stage_params(cfg=cfg, weights=w.data_ptr(), workspace=ws.data_ptr(),
                                         prepared=prep.data_ptr() if prep is not None else None, trace=None))
    xs = [B.to_device(synth.make_x(shape, 0, m), shape.dtype) for m in range(M)]
    dys = [B.to_device(synth.make_dy(shape, 0, m), shape.dtype) for m in range(M)]
    ys = [torch.empty_like(x) for x in xs]
    dxs = [torch.empty_like(x) for x in xs]
    slot = B.gpt_dpp_stash_slot_bytes(chunks)
    stash = torch.empty(slot * C * M, dtype=torch.uint8, device="cuda")
    act = torch.empty(B.gpt_dpp_act_slot_bytes(cfg) * (M + 2), dtype=torch.uint8, device="cuda")
    flops = B.gpt_stage_model_flops(cfg, True) * C * M
    rows = {}
    gslot = B.gpt_dpp_grad_slot_bytes(chunks)
    gpool = torch.empty(gslot * M, dtype=torch.uint8, device="cuda") if gslot else None
    # "+wp": backward tasks run the data phase, one weight phase per chunk and window
    for name, pol, cap, wp in (("dfc", B.GPT_DPP_DFC, 0, False), ("bfc", B.GPT_DPP_BFC, 0, False),
                               ("bfc_best_effort_cap_half", B.GPT_DPP_BFC_BEST_EFFORT, C * M // 2, False),
                               ("dfc+wp", B.GPT_DPP_DFC, 0, True), ("bfc+wp", B.GPT_DPP_BFC, 0, True),
                               ("bfc_best_effort_cap_half+wp", B.GPT_DPP_BFC_BEST_EFFORT, C * M // 2, True)):
        ev0 = torch.cuda.Event(enable_timing=True)
        ready = [torch.cuda.Event(enable_timing=True) for _ in range(C)]
        for e in [ev0] + ready:
            e.record()

        def step(timed_events):
            for j in range(C):
                if prepared[j] is not None:
                    B.gpt_stage_prepare(chunks[j], prepared[j])
            return B.gpt_dpp_run(pol, chunks, xs, dys, ys, dxs, dps, stash, act, max_live_stash=cap,
                                 grad_ready=ready if timed_events else None, grad_pool=gpool if wp else None)
        for _ in range(args.warmup):
            step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            rep = step(False)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ev0.record()
        rep = step(True)
        torch.cuda.synchronize()
        rows[name] = {"ms_per_iteration": ms, "TFLOP/s": flops / ms / 1e9,
                      "peak_live_stash": rep.peak_live_stash,
                      "peak_stash_GiB": rep.peak_live_stash * rep.stash_slot_bytes / 2**30,
                      "peak_boundary_buffers": rep.peak_live_act,
                      "grad_ready_ms_after_start": [ev0.elapsed_time(e) for e in ready]}
    print(json.dumps({"metric": "MegaDPP traversal policies on 1 MI355X", "unit": "ms per iteration",
                      "config": {"workload": shape.name, "chunks": C, "layers_per_chunk": Lc, "n_microbatches": M},
                      "steps": args.steps, "warmup": args.warmup, "policies": rows}))


def run_workload(args, shape):
    """Time K steps of one workload and return the result row."""
    import torch
    from paper_2507_19845_amd import binding as B
    from paper_2507_19845_amd import harness, synth
    n_mb = shape.n_microbatches
    decoupled = (n_mb > 1) if args.schedule == "auto" else (args.schedule == "decoupled")
    bufs = B.StageBuffers(shape, n_stash=n_mb if decoupled else 1)
    t0 = time.perf_counter()
    for l in range(shape.n_layers):   # one layer at a time keeps host memory small
        p = synth.make_layer_params(shape, l, 0)
        for tid, name in enumerate(synth.TENSOR_NAMES):
            off, n = B.gpt_stage_param_offset(bufs.cfg, l, tid)
            bufs.weights[off:off + n].copy_(B.to_device(p[name].reshape(-1), shape.dtype))
    xs = [B.to_device(synth.make_x(shape, 0, m), shape.dtype) for m in range(n_mb)]
    dys = [B.to_device(synth.make_dy(shape, 0, m), shape.dtype) for m in range(n_mb)]
    ys = [bufs.act() for _ in range(n_mb)]
    dxs = [bufs.act() for _ in range(n_mb)]
    gen_s = time.perf_counter() - t0
    runner = harness.StageRunner(bufs)
    split = decoupled and n_mb > 1 and args.wgrad != "per-microbatch" and shape.recompute != 2

    # Weight images are rebuilt once per step (the weights change once per step) and cost a read
    # and a write of twice the weight bytes; they make the forward and dgrad products of every
    # micro-batch about 6 % faster, which pays from three micro-batches per step on (measured:
    # with one micro-batch the 13B-shaped stage runs 893 TFLOP/s on raw weights, 824 on images).
    # fp16 forward activations read the weights through their (fp16) images only.
    prepare = shape.dtype == "bf16" and (shape.fwd_fp16 or args.force_prepare or (not args.no_prepare and n_mb >= 3))

    def step():
        # the weights change once per step in training, so their images are rebuilt once
        # per step, inside the timed region, and shared by all micro-batches
        if prepare:
            bufs.prepare()
        if decoupled:
            runner.decoupled(xs, dys, ys, dxs, split_wgrad=split)
        else:
            runner.coupled(xs, dys, ys, dxs)

    for _ in range(args.warmup):
        bufs.dparams.zero_()
        step()
    torch.cuda.synchronize()
    run_step = step
    use_graph = args.graph and not decoupled
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay
        run_step()
    bufs.dparams.zero_()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps

    flops = B.gpt_stage_model_flops(bufs.cfg, True) * n_mb
    flops_dense = B.gpt_stage_model_flops(bufs.cfg, False) * n_mb
    tflops = flops / (ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if shape.dtype == "bf16" else PEAK_FP32_TFLOPS
    ops_per_step = 28 * shape.n_layers * n_mb   # trace capacity (upper bound)
    roof, table = traced_pass(step, bufs, shape, ops_per_step, max(1, min(args.steps, 2)), split)
    stash = ("fp16 forward activations; LayerNorm/GeLU outputs rebuilt in backward" if shape.fwd_fp16 else
             "only each layer's input; backward re-runs the layer's forward" if shape.recompute == 2 else
             "recompute LayerNorm/GeLU outputs in backward" if shape.recompute else "full")
    out = {
        "metric": "model TFLOP/s for one stage fwd+bwd on 1 MI355X",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "pct_of_peak": 100.0 * tflops / peak, "peak_tflops": peak,
        "value_dense_attention_convention": flops_dense / (ms * 1e-3) / 1e12,
        "model_tflop_per_step": flops / 1e12,
        "config": {"workload": shape.name, "n_layers": shape.n_layers, "hidden": shape.hidden,
                   "n_heads": shape.n_heads, "head_dim": shape.head_dim, "ffn": shape.ffn,
                   "seq": shape.seq, "micro_batch": shape.batch, "n_microbatches": n_mb,
                   "schedule": "decoupled: all fwd on stream F, then all bwd on stream B" if decoupled
                               else "coupled fwd+bwd per micro-batch", "flop_count": "causal-aware",
                   "weight_gradients": "one weight phase over all micro-batches after their backward data phases "
                                       "(gpt_stage_bwd_data_only x n, gpt_stage_wgrad_flush)" if split
                                       else "inside every micro-batch's backward call",
                   "grad_stash_GiB_per_microbatch": B.gpt_stage_grad_stash_bytes(bufs.cfg) / 2**30 if split else 0.0,
                   "prepared_weights": "rebuilt every step (timed)" if prepare else "off (raw weights)",
                   "launch": "one HIP graph replay per step" if use_graph else "eager",
                   "forward_activations": "fp16" if shape.fwd_fp16 else shape.dtype,
                   "stash": stash,
                   "stash_GiB_per_microbatch": B.gpt_stage_stash_bytes(bufs.cfg) / 2**30,
                   "input_gen_seconds": gen_s},
        "roofline": roof,
        "kernels": table,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape)
    del bufs, xs, dys, ys, dxs, runner
    torch.cuda.empty_cache()
    return out


def op_bench(args, shape):
    """One operator alone, through its gpt_stage_op_* entry point, at the shapes it has in one
    layer of the workload; timed with events on the launch stream.  Meant to be run under
    `rocprofv3 --pmc ...` (the kernels of the operator are then the only ones in the trace) as
    well as on its own."""
    import torch
    from paper_2507_19845_amd import binding as B
    from paper_2507_19845_amd import synth
    dt = B.GPTS_BF16 if shape.dtype == "bf16" else B.GPTS_FP32
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    e = 2 if shape.dtype == "bf16" else 4
    T, H, P, F, S, Bt, a, d = (shape.tokens, shape.hidden, shape.attn_width, shape.ffn, shape.seq, shape.batch,
                               shape.n_heads, shape.head_dim)
    dev = "cuda"

    def rnd(shape_, std, tag):
        return B.to_device(synth.to_storage(synth.make_aux(0, tag, shape_, std), shape.dtype), shape.dtype)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(args.steps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / args.steps

    rows = {}
    if args.op == "attention":
        qkv = rnd((Bt, S, 3 * P), math.sqrt(H) * 0.02, 1)      # the spread a*W^T has in the workload
        out = torch.empty((Bt, S, P), dtype=tdt, device=dev)
        lse = torch.empty((Bt, a, S), dtype=torch.float32, device=dev)
        dout, dqkv = rnd((Bt, S, P), 1.0, 2), torch.empty_like(qkv)
        sc = [torch.empty(max(B.gpt_stage_op_attention_scratch_bytes(dt, Bt, S, a, d, ph), 256), dtype=torch.uint8,
                          device=dev) for ph in (0, 1)]
        fl = 4.0 * Bt * a * d * S * (S + 1) / 2
        ms = timed(lambda: B.gpt_stage_op_attention_fwd(dt, Bt, S, a, d, qkv, out, lse, sc[0]))
        rows["attention_fwd"] = {"ms": ms, "TFLOP/s": fl / ms / 1e9, "flops": fl, "bytes": T * 4.0 * P * e}
        ms = timed(lambda: B.gpt_stage_op_attention_bwd(dt, Bt, S, a, d, qkv, out, lse, dout, dqkv, sc[1]))
        rows["attention_bwd"] = {"ms": ms, "TFLOP/s": 2 * fl / ms / 1e9, "flops": 2 * fl, "bytes": T * 9.0 * P * e}
    elif args.op == "layernorm":
        x32 = shape.dtype == "bf16"     # inside a bf16 stage LayerNorm reads the fp32 residual stream
        x = torch.from_numpy(synth.make_aux(0, 3, (T, H))).to(dev) if x32 else rnd((T, H), 1.0, 3)
        g, b_ = rnd((H,), 1.0, 4), rnd((H,), 1.0, 5)
        out = torch.empty((T, H), dtype=tdt, device=dev)
        mean, rstd = (torch.empty(T, dtype=torch.float32, device=dev) for _ in range(2))
        dout, dres, dx = rnd((T, H), 1.0, 6), rnd((T, H), 1.0, 7), torch.empty((T, H), dtype=tdt, device=dev)
        dg, db, dxs = (torch.zeros(H, dtype=torch.float32, device=dev) for _ in range(3))
        part = torch.empty(B.gpt_stage_op_layernorm_bwd_scratch_bytes(T, H), dtype=torch.uint8, device=dev)
        xb = 4 if x32 else e
        ms = timed(lambda: B.gpt_stage_op_layernorm_fwd(dt, T, H, shape.ln_eps, x, g, b_, out, mean, rstd, x_f32=x32))
        by = T * H * (xb + e)
        rows["layernorm_fwd"] = {"ms": ms, "GB/s": by / ms / 1e6, "bytes": by}
        ms = timed(lambda: B.gpt_stage_op_layernorm_bwd(dt, T, H, dout, x, mean, rstd, g, dres, dx, dg, db, part,
                                                        x_f32=x32, dxsum=dxs))
        by = T * H * (3 * e + xb)
        rows["layernorm_bwd"] = {"ms": ms, "GB/s": by / ms / 1e6, "bytes": by}
    else:
        # the three forms at the layer's four linears, on raw weights (the image-fed variants of the
        # forward and dgrad products are reached through the stage calls only)
        for name, (N, K) in (("qkv", (3 * P, H)), ("out_proj", (H, P)), ("fc1", (F, H)), ("fc2", (H, F))):
            W = rnd((N, K), 0.02, 10)
            Ain, Gout = rnd((T, K), 1.0, 11), rnd((T, N), 1.0, 12)
            Cf, Cd = torch.empty((T, N), dtype=tdt, device=dev), torch.empty((T, K), dtype=tdt, device=dev)
            Cw = torch.zeros((N, K), dtype=torch.float32, device=dev)
            fl = 2.0 * T * N * K
            for form, fn in (("fwd", lambda: B.gpt_stage_op_gemm(dt, 0, T, N, K, Ain, W, Cf)),
                             ("dgrad", lambda: B.gpt_stage_op_gemm(dt, 1, T, K, N, Gout, W, Cd)),
                             ("wgrad", lambda: B.gpt_stage_op_gemm(dt, 2, N, K, T, Gout, Ain, Cw))):
                ms = timed(fn)
                rows[f"{name}_{form}"] = {"ms": ms, "TFLOP/s": fl / ms / 1e9, "flops": fl}
            del W, Ain, Gout, Cf, Cd, Cw
    print(json.dumps({"metric": f"operator {args.op} alone (gpt_stage_op_* entry points)", "unit": "ms per call",
                      "config": {"workload": shape.name, "tokens": T, "hidden": H, "attention_width": P, "ffn": F,
                                 "seq": S, "n_heads": a, "head_dim": d},
                      "steps": args.steps, "warmup": args.warmup, "dtype": shape.dtype, "operators": rows}))


def pmc_summary(path):
    """Per-kernel averages of every counter found in the counter_collection csv files that
    `rocprofv3 --pmc ... -d DIR --output-format csv` leaves under DIR (any depth)."""
    import csv
    acc = {}
    for root, _, files in os.walk(path):
        for f in files:
            if not f.endswith("counter_collection.csv"):
                continue
            with open(os.path.join(root, f), newline="") as fh:
                for r in csv.DictReader(fh):
                    k = r["Kernel_Name"].replace("(anonymous namespace)::", "").replace("void ", "")
                    k = k.split("(")[0]   # drop the argument list
                    row = acc.setdefault(k, {})
                    c = row.setdefault(r["Counter_Name"], [0.0, 0])
                    c[0] += float(r["Counter_Value"])
                    c[1] += 1
    names = sorted({c for row in acc.values() for c in row})
    print("| kernel | dispatches | " + " | ".join(names) + " |")
    print("|---|---:|" + "---:|" * len(names))
    for k, row in sorted(acc.items(), key=lambda kv: -max(v[1] for v in kv[1].values())):
        n = max(v[1] for v in row.values())
        print(f"| `{k[:90]}` | {n} | " + " | ".join(f"{row[c][0] / row[c][1]:.4g}" if c in row else "" for c in names) + " |")


def main():
    args = parse()
    if args.pmc_summary:
        return pmc_summary(args.pmc_summary)
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the stage has no collectives or sharding; run with --gpus 1")
    import torch
    from paper_2507_19845_amd import binding as B
    from paper_2507_19845_amd import synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    B.lib()
    shapes = list(synth.WORKLOADS) if args.workload == "all" else [pick_workload(args.workload)]
    if args.recompute:
        shapes = [s.with_(recompute=args.recompute) for s in shapes]
    if args.dpp:
        return dpp_bench(args, shapes[0])
    if args.op:
        return op_bench(args, shapes[0])
    for shape in shapes:
        print(json.dumps(run_workload(args, shape)), flush=True)


if __name__ == "__main__":
    main()
