#!/usr/bin/env python3
"""Benchmark of the SLA2 forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--quant fp8|int8|fp8v|none]

One "step" is one sla2_forward call (router -> kv state -> fused sparse + linear +
mix) on a synthetic Wan2.1-1.3B-shaped input set (B=1, H=12, N=32760, d=128,
b_q=128, b_kv=64, 3 % of the key blocks kept = 97 % sparsity) that is already
resident in HBM.  Prints ONE JSON line: dense-equivalent TFLOP/s (4 N^2 d H B / t,
the paper's C/t), ms per call, the roofline entry of the dominant kernel measured
live with HIP events (against the matrix-core peak, and against the bytes it has to
gather), the per-kernel breakdown, the in-build dense bf16 attention on the same
inputs, the training path (forward keeping its intermediates + sla2_backward; not
part of `value`), and the CPU oracle timed on the same workload.

Order of the legs: W warm-up + K timed calls first thing = `value`; the dense comparator (two untimed calls,
then five timed); the one-input-set pass and the per-kernel pass; the K calls once more = `settled`; the
backward pass.  An MI355X takes tens of milliseconds of load to reach its sustained clocks, more than a small
W covers: `value` then times that ramp along with the kernels, `settled` (labelled, never `value`) shows the
same loop afterwards, and the comparator is timed warm so that the ratio is not flattered.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "oracle")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0, "int8": 5000.0}   # dense; int8 in TOP/s


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="wan1.3b-97-fp8")
    ap.add_argument("--quant", choices=["fp8", "int8", "fp8v", "none"], default=None, help="override the workload's sparse-branch precision")
    ap.add_argument("--topk", type=float, default=None, help="override the kept fraction of key blocks")
    ap.add_argument("--input-sets", type=int, default=3, help="independent input copies rotated between calls")
    ap.add_argument("--packed-qkv", action="store_true",
                    help="q, k, v as slices of one [B, N, 3, H, d] tensor and out as [B, N, H, d], passed by strides")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true", help="skip the forward-for-training + backward timing")
    ap.add_argument("--cpu-heads", type=int, default=12, help="heads of the workload the oracle is timed on")
    ap.add_argument("--event-stride", type=int, default=1,
                    help="bracket the dominant kernel with HIP events on every n-th timed step")
    ap.add_argument("--block-q", type=int, default=None, choices=[64, 128], help="override the workload's query block size")
    ap.add_argument("--router-identity", action="store_true",
                    help="router weights Wq = Wk = I: the pooled-QK router of the Topk-router ablation (Sec. 9.4)")
    ap.add_argument("--sweep", action="store_true",
                    help="the sparsity sweep: kept fractions 0.15 ... 0.01 in bf16 and FP8 at N = 75,600 and 75,601 plus the "
                         "dense kernel on the same inputs; one JSON line per point, written to --sweep-out as well")
    ap.add_argument("--sweep-out", default="sweep.jsonl")
    ap.add_argument("--sweep-lengths", default="0,1", help="extra tokens after the 75,600-token grid, comma separated")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    return ap.parse_args()


TRAFFIC_FILE = os.path.join("profiles", "attn_mfma_traffic.txt")


def measured_traffic(workload, quant):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/attn_mfma_traffic.txt: lines `workload quant bytes`), or None.  It is a stored counter reading
    of an earlier profiled run of this same command, not a measurement of the present run."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and not line.startswith("#") and parts[0] == workload and parts[1] == quant:
                    return float(parts[2])
    except OSError:
        pass
    return None


def traffic_source():
    """Where `roofline.traffic` comes from: the file and the commit that last changed it."""
    import subprocess
    try:
        rev = subprocess.run(["git", "log", "-1", "--format=%h", "--", TRAFFIC_FILE], cwd=ROOT, capture_output=True,
                             text=True, timeout=10).stdout.strip()
    except Exception:
        rev = ""
    return "%s%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command; not measured in this run)" % (
        TRAFFIC_FILE, " @ " + rev if rev else "")


def cpu_baseline(inp, heads):
    """The oracle as it stands, timed on `heads` full heads of the workload."""
    import sla2_oracle as O
    import numpy as np
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    w = inp.workload
    quant = {"none": O.QUANT_NONE, "fp8": O.QUANT_FP8, "int8": O.QUANT_INT8, "fp8v": O.QUANT_FP8_V}[w.quant]
    Wq, Wk = inp.router_w[0].astype(np.float64), inp.router_w[1].astype(np.float64)
    t0 = time.perf_counter()
    for h in range(heads):
        O.forward_head(inp.values("q", 0, h), inp.values("k", 0, h), inp.values("v", 0, h), Wq, Wk,
                       float(inp.alpha[h]), w.topk_frac, w.block_q, w.block_kv, quant=quant)
    dt = time.perf_counter() - t0
    flops = 4.0 * w.N * w.N * w.d * heads
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": int(cores), "kind": "oracle",
            "sample": "%d of %d heads of the same workload, all query blocks, %.1f s; ms per full call extrapolated: %.0f"
                      % (heads, w.B * w.H, dt, dt / heads * w.B * w.H * 1e3)}


def backward_timing(api, W, torch, w, inp, dt, qm, tensors, rw, al, stream, ksel, reps=40):
    """Times sla2_forward with SLA2_FLAG_SAVE_FOR_BACKWARD and sla2_backward on the bench workload (contiguous
    layout).  Not part of `value`; a reported figure for the training path (Alg. 3)."""
    import numpy as np
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, quant_mode=qm,
                        flags=api.SLA2_FLAG_SAVE_FOR_BACKWARD)
    q, k, v, _ = tensors
    if not q.is_contiguous():
        q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
    out = torch.empty_like(q)
    g = np.random.default_rng(7).normal(size=inp.q.shape).astype(np.float32)
    dout = api.to_device(W.f32_to_bf16_bits(g) if w.dtype == "bf16" else g, dt)
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    dal = torch.empty_like(al)
    ws = api.alloc_workspace(p)

    def timed(f):
        for _ in range(15):                            # the clocks settle over a few dozen calls
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    fwd_ms = timed(lambda: api.sla2_forward(p, q, k, v, rw, al, out, workspace=ws, stream=stream))
    bwd_ms = timed(lambda: api.sla2_backward(p, q, k, v, al, dout, dq, dk, dv, dal, ws, stream=stream))
    api.sla2_profile_begin(["bwd_lists", "bwd_q", "bwd_kv", "bwd_rest"], reps)
    for _ in range(reps):
        api.sla2_backward(p, q, k, v, al, dout, dq, dk, dv, dal, ws, stream=stream)
    torch.cuda.synchronize()
    stage_ms = {name: round(ms / reps, 4) for name, (ms, n) in api.sla2_profile_end().items()}
    BH = w.B * w.H
    pair = 2.0 * w.block_q * w.block_kv * w.d                   # one product over a (query block, key block) pair
    # S, dP, dQ, dK, dV per selected pair; dQ^phi and dH_i per query block; dK^phi and the linear dV per key block
    flops = BH * (w.T_m * ksel * 5.0 * pair + w.T_m * 2 * 2.0 * w.block_q * w.d * w.d + w.T_n * 2 * 2.0 * w.block_kv * w.d * w.d)
    tf = flops / (bwd_ms * 1e-3) / 1e12
    res = {"ms": round(bwd_ms, 4), "forward_saving_ms": round(fwd_ms, 4), "stage_ms": stage_ms, "algorithmic_flops": flops,
           "TFLOP/s": round(tf, 1), "dtype": "bf16 MFMA products, fp32 elsewhere" if w.dtype == "bf16" else "f32",
           "workspace_bytes": int(ws.numel())}
    if w.dtype == "bf16":
        res["frac_of_bf16_mfma_peak"] = round(tf / MFMA_PEAK_TFLOPS["bf16"], 4)
    return res


def sweep(args, api, W, torch):
    """Config 5: B = 2, H = 40, d = 128, N = 75,600 (+ extra tokens), kept fractions 0.15 ... 0.01, bf16 and FP8
    sparse branch, and the dense bf16 kernel on the same inputs.  One JSON line per point."""
    stream = torch.cuda.current_stream()
    lines = []
    for extra in [int(x) for x in args.sweep_lengths.split(",") if x != ""]:
        base = W.SWEEP_BASE.replace(extra_tokens=extra)
        inp = W.generate(base)
        dt = api.SLA2_BF16
        sets = []
        for _ in range(max(1, min(args.input_sets, 2))):
            q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
            sets.append((q, k, v, torch.empty_like(q)))
        rw = torch.from_numpy(inp.router_w).cuda()
        al = torch.from_numpy(inp.alpha).cuda()
        dense_flops = 4.0 * base.N * base.N * base.d * base.H * base.B
        pd = api.make_params(base.B, base.H, base.N, base.d, base.block_q, base.block_kv, 1.0, dtype=dt)
        q, k, v, out = sets[0]
        api.sla2_dense_forward(pd, q, k, v, out, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2):
            api.sla2_dense_forward(pd, q, k, v, out, stream=stream)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) / 2 * 1e3
        dense = {"ms": round(dense_ms, 2), "TFLOP/s": round(dense_flops / (dense_ms * 1e-3) / 1e12, 1),
                 "frac_of_bf16_mfma_peak": round(dense_flops / (dense_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4)}
        for quant in ("none", "fp8"):
            for topk in W.SWEEP_TOPK:
                w = base.replace(quant=quant, topk_frac=topk)
                p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt,
                                    quant_mode=api.QUANT_MODES[quant])
                ws = api.alloc_workspace(p)

                def step(i):
                    q, k, v, out = sets[i % len(sets)]
                    api.sla2_forward(p, q, k, v, rw, al, out, workspace=ws, stream=stream)
                for i in range(args.warmup):
                    step(i)
                api.sla2_profile_begin([n for n in api.STAGES if n != "dense"], args.steps)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for i in range(args.steps):
                    step(i)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) / args.steps * 1e3
                stages = {name: round(t / n, 4) for name, (t, n) in api.sla2_profile_end().items()}
                ksel = api.sla2_num_selected(p)
                line = {"metric": "SLA2 forward, dense-equivalent throughput 4*N^2*d*H*B / t",
                        "value": round(dense_flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
                        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
                        "dtype": "bf16" if quant == "none" else "fp8", "data": "synthetic",
                        "config": {"workload": "wan14b-sweep", "B": w.B, "H": w.H, "N": w.N, "d": w.d, "block_q": w.block_q,
                                   "block_kv": w.block_kv, "topk_frac": topk, "k": ksel, "T_n": w.T_n,
                                   "sparsity": round(1.0 - ksel / w.T_n, 4), "quant": quant, "input_sets": len(sets)},
                        "stage_ms": stages, "dense_bf16": dense, "speedup_vs_dense_bf16": round(dense_ms / ms, 2)}
                lines.append(line)
                print(json.dumps(line), flush=True)
                del ws
        del sets, inp
        torch.cuda.empty_cache()
    with open(args.sweep_out, "w") as f:
        for line in lines:
            f.write(json.dumps(line) + "\n")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported - value is the throughput of a single MI355X" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2602_12675_amd import api, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    w = W.CONFIGS[args.workload]
    if args.quant is not None:
        w = w.replace(quant=args.quant)
    if args.topk is not None:
        w = w.replace(topk_frac=args.topk)
    if args.block_q is not None:
        w = w.replace(block_q=args.block_q)
    if args.sweep:
        return sweep(args, api, W, torch)
    inp = W.generate(w)
    if args.router_identity:
        inp.router_w[:] = np.eye(w.d, dtype=np.float32)
    dt = api.SLA2_BF16 if w.dtype == "bf16" else api.SLA2_F32
    qm = api.QUANT_MODES[w.quant]
    strides = {}
    if args.packed_qkv:
        strides = dict(in_stride=(w.N * 3 * w.H * w.d, w.d, 3 * w.H * w.d), out_stride=(w.N * w.H * w.d, w.d, w.H * w.d))
    p = api.make_params(w.B, w.H, w.N, w.d, w.block_q, w.block_kv, w.topk_frac, dtype=dt, quant_mode=qm, **strides)
    ksel = api.sla2_num_selected(p)
    sets = []
    for s in range(max(1, args.input_sets)):
        q, k, v = (api.to_device(a, dt) for a in (inp.q, inp.k, inp.v))
        if args.packed_qkv:
            qkv = torch.empty((w.B, w.N, 3, w.H, w.d), dtype=q.dtype, device="cuda")
            for x, t in enumerate((q, k, v)):
                qkv[:, :, x] = t.permute(0, 2, 1, 3)
            del q, k, v
            sets.append((qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2],
                         torch.empty((w.B, w.N, w.H, w.d), dtype=qkv.dtype, device="cuda")))
        else:
            sets.append((q, k, v, torch.empty_like(q)))
    rw = torch.from_numpy(inp.router_w).cuda()
    al = torch.from_numpy(inp.alpha).cuda()
    ws = api.alloc_workspace(p)
    stream = torch.cuda.current_stream()

    def step(i):
        q, k, v, out = sets[i % len(sets)]
        api.sla2_forward(p, q, k, v, rw, al, out, workspace=ws, stream=stream)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    dense_flops = 4.0 * w.N * w.N * w.d * w.H * w.B

    def timed(n_warm, n):
        """n_warm untimed calls, then exactly n calls between two synchronisations."""
        for i in range(n_warm):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3

    # `value`: W warm-up calls, then exactly K timed calls, first thing - on the chip as the process finds it.
    # With a small W that region lies inside the clock ramp of the first tens of milliseconds of load; the
    # `settled` object below times the same loop again at the end of the run and is never `value`.
    # The dominant kernel carries an event pair (on every step unless --event-stride says otherwise;
    # measured: the pairs do not change the step time).
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    stride = max(1, args.event_stride)
    api.sla2_profile_begin_sampled(["attn"], (args.steps + stride - 1) // stride, stride)
    # one event per step boundary (same stream as the kernels): the spread of the K calls, next to their mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = api.sla2_profile_end()
    ms_per_step = elapsed / args.steps * 1e3
    value = dense_flops / (ms_per_step * 1e-3) / 1e12
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    step_ms = {"median": round(per_step[len(per_step) // 2], 4), "min": round(per_step[0], 4), "max": round(per_step[-1], 4),
               "note": "GPU time between event marks after each of the K timed calls"}

    # The dense comparator, after two untimed calls of its own (the chip is at its sustained clocks by then:
    # a comparator timed cold would flatter the ratio).
    dense = None
    if not args.no_dense and w.dtype == "bf16":
        q, k, v, out = sets[0]
        reps = 5
        for _ in range(2):
            api.sla2_dense_forward(p, q, k, v, out, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            api.sla2_dense_forward(p, q, k, v, out, stream=stream)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) / reps * 1e3
        dense = {"ms": round(dense_ms, 3), "TFLOP/s": round(dense_flops / (dense_ms * 1e-3) / 1e12, 1),
                 "frac_of_mfma_peak": round(dense_flops / (dense_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS["bf16"], 4),
                 "reps": reps}

    # the same call on one input set only (its key/value state stays in the memory-side cache): reported
    # next to the headline figure, labelled, never as `value`
    warm = None
    if len(sets) > 1:
        n_warm = max(10, args.steps // 2)
        for _ in range(5):
            step(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_warm):
            step(0)
        torch.cuda.synchronize()
        warm_ms = (time.perf_counter() - t0) / n_warm * 1e3
        warm = {"ms_per_step": round(warm_ms, 4), "TFLOP/s": round(dense_flops / (warm_ms * 1e-3) / 1e12, 2),
                "steps": n_warm, "note": "one input set reused; `value` rotates over %d sets" % len(sets)}

    # per-kernel breakdown: a pass of its own, every kernel between event pairs
    api.sla2_profile_begin([n for n in api.STAGES if n != "dense"], args.steps)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    stages = {name: ms / n for name, (ms, n) in api.sla2_profile_end().items()}

    # the timed loop once more, now that the chip has had the comparator and 2 x steps more calls to reach its
    # sustained clocks: reported next to the headline figure, labelled, never as `value`
    settled_ms = timed(0, args.steps)
    settled = {"ms_per_step": round(settled_ms, 4), "TFLOP/s": round(dense_flops / (settled_ms * 1e-3) / 1e12, 2),
               "steps": args.steps,
               "note": "the same rotating-input loop as `value`, timed again at the end of the run (sustained clocks)"}
    if dense is not None:
        settled["speedup_vs_dense_bf16"] = round(dense["ms"] / settled_ms, 2)

    backward = None
    if not args.no_backward:
        backward = backward_timing(api, W, torch, w, inp, dt, qm, sets[0], rw, al, stream, ksel)

    BH, esz = w.B * w.H, (2 if w.dtype == "bf16" else 4)
    tile_iters = BH * w.T_m * ksel
    qk_flops = tile_iters * 2.0 * w.block_q * w.block_kv * w.d           # Q K^T: 8-bit products in the low-bit modes
    lin_flops = BH * w.T_m * 2.0 * w.block_q * w.d * w.d                 # Q^phi H_i: always bf16
    attn_flops = 2.0 * qk_flops + lin_flops                              # + P V, same count as Q K^T
    low_flops = {"none": 0.0, "fp8": qk_flops, "int8": qk_flops, "fp8v": 2.0 * qk_flops}[w.quant]
    rest_flops = attn_flops - low_flops
    attn_ms = prof["attn"][0] / prof["attn"][1]
    mm = {"none": "bf16", "fp8v": "fp8"}.get(w.quant, w.quant)
    achieved = attn_flops / (attn_ms * 1e-3) / 1e12
    if w.quant != "none":
        # each product priced at the peak of its own operand type: time-weighted (harmonic) blend
        low = "int8" if w.quant == "int8" else "fp8"
        peak = attn_flops / (low_flops / MFMA_PEAK_TFLOPS[low] + rest_flops / MFMA_PEAK_TFLOPS["bf16"])
        note = ("peak = harmonic blend of dense %s MFMA (%s, %.3g TFLOP) and dense bf16 MFMA (the rest, %.3g TFLOP)"
                % (low, "Q K^T and P V" if w.quant == "fp8v" else "Q K^T", low_flops / 1e12, rest_flops / 1e12))
    else:
        peak = MFMA_PEAK_TFLOPS["bf16"]
        note = "peak = dense bf16 MFMA"
    roofline = {"kernel": "attn_mfma (sparse + linear branch + mix)", "bound": "mfma", "achieved": round(achieved, 2),
                "peak": round(peak, 1), "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": measured_traffic(w.name, w.quant), "traffic_source": traffic_source(), "ms": round(attn_ms, 4),
                "launches_timed": prof["attn"][1],
                "algorithmic_flops": attn_flops, "note": note}
    if "attn" in stages:
        # the same kernel in the per-kernel pass later in the run (sustained clocks); labelled, not `frac`
        roofline["per_kernel_pass"] = {"ms": round(stages["attn"], 4),
                                       "frac": round(attn_flops / (stages["attn"] * 1e-3) / 1e12 / peak, 4)}
    # the same kernel against the other roof it can hit: bytes it has to gather per (query block, key block)
    # pair - the K tile (codes in the low-bit modes) and the V tile - plus Q read and out written once.
    # (The K^phi fragments it also loads, 16 KB per pair, are this design's choice and not counted.)
    k_tile = w.block_kv * w.d * (1 if w.quant != "none" else esz)
    v_tile = w.block_kv * w.d * esz + (w.block_kv * w.d if w.quant == "fp8v" else 0)
    gather_bytes = tile_iters * float(k_tile + v_tile) + 2.0 * BH * w.N * w.d * esz
    gather_gbs = gather_bytes / (attn_ms * 1e-3) / 1e9
    roofline["gathered_tiles"] = {"bound": "hbm", "achieved": round(gather_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "frac": round(gather_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": gather_bytes,
                                  "note": "K and V tiles of every selected pair + Q + out over the same kernel time; "
                                          "most tiles are served by L2 / Infinity Cache (see traffic)"}
    if roofline["traffic"]:
        # what the counters saw leave L2 for the fabric (profiles/), over the kernel time measured here
        t_gbs = roofline["traffic"] / (attn_ms * 1e-3) / 1e9
        roofline["traffic_rate"] = {"GB/s": round(t_gbs, 1), "frac_of_hbm_peak": round(t_gbs / HBM_PEAK_GBS, 4)}
    qk_bytes = 2.0 * BH * w.N * w.d * esz
    hbm = {}
    if "block_sums" in stages:
        gbs = qk_bytes / (stages["block_sums"] * 1e-3) / 1e9
        hbm["block_sums"] = {"GB/s": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4), "bytes": qk_bytes}
    if "kv_state" in stages:
        b = qk_bytes + BH * w.T_n * w.block_kv * w.d * {"none": 0, "fp8v": 2}.get(w.quant, 1)
        gbs = b / (stages["kv_state"] * 1e-3) / 1e9
        hbm["kv_state"] = {"GB/s": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4), "bytes": b}

    line = {
        "metric": "SLA2 forward, dense-equivalent throughput 4*N^2*d*H*B / t",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": mm, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "block_q": w.block_q,
                   "block_kv": w.block_kv, "topk_frac": w.topk_frac, "k": ksel, "T_n": w.T_n,
                   "sparsity": round(1.0 - ksel / w.T_n, 4), "quant": w.quant, "input_sets": len(sets),
                   "router": "identity weights (pooled-QK router)" if args.router_identity else "random projections",
                   "layout": "packed [B,N,3,H,d] -> [B,N,H,d]" if args.packed_qkv else "[B,H,N,d]"},
        "step_ms": step_ms,
        "roofline": roofline,
        "order": "W warm-up + K timed calls = value; dense comparator; one-input-set pass; per-kernel pass; the K calls again = settled; backward",
        "settled": settled,
        "warm_single_input_set": warm,
        "stage_ms": {k_: round(v_, 4) for k_, v_ in stages.items()},
        "hbm_kernels": hbm,
    }
    if dense is not None:
        line["dense_bf16"] = dense
        line["speedup_vs_dense_bf16"] = round(dense["ms"] / ms_per_step, 2)
    if backward is not None:
        line["backward"] = backward
    line["paper_context"] = "paper: 97 % sparsity, 18.6x attention speed-up over FlashAttn2 on an RTX5090 (other hardware; not a target)"
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(inp, max(1, min(args.cpu_heads, w.H)))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
