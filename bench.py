#!/usr/bin/env python3
"""Benchmark of the rank-local Domino layer (forward + backward) on one MI355X.

A step is one pass of the whole hot path: domino_layer_fwd + domino_layer_bwd over one batch of
synthetic input (all p x q pieces, all streams joined), inputs resident in HBM.  Prints ONE JSON line:
whole-job throughput in algorithmic TFLOP/s (causal attention counted at half the dense s^2,
backward = 2 x forward, no recomputation counted), the roofline of the dominant kernel measured with
HIP events on the kernel's own stream, and the fp64 CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt3-13b] [--streams 4]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

# The pool's streams only overlap if each has a hardware queue of its own; the HIP runtime's default of 4
# queues per process leaves one of them to the null stream, and two pool streams then share a queue and
# run their row slices one after the other.  Must be set before the runtime initialises (import torch).
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
DEFAULT_WORKLOAD = "gpt3-13b"      # the shard the throughput target is quoted on


def gemm_flops_per_launch(sc):
    """Algorithmic flops of one launch of each GEMM step class (one row slice; one column piece for
    the two row-parallel products; the weight gradients contract over one slice's rows for p <= 2 and over all rows
    of the block, in one launch per matrix, beyond that)."""
    Ms = sc.tokens // sc.p
    Mw = wgrad_rows(sc)
    h, hl, fl, upc, hq = sc.hidden, sc.h_local, sc.f_local, sc.up_cols, sc.hidden // sc.q
    return {
        "gemm_qkv": 2.0 * Ms * h * 3 * hl, "gemm_out": 2.0 * Ms * hl * hq, "gemm_up": 2.0 * Ms * h * upc,
        "gemm_down": 2.0 * Ms * fl * hq, "dgrad_down": 2.0 * Ms * h * fl, "wgrad_down": 2.0 * Mw * fl * h,
        "dgrad_up": 2.0 * Ms * upc * h, "wgrad_up": 2.0 * Mw * h * upc, "dgrad_out": 2.0 * Ms * h * hl,
        "wgrad_out": 2.0 * Mw * hl * h, "dgrad_qkv": 2.0 * Ms * 3 * hl * h, "wgrad_qkv": 2.0 * Mw * h * 3 * hl,
    }


def wgrad_rows(sc):
    """Rows one weight-gradient launch contracts over (the library's rule: merged over the slices when p > 2)."""
    return sc.tokens if sc.p > 2 and not sc.wgrad_per_slice else sc.tokens // sc.p


def algorithmic_flops(sc):
    M = sc.tokens
    gemm = 2.0 * M * (sc.hidden * 3 * sc.h_local + sc.h_local * sc.hidden + sc.hidden * sc.up_cols
                      + sc.f_local * sc.hidden)
    attn = 2.0 * sc.batch * sc.local_heads * sc.seq * sc.seq * sc.head_dim
    return 3.0 * (gemm + attn)


TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic_per_launch.md")


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE runs (lines
    'traffic[<workload>][<kernel>] = <bytes>' of the summary file), or None if it holds no such line."""
    key = f"traffic[{workload}][{kernel}] ="
    try:
        with open(TRAFFIC_FILE) as fh:
            for ln in fh:
                if ln.startswith(key):
                    return float(ln[len(key):].split()[0])
    except OSError:
        pass
    return None


def draw_inputs(sc):
    """The seeded inputs of a workload; the three groups of tensors are drawn side by side (NumPy's generators
    release the interpreter lock), which changes no value: every tensor has a random stream of its own."""
    from concurrent.futures import ThreadPoolExecutor
    from paper_2409_15241_amd import synth
    with ThreadPoolExecutor(max_workers=3) as ex:
        fp = ex.submit(synth.make_rank_params, sc)
        fa = ex.submit(synth.make_activations, sc)
        fo = ex.submit(synth.make_others, sc)
        x, dy = fa.result()
        return fp.result(), x, dy, fo.result()


def time_other_workloads(names, nstreams, pool, steps=10, warmup=3):
    """Forward + backward of the other configured shards as configured (their p and q), event-timed on the pool's
    first stream over `steps` steps in a row after `warmup` steps: ms per step, TFLOP/s, % of the nominal peak."""
    import torch
    from paper_2409_15241_amd import harness, synth
    out = {}
    for name in names:
        sc = synth.WORKLOADS[name]
        params, x, dy, others = draw_inputs(sc)
        buf = harness.LayerBuffers(sc, params, x, dy, others, streams=pool[:nstreams])
        del params, x, dy, others
        for _ in range(warmup):
            buf.forward()
            buf.backward(False)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(buf.streams[0])
        for _ in range(steps):
            buf.forward()
            buf.backward(False)
        e1.record(buf.streams[0])
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        tf = algorithmic_flops(sc) / (ms * 1e-3) / 1e12
        out[name] = {"ms_per_step": ms, "value": tf, "unit": "TFLOP/s", "pct_of_bf16_mfma_peak": 100.0 * tf / BF16_MFMA_PEAK_TFLOPS,
                     "p": sc.p, "q": sc.q, "tokens": sc.tokens, "steps": steps}
        del buf
        torch.cuda.empty_cache()
    return out


def measured_mfma_ceiling(stream, seconds=0.06):
    """TFLOP/s of back-to-back bf16 MFMAs (the library's MFMA-only probe) on operands drawn like the layer's
    (activations ~ N(0,1) against weights ~ N(0, 0.02^2)), sustained for about `seconds` so that the clock has
    settled where the power limit puts it."""
    import torch
    from paper_2409_15241_amd import domino
    g = torch.Generator(device="cuda").manual_seed(20240915)
    a = torch.randn(2048, device="cuda", generator=g).to(torch.bfloat16)
    b = (0.02 * torch.randn(2048, device="cuda", generator=g)).to(torch.bfloat16)
    blocks = 512                       # two workgroups of four waves per compute unit
    out = torch.empty(blocks * 256, device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    iters = 2000
    domino.domino_mfma_probe(a, b, out, blocks, iters, stream)          # warm-up and a first rate
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    fl = domino.domino_mfma_probe(a, b, out, blocks, iters, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    per_iter_ms = e0.elapsed_time(e1) / iters
    n = max(1, int(seconds * 1e3 / 6 / per_iter_ms))                    # six launches fill the span
    tot_fl = 0.0
    e0.record(stream)
    for k in range(6):
        if k == 2:
            e0.record(stream)                                           # the first two launches let the clock settle
            tot_fl = 0.0
        tot_fl += domino.domino_mfma_probe(a, b, out, blocks, n, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    return tot_fl / (e0.elapsed_time(e1) * 1e-3) / 1e12


def cpu_baseline(sc, budget_s=30.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import domino_oracle as O
    from paper_2409_15241_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    params = {k: (None if v is None else v.astype(np.float64)) for k, v in synth.make_rank_params(sc).items()}
    x, dy = synth.make_activations(sc)

    def run(sub):
        xs, dys = x[:sub.batch].astype(np.float64), dy[:sub.batch].astype(np.float64)
        t0 = time.perf_counter()
        F = O.rank_layer_fwd(sub, params, xs)
        O.rank_layer_bwd(sub, params, F, dys)
        return time.perf_counter() - t0

    # one row slice first; the whole batch (one full step of the workload) if that fits the budget
    sub = sc.replace(batch=sc.batch // sc.p, p=1, q=1)
    dt = run(sub)
    what = f"one row slice ({sub.batch} of {sc.batch} batch elements, {sub.tokens} tokens)"
    if dt * sc.p * 1.5 <= budget_s:
        sub = sc.replace(p=1, q=1)
        dt = run(sub)
        what = f"one full step (all {sc.batch} batch elements, {sub.tokens} tokens)"
    flops = algorithmic_flops(sub)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{what} fwd+bwd in fp64, {dt:.1f} s, within a {budget_s:.0f} s budget"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--streams", type=int, default=4)
    ap.add_argument("--layers", type=int, default=1,
                    help="blocks per step: above 1 the step is domino_stack_fwd + domino_stack_bwd over that many "
                         "blocks (row slices run on from block to block without joining)")
    ap.add_argument("--graph", action="store_true", help="capture the step in a HIP graph and replay it")
    ap.add_argument("--p", type=int, default=None)
    ap.add_argument("--q", type=int, default=None)
    ap.add_argument("--wgrad-per-slice", action="store_true",
                    help="weight gradients slice by slice behind each input gradient (the order of Sec. 4.1.2) also for p > 2")
    ap.add_argument("--stack-layers", type=int, default=4,
                    help="with --layers 1: also time a stack of this many blocks (0 = skip) and report it under 'stack'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the 10 timed steps of each of the other configured shards (key 'other_workloads')")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the MFMA-only probe (key 'measured_mfma_ceiling')")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="print the per-step-class timing table to stderr")
    ap.add_argument("--copy-check", type=int, default=0, metavar="MIB",
                    help="also run three plain device copies of this many MiB (a kernel of known HBM traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the one-GPU rank-local path; run it with --gpus 1 "
              "(the tensor-parallel all-reduce across GPUs is outside its scope)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2409_15241_amd import domino, harness, synth
    domino.load()
    sc = synth.WORKLOADS[args.workload]
    if args.p or args.q:
        sc = sc.replace(p=args.p or sc.p, q=args.q or sc.q)
    if args.wgrad_per_slice:
        sc = sc.replace(wgrad_per_slice=1)
    if args.graph and not domino.domino_capture_supported(args.streams, sc.p):
        print("bench.py: --graph is limited to pools of 1, 2 or 4 streams (graph instantiation of the other pool "
              "sizes aborted inside the runtime on this ROCm; the library refuses to be captured with them)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    params, x, dy, others = draw_inputs(sc)
    if args.layers > 1:
        params_l, others_l = synth.make_stack(sc, args.layers)
        buf = harness.StackBuffers(sc, params_l, x, dy, others_l, nstreams=args.streams)
    else:
        buf = harness.LayerBuffers(sc, params, x, dy, others, nstreams=args.streams)
    s0 = buf.streams[0]

    def eager_step():
        buf.forward()
        buf.backward(accumulate=False)

    step = eager_step
    if args.graph:
        # one pass of the path captured once on streams[0] (the library forks the other streams from it
        # and joins them back) and replayed: same kernels, launch order fixed by the graph's edges
        eager_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s0):
            eager_step()
        step = graph.replay             # on torch's current stream (replaying on streams[0] itself was measured 15 % slower)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps
    flops = algorithmic_flops(sc) * args.layers
    value = flops / (ms * 1e-3) / 1e12

    # forward-only / backward-only, event-timed on streams[0] (where the library joins its streams)
    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(s0)
        for _ in range(n):
            fn()
        e1.record(s0)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    # the step again, one event pair per step on streams[0]: spread of the single steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    ts = torch.cuda.current_stream() if args.graph else s0      # the stream the step is ordered on
    for e0, e1 in evs:
        e0.record(ts)
        step()
        e1.record(ts)
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_median, ms_min, ms_max = per_step[len(per_step) // 2], per_step[0], per_step[-1]
    fwd_ms = timed(buf.forward, max(3, args.steps // 3))
    bwd_ms = timed(lambda: buf.backward(False), max(3, args.steps // 3))

    roofline = None
    if not args.no_roofline:
        # the same K steps again with every launch bracketed by timing events on its own stream (eagerly also
        # when the timed steps were graph replays: a replay makes no library call that could be bracketed)
        domino.domino_profile_reset()
        domino.domino_profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            eager_step()
        torch.cuda.synchronize()
        inst_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        domino.domino_profile_enable(False)
        per = gemm_flops_per_launch(sc)
        table = {}
        for c in range(domino.domino_profile_classes()):
            tot, n = domino.domino_profile_read(c)
            if n:
                table[domino.domino_profile_name(c)] = (tot, n)
        domino.domino_profile_reset()
        # step classes that run the same kernel instantiation (= one line of a rocprofv3 kernel summary)
        llama = bool(sc.arch)
        instances = {
            "gemm_kernel<NN, store> (qkv, out-proj and mlp-down products)": ["gemm_qkv", "gemm_out", "gemm_down"],
            ("gemm_kernel<NN, swiglu> (mlp-up product)" if llama else "gemm_kernel<NN, bias+gelu> (mlp-up product)"): ["gemm_up"],
            "gemm_kernel<NT, store> (input gradients of mlp-up, out-proj, qkv)": ["dgrad_up", "dgrad_out", "dgrad_qkv"],
            ("gemm_kernel<NT, dswiglu> (input gradient of mlp-down)" if llama else "gemm_kernel<NT, dgelu> (input gradient of mlp-down)"): ["dgrad_down"],
            "gemm_kernel<TN, fp32 accumulate> (the four weight gradients)": ["wgrad_down", "wgrad_up", "wgrad_out", "wgrad_qkv"],
        }
        agg = {}
        for name, classes in instances.items():
            t = sum(table[c][0] for c in classes if c in table)
            n = sum(table[c][1] for c in classes if c in table)
            f = sum(per[c] * table[c][1] for c in classes if c in table)
            if n:
                agg[name] = (t, n, f)
        # the dominant kernel: most time on its streams; of those within 10 % of the longest (two instantiations can
        # trade places from run to run) the one that carries more of the step's flops
        longest = max(v[0] for v in agg.values())
        dom_name = max((k for k in agg if agg[k][0] >= 0.9 * longest), key=lambda k: agg[k][2])
        tot, n, f = agg[dom_name]
        avg_ms = tot / n
        achieved = f / (tot * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom_name, "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                    "traffic": measured_traffic(sc.name, dom_name),
                    "traffic_source": "profiles/hbm_traffic_per_launch.md: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of "
                                      "this kernel at this workload's shapes, scaled by a plain copy of known size; not "
                                      "re-measured by this run (null: no such run for this workload)",
                    "avg_launch_us": avg_ms * 1e3, "launches_per_step": n // args.steps,
                    "flops_per_launch": f / n, "ms_per_step_instrumented": inst_ms}
        if args.breakdown:
            print(f"{'class':14s} {'launch/step':>11s} {'us/launch':>10s} {'ms/step':>8s} {'TFLOP/s':>8s}", file=sys.stderr)
            for k, (t, m) in sorted(table.items(), key=lambda kv: -kv[1][0]):
                tf = per[k] / (t / m * 1e-3) / 1e12 if k in per else float("nan")
                print(f"{k:14s} {m // args.steps:11d} {t / m * 1e3:10.1f} {t / args.steps:8.3f} {tf:8.1f}", file=sys.stderr)

    if args.copy_check:
        src = torch.empty(args.copy_check << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if roofline is not None and roofline["kernel"].startswith("gemm_kernel<TN"):
        # context for `achieved`: the same launches with the chip to themselves (one stream, nothing else running)
        Ms = wgrad_rows(sc)
        shapes = [(sc.f_local, sc.hidden), (sc.hidden, sc.up_cols), (sc.h_local, sc.hidden), (sc.hidden, 3 * sc.h_local)]
        tile = 2 if min(args.streams, sc.p) >= 3 else -1       # the tile the layer call picks
        tot_ms, tot_fl = 0.0, 0.0
        for (Mw, Nw) in shapes:
            A = torch.randn(Ms, Mw, device="cuda").to(torch.bfloat16)
            B = torch.randn(Ms, Nw, device="cuda").to(torch.bfloat16)
            Cw = torch.zeros(Mw, Nw, device="cuda", dtype=torch.float32)
            torch.cuda.synchronize()
            run = lambda: domino.domino_gemm(domino.GEMM_TN, domino.EPI_ACC_F32, tile, A, Mw, B, Nw, Cw, Nw, Mw, Nw, Ms,
                                             beta=0 if Ms == sc.tokens else 1, stream=s0)
            run()
            tot_ms += timed(run, 10)
            tot_fl += 2.0 * Ms * Mw * Nw
        roofline["achieved_alone"] = tot_fl / (tot_ms * 1e-3) / 1e12
        roofline["frac_alone"] = roofline["achieved_alone"] / BF16_MFMA_PEAK_TFLOPS

    stack = None
    if args.layers == 1 and args.stack_layers > 1 and not args.graph:
        # the same blocks one after the other in one call (domino_stack_fwd / domino_stack_bwd): no fork and join
        # between blocks, so this is the rate a model of many blocks sees; same stand-in tensors for every block
        nl = args.stack_layers
        params_l = [synth.make_rank_params(sc, seed=synth.config_seed(sc) + l * synth.LAYER_SEED_STRIDE) for l in range(nl)]
        sbuf = harness.StackBuffers(sc, params_l, x, dy, [others] * nl, streams=buf.streams)   # the same pool
        for _ in range(max(2, args.warmup // 2)):
            sbuf.forward()
            sbuf.backward(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nrep = max(3, args.steps // 2)
        for _ in range(nrep):
            sbuf.forward()
            sbuf.backward(False)
        torch.cuda.synchronize()
        sms = (time.perf_counter() - t0) * 1e3 / nrep
        stack = {"layers": nl, "ms_per_step": sms, "ms_per_layer": sms / nl,
                 "value": algorithmic_flops(sc) * nl / (sms * 1e-3) / 1e12, "unit": "TFLOP/s"}

    ceiling = None if args.no_ceiling else measured_mfma_ceiling(s0)
    pool = buf.streams
    others_wl = None
    if not args.no_other_workloads and args.layers == 1:
        del buf
        torch.cuda.empty_cache()
        names = [n for n in ("tiny", "gpt3-2.7b", "gpt3-13b", "llama2-7b", "llama2-13b") if n != sc.name]
        others_wl = time_other_workloads(names, args.streams, pool)

    cpu = None if args.no_cpu_baseline else cpu_baseline(sc)

    line = {
        "metric": "layer fwd+bwd TFLOP/s per rank shard (1 MI355X); % of bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": sc.name, "hidden": sc.hidden, "heads": sc.heads, "tp": sc.tp, "rank": sc.rank,
                   "batch": sc.batch, "seq": sc.seq, "ffn": sc.ffn, "p": sc.p, "q": sc.q,
                   "arch": "llama" if sc.arch else "gpt", "streams": args.streams, "layers": args.layers,
                   "weight_gradients": "slice by slice" if sc.p <= 2 or sc.wgrad_per_slice else "once per block over all rows"},
        "pct_of_bf16_mfma_peak": 100.0 * value / BF16_MFMA_PEAK_TFLOPS,
        "algorithmic_gflop_per_step": flops / 1e9, "ms_per_step_median": ms_median, "ms_per_step_min": ms_min,
        "ms_per_step_max": ms_max, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "measured_mfma_ceiling": None if ceiling is None else {
            "value": ceiling, "unit": "TFLOP/s",
            "what": "back-to-back 32x32x16 bf16 MFMAs on N(0,1) x N(0,0.02) fragments, nothing else running (domino_mfma_probe)"},
        "pct_of_measured_mfma_ceiling": None if ceiling is None else 100.0 * value / ceiling,
        "other_workloads": others_wl,
        "stack": stack, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
