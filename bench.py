#!/usr/bin/env python3
"""Benchmark of the BCQ linear hot path on one MI355X.

Workload (default): the four linear layers of one GPT-2-medium-shaped block (h = 1024: QKV 1024->3072,
out 1024->1024, MLP 1024->4096->1024), q = 4 bit planes, bf16 activations, T = 8 x 512 = 4096 tokens,
W ~ N(0, 0.02^2) quantized once by the greedy quantizer, x, dy ~ N(0, 1).  One step = forward, input gradient
and alpha gradient of all four layers.  The quantizer, pack and transposed-twin passes run once before the
timed region (they are the one-time PTQ of the method) and are timed separately in "setup".

Prints ONE JSON line: effective TFLOP/s (6 T N K flops per layer and step), the roofline figures of the
dominant kernel family measured with HIP events inside the timed region, and the CPU oracle timed on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E peak
PEAK_FP32_VECTOR_TFLOPS = 157.3  # 256 compute units x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz

# HBM-side bytes per launch of the dominant kernel of the default workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter reads for a 256 MiB copy); see
# profiles/bench_config2_hbm_traffic.md for the commands and the table.  Not measured live: null for other workloads.
PMC_TRAFFIC_BYTES = {(2, 4096, 4, "bwd_alpha"): 5.12e7, (2, 4096, 4, "fwd"): 7.76e7, (2, 4096, 4, "bwd_input"): 7.76e7}
# the same for one whole step of `--config 5 --layer 16384x16384 --tokens 8` per layer copy (fwd 141.2 MB, dalpha 138.6 MB,
# dx 154.5 MB, the three activation pre-kernels 2.8 MB; profiles/stream_large_layer_kernel_stats.md)
PMC_TRAFFIC_STREAM_LAYER = {((16384, 16384), 8, 4): 4.252e8}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step is about half a millisecond: the defaults time 50 ms of steady state after the clocks have settled
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, help="workload number (2 = GPT-2-medium block, the headline)")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count of the workload")
    ap.add_argument("--q", type=int, default=0, help="override the number of bit planes")
    ap.add_argument("--g", type=int, default=0,
                    help="group size of the scales along K (Table 4); 0 = row-wise (g = h_in), the headline workload; "
                         "a layer with K < g uses g = K")
    ap.add_argument("--layer", type=str, default="",
                    help="time ONE layer of shape NxK (e.g. 16384x16384) instead of the workload's four layer shapes; "
                         "seeds, dtype and q still come from --config")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the two context measurements (device-to-device copy, plain bf16 GEMMs of the same "
                         "shapes through the vendor BLAS that PyTorch links)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="skip the per-op HIP events (pure step timing)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the whole step on one stream.  By default (32 tokens and more) a step is ordered like a "
                         "training step (all forwards, then the backward pass from the last layer) and the scale gradients "
                         "run on a second HIP stream of default priority beside the input gradients, joined at the end "
                         "of the step: in training dalpha "
                         "is a leaf of the backward pass (Eq. 4), only the optimizer waits for it")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every timed step from Python instead of replaying one captured HIP graph (a step is 32 "
                         "short launches: on a slow host the Python loop, not the GPU, then sets the pace)")
    ap.add_argument("--graph", action="store_true", help="accepted for compatibility: graph replay is the default")
    ap.add_argument("--replicas", type=int, default=0,
                    help="independent copies of the layer stack (own weights), so that the packed planes streamed per "
                         "step exceed the 256 MB Infinity Cache; default 1, or enough for 512 MB when tokens < 32")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives are part of "
              "the BCQ linear hot path: rows of W shard without any exchange except one all-reduce of dx)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2210_03858_amd as bcq
    from paper_2210_03858_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    bcq.load()

    cfg = synth.CONFIGS[args.config]
    h = cfg["h"]
    q = args.q or cfg["q"][-1]
    T = args.tokens or cfg["tokens"][-1]
    dtype = cfg["dtype"]
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = bcq.binding.BCQ_BF16 if dtype == "bf16" else bcq.binding.BCQ_F32
    kinds = cfg["kinds"]
    custom = None
    if args.layer:
        custom = tuple(int(v) for v in args.layer.lower().split("x"))
        assert len(custom) == 2 and custom[1] % 32 == 0, "--layer wants NxK with K % 32 == 0"
        kinds = ("out",)  # seeds of the (h, h) layer

    def shape_of(kind):
        return custom if custom else synth.layer_shape(h, kind)

    small = T < 32            # streaming regime: bound by HBM, measured over a stack of distinct layers
    use_graph = not args.no_graph
    block_packed = sum(shape_of(k)[0] * shape_of(k)[1] for k in kinds) * q // 8
    replicas = args.replicas or (max(1, -(-(512 << 20) // block_packed)) if small else 1)

    # ---------------- one-time setup: synthetic weights -> greedy BCQ on the GPU, twin, activations
    layers = []
    setup_ms = {"quantize": 0.0, "pack_transposed": 0.0}
    weights_total = 0
    for rep, kind in [(r, k) for r in range(replicas) for k in kinds]:
        N, K = shape_of(kind)
        W = torch.from_numpy(synth.weights(args.config, kind, N, K, outliers=cfg["outliers"], extra=rep)).cuda()
        g = min(args.g, K) if args.g else K
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        bcq.bcq_quantize_grouped(W, q, g)  # warm
        e0.record()
        alpha, packed, _ = bcq.bcq_quantize_grouped(W, q, g)
        e1.record()
        twin = bcq.bcq_pack_transposed(packed) if N % 32 == 0 else None
        e2.record()
        torch.cuda.synchronize()
        setup_ms["quantize"] += e0.elapsed_time(e1)
        setup_ms["pack_transposed"] += e1.elapsed_time(e2)
        weights_total += N * K
        x = torch.from_numpy(synth.activations(args.config, kind, T, K, 1, dtype)).cuda().to(tdtype)
        dy = torch.from_numpy(synth.activations(args.config, kind, T, N, 2, dtype)).cuda().to(tdtype)
        ws = {}
        for op in (1, 2, 3):
            nbytes = bcq.workspace_bytes_grouped(op, T, N, K, g, q, code)
            ws[op] = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        layers.append(dict(kind=kind, N=N, K=K, g=g, alpha=alpha, packed=packed, twin=twin, x=x, dy=dy, ws=ws,
                           y=torch.empty((T, N), dtype=tdtype, device="cuda"),
                           dx=torch.empty((T, K), dtype=tdtype, device="cuda"),
                           da=torch.empty((q, N, K // g), dtype=torch.float32, device="cuda")))
        del W

    ops = ("fwd", "bwd_input", "bwd_alpha")

    def run_op(L, op):
        # the row-wise C entry points forward to the grouped ones with g = K, so one call form serves both
        if op == "fwd":
            bcq.bcq_linear_fwd_grouped(L["packed"], L["alpha"], L["x"], L["g"], y=L["y"], workspace=L["ws"][1])
        elif op == "bwd_input":
            bcq.bcq_linear_bwd_input_grouped(L["packed"], L["alpha"], L["dy"], L["g"], packed_t=L["twin"], dx=L["dx"],
                                             workspace=L["ws"][2])
        else:
            bcq.bcq_linear_bwd_alpha_grouped(L["packed"], L["x"], L["dy"], L["g"], dalpha=L["da"],
                                             workspace=L["ws"][3])

    side = torch.cuda.Stream() if (not args.no_overlap and not small) else None

    def step_overlapped():
        """Ordered like a training step: the forward of every layer first; then, from the last layer back, the input
        gradient on the current stream and the scale gradient on the side stream (it is a leaf of the backward pass:
        only the optimizer waits for it); one join at the end."""
        main = torch.cuda.current_stream()
        for L in layers:
            run_op(L, "fwd")
        side.wait_stream(main)  # the backward pass starts when the forward is done
        for L in reversed(layers):
            with torch.cuda.stream(side):
                run_op(L, "bwd_alpha")
            run_op(L, "bwd_input")
        main.wait_stream(side)

    def step(events=None, only=None):
        """One pass of the hot path.  With `events`, HIP events bracket every op (or only the ops of family `only`)."""
        if side is not None and events is None:
            return step_overlapped()
        for L in layers:
            for op in ops:
                if events is not None and (only is None or op == only):
                    a = torch.cuda.Event(enable_timing=True)
                    b = torch.cuda.Event(enable_timing=True)
                    a.record()
                    run_op(L, op)
                    b.record()
                    events.append((op, L["kind"], a, b))
                else:
                    run_op(L, op)

    if args.calibrate_copy:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- warm-up: every op bracketed by events -> per-op table and the dominant op family
    warm_events = []
    n_warm = max(args.warmup, 2)  # at least two: the per-op figures skip the first step (one-time set-up of the kernels)
    for _ in range(n_warm):
        step(warm_events)
    torch.cuda.synchronize()
    graph = None
    if use_graph:  # the library neither allocates nor memsets, so a step can be captured as it is
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
    # per op family: time per step, median over the warm-up steps but the first (which pays one-time set-up)
    n_ev = len(ops) * len(layers)
    fam_steps = {op: [] for op in ops}
    for i in range(1, n_warm):
        sums = dict.fromkeys(ops, 0.0)
        for op, kind, a, b in warm_events[i * n_ev:(i + 1) * n_ev]:
            sums[op] += a.elapsed_time(b)
        for op in ops:
            fam_steps[op].append(sums[op])
    fam_ms = {op: sorted(v)[(len(v) - 1) // 2] for op, v in fam_steps.items()}  # lower median
    dom = max(fam_ms, key=lambda k: fam_ms[k])

    # ---------------- timed region: exactly --steps steps; events only around the dominant family's launches
    # (an event pair costs a few microseconds of GPU idle time, so bracketing all twelve ops would slow the step)
    events = None if (args.no_events or graph is not None or side is not None) else []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if graph is not None:
            graph.replay()
        else:
            step(events, only=dom)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # spread of single steps (not part of `value`): up to 50 more steps, each bracketed by HIP events
    spread = []
    for _ in range(min(args.steps, 50)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        if graph is not None:
            graph.replay()
        else:
            step()
        b.record()
        spread.append((a, b))
    torch.cuda.synchronize()
    spread = sorted(a.elapsed_time(b) for a, b in spread)

    flops_layer = {L["kind"]: 2.0 * T * L["N"] * L["K"] for L in layers}
    flops_step = 3.0 * sum(flops_layer.values())
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---------------- roofline of the dominant op family (timed region) and per-op table (warm-up steps)
    fam_flops = sum(flops_layer.values())  # every family runs every layer once per step
    per_op = {op: {"ms_per_step": round(fam_ms[op], 4), "tflops": round(fam_flops / (fam_ms[op] * 1e-3) / 1e12, 3)}
              for op in ops}
    roofline = None
    roofline_note = None
    if events is None and not small and not args.no_events:
        # graph replay (no events inside a graph) or two streams (kernels overlap): the per-launch figures come from
        # the eagerly launched one-stream warm-up steps of this run (all but the first, which pays one-time set-up)
        events = [e for e in warm_events[len(ops) * len(layers):] if e[0] == dom] or None
        roofline_note = ("per-launch figures from the %d eagerly launched one-stream warm-up steps of this run; the timed "
                         "region %s" % (n_warm - 1,
                                        " and ".join(([("replays a HIP graph of the same step")] if graph is not None else [])
                                                     + (["runs dalpha on a second stream"] if side is not None else []))))
    if events:
        # per step of the dominant family: median over the steps the events cover (robust against a stray slow launch)
        per_step = len(layers)
        step_ms = sorted(sum(a.elapsed_time(b) for _, _, a, b in events[i:i + per_step])
                         for i in range(0, len(events) - per_step + 1, per_step))
        ms = step_ms[(len(step_ms) - 1) // 2] * (len(events) / per_step)
        fl = sum(flops_layer[kind] for _, kind, _, _ in events)
        achieved = fl / (ms * 1e-3) / 1e12
        main_kernel = {"fwd": "gemm_kernel (+ expand_fwd_kernel)", "bwd_input": "gemm_kernel (+ expand_bwd_kernel)",
                       "bwd_alpha": "dalpha_kernel (+ transpose_frag_kernel, dalpha_reduce_kernel)"}[dom]
        if (dom == "fwd" and T <= 80) or (dom == "bwd_input" and T <= 48):  # the library streams the planes up to there
            main_kernel = "stream_kernel (+ quant_act_kernel), one pass over the planes per 16-token tile"
        bound, peak = "mfma", PEAK_BF16_MFMA_TFLOPS
        if dtype != "bf16":
            # fp32 activations take the any-shape vector-ALU kernels, which execute q plane products (2 q T N K lane
            # operations for 2 T N K effective flops): priced against the fp32 vector peak of the chip
            bound, peak, main_kernel = "alu", PEAK_FP32_VECTOR_TFLOPS, "%s_generic_kernel" % dom
        roofline = {"bound": bound, "kernel": main_kernel, "op": "bcq_linear_" + dom, "achieved": round(achieved, 3),
                    "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 5),
                    "traffic": PMC_TRAFFIC_BYTES.get((args.config, T, q, dom)) if not args.g else None,
                    "avg_launch_us": round(ms * 1e3 / len(events), 2), "launches": len(events),
                    "algorithmic": "2*T*N*K flops per launch, averaged over the %d layer shapes" % len(layers)}
        if roofline_note:
            roofline["note"] = roofline_note

    if small:
        # streaming regime: the planes are the only large operand; algorithmic bytes of one step
        sz = 2 if dtype == "bf16" else 4
        bytes_step = 0.0
        for L in layers:
            planes_b = q * L["N"] * L["K"] / 8
            bytes_step += 3 * planes_b + 2 * 4 * q * L["N"] + 2 * sz * T * (L["K"] + L["N"]) + sz * T * (L["K"] + L["N"])
        achieved = bytes_step / (ms_per_step * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "stream_kernel / stream_lds_kernel / stream_fused_kernel + quant_act_kernel (fwd, dalpha, dx; whole captured step)",
                    "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 5),
                    "traffic": (PMC_TRAFFIC_STREAM_LAYER.get((custom, T, q), 0.0) * replicas or None) if not args.g else None,
                    "packed_plane_GBps": round(3 * sum(q * L["N"] * L["K"] / 8 for L in layers) / (ms_per_step * 1e-3) / 1e9, 1),
                    "algorithmic": "per op and layer: q*N*K/8 plane bytes + 4*q*N + activations; planes are read once "
                                   "by each of fwd, dx, dalpha"}

    # ---------------- context (not a target, not part of the library): what a plain copy and plain bf16 GEMMs of
    # the same shapes reach on this GPU in this run
    context = None
    if not args.no_context and not small and dtype == "bf16":
        def timed(fn, n=10):
            fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / n
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        copy_ms = timed(lambda: dst.copy_(src))
        del src, dst
        gemm_ms = 0.0
        for L in layers[:len(kinds)]:
            Wd = torch.randn((L["N"], L["K"]), dtype=tdtype, device="cuda")
            gemm_ms += timed(lambda: torch.matmul(L["x"], Wd.t()))          # y  = x  W^T
            gemm_ms += timed(lambda: torch.matmul(L["dy"], Wd))             # dx = dy W
            gemm_ms += timed(lambda: torch.matmul(L["dy"].t(), L["x"]))     # dW-shaped product behind dalpha
            del Wd
        context = {"d2d_copy_GBps": round(2 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1),
                   "vendor_bf16_gemm_tflops": round(flops_step / replicas / (gemm_ms * 1e-3) / 1e12, 1),
                   "vendor_bf16_gemm_ms_per_step": round(gemm_ms, 4),
                   "note": "torch.matmul on dense bf16 weights of the same shapes (3 GEMMs per layer), events around "
                           "10 back-to-back calls each; read+write bytes for the 1 GiB copy"}

    # ---------------- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import bcq_oracle as oracle
        budget_s, spent, flops_done, done = 12.0, 0.0, 0.0, []
        for kind in sorted(kinds, key=lambda k: shape_of(k)[0] * shape_of(k)[1]):
            if spent > budget_s:
                break
            N, K = shape_of(kind)
            W = synth.weights(args.config, kind, N, K, outliers=cfg["outliers"])
            gl = min(args.g, K) if args.g else K
            a_ref, planes_ref = oracle.quantize(W, q, g=gl)
            Ts = min(T, 4096)
            xs = synth.activations(args.config, kind, T, K, 1, dtype)[:Ts]
            dys = synth.activations(args.config, kind, T, N, 2, dtype)[:Ts]
            c0 = time.perf_counter()
            oracle.fwd(a_ref, planes_ref, xs)
            oracle.bwd_input(a_ref, planes_ref, dys)
            oracle.bwd_alpha(planes_ref, xs, dys, g=gl)
            spent += time.perf_counter() - c0
            flops_done += 6.0 * Ts * N * K
            done.append("%s %dx%d x %d tokens" % (kind, N, K, Ts))
        cpu = {"value": round(flops_done / spent / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": round(spent, 2),
               "sample": "fwd+dx+dalpha, q=%d, fp64 naive loops, layers: %s" % (q, "; ".join(done))}

    out = {
        "metric": "BCQ linear fwd+bwd effective TFLOP/s",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(spread[len(spread) // 2], 4),
        "ms_per_step_min": round(spread[0], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype,
        "data": "synthetic",
        "config": {"workload": "config %d: %s-wide block layers %s, q=%d, %s scales, %s activations, T=%d tokens; "
                               "fwd+dx+dalpha" % (args.config, h, ("one %dx%d layer" % custom) if custom else "/".join(kinds), q,
                                                  ("g=%d group-wise" % args.g) if args.g else "row-wise", dtype, T),
                   "h": h, "q": q, "tokens": T, "g": args.g or "h_in", "weights_per_block": weights_total // replicas,
                   "layer_stack_replicas": replicas, "hip_graph": graph is not None,
                   "streams": 2 if side is not None else 1,
                   "order": ("training step: all forwards, then from the last layer back dx on the main stream and "
                             "dalpha on the second stream, one join") if side is not None else "fwd, dx, dalpha per layer"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "context": context,
        "per_op": per_op,
        "setup": {k: round(v, 4) for k, v in setup_ms.items()},
        "packed_weight_bytes": q * weights_total // 8,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
