#!/usr/bin/env python3
"""Benchmark of the BCQ linear hot path on one MI355X.

One step = forward, input gradient and alpha gradient of every layer of the workload.  The quantizer, pack,
transposed-twin and decode-layout passes run once before the timed regions (they are the one-time PTQ of the method)
and are timed separately in "setup".

The default run prints ONE JSON line:
  * headline (`value`, `config`, `roofline`): the largest large-token workload, number 4 of the benchmark definition:
    the four linear layers of an OPT-1.3B-shaped block (d = 2048, MLP 8192), q = 3, 0.1 % outlier rows, bf16
    activations, T = 8 x 2048 = 16384 tokens, full fwd + dx + dalpha.  `--steps` steps are timed exactly.
  * `regimes`: the other regimes the targets are stated on, each with ms_per_step, effective TFLOP/s, packed-weight
    GB/s and its own roofline object: workload 2 (GPT-2-medium block, T = 4096), workload 5 at 4096 tokens, and the
    small-token stacks (>= 512 MB of distinct packed planes, the batched entry points: one launch pair per operation
    for the whole stack) of workload 5 at 1, 8 and 16 tokens and workload 3 (q = 1 at 1 token, q = 4 at 8 tokens).
  * `cpu_baseline`: the CPU oracle timed on a bounded sample of the headline workload.
A single regime can be run alone with --config / --tokens / --q (and --regimes none).

Roofline figures: `achieved` is the algorithmic work of a kernel family (gemm_kernel = forward + input gradient calls,
dalpha_kernel = scale gradient calls; the one with the largest share of the step, the slowest operation beside it; each
C-ABI call with all its kernels) divided by its HIP-event time; for the large-token regimes the events bracket the calls in the eagerly launched one-stream
warm-up steps of the same run (the timed region replays a HIP graph over two streams, inside which no event can be
recorded); for the small-token stacks they bracket the batched calls themselves.  `traffic` is not measured live: it
is read from the table in profiles/hbm_traffic.md (rocprofv3 --pmc runs of this file's commands) and labelled so.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak
PEAK_FP32_VECTOR_TFLOPS = 157.3  # 256 compute units x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="headline workload number (4 = OPT-1.3B-shaped block, T = 16384)")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count of the workload")
    ap.add_argument("--q", type=int, default=0, help="override the number of bit planes")
    ap.add_argument("--g", type=int, default=0,
                    help="group size of the scales along K (Table 4); 0 = row-wise (g = h_in); a layer with K < g uses g = K")
    ap.add_argument("--layer", type=str, default="",
                    help="time ONE layer of shape NxK (e.g. 16384x16384) instead of the workload's four layer shapes; "
                         "seeds, dtype and q still come from --config")
    ap.add_argument("--regimes", type=str, default="all",
                    help="'all' (default), 'none', or a comma-separated list of regime names (see REGIMES)")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the two context measurements (device-to-device copy, plain bf16 GEMMs of the same "
                         "shapes through the vendor BLAS that PyTorch links)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="skip the per-op HIP events (pure step timing)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the whole step on one stream.  By default (32 tokens and more) a step is ordered like a "
                         "training step (all forwards, then the backward pass from the last layer) and the scale gradients "
                         "run on a second HIP stream of default priority beside the input gradients, joined at the end "
                         "of the step: in training dalpha is a leaf of the backward pass (Eq. 4), only the optimizer waits "
                         "for it")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every timed step from Python instead of replaying one captured HIP graph")
    ap.add_argument("--layer-by-layer", action="store_true",
                    help="small-token stacks: also time the same stack through the single-layer entry points (one call "
                         "per layer and operation, captured in one HIP graph)")
    ap.add_argument("--replicas", type=int, default=0,
                    help="small-token stacks: independent copies of the block (own weights); default: enough for 512 MB "
                         "of packed planes, beyond the 256 MB Infinity Cache")
    ap.add_argument("--setup-ops", type=int, default=-1,
                    help="workload whose two MLP shapes the set-up kernels (quantize, pack, unpack, transposed twin, "
                         "decode layout) are timed on, each alone; default: workload 5 in the default run, else none")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


# regimes of the default run besides the headline: name -> (kind, config, tokens, q)
REGIMES = {
    "config2_T4096": ("large", 2, 4096, 4),
    "config5_T4096": ("large", 5, 4096, 4),
    "config5_T8_stack": ("stack", 5, 8, 4),
    "config5_T1_stack": ("stack", 5, 1, 4),
    "config5_T16_stack": ("stack", 5, 16, 4),
    "config3_q1_T1_stack": ("stack", 3, 1, 1),
    "config3_q4_T8_stack": ("stack", 3, 8, 4),
}


def traffic_from_profile(key):
    """Bytes per launch from the committed table (lines `| key | fetched bytes | written bytes | ... |`), or None."""
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 3 and cells[0] == key:
                return float(cells[1]) + float(cells[2])
    except (OSError, ValueError):
        pass
    return None


def timed_events(torch, fn, n):
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


# ------------------------------------------------------------------------------------------------------------------
# large-token regime: the four layers of one block through the single-layer entry points

def run_large(args, env, config, T, q, steps, warmup, custom=None, context=True, headline=False):
    np, torch, bcq, synth = env
    cfg = synth.CONFIGS[config]
    h = cfg["h"]
    dtype = cfg["dtype"]
    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = bcq.binding.BCQ_BF16 if dtype == "bf16" else bcq.binding.BCQ_F32
    kinds = ("out",) if custom else cfg["kinds"]
    use_graph = not args.no_graph

    def shape_of(kind):
        return custom if custom else synth.layer_shape(h, kind)

    gen = torch.Generator(device="cuda")
    layers = []
    setup = {"quantize_ms": 0.0, "pack_transposed_ms": 0.0, "quantize_bytes": 0, "pack_transposed_bytes": 0}
    weights_total = 0
    for kind in kinds:
        N, K = shape_of(kind)
        W = torch.from_numpy(synth.weights(config, kind, N, K, outliers=cfg["outliers"])).cuda()
        g = min(args.g, K) if args.g else K
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        bcq.bcq_quantize_grouped(W, q, g)  # warm
        e0.record()
        alpha, packed, _ = bcq.bcq_quantize_grouped(W, q, g)
        e1.record()
        twin = bcq.bcq_pack_transposed(packed) if N % 32 == 0 else None
        e2.record()
        torch.cuda.synchronize()
        setup["quantize_ms"] += e0.elapsed_time(e1)
        setup["pack_transposed_ms"] += e1.elapsed_time(e2)
        setup["quantize_bytes"] += 4 * N * K + q * N * K // 8 + 4 * q * N * (K // g)   # W read once, planes + alpha written
        setup["pack_transposed_bytes"] += 2 * (q * N * K // 8) if twin is not None else 0
        weights_total += N * K
        # activations: seeded, drawn on the GPU (N(0,1) rounded to bf16); the CPU baseline below copies its sample back
        gen.manual_seed(synth.seed_for(config, kind, 1))
        x = torch.randn((T, K), generator=gen, device="cuda", dtype=torch.float32).to(tdtype)
        gen.manual_seed(synth.seed_for(config, kind, 2))
        dy = torch.randn((T, N), generator=gen, device="cuda", dtype=torch.float32).to(tdtype)
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

    side = torch.cuda.Stream() if not args.no_overlap else None

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

    def step(events=None):
        """One pass of the hot path.  With `events`, HIP events bracket every call (one stream, eager)."""
        if side is not None and events is None:
            return step_overlapped()
        for L in layers:
            for op in ops:
                if events is not None:
                    a = torch.cuda.Event(enable_timing=True)
                    b = torch.cuda.Event(enable_timing=True)
                    a.record()
                    run_op(L, op)
                    b.record()
                    events.append((op, L["kind"], a, b))
                else:
                    run_op(L, op)

    # warm-up: every call bracketed by events -> per-op table and the roofline of the dominant op family
    warm_events = []
    n_warm = max(warmup, 2)  # at least two: the per-op figures skip the first step (one-time set-up of the kernels)
    for _ in range(n_warm):
        step(None if args.no_events else warm_events)
    torch.cuda.synchronize()
    graph = None
    if use_graph:  # the library neither allocates nor memsets, so a step can be captured as it is
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()

    # timed region: exactly `steps` steps
    t0 = time.perf_counter()
    for _ in range(steps):
        if graph is not None:
            graph.replay()
        else:
            step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    # spread of single steps (not part of `value`): up to 20 more steps, each bracketed by HIP events
    spread = []
    for _ in range(min(steps, 20)):
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
    packed_bytes = q * weights_total // 8

    per_op, roofline = None, None
    if warm_events:
        n_ev = len(ops) * len(layers)
        fam_steps = {op: [] for op in ops}
        for i in range(1, n_warm):
            sums = dict.fromkeys(ops, 0.0)
            for op, kind, a, b in warm_events[i * n_ev:(i + 1) * n_ev]:
                sums[op] += a.elapsed_time(b)
            for op in ops:
                fam_steps[op].append(sums[op])
        fam_ms = {op: sorted(v)[(len(v) - 1) // 2] for op, v in fam_steps.items()}  # lower median
        fam_flops = sum(flops_layer.values())  # every family runs every layer once per step
        per_op = {op: {"ms_per_step": round(fam_ms[op], 4), "tflops": round(fam_flops / (fam_ms[op] * 1e-3) / 1e12, 3),
                       "frac_of_peak": round(fam_flops / (fam_ms[op] * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)}
                  for op in ops}
        # Kernel families of a step: gemm_kernel serves the forward and the input gradient (two calls per layer, each with
        # its short expand kernel), dalpha_kernel the scale gradient (one call per layer, with its transpose and reduce
        # kernels).  `roofline` is the family with the largest share of the step's time; the slowest single operation
        # family is reported beside it.
        kern = {"gemm": ("fwd", "bwd_input"), "dalpha": ("bwd_alpha",)}
        kern_ms = {k: sum(fam_ms[o] for o in v) for k, v in kern.items()}
        domk = max(kern_ms, key=lambda k: kern_ms[k])
        slow = max(fam_ms, key=lambda k: fam_ms[k])
        names = {"gemm": "gemm_kernel (+ expand_fwd_kernel / expand_bwd_kernel)",
                 "dalpha": "dalpha_kernel (+ transpose_frag_kernel, dalpha_reduce_kernel)"}
        bound, peak = "mfma", PEAK_BF16_MFMA_TFLOPS
        if dtype != "bf16":
            # fp32 activations take the any-shape vector-ALU kernels, which execute q plane products (2 q T N K lane
            # operations for 2 T N K effective flops): priced against the fp32 vector peak of the chip
            bound, peak = "alu", PEAK_FP32_VECTOR_TFLOPS
            names = {"gemm": "fwd_generic_kernel, bwd_input_generic_kernel", "dalpha": "bwd_alpha_generic_kernel"}
        calls = len(kern[domk]) * len(layers)
        achieved = len(kern[domk]) * fam_flops / (kern_ms[domk] * 1e-3) / 1e12
        traffic, tkeys = None, ["config%d_T%d_q%d_%s" % (config, T, q, o) for o in kern[domk]]
        if not (args.g or custom):
            rows = [traffic_from_profile(k) for k in tkeys]
            traffic = sum(rows) / len(rows) if all(r is not None for r in rows) else None
        slow_achieved = fam_flops / (fam_ms[slow] * 1e-3) / 1e12
        roofline = {"bound": bound, "kernel": names[domk], "op": " + ".join("bcq_linear_" + o for o in kern[domk]),
                    "time_share": round(kern_ms[domk] / sum(kern_ms.values()), 4),
                    "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 5),
                    "traffic": traffic,
                    "traffic_source": ("profiles/hbm_traffic.md rows %s (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE per call, "
                                       "copy-scaled; not measured in this run)" % ", ".join(tkeys)) if traffic else None,
                    "avg_launch_us": round(kern_ms[domk] * 1e3 / calls, 2), "launches_per_step": calls,
                    "algorithmic": "2*T*N*K flops per call, averaged over the %d layer shapes; the family's helper "
                                   "kernels are inside the event time" % len(layers),
                    "slowest_family": {"op": "bcq_linear_" + slow, "achieved": round(slow_achieved, 3),
                                       "frac": round(slow_achieved / peak, 5),
                                       "avg_launch_us": round(fam_ms[slow] * 1e3 / len(layers), 2)},
                    "note": "HIP events around each call in the %d eagerly launched one-stream warm-up steps of this run "
                            "(the family with the largest time share; the slowest operation family beside it); per-kernel "
                            "durations and matrix-core counters: profiles/large_token_kernel_stats.md, "
                            "profiles/large_token_mfma_counters.md" % (n_warm - 1)}

    ctx = None
    if context and not args.no_context and dtype == "bf16":
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        copy_ms = timed_events(torch, lambda: dst.copy_(src), 5)
        del src, dst
        gemm_ms = 0.0
        for L in layers:
            Wd = torch.randn((L["N"], L["K"]), dtype=tdtype, device="cuda")
            for fn in (lambda: torch.matmul(L["x"], Wd.t()), lambda: torch.matmul(L["dy"], Wd),
                       lambda: torch.matmul(L["dy"].t(), L["x"])):  # y = x W^T, dx = dy W, dW-shaped product behind dalpha
                fn()
                gemm_ms += timed_events(torch, fn, 5)
            del Wd
        ctx = {"d2d_copy_GBps": round(2 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1),
               "vendor_bf16_gemm_tflops": round(flops_step / (gemm_ms * 1e-3) / 1e12, 1),
               "vendor_bf16_gemm_ms_per_step": round(gemm_ms, 4),
               "note": "torch.matmul on dense bf16 weights of the same shapes (3 GEMMs per layer), events around "
                       "5 back-to-back calls each; read+write bytes for the 1 GiB copy"}

    res = {
        "workload": "config %d: %s-wide block layers %s, q=%d, %s scales, %s activations, T=%d tokens; fwd+dx+dalpha" % (
            config, h, ("one %dx%d layer" % custom) if custom else "/".join(kinds), q,
            ("g=%d group-wise" % args.g) if args.g else "row-wise", dtype, T),
        "h": h, "q": q, "tokens": T, "g": args.g or "h_in", "weights_per_block": weights_total,
        "hip_graph": graph is not None, "streams": 2 if side is not None else 1,
        "order": ("training step: all forwards, then from the last layer back dx on the main stream and dalpha on the "
                  "second stream, one join") if side is not None else "fwd, dx, dalpha per layer",
        "steps": steps, "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(spread[len(spread) // 2], 4),
        "ms_per_step_min": round(spread[0], 4), "tflops": round(value, 3),
        "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_MFMA_TFLOPS, 4),
        "packed_weight_bytes": packed_bytes,
        "packed_weight_GBps": round(3 * packed_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "roofline": roofline, "per_op": per_op, "context": ctx,
        "setup": {"quantize_ms": round(setup["quantize_ms"], 4),
                  "quantize_GBps": round(setup["quantize_bytes"] / (setup["quantize_ms"] * 1e-3) / 1e9, 1),
                  "pack_transposed_ms": round(setup["pack_transposed_ms"], 4),
                  "pack_transposed_GBps": round(setup["pack_transposed_bytes"] / max(setup["pack_transposed_ms"], 1e-6) / 1e6, 1),
                  "algorithmic": "quantize: 4NK read + qNK/8 + 4qN written; twin: qNK/8 read + written"},
    }
    return res, layers


# ------------------------------------------------------------------------------------------------------------------
# set-up operations (quantizer, Appendix C Eq. ap1-ap3; layouts of the planes): each kernel alone, on the two MLP shapes

def run_setup_ops(env, config, q, iters=10):
    np, torch, bcq, synth = env
    cfg = synth.CONFIGS[config]
    out = {}
    gen = torch.Generator(device="cuda")
    for kind in ("mlp_up", "mlp_down"):
        N, K = synth.layer_shape(cfg["h"], kind)
        gen.manual_seed(synth.seed_for(config, kind, 0))
        W = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
        alpha, packed, planes = bcq.bcq_quantize(W, q, want_planes=True)
        twin = bcq.bcq_pack_transposed(packed)
        tiled = bcq.bcq_pack_decode(packed)
        a2, p2 = torch.empty_like(alpha), torch.empty_like(packed)
        pb = q * N * K // 8
        ops = {
            # W read once; planes and scales written
            "quantize": (lambda: bcq.bcq_quantize(W, q, alpha=a2, packed=p2), 4 * N * K + pb + 4 * q * N),
            # one int8 per sign read, one bit written
            "pack": (lambda: bcq.bcq_pack(planes, packed=p2), q * N * K + pb),
            "unpack": (lambda: bcq.bcq_unpack(packed, planes_i8=planes), q * N * K + pb),
            "pack_transposed": (lambda: bcq.bcq_pack_transposed(packed, packed_t=twin), 2 * pb),
            "pack_decode": (lambda: bcq.bcq_pack_decode(packed, tiled=tiled), pb + tiled.numel() * tiled.element_size()),
        }
        r = {}
        for name, (fn, nbytes) in ops.items():
            fn()
            torch.cuda.synchronize()
            # one captured graph of `iters` calls: a call from Python costs more than these 10-30 us kernels run
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(iters):
                    fn()
            graph.replay()
            ms = timed_events(torch, graph.replay, 3) / iters
            del graph
            r[name] = {"us": round(ms * 1e3, 2), "algorithmic_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                       "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        out["%s_%dx%d_q%d" % (kind, N, K, q)] = r
        del W, alpha, packed, planes, twin, tiled, a2, p2
        torch.cuda.empty_cache()
    out["algorithmic"] = ("quantize 4NK + qNK/8 + 4qN; pack/unpack qNK + qNK/8; transposed twin 2*qNK/8; decode layout "
                          "qNK/8 read + the padded tiled size written; events around 3 replays of a HIP graph of %d calls" % iters)
    return out


# ------------------------------------------------------------------------------------------------------------------
# small-token regime: a stack of distinct layers through the batched entry points

def run_stack(args, env, config, T, q, custom=None, iters=20):
    np, torch, bcq, synth = env
    cfg = synth.CONFIGS[config]
    h = cfg["h"]
    kinds = ("out",) if custom else cfg["kinds"]
    shapes = [custom if custom else synth.layer_shape(h, k) for k in kinds]
    block_packed = sum(n * k for n, k in shapes) * q // 8
    replicas = args.replicas or max(1, -(-(512 << 20) // block_packed))
    gen = torch.Generator(device="cuda")
    layers = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for rep in range(replicas):
        for kind, (N, K) in zip(kinds, shapes):
            # weights: seeded N(0, 0.02^2) drawn on the GPU (a 512 MB stack at q = 1 is 4.3 G weights), quantized by
            # the library's greedy quantizer; only the packed planes are kept
            gen.manual_seed(synth.seed_for(config, kind, 0, rep))
            W = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
            alpha, packed, _ = bcq.bcq_quantize(W, q)
            del W
            twin = bcq.bcq_pack_transposed(packed)
            gen.manual_seed(synth.seed_for(config, kind, 1, rep))
            x = torch.randn((T, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            gen.manual_seed(synth.seed_for(config, kind, 2, rep))
            dy = torch.randn((T, N), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            L = dict(kind=kind, N=N, K=K, alpha=alpha, x=x, dy=dy, tiled=bcq.bcq_pack_decode(packed),
                     tiled_t=bcq.bcq_pack_decode(twin),
                     y=torch.empty((T, N), dtype=torch.bfloat16, device="cuda"),
                     dx=torch.empty((T, K), dtype=torch.bfloat16, device="cuda"),
                     dalpha=torch.empty((q, N), dtype=torch.float32, device="cuda"))
            if args.layer_by_layer:
                L["packed"], L["twin"] = packed, twin
            elif T == 1:  # the table look-up variant of the forward is timed beside the batched one
                L["packed"] = packed
            layers.append(L)
            del packed, twin
    e1.record()
    torch.cuda.synchronize()
    setup_ms = e0.elapsed_time(e1)

    names = {1: "fwd", 2: "bwd_input", 3: "bwd_alpha"}
    plans = {op: bcq.batch_plan(op, layers, T, q) for op in (1, 2, 3)}
    for _ in range(3):
        for op in (1, 2, 3):
            bcq.bcq_linear_batched(plans[op])
    torch.cuda.synchronize()
    op_ms = {names[op]: timed_events(torch, lambda: bcq.bcq_linear_batched(plans[op]), iters) for op in (1, 2, 3)}

    def step():
        for op in (1, 2, 3):
            bcq.bcq_linear_batched(plans[op])
    t0 = time.perf_counter()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / iters

    planes = sum(q * L["N"] * L["K"] // 8 for L in layers)
    # algorithmic bytes of one operation over the stack: planes + scales or their gradient + the two activations
    other = {"fwd": sum(4 * q * L["N"] + 2 * T * (L["K"] + L["N"]) for L in layers),
             "bwd_input": sum(4 * q * L["N"] + 2 * T * (L["K"] + L["N"]) for L in layers),
             "bwd_alpha": sum(4 * q * L["N"] + 2 * T * (L["K"] + L["N"]) for L in layers)}
    per_op = {}
    for name, ms in op_ms.items():
        tot = planes + other[name]
        per_op[name] = {"ms": round(ms, 4), "packed_weight_GBps": round(planes / (ms * 1e-3) / 1e9, 1),
                        "total_GBps": round(tot / (ms * 1e-3) / 1e9, 1),
                        "frac_of_hbm_peak": round(tot / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    dom = max(op_ms, key=lambda k: op_ms[k])
    tot_dom = planes + other[dom]
    tkey = "config%d_T%d_q%d_stack_%s" % (config, T, q, dom)
    traffic = traffic_from_profile(tkey) if not custom else None
    roofline = {"bound": "hbm", "kernel": "stream_tile_batched_kernel (+ quant_act_batched_kernel)",
                "op": "bcq_linear_batched " + dom, "achieved": round(tot_dom / (op_ms[dom] * 1e-3) / 1e9, 1),
                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(tot_dom / (op_ms[dom] * 1e-3) / 1e9 / PEAK_HBM_GBS, 5),
                "traffic": traffic,
                "traffic_source": ("profiles/hbm_traffic.md row %s (not measured in this run)" % tkey) if traffic else None,
                "avg_launch_us": round(op_ms[dom] * 1e3, 2), "launches_per_step": 1,
                "algorithmic": "per call over the stack: q*N*K/8 plane bytes + 4*q*N + 2*T*(K+N) per layer",
                "note": "HIP events around %d back-to-back batched calls of the slowest operation (pre-kernel + main "
                        "kernel); the planes are read once by each of fwd, dx, dalpha; per-kernel durations: "
                        "profiles/small_token_stack_kernel_stats.md" % iters}
    flops_step = 6.0 * T * sum(L["N"] * L["K"] for L in layers)
    res = {
        "workload": "config %d: stack of %d x (%s) layers of width %d (%d layers, %.1f MB of packed planes), q=%d, row-wise "
                    "scales, bf16 activations, T=%d tokens; fwd+dx+dalpha through the batched entry points (one launch pair "
                    "per operation)" % (config, replicas, ("%dx%d" % custom) if custom else "/".join(kinds), h, len(layers),
                                        planes / 1e6, q, T),
        "h": h, "q": q, "tokens": T, "layers": len(layers), "layer_stack_replicas": replicas,
        "ms_per_step": round(ms_per_step, 4), "tflops": round(flops_step / (ms_per_step * 1e-3) / 1e12, 3),
        "packed_weight_bytes": planes,
        "packed_weight_GBps": round(3 * planes / (ms_per_step * 1e-3) / 1e9, 1),
        "frac_of_hbm_peak": round(3 * planes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "roofline": roofline, "per_op": per_op,
        "setup": {"stack_ms": round(setup_ms, 2), "note": "random weights, greedy quantizer, twin and two decode layouts "
                                                           "per layer, launched from Python"},
    }
    if T == 1 and all("packed" in L and 8 * L["K"] <= 128 * 1024 for L in layers):
        # Section 6 "Inference Speed": forward by table look-up, one call per layer, the stack captured in one HIP graph
        def lut():
            for L in layers:
                bcq.bcq_linear_fwd_lut(L["packed"], L["alpha"], L["x"], y=L["y"])
        lut()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lut()
        graph.replay()
        ms = timed_events(torch, graph.replay, 5)
        del graph
        res["lut_forward"] = {"ms": round(ms, 4), "packed_weight_GBps": round(planes / (ms * 1e-3) / 1e9, 1),
                              "frac_of_hbm_peak": round((planes + other["fwd"]) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                              "note": "bcq_linear_fwd_lut per layer (lut_fwd_kernel), %d calls in one HIP graph; compare "
                                      "per_op.fwd (one batched call on the FP4 x FP8 matrix instruction)" % len(layers)}
    if args.layer_by_layer:
        ws = {}
        for L in layers:
            L["ws"] = {op: torch.empty((max(bcq.workspace_bytes(op, T, L["N"], L["K"], q, 1), 16),), dtype=torch.uint8,
                                       device="cuda") for op in (1, 2, 3)}

        def lbl():
            for L in layers:
                bcq.bcq_linear_fwd(L["packed"], L["alpha"], L["x"], y=L["y"], workspace=L["ws"][1])
                bcq.bcq_linear_bwd_input(L["packed"], L["alpha"], L["dy"], packed_t=L["twin"], dx=L["dx"], workspace=L["ws"][2])
                bcq.bcq_linear_bwd_alpha(L["packed"], L["x"], L["dy"], dalpha=L["dalpha"], workspace=L["ws"][3])
        lbl()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lbl()
        graph.replay()
        ms = timed_events(torch, graph.replay, 10)
        res["layer_by_layer"] = {"ms_per_step": round(ms, 4), "packed_weight_GBps": round(3 * planes / (ms * 1e-3) / 1e9, 1),
                                 "note": "single-layer entry points, %d calls in one HIP graph" % (3 * len(layers))}
    del plans, layers
    torch.cuda.empty_cache()
    return res


def cpu_baseline(env, config, T, q, layers, g_arg):
    """The oracle as it stands on a bounded token slice of the same layers and activations."""
    np, torch, bcq, synth = env
    from oracle import bcq_oracle as oracle
    cfg = synth.CONFIGS[config]
    total_nk = sum(L["N"] * L["K"] for L in layers)
    Ts = T
    while Ts > 1 and 6.0 * Ts * total_nk > 1.6e11:  # about 10 - 15 s of naive fp64 loops on 16 cores
        Ts //= 2
    spent, flops_done, done = 0.0, 0.0, []
    for L in layers:
        N, K = L["N"], L["K"]
        W = synth.weights(config, L["kind"], N, K, outliers=cfg["outliers"])
        gl = min(g_arg, K) if g_arg else K
        a_ref, planes_ref = oracle.quantize(W, q, g=gl)
        xs = L["x"][:Ts].float().cpu().numpy()
        dys = L["dy"][:Ts].float().cpu().numpy()
        c0 = time.perf_counter()
        oracle.fwd(a_ref, planes_ref, xs)
        oracle.bwd_input(a_ref, planes_ref, dys)
        oracle.bwd_alpha(planes_ref, xs, dys, g=gl)
        spent += time.perf_counter() - c0
        flops_done += 6.0 * Ts * N * K
        done.append("%s %dx%d" % (L["kind"], N, K))
    return {"value": round(flops_done / spent / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(spent, 2),
            "sample": "fwd+dx+dalpha on the first %d of the %d tokens, q=%d, fp64 naive loops, all layers: %s" % (
                Ts, T, q, "; ".join(done))}


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
    env = (np, torch, bcq, synth)

    cfg = synth.CONFIGS[args.config]
    q = args.q or cfg["q"][-1]
    T = args.tokens or cfg["tokens"][-1]
    custom = None
    if args.layer:
        custom = tuple(int(v) for v in args.layer.lower().split("x"))
        assert len(custom) == 2 and custom[1] % 32 == 0, "--layer wants NxK with K % 32 == 0"

    if args.calibrate_copy:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    small = T <= 16 and cfg["dtype"] == "bf16" and not args.g
    cpu = None
    if small:
        head = run_stack(args, env, args.config, T, q, custom=custom, iters=max(args.steps, 1))
        value, unit, metric = head["packed_weight_GBps"], "GB/s", "BCQ linear fwd+bwd packed-weight GB/s"
    else:
        head, layers = run_large(args, env, args.config, T, q, args.steps, args.warmup, custom=custom, headline=True)
        value, unit, metric = head["tflops"], "TFLOP/s", "BCQ linear fwd+bwd effective TFLOP/s"
        if not args.no_cpu_baseline:
            cpu = cpu_baseline(env, args.config, T, q, layers, args.g)
        del layers
        torch.cuda.empty_cache()

    regimes = {}
    wanted = [] if args.regimes == "none" else (list(REGIMES) if args.regimes == "all" else args.regimes.split(","))
    if args.regimes == "all" and (args.tokens or args.q or args.g or args.layer or args.config != 4):
        wanted = []  # a single regime was asked for
    for name in wanted:
        kind, c, t, qq = REGIMES[name]
        if kind == "large":
            if (c, t, qq) == (args.config, T, q):
                continue
            r, _ = run_large(args, env, c, t, qq, min(args.steps, 20), min(max(args.warmup, 3), 5), context=True)
            del _
        else:
            r = run_stack(args, env, c, t, qq)
        torch.cuda.empty_cache()
        regimes[name] = r

    setup_ops = None
    so = args.setup_ops if args.setup_ops >= 0 else (5 if wanted and args.regimes == "all" else 0)
    if so:
        setup_ops = run_setup_ops(env, so, synth.CONFIGS[so]["q"][-1])

    out = {
        "metric": metric,
        "value": value,
        "unit": unit,
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg["dtype"],
        "data": "synthetic",
        "config": {k: head[k] for k in head if k not in ("roofline", "per_op", "context", "setup", "ms_per_step", "tflops")},
        "packed_weight_GBps": head["packed_weight_GBps"],
        "roofline": head["roofline"],
        "cpu_baseline": cpu,
        "context": head.get("context"),
        "per_op": head["per_op"],
        "setup": head["setup"],
        "setup_ops": setup_ops,
        "regimes": regimes,
        "targets": {"large_token": ">= 0.50 of the bf16 MFMA peak at >= 2048 tokens", "small_token": ">= 0.70 of the HBM peak "
                    "at <= 8 tokens", "status": "both open: see roofline.frac of the headline and of the regimes"},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
