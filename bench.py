#!/usr/bin/env python3
"""Benchmark of the XNOR-Net binary convolution forward pass on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic input that already
lives in HBM: binarise+pack the input and its scaling map K (one pass over I), binarise+pack the
filters and their alpha (one pass over Wt; for the matrix-core kernel also their expansion into its
operand order), XNOR convolution with the K*alpha epilogue.  With
--unfused the four pre-stage calls run separately (pack_I, scale_K, alpha, pack_W).  Prints ONE JSON line: whole-step throughput in binary
GMAC/s, the convolution kernel's roofline figures (timed live with events on the launch stream)
and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer c5] [--algo auto]

The timing protocol is the paper's (Sec. IV: compute only, the mean over repeated runs), with buffers
allocated and filled before the timed region and reused every step.  Defaults: 1000 warm-up and 1000
timed steps (a third of a second of GPU time): in a process that has just started, the first one to
two hundred steps run about 10 % slower than the rate the chip then holds (with 10 warm-up and 100
timed steps the c5 step measures 165-168 us instead of 151 us).
Other modes: --sweep (all layers, both kernels, with HIP-graph replay times), --chain (chained
layer), --image (the paper's single-channel workload, Tables I-III), --bwn (Binary-Weight-Network
layer), --unfused (separate pre-stage calls), --peaks (the ceilings this GPU sustains), --vanilla (the real-valued convolution beside the XNOR one).
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

# MI355X published peaks used as roofline denominators.
PEAK_FP4_MFMA_TFLOPS = 10100.0      # dense FP4 MFMA, 2 flops per multiply-accumulate
PEAK_HBM_GBS = 8000.0
# v_xor_b32 + v_bcnt_u32_b32 retire 32 binary MACs per lane: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz
# = 3.93e13 lane-ops/s -> 6.29e14 binary MAC/s -> 1258 T binary op/s counting 2 ops per MAC.
PEAK_VALU_POPCOUNT_TOPS = 256 * 4 * 16 * 2.4e9 / 2 * 32 * 2 / 1e12
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "forward_c5_hbm_traffic_pmc.md")
CONV_SOURCES = ("conv_mfma_persistent.hip", "conv_mfma.hip", "conv_mfma_common.hpp")


def conv_source_digest() -> str:
    """Fingerprint of the matrix-core convolution's sources: a counter reading belongs to the kernel
    it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in CONV_SOURCES:
        with open(os.path.join(ROOT, "paper_2007_14178_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_conv_traffic(layer_name: str, algo_name: str):
    """HBM bytes per convolution launch from the tracked rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, each scaled by a plain copy of known size).  The summary carries one line
    `traffic: layer=<l> algo=<a> fetch_bytes=<n> write_bytes=<n> commit=<hash> conv_sources=<digest>`
    per measured kernel; a reading taken on other kernel sources than the ones at hand is not
    reported (None), and neither is a missing one."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            lines = [ln.strip() for ln in f if ln.strip().startswith("traffic:")]
    except OSError:
        return None, None
    for ln in lines:
        kv = dict(item.split("=", 1) for item in ln.split()[1:] if "=" in item)
        if kv.get("layer") == layer_name and kv.get("algo") == algo_name:
            if kv.get("conv_sources") != conv_source_digest():
                return None, f"stale: measured at commit {kv.get('commit')} on other kernel sources"
            return float(kv["fetch_bytes"]) + float(kv["write_bytes"]), f"measured at commit {kv.get('commit')}"
    return None, None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--layer", default="c5", help="workload name (see paper_2007_14178_amd/workloads.py)")
    ap.add_argument("--algo", default="auto", choices=["auto", "direct", "tiled", "mfma", "split"],
                    help="the convolution kernel (split: --bwn only, the three-term bf16 form)")
    ap.add_argument("--unfused", action="store_true", help="run the four pre-stage calls separately")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-prepare", action="store_true",
                    help="xnor_input_prepare and xnor_filter_prepare as two calls instead of xnor_prepare")
    ap.add_argument("--sweep", action="store_true",
                    help="not the benchmark line: one JSON line per (layer, conv kernel) for all 11 layers, no CPU baseline")
    ap.add_argument("--chain", action="store_true",
                    help="not the benchmark line: time the layer as a chained one (K from a given A, convolution with "
                         "packed-sign + channel-mean output; no fp32 tensor read or written)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 1 GiB device copies before the timed loop (calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run against known traffic)")
    ap.add_argument("--bwn", action="store_true",
                    help="the Binary-Weight-Network layer (Eq. 1: real input, binary weights) on --layer "
                         "(or on every layer with --sweep): filter_prepare + xnor_bwn_conv2d_fwd")
    ap.add_argument("--image", action="store_true",
                    help="the paper's own workload (Tables I-III): one channel, one 3x3 filter, zero padding, "
                         "square images of 256, 512, 1024 and 2048 pixels; one JSON line per size, latency in ms")
    ap.add_argument("--image-sides", default="256,512,1024,2048")
    ap.add_argument("--vanilla", action="store_true",
                    help="not the benchmark line: the real-valued fp32 convolution (Table I's comparison column) on "
                         "--layer beside the XNOR forward pass of the same layer, and on the paper's single-channel "
                         "images (--image-sides); one JSON line each, with the XNOR-vs-float ratio")
    ap.add_argument("--k-in-conv", action="store_true",
                    help="form K inside the convolution kernel from the channel mean (one launch less, a slower "
                         "convolution) instead of with the box-filter launch of the prepare call; by default this is "
                         "done where the layer is one round of the matrix-core kernel's items (there a launch costs "
                         "more than the kernel gains)")
    ap.add_argument("--k-in-prepare", action="store_true", help="form K with the box-filter launch on every layer")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the HIP-graph replay of the step (its time is reported beside the eager one)")
    ap.add_argument("--conv-events-every", type=int, default=-1,
                    help="bracket the convolution launch with events on every n-th timed step only (0: never; "
                         "default: about 250 of the timed steps, evenly spread: on the small layers two event "
                         "records per step cost the host more than the step costs the GPU)")
    ap.add_argument("--peaks", action="store_true",
                    help="not the benchmark line: the ceilings this GPU sustains (register-only FP4 matrix loop, "
                         "bf16 matrix loop, v_xor + v_bcnt loop, plain copies of 64 MiB and 1 GiB) and the cost of replaying "
                         "a HIP graph of one or two tiny kernels, one JSON line")
    ap.add_argument("--print-conv-digest", action="store_true",
                    help="print the fingerprint of the convolution sources (for the traffic line of a counter summary)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def cpu_baseline(layer, Wt, target_s: float, gpu_out=None, gpu_dot=None):
    """The oracle as it stands, on the host cores, on the first images of the same workload.  Its
    results are kept and the GPU's outputs for the same images (`gpu_out`, `gpu_dot`: device
    tensors of the whole batch) are compared with them, element by element: the second value
    returned is {"images", "elements", "dot_mismatches", "worst_rel", "outside_1e-5"}."""
    import numpy as np
    import oracle
    from paper_2007_14178_amd.workloads import make_input

    def run(n):
        I = make_input(layer, n)
        s = oracle.Shape(n, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                         layer.sh, layer.sw, layer.ph, layer.pw)
        t0 = time.perf_counter()
        res = oracle.forward(I, Wt, s)
        return time.perf_counter() - t0, res

    t1, res = run(1)
    n = max(1, min(layer.N, int(target_s / max(t1, 1e-3))))
    t = t1
    if n > 1:
        t, res = run(n)
    macs = layer.binary_macs // layer.N * n
    base = {"value": macs / t / 1e9, "unit": "binary GMAC/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {n} of {layer.N} images of {layer.name}, all {layer.F} filters, whole forward "
                      f"pass (sign conv + K + alpha + rescale), {t:.2f} s"}
    parity = None
    if gpu_out is not None:
        d_ref, _, _, O_ref = res
        got = gpu_out[:n].cpu().numpy().astype(np.float64)
        ref = O_ref.astype(np.float64)
        err = np.abs(got - ref)
        nz = ref != 0
        rel = np.zeros_like(err)
        rel[nz] = err[nz] / np.abs(ref[nz])
        rel[~nz & (got != 0)] = np.inf
        parity = {"images": n, "elements": int(ref.size),
                  "dot_mismatches": int((gpu_dot[:n].cpu().numpy() != d_ref).sum()) if gpu_dot is not None else None,
                  "worst_rel": float(rel.max()), "outside_1e-5": int((rel > 1e-5).sum())}
    return base, parity


def run_layer(args, xb, torch, layer, algo_name, make_input, make_weights):
    algo = {"auto": xb.ALGO_AUTO, "direct": xb.ALGO_DIRECT, "tiled": xb.ALGO_TILED, "mfma": xb.ALGO_MFMA}[algo_name]
    s = xb.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                 layer.sh, layer.sw, layer.ph, layer.pw)
    OH, OW = xb.xnor_out_dim(s)
    ws_bytes = xb.xnor_conv2d_workspace_bytes(s)
    used_algo = xb.xnor_conv2d_pick_algo(s, ws_bytes) if algo == xb.ALGO_AUTO else algo

    Wt_host = make_weights(layer)
    dI = torch.from_numpy(make_input(layer)).cuda()
    dW = torch.from_numpy(Wt_host).cuda()
    Ipk = torch.empty((s.N, s.H, s.W, s.Cw), dtype=torch.int32, device="cuda")
    Wpk = torch.empty((s.F, s.kh, s.kw, s.Cw), dtype=torch.int32, device="cuda")
    A = torch.empty((s.N, s.H, s.W), dtype=torch.float32, device="cuda")
    K = torch.empty((s.N, OH, OW), dtype=torch.float32, device="cuda")
    alpha = torch.empty((s.F,), dtype=torch.float32, device="cuda")
    out = torch.empty((s.N, s.F, OH, OW), dtype=torch.float32, device="cuda")
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda") if ws_bytes else None

    M = torch.empty((s.F, s.kh, s.kw), dtype=torch.float32, device="cuda")
    # with the matrix-core kernel the convolution is two calls, so that the timed "conv" stage is
    # that one kernel launch (what the roofline figures are about)
    two_phase = used_algo == xb.ALGO_MFMA and not args.chain
    # (items of the matrix-core kernel: bands of up to 256 output pixels x tiles of 128 filters; one
    #  round = two per compute unit)
    items = -(-(s.N * OH) // max(1, 256 // OW)) * -(-s.F // 128)
    k_in_conv = two_phase and not args.unfused and not args.k_in_prepare and (args.k_in_conv or items <= 512)
    if args.chain:
        xb.xnor_input_prepare(dI, s, Ipk, A, K)
        xb.xnor_filter_prepare(dW, Wpk, M, alpha)
        Opk = torch.empty((s.N, OH, OW, (s.F + 31) // 32), dtype=torch.int32, device="cuda")
        A_next = torch.empty((s.N, OH, OW), dtype=torch.float32, device="cuda")
        ws = torch.empty((xb.xnor_conv2d_chain_workspace_bytes(s),), dtype=torch.uint8, device="cuda")
        # a chained network's filters are constants: packed, scaled and expanded once, outside the step
        xb.xnor_filter_expand(Wpk, s, ws)
    # input side and filter side as one call (one launch where the shapes allow it)
    one_prepare = not (args.chain or args.unfused or args.separate_prepare)
    if args.chain:
        names = ["conv"]
    else:
        names = (["pack_I", "scale_K", "alpha", "pack_W"] if args.unfused else
                 ["prepare"] if one_prepare else ["input_prepare", "filter_prepare"]) + \
                (["conv"] if one_prepare or not two_phase else ["filter_expand", "conv"])

    n_marks = len(names) + 1

    def step(events=None, conv_only=False):
        marks = []

        def mark():
            if events is None:
                return
            if conv_only and len(marks) < n_marks - 2:
                marks.append(None)              # only the two events that bracket the convolution (the last stage)
                return
            e = torch.cuda.Event(enable_timing=True)
            e.record()                          # recorded on the stream the kernels are launched on
            marks.append(e)

        if args.chain:
            # a chained layer receives packed signs and the channel mean; K is formed inside the kernel
            mark(); xb.xnor_conv2d_fwd_chain(Ipk, None, None, alpha, s, Opk, A_next, workspace=ws, A=A)
            mark()
            if events is not None:
                events.append(marks)
            return
        if args.unfused:
            mark(); xb.xnor_binarize_pack(dI, Ipk)
            mark(); xb.xnor_scale_K(dI, s, A, K)
            mark(); xb.xnor_alpha(dW, alpha)
            mark(); xb.xnor_binarize_pack(dW, Wpk)
        else:
            # with the matrix-core kernel K is formed inside the convolution from A (same arithmetic
            # as the box-filter kernel, bit-identical output): one launch less per step
            if one_prepare:
                # (with the matrix-core kernel the call also leaves the filters expanded in `ws`)
                mark(); xb.xnor_prepare(dI, dW, s, Ipk, A, K, Wpk, M, alpha, want_K=not k_in_conv,
                                        workspace=ws if two_phase else None)
            else:
                mark(); xb.xnor_input_prepare(dI, s, Ipk, A, K, want_K=not k_in_conv)
                mark(); xb.xnor_filter_prepare(dW, Wpk, M, alpha)
        if two_phase:
            # per-model work ends with the filters in the matrix-core kernel's operand order
            if not one_prepare:
                mark(); xb.xnor_filter_expand(Wpk, s, ws)
            if not k_in_conv:
                mark(); xb.xnor_conv2d_fwd_expanded(Ipk, ws, K, alpha, s, out=out)
            else:
                mark(); xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, out=out, A=A)
        else:
            mark(); xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, out=out, algo=algo, workspace=ws)
        mark()
        if events is not None:
            events.append(marks)

    if args.copy_probe:
        src = torch.empty((1 << 28,), dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            xb.xnor_probe_copy(src, dst)       # probe_copy_kernel: 1 GiB read + 1 GiB written per launch
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: K steps, with a pair of events around the convolution launch on about 250 of
    # them, evenly spread (the roofline figure).  The other stages' times come from a second, untimed pass with an event
    # after every call: five event records per step cost the host about as much as the launches.
    events: list = []
    every = args.conv_events_every if args.conv_events_every >= 0 else max(1, args.steps // 250)
    t0 = time.perf_counter()
    for k in range(args.steps):
        if every and k % every == 0:
            step(events, conv_only=True)
        else:
            step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    conv_events = [(m[-2], m[-1]) for m in events]
    events = []
    for _ in range(min(args.steps, 250)):
        step(events)
    torch.cuda.synchronize()

    # An eager step pays the host's launches and the dispatch gaps between dependent kernels (the small
    # layers finish faster than the host can issue their launches): unless --no-graph, the step is
    # also captured into a HIP graph (the library allocates nothing and records no memset), each
    # replay is checked against the eager result, and the replay time is reported beside the eager one.
    graph_ms, graph_ok = None, None
    if not args.no_graph and not args.copy_probe:
        eager = out.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        graph_ok = True
        for _ in range(3):
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            graph_ok = graph_ok and bool(torch.equal(out, eager))
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) / args.steps * 1e3
        del graph

    # untimed: the convolution once more with the raw dot products as well (for the parity check
    # against the oracle's sample; the step itself does not write them)
    dot = None
    if not args.sweep and not args.chain and not args.no_cpu_baseline:
        dot = torch.empty((s.N, s.F, OH, OW), dtype=torch.int32, device="cuda")
        step()
        if two_phase:
            xb.xnor_conv2d_fwd_expanded(Ipk, ws, K, alpha, s, out=out, dot=dot) if not k_in_conv else \
                xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, out=out, dot=dot, A=A)
        else:
            xb.xnor_conv2d_fwd(Ipk, Wpk, K, alpha, s, out=out, dot=dot, algo=algo, workspace=ws)
        torch.cuda.synchronize()

    ms_per_step = elapsed / args.steps * 1e3
    stage_ms = {n: sum(m[i].elapsed_time(m[i + 1]) for m in events) / len(events) for i, n in enumerate(names)}
    conv_times = sorted(a.elapsed_time(b) for a, b in conv_events)
    stage_ms["conv"] = sum(conv_times) / len(conv_times)
    conv_ms = stage_ms["conv"]
    macs = layer.binary_macs
    value = macs / (ms_per_step * 1e-3) / 1e9

    ops = 2.0 * macs                                           # algorithmic ops of one conv launch
    achieved = ops / (conv_ms * 1e-3) / 1e12
    if used_algo == xb.ALGO_MFMA:
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP4_MFMA_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "alu", "achieved": achieved, "peak": PEAK_VALU_POPCOUNT_TOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM bytes per conv launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by a
    # plain copy of known size), read from the tracked summary; null where no reading of this
    # kernel as it stands exists
    roof["traffic"], roof["traffic_note"] = measured_conv_traffic(layer.name, xb.ALGO_NAMES[used_algo])
    roof["kernel"] = ("matrix-core convolution kernel (xnor_conv2d_fwd_expanded" + (", K formed from A" if k_in_conv else "") + ")") if two_phase else f"xnor_conv2d_fwd[{xb.ALGO_NAMES[used_algo]}]"
    roof["kernel_ms"] = conv_ms                                # mean over the timed steps (what `achieved` uses)
    roof["kernel_ms_median"] = conv_times[len(conv_times) // 2]
    roof["kernel_ms_min"] = conv_times[0]
    # what a pair of events reads with nothing between them, and with a tiny kernel between them:
    # the part of kernel_ms that is the bracket's own (reported, not subtracted)
    a16 = torch.zeros((64,), dtype=torch.float32, device="cuda")
    b16 = torch.zeros_like(a16)
    pairs = []
    for tiny in (False, True):
        evs = []
        for _ in range(200):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if tiny:
                xb.xnor_probe_copy(a16, b16)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        pairs.append(sum(a.elapsed_time(b) for a, b in evs[50:]) / len(evs[50:]))
    roof["event_pair_ms_empty"], roof["event_pair_ms_tiny_kernel"] = pairs
    # (`achieved` and `frac` stay on the raw event time; net of the empty bracket the launch is what
    #  the kernel trace of the same command shows)
    if two_phase and conv_ms > pairs[0]:
        roof["kernel_ms_net_of_empty_pair"] = conv_ms - pairs[0]
        roof["frac_net_of_empty_pair"] = roof["frac"] * conv_ms / (conv_ms - pairs[0])
    if two_phase:
        # the same launch 200 times in a row inside ONE pair of events (the bracket's cost spread
        # over 200 launches, the dispatch gap between two of them included): how long the launch
        # is when nothing else runs between two of them.  Not the step's conditions: there the
        # HBM-bound prepare launches sit between two convolutions.
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            if not k_in_conv:
                xb.xnor_conv2d_fwd_expanded(Ipk, ws, K, alpha, s, out=out)
            else:
                xb.xnor_conv2d_fwd_expanded(Ipk, ws, None, alpha, s, out=out, A=A)
        e1.record()
        torch.cuda.synchronize()
        roof["kernel_ms_back_to_back"] = e0.elapsed_time(e1) / 200
    roof["binary_gmacs"] = macs / (conv_ms * 1e-3) / 1e9
    roof["frac_of_valu_popcount_peak"] = achieved / PEAK_VALU_POPCOUNT_TOPS
    # the same launch against the HBM roof: packed operands in, fp32 out
    conv_bytes = 4.0 * (Ipk.numel() + Wpk.numel() + K.numel() + alpha.numel() + out.numel())
    roof["hbm_gbs"] = conv_bytes / (conv_ms * 1e-3) / 1e9
    roof["hbm_frac"] = roof["hbm_gbs"] / PEAK_HBM_GBS

    # the whole step against the HBM roof: the fp32 input read once, the packed input written and
    # read once, the fp32 output written once (filters, K and alpha are under 3 % of that)
    step_bytes = 4.0 * (dI.numel() + 2 * Ipk.numel() + out.numel())
    step_roof = {"bound": "hbm", "achieved": step_bytes / (ms_per_step * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                 "unit": "GB/s", "algorithmic_bytes": step_bytes, "floor_ms": step_bytes / PEAK_HBM_GBS / 1e6}
    step_roof["frac"] = step_roof["achieved"] / PEAK_HBM_GBS

    rec = {
        "metric": ("binary GMAC/s, chained layer (XNOR conv taking packed signs + channel mean and expanded filters, emitting packed signs + channel mean for the next layer)" if args.chain
                   else "binary GMAC/s, whole forward pass (pack + K + alpha + XNOR conv + rescale)"),
        "pre_stages": ("separate calls" if args.unfused else
                       "one pass over I, one pass over Wt" + (", issued as one call" if one_prepare else "")),
        "value": value, "unit": "binary GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-packed +-1 (FP4 in the MFMA kernel), int32 dot, fp32 scale",
        "data": "synthetic (seeded; shapes and value distributions of the benchmark layer)",
        "config": {"workload": f"{layer.name}: N={layer.N} C={layer.C} {layer.H}x{layer.W} F={layer.F} "
                               f"{layer.kh}x{layer.kw} stride {layer.sh} pad {layer.ph}",
                   "binary_macs": macs, "conv_algo": xb.ALGO_NAMES[used_algo],
                   "buffers": f"reused every step (fp32 input {dI.numel() * 4 / 1e6:.1f} MB, output "
                              f"{out.numel() * 4 / 1e6:.1f} MB; the last-level cache holds 256 MB)"},
        "stage_ms": stage_ms,
        **({"graph_ms_per_step": graph_ms, "graph_replays_match_eager": graph_ok} if graph_ms is not None else {}),
        "roofline": roof,
        **({} if args.chain else {"step_roofline": step_roof}),
    }
    rec["_Wt_host"] = Wt_host
    rec["_out"], rec["_dot"] = (out, dot) if dot is not None else (None, None)
    del dI
    return rec


PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0      # dense bf16 MFMA


def run_bwn(args, xb, torch, layer, make_input, make_weights):
    """Eq. 1 on a benchmark layer: one step = filter_prepare (signs + alpha, one pass over Wt) and
    the BWN convolution reading the fp32 input directly (no input stage: nothing is binarised)."""
    import oracle

    s = xb.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                 layer.sh, layer.sw, layer.ph, layer.pw)
    OH, OW = xb.xnor_out_dim(s)
    Wt_host = make_weights(layer)
    dI = torch.from_numpy(make_input(layer)).cuda()
    dW = torch.from_numpy(Wt_host).cuda()
    Wpk = torch.empty((s.F, s.kh, s.kw, s.Cw), dtype=torch.int32, device="cuda")
    M = torch.empty((s.F, s.kh, s.kw), dtype=torch.float32, device="cuda")
    alpha = torch.empty((s.F,), dtype=torch.float32, device="cuda")
    out = torch.empty((s.N, s.F, OH, OW), dtype=torch.float32, device="cuda")
    algo = {"auto": xb.ALGO_AUTO, "direct": xb.ALGO_DIRECT, "mfma": xb.ALGO_MFMA, "split": xb.ALGO_MFMA_SPLIT}[args.algo]
    # which kernel that is for this shape: the three-term bf16 form, else the fp32 matrix form, else direct
    kernel = args.algo
    if kernel == "auto":
        kernel = "direct"
        for cand, cand_id in (("mfma", xb.ALGO_MFMA), ("split", xb.ALGO_MFMA_SPLIT)):
            try:
                xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, out=out, algo=cand_id)
                kernel = cand
            except xb.XnorError as e:
                if e.status != xb.E_UNSUPPORTED:
                    raise
        torch.cuda.synchronize()

    def step(events=None):
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if events is not None else None
        if marks: marks[0].record()
        xb.xnor_filter_prepare(dW, Wpk, M, alpha)
        if marks: marks[1].record()
        xb.xnor_bwn_conv2d_fwd(dI, Wpk, alpha, s, out=out, algo=algo)
        if marks:
            marks[2].record()
            events.append(marks)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events: list = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    stage_ms = {n: sum(m[i].elapsed_time(m[i + 1]) for m in events) / len(events)
                for i, n in enumerate(["filter_prepare", "conv"])}
    macs = layer.binary_macs
    conv_ms = stage_ms["conv"]
    # the three-term form executes three bf16 multiply-accumulates per fp32 one and is priced against
    # the bf16 peak with what it executes; the other kernels against the fp32 peak
    terms = 3 if kernel == "split" else 1
    peak = PEAK_BF16_MFMA_TFLOPS if kernel == "split" else PEAK_FP32_MFMA_TFLOPS
    achieved = terms * 2.0 * macs / (conv_ms * 1e-3) / 1e12
    rec = {
        "metric": "GMAC/s (real input x binary weight), Binary-Weight-Network layer (sign + alpha of the filters, add/subtract convolution, rescale)",
        "value": macs / (ms_per_step * 1e-3) / 1e9, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp32 input as three bf16 terms (exact), 1-bit weights, fp32 accumulate (v_mfma_f32_32x32x16_bf16)"
                 if kernel == "split" else "fp32 input, 1-bit weights, fp32 accumulate (v_mfma_f32_32x32x2_f32)",
        "data": "synthetic (seeded; shapes and value distributions of the benchmark layer)",
        "config": {"workload": f"{layer.name} as a BWN layer: N={layer.N} C={layer.C} {layer.H}x{layer.W} F={layer.F} "
                               f"{layer.kh}x{layer.kw} stride {layer.sh} pad {layer.ph}", "macs": macs},
        "stage_ms": stage_ms,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": None,
                     "kernel": {"split": "bwn_split_kernel", "mfma": "bwn_mfma_kernel", "direct": "bwn_direct_kernel"}[kernel]
                               + " (xnor_bwn_conv2d_fwd)",
                     "executed_flops_per_mac": 2 * terms, "kernel_ms": conv_ms},
    }
    if not args.no_cpu_baseline and not args.sweep:
        def run(n):
            I = make_input(layer, n)
            osh = oracle.Shape(n, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                               layer.sh, layer.sw, layer.ph, layer.pw)
            t0 = time.perf_counter()
            oracle.bwn(I, Wt_host, osh)
            return time.perf_counter() - t0
        t1 = run(1)
        n = max(1, min(layer.N, int(args.cpu_seconds / max(t1, 1e-3))))
        t = run(n) if n > 1 else t1
        rec["cpu_baseline"] = {"value": macs // layer.N * n / t / 1e9, "unit": "GMAC/s", "cores": oracle.threads(),
                               "kind": "oracle", "sample": f"first {n} of {layer.N} images of {layer.name}, all "
                                                           f"{layer.F} filters, oracle.bwn, {t:.2f} s"}
    return rec


# Table I (GTX 1080 Ti, mean of 100 runs, compute only), ms: vanilla convolution and XNOR convolution
PAPER_GPU_VANILLA_MS = {256: 0.062, 512: 0.186, 1024: 0.671, 2048: 2.641}


def time_call(torch, fn, warmup, steps):
    """Mean time of one call in ms, by events on the launch stream, after `warmup` calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def run_vanilla_layer(args, xb, torch, layer, make_input, make_weights):
    """The float comparison on a benchmark layer: xnor_conv2d_fp32_fwd on the fp32 input and weights
    (nothing to prepare), beside the whole XNOR forward pass of the same layer."""
    import numpy as np
    import oracle

    s = xb.Shape(layer.N, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                 layer.sh, layer.sw, layer.ph, layer.pw)
    OH, OW = xb.xnor_out_dim(s)
    Wt_host = make_weights(layer)
    dI = torch.from_numpy(make_input(layer)).cuda()
    dW = torch.from_numpy(Wt_host).cuda()
    out = torch.empty((s.N, s.F, OH, OW), dtype=torch.float32, device="cuda")
    ms = time_call(torch, lambda: xb.xnor_conv2d_fp32_fwd(dI, dW, s, out=out), args.warmup, args.steps)
    macs = layer.binary_macs                      # the same count of multiply-accumulates, now real-valued
    achieved = 2.0 * macs / (ms * 1e-3) / 1e12
    rec = {
        "metric": "GMAC/s, real-valued fp32 convolution (the float comparison of Table I)",
        "value": macs / (ms * 1e-3) / 1e9, "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp32 input and weights, fp32 accumulate (v_mfma_f32_32x32x2_f32)",
        "data": "synthetic (seeded; shapes and value distributions of the benchmark layer)",
        "config": {"workload": f"{layer.name} as a real-valued layer: N={layer.N} C={layer.C} {layer.H}x{layer.W} "
                               f"F={layer.F} {layer.kh}x{layer.kw} stride {layer.sh} pad {layer.ph}", "macs": macs},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": None,
                     "kernel": "bwn_mfma_kernel<.., real weights> (xnor_conv2d_fp32_fwd)", "kernel_ms": ms},
    }
    if not args.no_cpu_baseline:
        def run(n):
            I = make_input(layer, n)
            osh = oracle.Shape(n, layer.C, layer.H, layer.W, layer.F, layer.kh, layer.kw,
                               layer.sh, layer.sw, layer.ph, layer.pw)
            t0 = time.perf_counter()
            res = oracle.conv_fp32(I, Wt_host, osh, want_scale=True)
            return time.perf_counter() - t0, res
        t1, res = run(1)
        n = max(1, min(layer.N, int(args.cpu_seconds / max(t1, 1e-3))))
        t = t1
        if n > 1:
            t, res = run(n)
        rec["cpu_baseline"] = {"value": macs // layer.N * n / t / 1e9, "unit": "GMAC/s", "cores": oracle.threads(),
                               "kind": "oracle", "sample": f"first {n} of {layer.N} images of {layer.name}, all "
                                                           f"{layer.F} filters, oracle.conv_fp32, {t:.2f} s"}
        O_ref, S = res
        err = np.abs(out[:n].cpu().numpy().astype(np.float64) - O_ref.astype(np.float64))
        rec["parity"] = {"images": n, "elements": int(err.size), "worst_err_over_scale": float((err / np.maximum(S, 1e-300)).max()),
                         "outside_1e-5_of_scale": int((err > 1e-5 * S).sum()),
                         "scale": "sum |I * Wt| over the output's terms"}
    del dI, dW, out
    # the XNOR forward pass of the same layer (all of it: binarisation, K, alpha, convolution, rescale)
    sub = argparse.Namespace(**{**vars(args), "no_cpu_baseline": True, "sweep": True, "chain": False})
    x = run_layer(sub, xb, torch, layer, "auto", make_input, make_weights)
    rec["xnor_vs_float"] = {"float_conv_ms": ms, "xnor_step_ms": x["ms_per_step"], "xnor_conv_kernel_ms": x["stage_ms"]["conv"],
                            "speedup_whole_step": ms / x["ms_per_step"], "speedup_conv_only": ms / x["stage_ms"]["conv"],
                            "paper": "2.57x to 2.69x (Table I: one channel, 3x3, GTX 1080 Ti; another machine and shape, context only)"}
    return rec


def run_vanilla_image(args, xb, torch, side):
    """The paper's own shape (Table I): one channel, one 3x3 filter, pad 1; the float convolution
    beside xnor_forward_image on the same image."""
    import numpy as np

    rng = np.random.default_rng(20200714 * 100 + side)
    I = rng.standard_normal(size=(1, 1, side, side), dtype=np.float32)
    Wt = rng.standard_normal(size=(1, 1, 3, 3), dtype=np.float32)
    s = xb.Shape(1, 1, side, side, 1, 3, 3, 1, 1, 1, 1)
    dI, dW = torch.from_numpy(I).cuda(), torch.from_numpy(Wt).cuda()
    out = torch.empty((1, 1, side, side), dtype=torch.float32, device="cuda")
    Wpk, alpha, _ = xb.xnor_filter_prepare(dW)
    # both kernels are shorter than a launch: 20 back-to-back launches per HIP-graph replay
    reps = 20
    res = {}
    for name, fn in (("float", lambda: xb.xnor_conv2d_fp32_fwd(dI, dW, s, out=out)),
                     ("xnor", lambda: xb.xnor_forward_image(dI, Wpk, alpha, s, out=out))):
        fn()
        torch.cuda.synchronize()
        side_stream = torch.cuda.Stream()
        side_stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side_stream):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side_stream):
                for _ in range(reps):
                    fn()
        torch.cuda.current_stream().wait_stream(side_stream)
        res[name] = time_call(torch, g.replay, 3, args.steps) / reps
        del g
    gbs = 8.0 * side * side / (res["float"] * 1e-3) / 1e9
    return {
        "metric": "real-valued fp32 convolution latency, one image (the float comparison of Table I)",
        "value": res["float"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["float"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": res["float"] / PAPER_GPU_VANILLA_MS[side] if side in PAPER_GPU_VANILLA_MS else None,
        "baseline_note": "Table I, vanilla column (GTX 1080 Ti, compute only, mean of 100 runs): another machine, context only",
        "dtype": "fp32", "data": "synthetic (seeded N(0,1) image and filter)",
        "config": {"workload": f"image {side}x{side}: N=1 C=1 F=1 3x3 stride 1 pad 1 (Table I)", "macs": 9 * side * side},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                     "traffic": None, "kernel": "conv_fp32_rows_kernel (xnor_conv2d_fp32_fwd)", "kernel_ms": res["float"],
                     "timing": f"{reps} back-to-back launches per graph replay, events on the launch stream"},
        "xnor_vs_float": {"float_conv_ms": res["float"], "xnor_image_kernel_ms": res["xnor"],
                          "speedup": res["float"] / res["xnor"],
                          "paper": f"{PAPER_GPU_VANILLA_MS.get(side)} ms vs {PAPER_GPU_XNOR_MS.get(side)} ms on a GTX 1080 Ti (Table I)"},
    }


# Table III's "GPU" column for the XNOR convolution (GTX 1080 Ti, mean of 100 runs, compute only), ms
PAPER_GPU_XNOR_MS = {256: 0.0237, 512: 0.0692, 1024: 0.2519, 2048: 0.9859}


def run_image(args, xb, torch, side):
    """One channel, one 3x3 filter, pad 1 (the paper times nothing else): filter_prepare (per-model)
    + xnor_forward_image (per image: signs, K, XNOR convolution, rescale in one kernel)."""
    import numpy as np
    import oracle

    rng = np.random.default_rng(20200714 * 100 + side)
    I = rng.standard_normal(size=(1, 1, side, side), dtype=np.float32)
    Wt = rng.standard_normal(size=(1, 1, 3, 3), dtype=np.float32)
    s = xb.Shape(1, 1, side, side, 1, 3, 3, 1, 1, 1, 1)
    dI, dW = torch.from_numpy(I).cuda(), torch.from_numpy(Wt).cuda()
    Wpk = torch.empty((1, 3, 3, 1), dtype=torch.int32, device="cuda")
    alpha = torch.empty((1,), dtype=torch.float32, device="cuda")
    M = torch.empty((1, 3, 3), dtype=torch.float32, device="cuda")
    out = torch.empty((1, 1, side, side), dtype=torch.float32, device="cuda")

    def step():
        xb.xnor_filter_prepare(dW, Wpk=Wpk, M_work=M, alpha=alpha)
        xb.xnor_forward_image(dI, Wpk, alpha, s, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    eager = out.clone()

    # The kernels are shorter than the host's launch path, so the GPU's own time comes from HIP
    # graphs (the library allocates nothing and records no memset): one graph of the step, and one
    # of 20 back-to-back launches of the image kernel alone, timed with events on the launch stream.
    side_stream = torch.cuda.Stream()
    side_stream.wait_stream(torch.cuda.current_stream())
    reps = 20
    with torch.cuda.stream(side_stream):
        g_step, g_kernel = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_step, stream=side_stream):
            step()
        with torch.cuda.graph(g_kernel, stream=side_stream):
            for _ in range(reps):
                xb.xnor_forward_image(dI, Wpk, alpha, s, out=out)
    torch.cuda.current_stream().wait_stream(side_stream)
    ok = True
    for g in (g_step, g_kernel, g_step):
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ok = ok and bool(torch.equal(out, eager))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g_step.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        g_kernel.replay()
    e1.record()
    torch.cuda.synchronize()
    kernel_ms = e0.elapsed_time(e1) / (args.steps * reps)

    bytes_alg = 8.0 * side * side                       # 4 B read + 4 B written per pixel
    gbs = bytes_alg / (kernel_ms * 1e-3) / 1e9
    rec = {
        "metric": "XNOR convolution latency, one image (signs + K + XNOR conv + rescale; filter packing and alpha included)",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": ms_per_step / PAPER_GPU_XNOR_MS[side] if side in PAPER_GPU_XNOR_MS else None,
        "baseline_note": "Table III, GPU column (GTX 1080 Ti, compute only, mean of 100 runs); the paper does not say "
                         "how many filters it timed (one assumed) nor whether binarisation is inside its figure",
        "dtype": "fp32 in, sign bits in spatially packed windows, int32 dot, fp32 scale",
        "data": "synthetic (seeded N(0,1) image and filter; the paper's images are not specified)",
        "config": {"workload": f"image {side}x{side}: N=1 C=1 F=1 3x3 stride 1 pad 1 (Tables I-III)",
                   "binary_macs": 9 * side * side},
        "graph_ms_per_step": graph_ms, "graph_replays_match_eager": ok,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                     "traffic": None, "kernel": "conv_image_kernel (xnor_forward_image)", "kernel_ms": kernel_ms,
                     "timing": f"{reps} back-to-back launches per graph replay, events on the launch stream"},
    }
    if not args.no_cpu_baseline:
        osh = oracle.Shape(1, 1, side, side, 1, 3, 3, 1, 1, 1, 1)
        oracle.forward(I, Wt, osh)
        n, t0 = 0, time.perf_counter()
        while n < 3 or time.perf_counter() - t0 < 1.0:
            oracle.forward(I, Wt, osh)
            n += 1
        t = (time.perf_counter() - t0) / n
        rec["cpu_baseline"] = {"value": t * 1e3, "unit": "ms", "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"the same {side}x{side} image, whole forward pass, mean of {n} runs"}
    return rec


def run_peaks(args, xb, torch):
    """The ceilings this GPU sustains, each timed with events on the launch stream over repeated
    launches: the FP4 matrix instruction in registers, the v_xor + v_bcnt pair in registers, and a
    plain copy at a size the last-level cache holds and at one it does not."""
    def timed(fn, reps):
        # (a third of a second of the same work first: the chip holds its rate only after that)
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.3:
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    sink_f = torch.zeros((4,), dtype=torch.float32, device="cuda")
    sink_i = torch.zeros((4,), dtype=torch.int32, device="cuda")
    out = {"metric": "measured ceilings of this GPU (not the benchmark line)", "n_gpus": 1}
    for wgs in (256, 512, 1024):      # one, two and four 4-wave workgroups per compute unit
        flops = [0.0]
        t = timed(lambda: flops.__setitem__(0, xb.xnor_probe_mfma_fp4(wgs, 4000, sink_f)), 20)
        out[f"mfma_fp4_tflops_{wgs}wg"] = flops[0] / t / 1e12
    out["mfma_fp4_published_tflops"] = PEAK_FP4_MFMA_TFLOPS
    # the bf16 instruction of the Binary-Weight-Network kernel: +-1.0 against +-1.0, and +-1.0 against
    # values with random significands (two workgroups per compute unit, as the kernel runs)
    for name, rnd in (("pm1", False), ("random", True)):
        flops = [0.0]
        t = timed(lambda: flops.__setitem__(0, xb.xnor_probe_mfma_bf16(512, 8000, rnd, sink_f)), 20)
        out[f"mfma_bf16_tflops_b_{name}"] = flops[0] / t / 1e12
    out["mfma_bf16_published_tflops"] = PEAK_BF16_MFMA_TFLOPS
    macs = [0.0]
    t = timed(lambda: macs.__setitem__(0, xb.xnor_probe_xor_popcount(256 * 8, 20000, sink_i)), 10)
    out["xor_popcount_binary_tops"] = 2.0 * macs[0] / t / 1e12
    out["xor_popcount_derived_peak_tops"] = PEAK_VALU_POPCOUNT_TOPS
    for mib in (64, 1024):
        src = torch.empty((mib << 18,), dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        t = timed(lambda: xb.xnor_probe_copy(src, dst), 10)
        out[f"copy_{mib}MiB_gbs_read_plus_write"] = 2.0 * (mib << 20) / t / 1e9
        t = timed(lambda: xb.xnor_probe_read(src, sink_i), 10)
        out[f"read_{mib}MiB_gbs"] = (mib << 20) / t / 1e9
        del src, dst
    out["hbm_published_gbs"] = PEAK_HBM_GBS
    # what one replay of a captured HIP graph costs when the graph holds next to nothing (one or two
    # 256-byte copies): the floor under every graph-replayed step time
    a = torch.zeros((64,), dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    for n in (1, 2):
        def tiny():
            xb.xnor_probe_copy(a, b)
            if n == 2:
                xb.xnor_probe_copy(b, a)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            tiny()
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                tiny()
            for _ in range(200):
                graph.replay()
            stream.synchronize()
            t0 = time.perf_counter()
            for _ in range(2000):
                graph.replay()
            stream.synchronize()
            out[f"graph_replay_us_{n}_tiny_kernels"] = (time.perf_counter() - t0) / 2000 * 1e6
    # what the stores of a convolution item (128 KB per four waves) cost a wave group while the
    # other four waves of its compute unit run matrix instructions: shader-clock cycles per 128 KB,
    # mean over the storing waves, one workgroup per compute unit and 16 workgroups on the chip
    reps = 8
    sink = torch.zeros((4,), dtype=torch.float32, device="cuda")
    for wgs in (16, 256):
        dst = torch.empty((wgs * reps * 32768,), dtype=torch.float32, device="cuda")
        cycles = torch.zeros((wgs, 4), dtype=torch.int64, device="cuda")
        for wide in (False, True):
            for loop, name in ((0, "alone"), (1, "beside_back_to_back_mfma"), (2, "beside_mfma_with_pipe_idle_an_eighth")):
                for _ in range(2):
                    xb.xnor_probe_store_beside_mfma(wgs, reps, wide, loop, dst, cycles, sink)
                torch.cuda.synchronize()
                out[f"store_cycles_per_128KB_{'16B' if wide else '4B'}_stores_{name}_{wgs}wg"] = \
                    float(cycles.to(torch.float64).mean()) / reps
        del dst
    return out


def main():
    args = parse()
    if args.print_conv_digest:
        print(conv_source_digest())
        return
    world = int(os.environ.get("WORLD_SIZE", "1"))
    if args.gpus != 1 or world != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2007_14178_amd import binding as xb
    from paper_2007_14178_amd.workloads import LAYERS, make_input, make_weights

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.peaks:
        print(json.dumps(run_peaks(args, xb, torch)), flush=True)
        return
    if args.vanilla:
        print(json.dumps(run_vanilla_layer(args, xb, torch, LAYERS[args.layer], make_input, make_weights)), flush=True)
        for side in (int(v) for v in args.image_sides.split(",")):
            print(json.dumps(run_vanilla_image(args, xb, torch, side)), flush=True)
        return
    if args.image:
        for side in (int(v) for v in args.image_sides.split(",")):
            print(json.dumps(run_image(args, xb, torch, side)), flush=True)
        return
    if args.bwn:
        for lname in (list(LAYERS) if args.sweep else [args.layer]):
            print(json.dumps(run_bwn(args, xb, torch, LAYERS[lname], make_input, make_weights)), flush=True)
        return
    layers = list(LAYERS) if args.sweep else [args.layer]
    algos = ["tiled", "mfma"] if args.sweep else [args.algo]
    for lname in layers:
        for aname in algos:
            rec = run_layer(args, xb, torch, LAYERS[lname], aname, make_input, make_weights)
            Wt_host = rec.pop("_Wt_host")
            gpu_out, gpu_dot = rec.pop("_out"), rec.pop("_dot")
            if args.sweep:
                print(json.dumps(rec), flush=True)
    if args.sweep:
        return
    layer = LAYERS[args.layer]
    if not args.no_cpu_baseline:
        rec["cpu_baseline"], rec["parity"] = cpu_baseline(layer, Wt_host, args.cpu_seconds, gpu_out, gpu_dot)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
