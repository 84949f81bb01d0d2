#!/usr/bin/env python3
"""Benchmark of the width-folded convolution hot path on one MI355X.

One step = one pass of the hot path over one batch of the headline layer
(VGG-style first layer, N=64, 224x224, C_in=3 -> 64, 3x3, fp16, F=16):
fold (x' aliases x: identical bytes, nothing to launch) -> folded MFMA
convolution with bias -> reconstruct fused into the store.  The filter is
expanded and packed once before timing (the rewrite is post-training).
Inputs are seeded synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is useful conv TFLOP/s (padding and
structural-zero FLOPs excluded).  `roofline` describes the convolution
kernel (HIP events around every launch in the timed region);
`cpu_baseline` is the fp64 oracle timed on the host cores.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0  # dense fp16/bf16
KERNEL_NAMES = ["gather", "tiled", "stream"]
EXTRAS = ["dense_k", "padded", "pacing", "repack", "compact_filter", "copies", "c5_stack", "small_configs", "gemm_1x1", "fp32", "nchw",
          "fold_choice", "operand_values"]


def measured_traffic_bytes():
    """HBM bytes per launch of the headline kernel from the committed counter summary
    (profiles/conv_stream_c2_fp16.json), or None when the kernel's sources have changed since the
    counters were taken (the summary records a hash of the files the kernel is built from)."""
    path = os.path.join(ROOT, "profiles", "conv_stream_c2_fp16.json")
    try:
        rec = json.load(open(path))
        h = hashlib.sha256()
        for rel in rec["sources"]:
            h.update(open(os.path.join(ROOT, rel), "rb").read())
        if h.hexdigest() != rec["sources_sha256"]:
            return None
        return float(rec["hbm_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


SETTLE_MS = 15.0  # extras keep warming up until this much time has passed since their first call


def time_events(fn, steps, warmup, settle_ms=None):
    """Runs fn warmup+steps times.  Returns (wall ms/step, device ms/step): wall clock between
    two synchronisations around exactly `steps` calls, and HIP-event time over the same region
    on the stream the kernels are launched on, both divided by `steps`.
    settle_ms (default SETTLE_MS; the headline passes 0 and warms up exactly `warmup` times): further
    warm-up calls until that long after the first one, so that the timed region is past the clock dip
    the GPU goes through 2-10 ms after it leaves idle."""
    import torch

    settle_ms = SETTLE_MS if settle_ms is None else settle_ms
    t_first = time.perf_counter()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    while (time.perf_counter() - t_first) * 1e3 < settle_ms:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return wall_ms, e0.elapsed_time(e1) / steps


def per_launch_ms(fn, launches, warmup):
    """One event pair per launch: sorted list of device times in ms."""
    import torch

    t_first = time.perf_counter()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    while (time.perf_counter() - t_first) * 1e3 < SETTLE_MS:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    return sorted(e0.elapsed_time(e1) for e0, e1 in evs)


def graph_us_per_launch(fns, min_launches=16, replays=10, warmup=3):
    """Captures the calls of `fns` (one per rotating buffer set, repeated until there are at least
    min_launches) into one HIP graph and times its replay: device time per call in microseconds,
    without the per-launch host work of the Python binding."""
    import torch

    reps = max(1, -(-min_launches // len(fns)))

    def burst():
        for _ in range(reps):
            for f in fns:
                f()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        burst()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        burst()
    _, ms = time_events(gr.replay, replays, warmup)
    return ms * 1e3 / (reps * len(fns))


def rotating_sets(set_bytes, lo=4, hi=32, beyond=512e6):
    """How many buffer sets to rotate so that the 256 MB cache cannot hold them."""
    return int(min(hi, max(lo, -(-beyond // max(set_bytes, 1)))))


def cpu_baseline(layer, x, w, b):
    """The fp64 oracle, as it stands, on this host's cores over the whole batch."""
    from oracle import oracle as orc

    xs, wd, bd = x.double().numpy(), w.double().numpy(), None if b is None else b.double().numpy()
    ph, pw = orc.axis_pads(layer.KH, layer.KW, layer.pad)
    orc.conv_direct(xs[:1], wd, bd, ph, pw)  # page in
    t0 = time.perf_counter()
    ref = orc.conv_direct(xs, wd, bd, ph, pw)
    dt = time.perf_counter() - t0
    return ref, dt


def stats(ms_sorted):
    n = len(ms_sorted)
    return {"mean_ms": sum(ms_sorted) / n, "median_ms": ms_sorted[n // 2], "min_ms": ms_sorted[0], "launches": n}


def fold_choice_table(fc, runner, wl, torch):
    """Every legal power-of-two fold factor of the benchmark layers, timed (band walk, prepared
    filter, rotating buffers, graph replay), beside the cost model's estimate and its pick."""
    named = [("c2", wl.CONFIGS["c2"][0]), ("c3", wl.CONFIGS["c3"][0]), ("c4", wl.CONFIGS["c4"][0])]
    named += [("c5_L%d" % (i + 1), l) for i, l in enumerate(wl.CONFIGS["c5"])]
    # the fp32 path: the small fp32 configuration, and the headline shape in fp32
    c2_f32 = wl.Layer(**{**wl.CONFIGS["c2"][0].__dict__})
    c2_f32.dtype = "f32"
    named += [("c1", wl.CONFIGS["c1"][0]), ("c2_f32", c2_f32)]
    table = {}
    for name, base in named:
        pick = fc.foldconv_choose_fold(base.N, base.H, base.W, base.C_in, base.C_out, base.KH, base.KW, base.pad,
                                       wl.DTYPES[base.dtype])
        row = {"config_F": base.F, "model_pick": pick, "measured_us": {}, "model_us": {}, "kernel": {}}
        F = 1
        while F <= 64 and base.W % F == 0:
            l = wl.Layer(**{**base.__dict__})
            l.F = F
            plan = fc.foldconv_plan(*l.plan_args(), wl.DTYPES[l.dtype])
            s = plan.shapes
            row["model_us"][str(F)] = s.model_seconds * 1e6
            row["kernel"][str(F)] = KERNEL_NAMES[s.conv_kernel]
            if s.model_seconds > 5e-3 or s.w_exp_bytes > (1 << 30):
                row["measured_us"][str(F)] = None  # element-gather kernel on a large layer: not worth timing
                F *= 2
                continue
            x, w, b = wl.make_layer(l, 3000 + F)
            L = runner.FoldedLayer(l, w, b)
            nb = rotating_sets(s.x_bytes + s.y_bytes, hi=12)
            xs = [x.cuda() for _ in range(nb)]
            ys = [L.new_output() for _ in range(nb)]
            fns = [(lambda xi=xi, yi=yi: L.forward(xi, yi, compact=None)) for xi, yi in zip(xs, ys)]
            row["measured_us"][str(F)] = graph_us_per_launch(fns, min_launches=nb, replays=6, warmup=2)
            del L, xs, ys, fns
            F *= 2
        timed = {k: v for k, v in row["measured_us"].items() if v is not None}
        best = min(timed, key=timed.get)
        row["measured_best"] = int(best)
        row["pick_over_best"] = timed[str(pick)] / timed[best] if str(pick) in timed else None
        table[name] = row
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: long enough a warm-up to be past the first ~10 ms after the GPU leaves idle, where its
    # clocks dip and every memory-bound launch runs 10-30 % slower than before and after
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline step (profiling runs)")
    ap.add_argument("--extras", default=",".join(EXTRAS), help="comma-separated subset of: " + ", ".join(EXTRAS))
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: libfoldconv is measured on one GPU only; --gpus N with N > 1 is not supported "
              "(the path shards over the batch without collectives).", file=sys.stderr)
        sys.exit(2)
    want = set() if args.no_extras else set(e for e in args.extras.split(",") if e)
    if want - set(EXTRAS):
        print("bench.py: unknown extras %s" % sorted(want - set(EXTRAS)), file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_11608_amd as fc
    from paper_2601_11608_amd import runner
    from paper_2601_11608_amd import workloads as wl

    fc.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    layers, x, ws, bs = wl.make_config("c2")
    layer = layers[0]
    L = runner.FoldedLayer(layer, ws[0], bs[0])
    s = L.plan.shapes
    xd = x.cuda()
    y = L.new_output()

    def step():
        L.forward(xd, y)

    wall_ms, dev_ms = time_events(step, args.steps, args.warmup, settle_ms=0)
    useful_tflops = s.useful_flops / (wall_ms * 1e-3) / 1e12
    algo_bytes = s.x_bytes + s.w_exp_bytes + s.bias_bytes + s.y_bytes  # x + packed w' + b read once, y written once
    achieved_gbs = algo_bytes / (dev_ms * 1e-3) / 1e9

    # per-launch distribution (one event pair per launch, after the timed region): median and minimum
    per_launch = per_launch_ms(step, max(args.steps, 50), 0)

    out = {
        "metric": "useful conv TFLOP/s (fold vs zero-pad) + % MFMA peak, C_in=3 224^2 3x3 fp16",
        "value": useful_tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "c2: Conv2d NHWC fp16 N=64 224x224 C_in=3 C_out=64 3x3 s1 p1 bias, F=16 "
                               "(x' [64,224,14,48], w' [3,3,48,1024])",
                   "kernel": KERNEL_NAMES[s.conv_kernel], "k_walk": "band"},
        "roofline": {
            "bound": "hbm",
            "achieved": achieved_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            "traffic": measured_traffic_bytes(),
            "kernel_ms": dev_ms,
            "kernel_ms_median": per_launch[len(per_launch) // 2],
            "kernel_ms_min": per_launch[0],
            "algorithmic_bytes": algo_bytes,
        },
        "useful_pct_of_mfma_peak": 100.0 * useful_tflops / MFMA_PEAK_TFLOPS,
        "issued_tflops_band": s.issued_flops_band / (dev_ms * 1e-3) / 1e12,
    }

    extras = {}
    if "dense_k" in want:
        # dense walk of w' (every structural zero multiplied): the MFMA-bound figure.  Launches back to
        # back after a warm-up, as a serving loop would issue them.
        def step_dense():
            L.forward(xd, y, flags=fc.FLAG_DENSE_K)

        _, d_ms = time_events(step_dense, max(30, args.steps), 10)
        d_sorted = per_launch_ms(step_dense, 30, 0)
        extras["dense_k"] = {
            "kernel_ms": d_ms,
            "per_launch": stats(d_sorted),
            "useful_tflops": s.useful_flops / (d_ms * 1e-3) / 1e12,
            "issued_tflops": s.issued_flops_dense / (d_ms * 1e-3) / 1e12,
            "issued_pct_of_mfma_peak": 100.0 * s.issued_flops_dense / (d_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
            "note": "%d launches back to back after a %d ms warm-up" % (max(30, args.steps), int(SETTLE_MS)),
        }
    if "padded" in want:
        # zero-padded reference path (pad pass + conv), same kernels; and its convolution alone, on an
        # input that already has C_pad channels (the same kernel instance through the F = 1 plan)
        def step_padded():
            L.forward_padded(xd, y)

        _, p_ms = time_events(step_padded, max(20, args.steps // 2), 5)
        lp = wl.Layer(**{**layer.__dict__})
        lp.C_in, lp.F = s.C_pad, 1
        xp, wp_, bp = wl.make_layer(lp, 1500)
        Lp = runner.FoldedLayer(lp, wp_, bp)
        xpd = xp.cuda()
        _, pc_ms = time_events(lambda: Lp.forward(xpd, y), max(20, args.steps // 2), 5)
        extras["padded"] = {
            "ms": p_ms,
            "conv_only_ms": pc_ms,
            "C_pad": s.C_pad,
            "useful_tflops": s.useful_flops / (p_ms * 1e-3) / 1e12,
            "useful_tflops_conv_only": s.useful_flops / (pc_ms * 1e-3) / 1e12,
            "folded_speedup": p_ms / dev_ms,
            "folded_speedup_vs_conv_only": pc_ms / dev_ms,
        }
        del Lp, xpd
    if "pacing" in want:
        # the store pacing of the streaming kernel, A/B in steady state (200 warm-up launches each):
        # the library's default, the same launch with FOLDCONV_FLAG_UNPACED, and a plain fill of y
        _, on_ms = time_events(step, 100, 200)
        _, off_ms = time_events(lambda: L.forward(xd, y, flags=fc.FLAG_UNPACED), 100, 200)
        _, fill_ms = time_events(lambda: y.zero_(), 100, 200)
        extras["pacing"] = {
            "paced_ms": on_ms, "unpaced_ms": off_ms, "fill_ms": fill_ms,
            "paced_GBps": algo_bytes / (on_ms * 1e-3) / 1e9, "unpaced_GBps": algo_bytes / (off_ms * 1e-3) / 1e9,
            "fill_GBps": s.y_bytes / (fill_ms * 1e-3) / 1e9,
            "note": "100 launches after 200 warm-ups each; fill = torch's zero_() on the %d MB output" % (s.y_bytes // 1000000),
        }
    if "repack" in want:
        # per-call filter re-pack included (stateless call)
        _, r_ms = time_events(lambda: L.forward(xd, y, repack=True), max(20, args.steps // 2), 5)
        extras["with_filter_repack_ms"] = r_ms
    if "compact_filter" in want:
        # compact filter storage (non-zero blocks of w' only)
        _, c_ms = time_events(lambda: L.forward(xd, y, compact=True), max(20, args.steps // 2), 5)
        extras["compact_filter"] = {"kernel_ms": c_ms, "filter_bytes": int(s.filter_compact_bytes),
                                    "expanded_filter_bytes": int(s.w_exp_bytes)}
    if "copies" in want:
        # materialised fold and reconstruct copies (not on the timed path: both alias)
        nbuf = 8
        xs_rot = [torch.empty_like(xd) for _ in range(nbuf)]
        xs_src = [xd.clone() for _ in range(nbuf)]
        k = [0]

        def step_fold():
            fc.foldconv_fold_input(L.plan, xs_src[k[0] % nbuf], xs_rot[k[0] % nbuf])
            k[0] += 1

        _, f_ms = time_events(step_fold, 40, 8)
        extras["fold_copy"] = {"ms": f_ms, "GBps": 2 * s.x_bytes / (f_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": 2 * s.x_bytes / (f_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               "note": "rotating %d buffer pairs (%.0f MB) to defeat the 256 MB cache" % (nbuf, 2 * nbuf * s.x_bytes / 1e6)}
        y2 = torch.empty_like(y)
        _, u_ms = time_events(lambda: fc.foldconv_unfold_output(L.plan, y, y2), 10, 2)
        extras["unfold_copy"] = {"ms": u_ms, "GBps": 2 * s.y_bytes / (u_ms * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": 2 * s.y_bytes / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del xs_rot, xs_src, y2
    if "c5_stack" in want:
        # the 5-layer bf16 stack (3->20->36->68->132->256, 112x112, N=32), folded vs zero-padded
        l5, x5, w5, b5 = wl.make_config("c5")
        stack = runner.FoldedStack(l5, w5, b5)
        x5d = x5.cuda()
        flops5 = sum(L5.plan.shapes.useful_flops for L5 in stack.layers)
        # the stack as a user would run it: every layer from the filter form its plan prefers (packed w' for
        # the small layers, the compact form for the two large ones); then all-packed and all-compact
        # (long warm-up first: the launches after the GPU has idled run slower, whichever variant they are)
        _, spk_ms = time_events(lambda: stack.forward(x5d, compact=False), 20, 15)
        _, sc_ms = time_events(lambda: stack.forward(x5d, compact=True), 20, 5)
        _, s_ms = time_events(lambda: stack.forward(x5d, compact=None), 20, 5)
        _, sp_ms = time_events(lambda: stack.forward(x5d, padded=True), 20, 5)
        # each layer on its own (events around 20 launches, input = the previous layer's output)
        per_layer = []
        a = x5d
        for L5, y5 in zip(stack.layers, stack.outs):
            _, l_ms = time_events(lambda: L5.forward(a, y5, compact=None), 20, 3)
            s5 = L5.plan.shapes
            per_layer.append({"ms": l_ms, "F": s5.F, "kernel": KERNEL_NAMES[s5.conv_kernel],
                              "filter": "compact" if s5.prefer_compact else "packed",
                              "useful_tflops": s5.useful_flops / (l_ms * 1e-3) / 1e12,
                              "issued_tflops": s5.issued_flops_band / (l_ms * 1e-3) / 1e12,
                              "issued_over_useful": s5.issued_flops_band / s5.useful_flops})
            a = y5
        # the same five launches replayed from a captured HIP graph (no per-launch host work)
        sg_ms = graph_us_per_launch([lambda: stack.forward(x5d, compact=None)], min_launches=1, replays=20, warmup=5) * 1e-3
        extras["c5_stack"] = {"folded_ms": s_ms, "padded_ms": sp_ms, "folded_packed_filter_ms": spk_ms,
                              "folded_compact_filter_ms": sc_ms, "folded_graph_ms": sg_ms,
                              "per_layer": per_layer,
                              "filter_bytes": {"expanded": sum(int(L5.plan.shapes.w_exp_bytes) for L5 in stack.layers),
                                               "compact": sum(int(L5.plan.shapes.filter_compact_bytes) for L5 in stack.layers)},
                              "useful_tflops": flops5 / (s_ms * 1e-3) / 1e12,
                              "useful_pct_of_mfma_peak": 100.0 * flops5 / (s_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                              "kernels": [KERNEL_NAMES[L5.plan.shapes.conv_kernel] for L5 in stack.layers]}
        del stack, x5d
    if "operand_values" in want:
        # The MFMA-bound layer of the stack (132 -> 256 channels) with its seeded operands and with all-zero
        # operands: same kernel, same launch, same memory traffic; what differs is the clock the power
        # management allows (profiles/conv_tiled_c5_bf16.md reads the cycle counters of these launches).
        l5 = wl.CONFIGS["c5"][4]
        x5, w5, b5 = wl.make_layer(l5, 4005)
        ov = {}
        for name, xv, wv in (("seeded", x5, w5), ("zero", torch.zeros_like(x5), torch.zeros_like(w5))):
            Lv = runner.FoldedLayer(l5, wv, b5)
            xvd = xv.cuda()
            yv = Lv.new_output()
            _, v_ms = time_events(lambda: Lv.forward(xvd, yv, compact=None), 40, 10)
            sv = Lv.plan.shapes
            ov[name] = {"kernel_ms": v_ms, "issued_tflops": sv.issued_flops_band / (v_ms * 1e-3) / 1e12,
                        "issued_pct_of_mfma_peak": 100.0 * sv.issued_flops_band / (v_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS}
            del Lv, xvd, yv
        ov["note"] = "c5 layer 5 alone, 40 launches back to back after a %d ms warm-up, per operand values" % int(SETTLE_MS)
        extras["operand_values"] = ov
    if "small_configs" in want:
        # the small configurations (parity-test cases, not the headline) and the first layer of the stack:
        # launches replayed from a captured graph (so that the per-launch host work of the Python binding
        # is not what is timed), each launch on its own input/output pair out of a rotating set larger
        # than the 256 MB cache, so that the GB/s are HBM figures
        small = {}
        for cname, lidx in (("c1", 0), ("c3", 0), ("c4", 0), ("c5", 0)):
            ls, xs_, ws_, bs_ = wl.make_config(cname)
            Ls = runner.FoldedLayer(ls[lidx], ws_[lidx], bs_[lidx])
            ss = Ls.plan.shapes
            nb = rotating_sets(ss.x_bytes + ss.y_bytes)
            xs_d = [xs_.cuda() for _ in range(nb)]
            ys_d = [Ls.new_output() for _ in range(nb)]
            res = {"buffer_sets": nb, "rotated_MB": nb * (ss.x_bytes + ss.y_bytes) / 1e6}
            res["folded_us"] = graph_us_per_launch([(lambda a=a, b=b: Ls.forward(a, b)) for a, b in zip(xs_d, ys_d)])
            res["padded_us"] = graph_us_per_launch([(lambda a=a, b=b: Ls.forward_padded(a, b)) for a, b in zip(xs_d, ys_d)])
            res["useful_tflops"] = ss.useful_flops / (res["folded_us"] * 1e-6) / 1e12
            res["GBps"] = (ss.x_bytes + ss.y_bytes + ss.w_exp_bytes) / (res["folded_us"] * 1e-6) / 1e9
            res["frac_of_hbm_peak"] = res["GBps"] / HBM_PEAK_GBS
            res["kernel"] = KERNEL_NAMES[ss.conv_kernel]
            small[cname if cname != "c5" else "c5_L1"] = res
            del Ls, xs_d, ys_d
        extras["small_configs"] = small
    if "gemm_1x1" in want:
        # tall-skinny GEMM as a folded 1x1 convolution: A[2^21, 12] x B[12, 64], fp16, F = 4
        Mg, Kg, Ng, Fg = 1 << 21, 12, 64, 4
        gp = fc.foldconv_plan_gemm(Mg, Kg, Ng, Fg, torch.float16)
        gs = gp.shapes
        gl = wl.Layer("gemm", 1, gs.H, gs.W, Kg, Ng, 1, 1, 0, Fg, "f16", False, "normal")
        gx, gw, _ = wl.make_layer(gl, 2001)
        G = runner.FoldedLayer(gl, gw, None)
        gxd = gx.cuda()
        gy = G.new_output()
        _, g_ms = time_events(lambda: G.forward(gxd, gy), 50, 5)
        _, gp_ms = time_events(lambda: G.forward_padded(gxd, gy), 20, 3)
        extras["gemm_1x1"] = {"M": Mg, "K": Kg, "N": Ng, "F": Fg, "ms": g_ms, "padded_ms": gp_ms,
                              "useful_tflops": gs.useful_flops / (g_ms * 1e-3) / 1e12,
                              "GBps": (gs.x_bytes + gs.y_bytes) / (g_ms * 1e-3) / 1e9,
                              "frac_of_hbm_peak": (gs.x_bytes + gs.y_bytes) / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del G, gxd, gy
    if "fp32" in want:
        # the headline layer in fp32 (the precision of the paper's appendix listing): the streaming kernel with
        # steps of 8 K values as four MFMAs of K = 2; bound by the fp32 matrix rate, not by the 822 MB output
        lf = wl.Layer(**{**layer.__dict__})
        lf.dtype = "f32"
        Lf = runner.FoldedLayer(lf, ws[0].float(), None if bs[0] is None else bs[0].float())
        sf = Lf.plan.shapes
        xfd = x.float().cuda()
        yf = Lf.new_output()
        _, f_ms = time_events(lambda: Lf.forward(xfd, yf), 30, 5)
        _, fp_ms = time_events(lambda: Lf.forward_padded(xfd, yf), 10, 3)
        extras["fp32"] = {"kernel": KERNEL_NAMES[sf.conv_kernel], "ms": f_ms, "padded_ms": fp_ms,
                          "useful_tflops": sf.useful_flops / (f_ms * 1e-3) / 1e12,
                          "issued_tflops": sf.issued_flops_band / (f_ms * 1e-3) / 1e12,
                          "issued_pct_of_fp32_mfma_peak": 100.0 * sf.issued_flops_band / (f_ms * 1e-3) / 1e12 / 157.3,
                          "GBps": (sf.x_bytes + sf.y_bytes) / (f_ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": (sf.x_bytes + sf.y_bytes) / (f_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del Lf, xfd, yf
    if "nchw" in want:
        # the headline layer handed over channels-first (NCHW / OIHW): fold and reconstruct are real
        # re-indexing kernels here, the convolution between them is the same kernel as above
        xn = x.permute(0, 3, 1, 2).contiguous().cuda()
        wn = ws[0].permute(3, 2, 0, 1).contiguous().cuda()
        nchw = {}
        for axis_name, axis in (("fold_w", fc.FOLD_W), ("fold_h", fc.FOLD_H)):
            l = layer
            pn = fc.foldconv_plan_nchw(l.N, l.C_in, l.H, l.W, l.C_out, l.KH, l.KW, l.pad, l.F, axis, xn.dtype)
            sn = pn.shapes
            w_exp_n = torch.empty(sn.w_exp_bytes // sn.elem_bytes, dtype=xn.dtype, device="cuda")
            fc.foldconv_expand_filter_oihw(pn, wn, w_exp_n)
            ws_n = torch.empty(max(int(sn.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
            fc.foldconv_pack_filter(pn, w_exp_n, ws_n)
            xf_n = torch.empty_like(xn)
            yn = torch.empty(y.numel(), dtype=xn.dtype, device="cuda")
            bn = L.b

            def step_nchw():
                fc.foldconv_fold_input_nchw(pn, xn, xf_n)
                fc.foldconv_forward(pn, xf_n, w_exp_n, bn, y, ws_n, fc.FLAG_KEEP_FOLDED | fc.FLAG_FILTER_PACKED)
                fc.foldconv_unfold_output_nchw(pn, y, yn)

            _, n_ms = time_events(step_nchw, 10, 2)
            _, nf_ms = time_events(lambda: fc.foldconv_fold_input_nchw(pn, xn, xf_n), 20, 3)
            _, nu_ms = time_events(lambda: fc.foldconv_unfold_output_nchw(pn, y, yn), 10, 2)
            # total_ms / route: the fastest route the library offers for this layer (filled in below);
            # three_pass_ms: fold pass + convolution to the folded output + reconstruct pass
            nchw[axis_name] = {"total_ms": n_ms, "route": "fold pass + convolution + reconstruct pass",
                               "three_pass_ms": n_ms, "fold_ms": nf_ms, "unfold_ms": nu_ms,
                               "unfold_GBps": 2 * sn.y_bytes / (nu_ms * 1e-3) / 1e9}
            if sn.out_nchw_fused:
                # the convolution writes y channels-first itself: no folded output, no reconstruct pass
                def step_fused():
                    fc.foldconv_fold_input_nchw(pn, xn, xf_n)
                    fc.foldconv_forward(pn, xf_n, w_exp_n, bn, yn, ws_n, fc.FLAG_OUT_NCHW | fc.FLAG_FILTER_PACKED)

                _, fz_ms = time_events(step_fused, 20, 5)
                _, fk_ms = time_events(lambda: fc.foldconv_forward(pn, xf_n, w_exp_n, bn, yn, ws_n,
                                                                   fc.FLAG_OUT_NCHW | fc.FLAG_FILTER_PACKED), 20, 5)
                nchw[axis_name].update({"fused_total_ms": fz_ms, "fused_forward_ms": fk_ms,
                                        "fused_forward_GBps": (sn.x_bytes + sn.y_bytes) / (fk_ms * 1e-3) / 1e9,
                                        "fused_useful_tflops": sn.useful_flops / (fz_ms * 1e-3) / 1e12})
                # ... and reads x channels-first itself: one launch, no folded copy of the input either
                _, fi_ms = time_events(lambda: fc.foldconv_forward(pn, xn, w_exp_n, bn, yn, ws_n,
                                                                   fc.FLAG_IN_NCHW | fc.FLAG_OUT_NCHW | fc.FLAG_FILTER_PACKED), 20, 5)
                nchw[axis_name].update({"one_launch_ms": fi_ms,
                                        "one_launch_useful_tflops": sn.useful_flops / (fi_ms * 1e-3) / 1e12})
                if fz_ms < fi_ms:
                    nchw[axis_name].update({"total_ms": fz_ms, "route": "fold pass + convolution writing NCHW"})
                else:
                    nchw[axis_name].update({"total_ms": fi_ms, "route": "one launch: reads and writes NCHW"})
            nchw[axis_name]["useful_tflops"] = sn.useful_flops / (nchw[axis_name]["total_ms"] * 1e-3) / 1e12
            nchw[axis_name]["total_over_nhwc"] = nchw[axis_name]["total_ms"] / wall_ms   # against the channels-last step of the headline
            del w_exp_n, ws_n, xf_n, yn
        extras["nchw"] = nchw
    if "fold_choice" in want:
        extras["fold_choice"] = fold_choice_table(fc, runner, wl, torch)
    if want:
        out["extras"] = extras

    if not args.no_cpu_baseline:
        import numpy as np

        step()
        torch.cuda.synchronize()
        ref, dt = cpu_baseline(layer, x, ws[0], bs[0])
        cores = os.cpu_count()
        try:
            cores = len(os.sched_getaffinity(0))
        except Exception:
            pass
        cores = int(os.environ.get("OMP_NUM_THREADS", cores))
        out["cpu_baseline"] = {
            "value": s.useful_flops / dt / 1e12,
            "unit": "TFLOP/s",
            "cores": cores,
            "kind": "oracle",
            "sample": "whole batch (64 images), fp64 direct loops, %.2f s wall" % dt,
        }
        got = y[:4].cpu().double().numpy()
        err = max(float(np.linalg.norm(got[n] - ref[n]) / np.linalg.norm(ref[n])) for n in range(4))
        out["rel_l2_vs_oracle_first4"] = err

    print(json.dumps(out))


if __name__ == "__main__":
    main()
