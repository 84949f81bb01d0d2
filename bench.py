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
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the folded convolution on the headline layer from rocprofv3 counters
# (profiles/conv_stream_c2_fp16.md: WRITE_SIZE x 1.000 + FETCH_SIZE x 1.998).  Set to None whenever
# the convolution kernel changes after the counters were taken.
MEASURED_TRAFFIC_BYTES = 439.2e6
MFMA_PEAK_TFLOPS = 2500.0  # dense fp16/bf16


def time_events(fn, steps, warmup):
    """Runs fn warmup+steps times.  Returns (wall ms/step, device ms/step): wall clock between
    two synchronisations around exactly `steps` calls, and HIP-event time over the same region
    on the stream the kernels are launched on, both divided by `steps`."""
    import torch

    for _ in range(warmup):
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline step (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: libfoldconv is measured on one GPU only; --gpus N with N > 1 is not supported "
              "(the path shards over the batch without collectives).", file=sys.stderr)
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

    wall_ms, dev_ms = time_events(step, args.steps, args.warmup)
    useful_tflops = s.useful_flops / (wall_ms * 1e-3) / 1e12
    algo_bytes = s.x_bytes + s.w_exp_bytes + s.bias_bytes + s.y_bytes  # x + packed w' + b read once, y written once
    achieved_gbs = algo_bytes / (dev_ms * 1e-3) / 1e9

    # per-launch distribution (one event pair per launch, after the timed region): median and minimum
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.steps, 50))]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_launch = sorted(e0.elapsed_time(e1) for e0, e1 in evs)

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
                   "kernel": ["gather", "tiled", "stream"][s.conv_kernel], "k_walk": "band"},
        "roofline": {
            "bound": "hbm",
            "achieved": achieved_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES,
            "kernel_ms": dev_ms,
            "kernel_ms_median": per_launch[len(per_launch) // 2],
            "kernel_ms_min": per_launch[0],
            "algorithmic_bytes": algo_bytes,
        },
        "useful_pct_of_mfma_peak": 100.0 * useful_tflops / MFMA_PEAK_TFLOPS,
        "issued_tflops_band": s.issued_flops_band / (dev_ms * 1e-3) / 1e12,
    }

    if not args.no_extras:
        extras = {}
        # dense walk of w' (every structural zero multiplied): MFMA-bound figure
        def step_dense():
            L.forward(xd, y, flags=fc.FLAG_DENSE_K)

        _, d_ms = time_events(step_dense, max(3, args.steps // 5), 2)
        extras["dense_k"] = {
            "kernel_ms": d_ms,
            "useful_tflops": s.useful_flops / (d_ms * 1e-3) / 1e12,
            "issued_tflops": s.issued_flops_dense / (d_ms * 1e-3) / 1e12,
            "issued_pct_of_mfma_peak": 100.0 * s.issued_flops_dense / (d_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
        }
        # zero-padded reference path (pad pass + conv), same kernels
        def step_padded():
            L.forward_padded(xd, y)

        _, p_ms = time_events(step_padded, max(3, args.steps // 5), 2)
        extras["padded"] = {
            "ms": p_ms,
            "C_pad": s.C_pad,
            "useful_tflops": s.useful_flops / (p_ms * 1e-3) / 1e12,
            "folded_speedup": p_ms / dev_ms,
        }
        # per-call filter re-pack included (stateless call)
        def step_repack():
            L.forward(xd, y, repack=True)

        _, r_ms = time_events(step_repack, max(3, args.steps // 5), 2)
        extras["with_filter_repack_ms"] = r_ms
        # compact filter storage (non-zero blocks of w' only), headline layer and the stack below
        def step_compact():
            L.forward(xd, y, compact=True)

        _, c_ms = time_events(step_compact, max(3, args.steps // 5), 2)
        extras["compact_filter"] = {"kernel_ms": c_ms, "filter_bytes": int(s.filter_compact_bytes),
                                    "expanded_filter_bytes": int(s.w_exp_bytes)}
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

        def step_unfold():
            fc.foldconv_unfold_output(L.plan, y, y2)

        _, u_ms = time_events(step_unfold, 10, 2)
        extras["unfold_copy"] = {"ms": u_ms, "GBps": 2 * s.y_bytes / (u_ms * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": 2 * s.y_bytes / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del xs_rot, xs_src, y2
        # the 5-layer bf16 stack (3->20->36->68->132->256, 112x112, N=32), folded vs zero-padded
        l5, x5, w5, b5 = wl.make_config("c5")
        stack = runner.FoldedStack(l5, w5, b5)
        x5d = x5.cuda()
        flops5 = sum(L5.plan.shapes.useful_flops for L5 in stack.layers)
        _, s_ms = time_events(lambda: stack.forward(x5d), 20, 15)  # long warm-up: the first launches after idling run slower
        _, sp_ms = time_events(lambda: stack.forward(x5d, padded=True), 20, 5)
        _, sc_ms = time_events(lambda: stack.forward(x5d, compact=True), 20, 5)
        # the same five launches replayed from a captured HIP graph (no per-launch host work)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stack.forward(x5d, compact=True)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            stack.forward(x5d, compact=True)
        _, sg_ms = time_events(graph.replay, 20, 5)
        extras["c5_stack"] = {"folded_ms": s_ms, "padded_ms": sp_ms, "folded_compact_filter_ms": sc_ms,
                              "folded_compact_filter_graph_ms": sg_ms,
                              "filter_bytes": {"expanded": sum(int(L5.plan.shapes.w_exp_bytes) for L5 in stack.layers),
                                               "compact": sum(int(L5.plan.shapes.filter_compact_bytes) for L5 in stack.layers)},
                              "useful_tflops": flops5 / (s_ms * 1e-3) / 1e12,
                              "useful_pct_of_mfma_peak": 100.0 * flops5 / (s_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                              "kernels": [["gather", "tiled", "stream"][L5.plan.shapes.conv_kernel] for L5 in stack.layers]}
        # the small configurations (parity-test cases, not the headline): 20 launches replayed from a
        # captured graph so that the per-launch host work of the Python binding is not what is timed
        small = {}
        for cname in ("c1", "c3", "c4"):
            ls, xs_, ws_, bs_ = wl.make_config(cname)
            Ls = runner.FoldedLayer(ls[0], ws_[0], bs_[0])
            xsd = xs_.cuda()
            ys = Ls.new_output()
            ss = Ls.plan.shapes

            def burst(padded=False):
                for _ in range(20):
                    if padded:
                        Ls.forward_padded(xsd, ys)
                    else:
                        Ls.forward(xsd, ys)

            res = {}
            for key, padded in (("folded_us", False), ("padded_us", True)):
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    burst(padded)
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr):
                    burst(padded)
                _, b_ms = time_events(gr.replay, 10, 3)
                res[key] = b_ms * 1e3 / 20
            res["useful_tflops"] = ss.useful_flops / (res["folded_us"] * 1e-6) / 1e12
            res["GBps"] = (ss.x_bytes + ss.y_bytes + ss.w_exp_bytes) / (res["folded_us"] * 1e-6) / 1e9
            res["kernel"] = ["gather", "tiled", "stream"][ss.conv_kernel]
            small[cname] = res
        extras["small_configs"] = small
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
            nchw[axis_name] = {"total_ms": n_ms, "fold_ms": nf_ms, "unfold_ms": nu_ms,
                               "unfold_GBps": 2 * sn.y_bytes / (nu_ms * 1e-3) / 1e9,
                               "useful_tflops": sn.useful_flops / (n_ms * 1e-3) / 1e12}
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
            del w_exp_n, ws_n, xf_n, yn
        extras["nchw"] = nchw
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
