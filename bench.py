#!/usr/bin/env python3
"""Benchmark: Moonwalk gradient steps per second on one MI355X.

One "step" is one full moonwalk_grad call (Phase I forward, loss, Phase II reverse, Phase III
forward vijp sweep with weight and bias gradients) on one batch of synthetic input that is
already resident in HBM. Default workload: the deep square MLP (depth 64, width 1024, batch
256, leaky slope 0.1, re-seed interval 4).

Prints ONE JSON line. `value` is gradient steps/s of moonwalk_grad; the same line carries
TFLOP/s (10 B sum d_in d_out flop per step), the library's own backprop_grad timed the same
way, itemised and peak device bytes of both, the roofline of the dominant kernel measured live
with HIP events, and the fp64 CPU oracle timed on the host cores as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak (256 CUs x 256 flop/clk x 2.4 GHz)

# Bytes that cross the L2 per Phase-III launch (the layer kernels of four stretches + the weight gradients of the
# position before; average over the 17 launches of a step), from the two rocprofv3 --pmc runs summarised in
# profiles/bench_deep_square_hbm_traffic.txt (FETCH_SIZE 33096.8 KiB scaled x2.0 by the copy-kernel calibration,
# WRITE_SIZE 27000.5 KiB scaled x1.0). Offline counters: known only for the default workload in its default
# launch configuration (re-seed interval, group width), null otherwise.
PHASE3_TRAFFIC_BYTES = {"deep_square": int(33096.8 * 1024 * 2.0 + 27000.5 * 1024 * 1.0)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="deep_square")
    ap.add_argument("--depth", type=int, default=None, help="truncate the configuration to this many layers")
    ap.add_argument("--reseed", type=int, default=None, help="override the re-seed interval K")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backprop", action="store_true")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (convolutional configurations)")
    ap.add_argument("--block", type=int, default=None, help="conv1d configurations: positions per block of the fragment store")
    ap.add_argument("--h0", choices=["full", "as_read"], default="full",
                    help="convolutional configurations: compute the input cotangent for every input element (a network with "
                         "layers before the chain needs it; backprop then computes it too), or only what the first vijp reads")
    ap.add_argument("--segment", type=int, default=0,
                    help="segment length S of Moonwalk with rematerialisation (0 = off: the metric's configuration)")
    ap.add_argument("--group", type=int, default=0,
                    help="Phase III side by side: most stretches between re-seed points per launch (1: off, 0: chosen by the library)")
    ap.add_argument("--overlap", type=int, default=1, choices=[0, 1],
                    help="1: the grouped Phase-III sweeps run on the library's second stream while Phase II goes on")
    ap.add_argument("--no-train", action="store_true", help="skip the timing of the in-place training step")
    ap.add_argument("--refresh", choices=["fp32", "bf16"], default="bf16",
                    help="training step only: operand precision of the correction product of the Schulz refresh "
                         "(the residual it corrects is formed in fp32 either way; the gradient step is fp32 always)")
    ap.add_argument("--unfused", action="store_true", help="plain GEMMs + stand-alone elementwise kernels")
    ap.add_argument("--gen", choices=["numpy", "torch"], default="numpy",
                    help="numpy: host generator (the one the parity tests use); torch: same recipe drawn on the GPU "
                         "(for the large configurations; the CPU baseline is then skipped)")
    return ap.parse_args()


def time_steps(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return start.elapsed_time(stop) / steps, wall * 1e3 / steps   # ms/step by events, by wall clock


def cpu_baseline(wl, flops):
    """The fp64 oracle's Moonwalk step as it stands, on the host cores (right inverses excluded,
    as for the GPU). Sample: whole steps of the same workload, at least one, about 10-30 s."""
    from oracle import moonwalk_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ps = [O.right_inverse(W) for W in wl.W]
    n, elapsed = 0, 0.0
    while n < 1 or (elapsed < 10.0 and n < 50):
        t0 = time.perf_counter()
        O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, reseed_interval=wl.reseed_interval,
                   loss_scale=wl.loss_scale, Ps=Ps)
        elapsed += time.perf_counter() - t0
        n += 1
    per = elapsed / n
    return {"value": 1.0 / per, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} full fp64 oracle Moonwalk step(s) of the same workload (numpy, right inverses precomputed)",
            "gflops": flops / per / 1e9}


def bench_conv(args):
    """The convolutional configurations (--config conv2d, conv2d_small): the same JSON line for Moonwalk on
    submersive 2-D convolutional layers. These are additional workloads, not the headline metric's."""
    import numpy as np
    import torch
    import paper_2402_14212_amd as mw
    from workloads import (CONV_CONFIGS, FRAG_CONFIGS, make_convnet, make_convnet_on_device, make_fragnet, conv_moonwalk_flops,
                           conv_backprop_flops, frag_moonwalk_flops, frag_backprop_flops)

    frag1d = args.config.startswith("conv1d")
    c = dict((FRAG_CONFIGS if frag1d else CONV_CONFIGS)[args.config])
    if args.depth is not None:
        c["depth"] = args.depth
    if args.batch is not None:
        c["batch"] = args.batch
    if args.block is not None:
        c["block"] = args.block
    torch.cuda.set_device(0)
    on_device = (args.gen == "torch" or args.config == "conv2d") and not frag1d
    if frag1d:
        wl = make_fragnet(c["batch"], c["length"], c["channels"], c["depth"], block=c["block"], alpha=c["alpha"], seed=0,
                          name=args.config)
        h0_full = True
        flops_mw, flops_bp = frag_moonwalk_flops(wl), frag_backprop_flops(wl, True)
    else:
        wl = (make_convnet_on_device if on_device else make_convnet)(c["batch"], c["side"], c["channels"], c["depth"],
                                                                     k=c.get("k", 3), s=c.get("s", 2), p=c.get("p", 1),
                                                                     alpha=c["alpha"], seed=0, name=args.config)
        h0_full = args.h0 == "full"
        flops_mw, flops_bp = conv_moonwalk_flops(wl, h0_full), conv_backprop_flops(wl, h0_full)
    K = args.reseed if args.reseed is not None else (0 if frag1d else 2)
    h0_mode = mw.CONV_H0_FULL if h0_full else mw.CONV_H0_AS_READ
    grads_probe = None
    # --- Moonwalk handle only (so that its memory is its own)
    t0 = time.perf_counter()
    net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, plan=mw.PLAN_MOONWALK, input_cotangent=h0_mode)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0
    grads = net.new_grads()
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ms_mw, wall_mw = time_steps(lambda: net.moonwalk_grad(net.x, net.t, grads, loss), args.steps, args.warmup)
    st = net.memory_stats()
    bp = {}
    mem_bp = {}
    if not args.no_backprop:
        grads_probe = grads.clone()
        net.close()
        net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_BACKPROP, input_cotangent=h0_mode)
        ms_bp, _ = time_steps(lambda: net.backprop_grad(net.x, net.t, grads, loss), args.steps, args.warmup)
        sb = net.memory_stats()
        # the two paths' gradients against each other (each is checked against the oracle in the tests)
        agree = float(((grads - grads_probe).double().norm() / grads.double().norm()).item())
        bp = {"steps_per_s": 1e3 / ms_bp, "ms_per_step": ms_bp, "tflops": flops_bp / (ms_bp * 1e-3) / 1e12,
              "flop_per_step": flops_bp, "moonwalk_vs_backprop_grad_rel_diff": agree}
        mem_bp = {"bytes_residual": sb["bytes_bp_activations"], "bytes_input_cotangent": sb["bytes_input_cotangent"],
                  "bytes_scratch": sb["bytes_bp_scratch"] + sb["bytes_scratch"] + sb["bytes_patches"],
                  "bytes_packed_weights": sb["bytes_packed_weights"], "bytes_total": sb["bytes_peak"]}
    train = {}
    if not args.no_train:
        # the training step in place (gradients applied in the weight-gradient reduction, constrained taps
        # projected, derived matrices refreshed); a step that moves the weights by about 1e-4 of their size
        net.close()
        net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, plan=mw.PLAN_MOONWALK, input_cotangent=h0_mode)
        gn = float(grads.double().norm().item()) if grads_probe is None else float(grads_probe.double().norm().item())
        wn = float(torch.sqrt(sum((w.double() ** 2).sum() for w in net.ws)).item())
        lr = 1e-4 * wn / max(gn, 1e-30)
        ms_tr, _ = time_steps(lambda: net.sgd_step(net.x, net.t, lr, loss), args.steps, args.warmup)
        train = {"ms_per_step": ms_tr, "steps_per_s": 1e3 / ms_tr, "lr": lr,
                 "note": "moonwalk_conv_sgd_step: gradients applied in place, no gradient buffer; includes the refresh of the "
                         "tap inverses and regrouped taps and its synchronisation"}
    achieved = flops_mw / (ms_mw * 1e-3) / 1e12
    residual_mw = st["bytes_masks"] + st["bytes_checkpoints"] + st["bytes_fragments"]
    if frag1d:
        what = (f"{args.config}: {wl.depth} layers of 1-D convolution {wl.k}x{wl.channels}x{wl.channels}, stride 1, padding {(wl.k - 1) // 2}, "
                f"input {wl.length}x{wl.channels}, batch {wl.batch}, alpha {wl.alphas[0]}, fragment blocks of {wl.block}, reseed K={K}")
        metric = ("gradient steps/s (mixed-mode Moonwalk with fragmental checkpointing on 1-D convolutional layers, one full "
                  "moonwalk_conv_grad per step)")
    else:
        what = (f"{args.config}: {wl.depth} layers of {wl.k}x{wl.k}x{wl.channels}x{wl.channels} convolution, stride {wl.s}, "
                f"padding {wl.p}, input {wl.side}x{wl.side}x{wl.channels}, batch {wl.batch}, alpha {wl.alphas[0]}, "
                f"reseed K={K}, input cotangent {'for every input element' if h0_full else 'as the first vijp reads it'}")
        metric = "gradient steps/s (mixed-mode Moonwalk on submersive 2-D convolutional layers, one full moonwalk_conv_grad per step)"
    out = {
        "metric": metric,
        "value": 1e3 / ms_mw, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_mw, "ms_per_step_wall": wall_mw, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic (seeded, generator: %s)" % ("torch" if on_device else "numpy"),
        "config": {"workload": what},
        "tflops": achieved, "flop_per_step": flops_mw,
        "mfma_frac_whole_step": achieved / MFMA_F32_PEAK_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "whole step (products with gathered patch matrices, reductions and elementwise kernels included)",
                     "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_F32_PEAK_TFLOPS, "traffic": None},
        "setup_s": setup_s,
        "memory": {"moonwalk": {"bytes_masks": st["bytes_masks"], "bytes_fragments": st["bytes_fragments"],
                                "bytes_checkpoints": st["bytes_checkpoints"],
                                "bytes_residual": residual_mw, "bytes_tap_inverses": st["bytes_tap_inverses"],
                                "bytes_packed_weights": st["bytes_packed_weights"],
                                "bytes_input_cotangent": st["bytes_input_cotangent"],
                                "bytes_scratch": st["bytes_scratch"] + st["bytes_patches"], "bytes_total": st["bytes_peak"]},
                   "backprop": mem_bp,
                   "bytes_input": int(wl.x.numel() if hasattr(wl.x, "numel") else wl.x.size) * 4},
        "backprop": bp,
        "train_step": train,
    }
    net.close()
    if not args.no_cpu_baseline and frag1d:
        from oracle import frag_oracle as FO
        sample = make_fragnet(2, min(wl.length, 256), wl.channels, min(wl.depth, 3), block=wl.block, alpha=c["alpha"], seed=0)
        t0, n = time.perf_counter(), 0
        while n < 1 or time.perf_counter() - t0 < 10.0:
            FO.frag_moonwalk(sample.w, sample.b, sample.alphas, sample.x, sample.t, sample.block)
            n += 1
        per = (time.perf_counter() - t0) / n
        fl = frag_moonwalk_flops(sample)
        out["cpu_baseline"] = {"value": (fl / per) / flops_mw, "unit": "steps/s", "cores": int(os.cpu_count() or 1), "kind": "oracle",
                               "sample": f"{n} fp64 oracle step(s) of a {sample.depth}-layer, {sample.length}x{sample.channels}, "
                                         f"batch-2 cut of the workload; steps/s scaled by the flop ratio to the full workload",
                               "gflops": fl / per / 1e9}
    elif not args.no_cpu_baseline:
        from oracle import conv_oracle as CO
        sample = make_convnet(1, min(wl.side, 32), wl.channels, min(wl.depth, 3), k=wl.k, s=wl.s, p=wl.p, alpha=c["alpha"], seed=0)
        t0, n = time.perf_counter(), 0
        while n < 1 or time.perf_counter() - t0 < 10.0:
            CO.conv_moonwalk(sample.w, sample.b, sample.alphas, sample.s, sample.p, sample.x, sample.t)
            n += 1
        per = (time.perf_counter() - t0) / n
        fl = conv_moonwalk_flops(sample)
        out["cpu_baseline"] = {"value": (fl / per) / flops_mw, "unit": "steps/s", "cores": int(os.cpu_count() or 1), "kind": "oracle",
                               "sample": f"{n} fp64 oracle Moonwalk step(s) of a {sample.depth}-layer, {sample.side}x{sample.side}x{sample.channels}, "
                                         f"batch-1 cut of the workload; steps/s scaled by the flop ratio to the full workload",
                               "gflops": fl / per / 1e9}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.config.startswith("conv2d") or args.config.startswith("conv1d"):
        return bench_conv(args)
    import torch
    import paper_2402_14212_amd as mw
    from workloads import make_config, moonwalk_flops, backprop_flops, CONFIGS

    wl = make_config(args.config, depth=args.depth, device="cuda:0" if args.gen == "torch" else None)
    if args.reseed is not None:
        wl.reseed_interval = args.reseed
    B, widths, L = wl.batch, wl.widths, wl.depth
    flops_mw, flops_bp = moonwalk_flops(widths, B), backprop_flops(widths, B)

    torch.cuda.set_device(0)
    torch.cuda.reset_peak_memory_stats()
    base_bytes = torch.cuda.memory_allocated()

    # --- Moonwalk handle only (so that its peak memory is its own)
    t0 = time.perf_counter()
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, fuse=not args.unfused, segment_length=args.segment,
                                       phase3_parallel_segments=args.group, phase3_overlap=bool(args.overlap),
                                       refresh_bf16=args.refresh == "bf16")
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0
    grads = net.new_grads()
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ms_mw, wall_mw = time_steps(lambda: net.moonwalk_grad(net.x, net.t, grads, loss), args.steps, args.warmup)
    st = net.memory_stats()
    mw_peak_lib = st["bytes_live"]
    mw_peak_torch = torch.cuda.max_memory_allocated() - base_bytes

    # --- roofline of the dominant kernel: the Phase-III launch, which carries layer i's kernel
    # (recompute + vijp + epilogue: two products) and layer i-1's weight-gradient product: three of
    # the five GEMMs of the step. Each kernel class is timed alone: only its launches run, back to
    # back over the real buffers (all layers, cold weights), between two events on the launch stream.
    prof_steps = max(1, min(args.steps, 20))
    sum_dd = sum(a * b for a, b in zip(widths[:-1], widths[1:]))
    class_flops = {"fwd": 2.0, "rev": 2.0, "vijp": 4.0, "dw": 2.0, "phase3": 6.0}
    per_class = {}
    for k in ("fwd", "rev", "vijp", "dw", "ew", "phase3"):
        net.profile_filter(k)
        ms_k, _ = time_steps(lambda: net.moonwalk_grad(net.x, net.t, grads, loss), prof_steps, 2)
        n_k = net.profile_launches()[k]
        per_class[k] = {"launches_per_step": n_k, "avg_us": (ms_k / n_k * 1e3 if n_k else None),
                        "ms_per_step": ms_k}
        if k in class_flops and n_k:
            per_class[k]["tflops"] = class_flops[k] * B * sum_dd / (ms_k * 1e-3) / 1e12
    net.profile_filter(None)
    # The few small elementwise launches run alone are bound by the host's launch rate, not by the
    # GPU: report that class as what is left of the step after the GEMM classes.
    ew = per_class["ew"]
    ew["ms_per_step_alone"] = ew["ms_per_step"]
    gemm_ms = sum(per_class[k]["ms_per_step"] for k in ("fwd", "rev", "phase3"))
    if per_class["phase3"]["launches_per_step"] == 0:
        gemm_ms += per_class["vijp"]["ms_per_step"] + per_class["dw"]["ms_per_step"]
    ew["ms_per_step"] = max(0.0, ms_mw - gemm_ms)
    ew["avg_us"] = ew["ms_per_step"] / ew["launches_per_step"] * 1e3 if ew["launches_per_step"] else None
    ew["method"] = "step time minus the GEMM classes"
    # dominant kernel: the paired Phase-III launch; in unfused runs (no layer kernel at all) the plain
    # GEMM that serves Phase I and both Phase-III products, three launches per layer
    if per_class["phase3"]["launches_per_step"]:
        grouped = net.memory_stats()["phase3_group_width"]
        dom, dom_flops, dom_name = "phase3", class_flops["phase3"], (
            ("task_pair_kernel_resident<GroupedVijpTask, GroupedDwTask> (Phase-III launch: one layer position of up to %d "
             "stretches side by side = recompute + vijp + epilogue each, plus the weight-gradient GEMMs of the position "
             "before)" % grouped) if grouped > 1 else
            "task_pair_kernel (Phase-III launch: layer kernel = recompute + vijp + epilogue, plus the previous "
            "layer's weight-gradient GEMM)")
    elif per_class["vijp"]["launches_per_step"]:
        dom, dom_flops, dom_name = "vijp", class_flops["vijp"], "Phase-III layer kernel"
    else:
        dom, dom_flops, dom_name = "fwd", 2.0 * per_class["fwd"]["launches_per_step"] / L, "plain NT GEMM (unfused path)"
        per_class["fwd"]["tflops"] = dom_flops * B * sum_dd / (per_class["fwd"]["ms_per_step"] * 1e-3) / 1e12
    n_v = per_class[dom]["launches_per_step"]
    avg_ms = per_class[dom]["ms_per_step"] / max(n_v, 1)
    flop_per_launch = dom_flops * B * sum_dd / max(n_v, 1)
    achieved = flop_per_launch / (avg_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma",
                "kernel": dom_name,
                "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_F32_PEAK_TFLOPS,
                "traffic": PHASE3_TRAFFIC_BYTES.get(args.config) if args.depth is None and args.reseed is None and not args.segment and dom == "phase3" and args.group == 0 else None,
                "avg_launch_ms": avg_ms, "launches": n_v * prof_steps,
                "flop_per_launch": flop_per_launch}
    # --- training step in place (gradients applied as Phase III produces them, then the right inverses
    # refreshed by two Schulz iterations): reported next to the metric, not part of it. The step size is
    # tiny so that the weights of the timed run stay where they are; the work does not depend on it.
    train = None
    if not args.unfused and not args.no_train:
        resid = torch.empty(1, dtype=torch.float32, device="cuda")
        tsteps = max(1, min(args.steps, 20))
        ms_train, _ = time_steps(lambda: net.sgd_step(net.x, net.t, 1e-7, 2, loss, resid), tsteps, 2)
        ms_apply, _ = time_steps(lambda: net.sgd_step(net.x, net.t, 1e-7, -1, loss, resid), tsteps, 2)
        ms_ref, _ = time_steps(lambda: net.refresh_incremental(2, resid), tsteps, 1)
        t0 = time.perf_counter()
        net.refresh()
        torch.cuda.synchronize()
        full_ms = (time.perf_counter() - t0) * 1e3
        train = {"ms_per_step": ms_train, "steps_per_s": 1e3 / ms_train, "refresh_iters": 2,
                 "refresh_correction_operands": args.refresh,
                 "ms_grad_and_apply": ms_apply, "ms_refresh_incremental": ms_ref, "ms_refresh_full": full_ms,
                 "residual_before_last_iteration": float(resid.item()),
                 "gradient_buffer_bytes_saved": int(net.total_floats) * 4}
    net.close()
    del net
    if train is not None and args.refresh == "bf16":
        # the same step with every product of the refresh in fp32, on a handle of its own
        net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, segment_length=args.segment,
                                           phase3_parallel_segments=args.group, phase3_overlap=bool(args.overlap))
        ms32, _ = time_steps(lambda: net.sgd_step(net.x, net.t, 1e-7, 2, loss, resid), tsteps, 2)
        ms_ref32, _ = time_steps(lambda: net.refresh_incremental(2, resid), tsteps, 1)
        train["fp32_refresh"] = {"ms_per_step": ms32, "ms_refresh_incremental": ms_ref32,
                                 "residual_before_last_iteration": float(resid.item())}
        net.close()
        del net

    # --- the library's own backprop, timed the same way on a handle of its own
    bp = {}
    if not args.no_backprop:
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        base2 = torch.cuda.memory_allocated()
        net_bp = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_BACKPROP)
        ms_bp, _ = time_steps(lambda: net_bp.backprop_grad(net_bp.x, net_bp.t, grads, loss), args.steps, args.warmup)
        st_bp = net_bp.memory_stats()
        bp = {"steps_per_s": 1e3 / ms_bp, "ms_per_step": ms_bp, "tflops": flops_bp / (ms_bp * 1e-3) / 1e12,
              "bytes_residual": st_bp["bytes_bp_activations"] + st_bp["bytes_bp_scratch"],
              "bytes_library": st_bp["bytes_live"],
              "bytes_peak_torch": torch.cuda.max_memory_allocated() - base2}
        net_bp.close()

    out = {
        "metric": "gradient steps/s (mixed-mode Moonwalk, one full moonwalk_grad per step)",
        "value": 1e3 / ms_mw, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_mw, "ms_per_step_wall": wall_mw, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic (seeded, generator: %s)" % args.gen,
        "config": {"workload": f"{wl.name}: depth {L}, widths {widths[0]}->{widths[-1]}, batch {B}, "
                               f"alpha {wl.alphas[0]}, reseed K={wl.reseed_interval}, loss_scale {wl.loss_scale:g}, "
                               f"{'unfused' if args.unfused else 'fused'} kernels"
                               + (f", segments of {args.segment} layers" if args.segment else "")
                               + (f", Phase III of up to {st['phase3_group_width']} stretches side by side"
                                  f"{' on a second stream under Phase II' if args.overlap else ''}"
                                  if st["phase3_group_width"] > 1 else "")},
        "tflops": flops_mw / (ms_mw * 1e-3) / 1e12,
        "flop_per_step": flops_mw,
        "mfma_frac_whole_step": flops_mw / (ms_mw * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS,
        "roofline": roofline,
        "per_kernel_class": per_class,
        "setup_s": setup_s,
        "memory": {
            "moonwalk": {"bytes_P": st["bytes_P"], "bytes_masks": st["bytes_masks"],
                         "bytes_fragments": st["bytes_fragments"], "bytes_frag_index": st["bytes_frag_index"],
                         "bytes_checkpoints": st["bytes_checkpoints"], "bytes_scratch": st["bytes_mw_scratch"],
                         "bytes_residual": st["bytes_masks"] + st["bytes_fragments"] + st["bytes_frag_index"]
                                           + st["bytes_checkpoints"] + st["bytes_mw_scratch"],
                         "bytes_library": mw_peak_lib, "bytes_setup_peak": st["bytes_setup_peak"],
                         "bytes_peak_torch": mw_peak_torch},
            "backprop": {k: v for k, v in bp.items() if k.startswith("bytes")},
        },
        "backprop": {k: v for k, v in bp.items() if not k.startswith("bytes")},
    }
    if train is not None:
        out["train_step"] = train
    if not args.no_cpu_baseline and args.gen == "numpy":
        out["cpu_baseline"] = cpu_baseline(wl, flops_mw)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
