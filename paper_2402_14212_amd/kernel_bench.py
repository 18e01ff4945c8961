#!/usr/bin/env python3
"""Kernel-level microbenchmarks of libmoonwalk on one MI355X.

    python -m paper_2402_14212_amd.kernel_bench gemm          # fp32 MFMA GEMMs at the layer shapes
    python -m paper_2402_14212_amd.kernel_bench elementwise   # HBM-bound elementwise / pack / compaction kernels
    python -m paper_2402_14212_amd.kernel_bench fill          # load-only model of the tiled products: operand-panel fill rate
    python -m paper_2402_14212_amd.kernel_bench all
    python -m paper_2402_14212_amd.kernel_bench one --op nt --tile 3 --m 256 --n 1024 --k 1024   # one GEMM, for counter runs

Every kernel is launched `--iters` times back to back between two events on the current stream;
the figure printed is the mean time per launch (launch gaps included, so short kernels read
pessimistically). GEMM rates are against the 157.3 TFLOP/s fp32 matrix peak, elementwise rates
are ALGORITHMIC bytes (what the step has to move, stated per kernel below) over the time, against
8 TB/s. Elementwise tensors are cycled through a pool larger than the 256 MiB last-level cache,
so the bytes really come from HBM.
"""
import argparse
import sys

import numpy as np
import torch

import paper_2402_14212_amd as mw

MFMA_PEAK = 157.3e12
HBM_PEAK = 8.0e12


def timed(fn, iters, warmup=3):
    for _ in range(warmup):
        fn(0)
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for i in range(iters):
        fn(i)
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / iters * 1e-3      # seconds per launch


GEMM_SHAPES = [
    # (label, op, M, N, K)  -- forward/vijp (NT), reverse (NN), weight gradient (TN) per configuration
    ("deep_square fwd", mw.GEMM_NT, 256, 1024, 1024), ("deep_square rev", mw.GEMM_NN, 256, 1024, 1024),
    ("deep_square dW", mw.GEMM_TN, 1024, 1024, 256),
    ("narrowing fwd", mw.GEMM_NT, 512, 3968, 4096), ("narrowing rev", mw.GEMM_NN, 512, 4096, 3968),
    ("narrowing dW", mw.GEMM_TN, 3968, 4096, 512),
    ("relu_frag fwd", mw.GEMM_NT, 512, 2048, 2048), ("relu_frag rev", mw.GEMM_NN, 512, 2048, 2048),
    ("relu_frag dW", mw.GEMM_TN, 2048, 2048, 512),
    ("very_deep fwd", mw.GEMM_NT, 1024, 4096, 4096), ("very_deep rev", mw.GEMM_NN, 1024, 4096, 4096),
    ("very_deep dW", mw.GEMM_TN, 4096, 4096, 1024),
    ("square 4096", mw.GEMM_NT, 4096, 4096, 4096),
]
TILES = {0: "auto", 1: "128x128", 2: "64x64", 3: "32x32 K/4", 4: "32x32 K/8", 5: "64x64 K/2", 6: "128x128 w8", 7: "64x128 w8"}


def bench_gemm(iters):
    print(f"{'shape':18s} {'M':>5s} {'N':>5s} {'K':>5s} {'tile':>10s} {'us':>9s} {'TFLOP/s':>8s} {'of peak':>8s}")
    for label, op, M, N, K in GEMM_SHAPES:
        if op == mw.GEMM_NT:
            A, B = torch.randn(M, K, device="cuda"), torch.randn(N, K, device="cuda")
        elif op == mw.GEMM_NN:
            A, B = torch.randn(M, K, device="cuda"), torch.randn(K, N, device="cuda")
        else:
            A, B = torch.randn(K, M, device="cuda"), torch.randn(K, N, device="cuda")
        C = torch.empty(M, N, device="cuda")
        for tile in TILES:
            t = timed(lambda i: mw.gemm_f32(op, A, B, C_out=C, tile=tile), iters)
            tf = 2.0 * M * N * K / t
            print(f"{label:18s} {M:5d} {N:5d} {K:5d} {TILES[tile]:>10s} {t * 1e6:9.1f} {tf / 1e12:8.2f} {tf / MFMA_PEAK:8.1%}",
                  flush=True)


def bench_elementwise(iters, max_log2):
    print(f"{'kernel':26s} {'elements':>11s} {'B/elt':>7s} {'us':>9s} {'GB/s':>8s} {'of 8 TB/s':>9s}")
    d = 4096
    for log2n in range(18, max_log2 + 1, 2):
        n = 1 << log2n
        rows = n // d if n >= d else 1
        dd = d if n >= d else n
        pool = max(2, min(16, (1 << 30) // (n * 4)))      # >= 1 GiB of distinct inputs when they are large
        zs = [torch.randn(rows, dd, device="cuda") for _ in range(pool)]
        hs = [torch.randn(rows, dd, device="cuda") for _ in range(pool)]
        bias = torch.randn(dd, device="cuda")
        x = torch.empty(rows, dd, device="cuda")
        y = torch.empty(rows, dd, device="cuda")
        lib = mw.load_library()
        stream = torch.cuda.current_stream().cuda_stream
        n_words = (n + 63) // 64
        mask = torch.zeros(n_words, dtype=torch.int64, device="cuda")
        off = torch.empty(n_words + 1, dtype=torch.int32, device="cuda")
        frag = torch.empty(n, dtype=torch.float32, device="cuda")
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        scratch = torch.empty(int(lib.mw_loss_scratch_doubles()), dtype=torch.float64, device="cuda")
        loss = torch.empty(1, device="cuda")
        cswork = torch.empty(int(lib.mw_colsum_work_floats(128)), dtype=torch.float32, device="cuda")
        P = lambda t: t.data_ptr()

        def report(name, bytes_per_elt, t):
            bw = bytes_per_elt * n / t
            print(f"{name:26s} {n:11d} {bytes_per_elt:7.3f} {t * 1e6:9.1f} {bw / 1e9:8.0f} {bw / HBM_PEAK:9.1%}", flush=True)

        # plain copy: the yardstick (4 B read + 4 B written per element)
        report("copy", 8.0, timed(lambda i: lib.mw_copy_f32(P(zs[i % pool]), P(x), n, stream), iters))
        # Phase I epilogue: read z, write x, write 1 bit
        report("bias_act_mask", 8.125,
               timed(lambda i: lib.mw_bias_act_mask(P(zs[i % pool]), P(bias), rows, dd, 0.1, P(x), P(mask), stream), iters))
        # Phase II scaling: read h and 1 bit, write ct_z
        report("rev_scale", 8.125, timed(lambda i: lib.mw_rev_scale(P(hs[i % pool]), P(mask), n, 0.1, P(x), stream), iters))
        # fragment index (integer scan over the mask words only)
        if n <= (1 << 28):   # fragment kernels (the largest layer of the configurations has B * d = 2^22)
            swork = torch.empty(int(lib.mw_frag_offsets_work_words(n)), dtype=torch.int32, device="cuda")
            lib.mw_frag_offsets(P(mask), n, P(off), P(swork), stream)
            report("frag_offsets", 0.125 + 0.0625,
                   timed(lambda i: lib.mw_frag_offsets(P(mask), n, P(off), P(swork), stream), iters))
            # compaction: read h, 1 bit, offsets; write the erased half
            frac0 = 1.0 - float(torch.mean((zs[0] > 0).float()))
            report("frag_compact", 4 + 0.125 + 0.0625 + 4 * frac0,
                   timed(lambda i: lib.mw_frag_compact(P(hs[i % pool]), P(mask), P(off), n, P(frag), n, P(flag), stream), iters))
            # Phase III epilogue, ReLU: read z, ct_z, mask, offsets, erased half; write x, h, ct_z
            report("vijp_epilogue relu", 4 + 4 + 0.125 + 0.0625 + 4 * frac0 + 12,
                   timed(lambda i: lib.mw_vijp_epilogue(P(zs[i % pool]), P(hs[i % pool]), rows, dd, 0.0, P(mask), P(off),
                                                        P(frag), P(x), P(y), stream), iters))
        # Phase III epilogue, leaky: read z and ct_z, write x and h
        report("vijp_epilogue leaky", 16.0,
               timed(lambda i: lib.mw_vijp_epilogue(P(zs[i % pool]), P(hs[i % pool]), rows, dd, 0.1, None, None, None,
                                                    P(x), P(y), stream), iters))
        report("colsum", 4.0, timed(lambda i: lib.mw_colsum(P(hs[i % pool]), rows, dd, 1.0, P(bias), stream), iters))
        # the tall-matrix form (bias gradient of a convolutional layer): as many rows as fit 128 columns
        report("colsum tall, 128 columns", 4.0,
               timed(lambda i: lib.mw_colsum_wide(P(hs[i % pool]), n // 128, 128, 1.0, P(bias), P(cswork), stream), iters))
        report("loss_grad", 12.0,
               timed(lambda i: lib.mw_loss_grad(P(zs[i % pool]), P(hs[i % pool]), rows, dd, 1.0, P(x), P(loss), P(scratch),
                                                stream), iters))
        del zs, hs


def bench_fill(iters):
    """Operand-panel fill rate: every workgroup of a tile x tile output tiling reads its two K-long
    row panels and computes nothing. Bytes = what the workgroups load, (M/tile)(N/tile) * 2 tile K 4.
    Each timed call launches the kernel 32 times inside the library (the operands stay in the L2
    caches / Infinity Cache: what is measured is the path into the CUs, not HBM)."""
    reps = 32
    print(f"{'shape':22s} {'tile':>5s} {'WGs':>6s} {'us':>8s} {'MB loaded':>10s} {'TB/s':>7s} {'B/clk/CU':>9s}")
    for (M, N, K) in [(256, 1024, 1024), (512, 2048, 2048), (1024, 4096, 4096)]:
        A, B = torch.randn(M, K, device="cuda"), torch.randn(N, K, device="cuda")
        for tile in (16, 32, 64):
            wgs = (M // tile) * (N // tile)
            sink = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
            loaded = wgs * 2 * tile * K * 4
            t = timed(lambda i: mw.probe_operand_stream(A, B, tile, sink, repeats=reps), max(4, iters // 4)) / reps
            print(f"{M:5d}x{N:5d}x{K:5d}     {tile:5d} {wgs:6d} {t * 1e6:8.2f} {loaded / 1e6:10.1f} {loaded / t / 1e12:7.2f} "
                  f"{loaded / t / 256 / 2.4e9:9.1f}", flush=True)


def bench_one(args):
    op = {"nt": mw.GEMM_NT, "nn": mw.GEMM_NN, "tn": mw.GEMM_TN}[args.op]
    M, N, K = args.m, args.n, args.k
    A = torch.randn((K, M) if op == mw.GEMM_TN else (M, K), device="cuda")
    B = torch.randn((N, K) if op == mw.GEMM_NT else (K, N), device="cuda")
    C = torch.empty(M, N, device="cuda")
    t = timed(lambda i: mw.gemm_f32(op, A, B, C_out=C, tile=args.tile), args.iters)
    tf = 2.0 * M * N * K / t
    print(f"{args.op} M={M} N={N} K={K} tile={TILES[args.tile]}: {t * 1e6:.1f} us/launch, {tf / 1e12:.2f} TFLOP/s "
          f"({tf / MFMA_PEAK:.1%} of the fp32 MFMA peak)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["gemm", "elementwise", "fill", "all", "one"])
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--max-log2", type=int, default=28, help="largest elementwise tensor, log2(elements)")
    ap.add_argument("--op", choices=["nt", "nn", "tn"], default="nt")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--m", type=int, default=256)
    ap.add_argument("--n", type=int, default=1024)
    ap.add_argument("--k", type=int, default=1024)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("kernel_bench needs a GPU")
    print(f"# device: {torch.cuda.get_device_name(0)}; iters={args.iters}", flush=True)
    if args.what == "one":
        bench_one(args)
    if args.what in ("gemm", "all"):
        bench_gemm(args.iters)
    if args.what in ("fill", "all"):
        bench_fill(args.iters)
    if args.what in ("elementwise", "all"):
        bench_elementwise(args.iters, args.max_log2)


if __name__ == "__main__":
    main()
