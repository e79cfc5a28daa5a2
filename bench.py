#!/usr/bin/env python3
"""Benchmark of the block-sparse convolution hot path on one MI355X.

A step is one launch of bsp_conv2d (activation staging, gathered block-row
contraction, bias epilogue) on one batch of the named workload, inputs and the
packed weights already resident in HBM.  Packing (host, once per layer) is
timed separately and reported as ``pack_ms``.  Prints ONE JSON line.

  python bench.py [--steps K] [--warmup W] [--workload c1|c2|...]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
# HBM bytes per launch of the dispatcher's kernel for the default workload, from two
# rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE), each scaled by the same
# counter's reading for a device copy of known size; the summary names the commit it was
# taken at (profiles/conv_band3_bf16_c1.md)
MEASURED_TRAFFIC = {"c1": {"bytes": 26_250_297, "commit": "4633f0f"}}


def measured_peaks(dev):
    """What this GPU sustains: a stream copy through HBM (GB/s, read + write) and a loop of
    independent bf16 MFMAs on register operands (TFLOP/s), each the best of a few launches."""
    import torch
    import paper_2407_09453_amd as bsp
    st = torch.cuda.current_stream(dev)
    n = 512 << 20
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    src.fill_(1)
    sink = torch.zeros(8192, dtype=torch.float32, device=dev)
    waves, iters = 8192, 2000

    def best(fn, reps=5):
        out = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(st)
            fn()
            b.record(st)
            torch.cuda.synchronize()
            out.append(a.elapsed_time(b))
        return min(out)

    copy_ms = best(lambda: bsp.bsp_bench_copy(dst.data_ptr(), src.data_ptr(), n, st.cuda_stream))
    mfma_ms = best(lambda: bsp.bsp_bench_mfma_bf16(sink.data_ptr(), waves, iters, None, st.cuda_stream))
    del src, dst
    return {"hbm_copy_GBs": round(2 * n / copy_ms / 1e6, 1),
            "mfma_bf16_TFLOPs": round(waves * iters * 8 * 16384 / mfma_ms / 1e9, 1)}


def time_launches(launch, steps, warmup, dev, use_graph=True):
    """Average time of one step, ms: `steps` back-to-back calls of launch(i, stream) timed
    between synchronisations (wall clock) and with HIP events on the launch stream.  With
    use_graph the calls are captured once into a HIP graph on a side stream and the graph
    is replayed: what remains between kernels is the GPU's own dispatch, not the Python loop;
    the `warmup` untimed steps are then whole replays (rounded up to a multiple of `steps`)."""
    import torch
    # (at least one launch outside the capture: a kernel's first launch sets attributes that a
    # capture does not record)
    for i in range(max(1, min(warmup, 20)) if use_graph else warmup):
        launch(i, None)
    torch.cuda.synchronize()
    if use_graph:
        side = torch.cuda.Stream(device=dev)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    launch(i, side.cuda_stream)
        torch.cuda.synchronize()
        # the warm-up steps are replays of the same graph, right before the timed one: capturing
        # takes the host milliseconds in which the GPU idles, and warm-up done before it is lost
        # (the GPU reaches its sustained state only after tens of milliseconds under load)
        for _ in range(max(1, -(-warmup // max(steps, 1)))):
            graph.replay()
        torch.cuda.synchronize()
        run = graph.replay
    else:
        def run():
            for i in range(steps):
                launch(i, None)
    stream = torch.cuda.current_stream(dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t = time.perf_counter()
    e0.record(stream)
    run()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t
    return wall * 1e3 / steps, e0.elapsed_time(e1) / steps


def algorithmic_bytes(c, nnzb: int) -> int:
    """Bytes the method itself must move for one launch: X read once, Y written
    once, kept blocks + indices + bias read once."""
    es = 4 if c.dtype == "f32" else 2
    nbr = -(-c.O // c.bo)
    return (c.B * c.L * c.J * c.I * es + c.P * c.O * es
            + nnzb * c.bo * c.bi * c.H * c.K * es + 4 * (nnzb + nbr + 1) + 4 * c.O)


def flops_nonzero(c, nnzb: int) -> int:
    return 2 * c.P * nnzb * c.bo * c.bi * c.H * c.K


def pick_case(name: str):
    from synthetic import config_cases
    if name == "c1":
        return next(config_cases(1)), "config1: conv3x3 s1 p1, X 32x56x56x64 NHWC bf16, W 64x3x3x64, 8x8 blocks, 32 of 64 kept"
    if name == "c0":
        return next(config_cases(0)), "config0: FC fp32 64x256 -> 256, 8x8 blocks, Bernoulli(0.5)"
    if name.startswith("c2"):
        want = name[3:] if len(name) > 3 else "8x8.d0.5"
        for c in config_cases(2):
            if c.name.endswith(want):
                return c, f"config2: conv1x1 256->1024 @14x14 batch 32 bf16, {want}"
    if ":" in name:      # one layer of a network-shaped stack, e.g. resnet50:layer3.1.conv2
        net, lname = name.split(":", 1)
        cfg = 3 if net == "resnet50" else 4
        for c in config_cases(cfg):
            if c.meta.get("net") == net and c.name == lname:
                return c, (f"{net} {lname}: conv{c.H}x{c.K} s{c.stride[0]} {c.I}->{c.O} on "
                           f"{c.B}x{c.L}x{c.J}, 8x8 blocks, half kept")
    raise SystemExit(f"unknown workload {name}")


def bench_i8(args) -> int:
    """Config 1's shape as an 8-bit integer layer: weights quantized by Eq. (8), int8
    activations, int32 bias, int8 output after a power-of-two rescale."""
    import torch
    import paper_2407_09453_amd as bsp
    from synthetic import config_cases

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    c = next(config_cases(1))
    rng = np.random.default_rng(240709453 + 1001)
    Wq, delta = bsp.bsp_quantize(c.W)
    Xq = np.clip(np.rint(c.X * 32.0), -128, 127).astype(np.int8)      # N(0,1) at scale 2^-5
    bias = rng.integers(-2 ** 12, 2 ** 12, c.O).astype(np.int32)
    shift = 9
    layer = bsp.BspLayerI8(Wq, c.gamma, c.bo, c.bi, bias=bias)
    dense = bsp.BspLayerI8(Wq, np.ones_like(c.gamma), c.bo, c.bi, bias=bias)
    nbr = -(-c.O // c.bo)
    nbytes = (Xq.size + c.P * c.O + layer.nnzb * c.bo * c.bi * c.H * c.K
              + 4 * (layer.nnzb + nbr + 1) + 4 * c.O)
    nsets = args.sets or max(2, int(np.ceil(300e6 / nbytes)))
    X0 = torch.from_numpy(Xq).to(dev)
    Xs = [X0] + [X0.clone() for _ in range(nsets - 1)]
    Ys = [torch.empty(layer.out_shape(c.B, c.L, c.J, c.stride, c.pad), dtype=torch.int8, device=dev)
          for _ in range(nsets)]
    stream = torch.cuda.current_stream(dev)

    def timed(lay):
        def launch(i, st):
            lay.conv2d(Xs[i % nsets], c.stride, c.pad, shift=shift, out=Ys[i % nsets], stream=st)
        return time_launches(launch, args.steps, args.warmup, dev, use_graph=args.graph)

    ms_wall, ms_ev = timed(layer)
    ms_wall_d, _ = timed(dense)
    ops = 2 * c.P * layer.nnzb * c.bo * c.bi * c.H * c.K
    achieved = nbytes / (ms_ev * 1e-3) / 1e9
    out = {
        "metric": "effective nonzero TOP/s (2*P*nnzb*bo*bi*H*K / t), 50% 8x8 block-sparse int8 conv",
        "value": round(ops / (ms_wall * 1e-3) / 1e12, 4), "unit": "TOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_wall, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i8",
        "data": "synthetic",
        "config": {"workload": "config1's shape as an int8 layer: conv3x3 s1 p1, X 32x56x56x64 "
                               "int8, W 64x3x3x64 int8 codes (Eq. 8), int32 bias, int8 out >> 9",
                   "block": "8x8", "nnzb": layer.nnzb, "buffer_sets": nsets,
                   "kernel": "dispatch", "delta": delta},
        "speedup_vs_dense_mask": None if ms_wall_d is None else round(ms_wall_d / ms_wall, 4),
        "dense_mask_ms_per_step": None if ms_wall_d is None else round(ms_wall_d, 6),
        "event_ms_per_step": round(ms_ev, 6),
        "timing": ("K launches captured into one HIP graph, one replay timed between synchronisations"
                   if args.graph else "K launches issued from the Python loop"),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": None,
                     "algorithmic_bytes": int(nbytes)},
        "int8_mfma_frac_of_peak": round(ops / (ms_ev * 1e-3) / 1e12 / 5000.0, 5),
    }
    if not args.no_cpu_baseline:
        import oracle
        reps, dt = 0, 0.0
        while reps < 12 and dt * 16 < 12.0:
            t = time.perf_counter()
            oracle.conv2d_i8(Xq, Wq, bias, c.gamma, c.bo, c.bi, c.stride, c.pad, shift=shift)
            dt += time.perf_counter() - t
            reps += 1
        out["cpu_baseline"] = {"value": round(ops * reps / dt / 1e12, 6), "unit": "TOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": f"the full workload {reps} times ({dt:.2f} s wall); the integer "
                                         "oracle takes the dense masked sum exactly and skips nothing"}
    print(json.dumps(out))
    return 0


def bench_spgemm(args) -> int:
    """Block-sparse x block-sparse product (Section III-A): square operands of 4096 x 4096 bf16
    in 8x8 blocks, each with a Bernoulli(0.5) block mask; C = (Gamma A)(Omega B)^t in fp32."""
    import torch
    import paper_2407_09453_amd as bsp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    n = 512                                    # block rows = block columns
    rng = np.random.default_rng(240709453 + 9000)
    A = rng.standard_normal((n * 8, n * 8)).astype(np.float32).view(np.uint32)
    B = rng.standard_normal((n * 8, n * 8)).astype(np.float32).view(np.uint32)
    A = (A & np.uint32(0xFFFF0000)).view(np.float32)      # onto the bf16 grid
    B = (B & np.uint32(0xFFFF0000)).view(np.float32)
    gamma = (rng.random((n, n)) < 0.5).astype(np.uint8)
    omega = (rng.random((n, n)) < 0.5).astype(np.uint8)
    Am, Bm = bsp.BspMatrix(A, gamma), bsp.BspMatrix(B, omega)
    ones = np.ones((n, n), dtype=np.uint8)
    Ad, Bd = bsp.BspMatrix(A, ones), bsp.BspMatrix(B, ones)
    C = torch.empty((n * 8, n * 8), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()

    def timed(x, y):
        def launch(i, st):
            x.matmul_nt(y, out=C, stream=st)
        return time_launches(launch, args.steps, args.warmup, torch.device("cuda:0"),
                             use_graph=args.graph)

    ms, ms_ev = timed(Am, Bm)
    ms_d, _ = timed(Ad, Bd)
    quarter = (rng.random((n, n)) < 0.25).astype(np.uint8), (rng.random((n, n)) < 0.25).astype(np.uint8)
    ms_q, _ = timed(bsp.BspMatrix(A, quarter[0]), bsp.BspMatrix(B, quarter[1]))
    pairs = int((gamma.astype(np.int64) @ omega.astype(np.int64).T).sum())
    flops = 2 * 512 * pairs                                   # 8x8x8 multiply-adds per block pair
    nbytes = (Am.nnzb + Bm.nnzb) * (128 + 4) + Am.seg_ptr.nbytes + Bm.seg_ptr.nbytes + C.numel() * 4
    out = {
        "metric": "effective TFLOP/s of the block-sparse x block-sparse product (2*8^3 per matching block pair)",
        "value": round(flops / (ms * 1e-3) / 1e12, 4), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "C = (Gamma A)(Omega B)^t, A and B 4096x4096 bf16 in 8x8 blocks, "
                               "Bernoulli(0.5) masks, C fp32", "matching_block_pairs": pairs,
                   "nnzb_a": Am.nnzb, "nnzb_b": Bm.nnzb},
        "speedup_vs_dense_mask": round(ms_d / ms, 4), "dense_mask_ms_per_step": round(ms_d, 6),
        "quarter_density_ms_per_step": round(ms_q, 6),
        "event_ms_per_step": round(ms_ev, 6),
        "timing": "one HIP graph of K launches" if args.graph else "K launches from the Python loop",
        "roofline": {"bound": "mfma", "achieved": round(flops / (ms_ev * 1e-3) / 1e12, 3),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (ms_ev * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5),
                     "traffic": None, "algorithmic_bytes": int(nbytes)},
    }
    if not args.no_cpu_baseline:
        import oracle
        m = n                                     # the whole problem: a masked fp64 matmul
        t = time.perf_counter()
        oracle.spgemm_nt(A[:m * 8], gamma[:m], B[:m * 8], omega[:m], 8)
        dt = time.perf_counter() - t
        sub = int((gamma[:m].astype(np.int64) @ omega[:m].astype(np.int64).T).sum())
        out["cpu_baseline"] = {"value": round(2 * 512 * sub / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": f"the first {m} block rows of A against the first {m} of B "
                                         f"({dt:.2f} s; masked dense fp64 matmul, nothing skipped)"}
    print(json.dumps(out))
    return 0


def bench_bottleneck(args) -> int:
    """ResNet50-shaped bottlenecks (layer1: 256 -> 64 -> 256 on 56x56, layer2: 512 -> 128 -> 512 on
    28x28, layer3: 1024 -> 256 -> 1024 on 14x14; batch 32, 8x8 blocks, half kept): bsp_bottleneck, which keeps the two
    intermediates in LDS, against the same three layers launched one by one."""
    import torch
    import paper_2407_09453_amd as bsp
    from synthetic import draw_layer

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(2407)
    out = []
    for name, (B, L, J, I, C, O) in (("layer1", (32, 56, 56, 256, 64, 256)),
                                     ("layer2", (32, 28, 28, 512, 128, 512)),
                                     ("layer3", (32, 14, 14, 1024, 256, 1024))):
        specs = ((I, C, 1, 0), (C, C, 3, 1), (C, O, 1, 0))
        cs = [draw_layer(f"{name}.{k}", B=1, L=3, J=3, I=i, O=o, H=h, K=h, pad=p, dtype="bf16",
                         mask_kind="exact", density=0.5, seed=7700 + k, b_std=0.3)
              for k, (i, o, h, p) in enumerate(specs)]
        ls = [bsp.BspLayer(c.W, c.gamma, 8, 8, "bf16", bias=c.bias) for c in cs]
        nb = 3
        Xs = [torch.randn((B, L, J, I), device=dev, generator=gen).to(torch.bfloat16) for _ in range(nb)]
        Ys = [torch.empty((B, L, J, O), dtype=torch.bfloat16, device=dev) for _ in range(nb)]
        T1 = torch.empty((B, L, J, C), dtype=torch.bfloat16, device=dev)
        T2 = torch.empty_like(T1)

        def fused(i, st):
            bsp.bottleneck(ls[0], ls[1], ls[2], Xs[i % nb], residual=Xs[i % nb], relu=True,
                           out=Ys[i % nb], stream=st, force=True)

        def separate(i, st):
            ls[0].conv2d(Xs[i % nb], out=T1, relu=True, stream=st)
            ls[1].conv2d(T1, (1, 1), (1, 1), out=T2, relu=True, stream=st)
            ls[2].conv2d(T2, out=Ys[i % nb], residual=Xs[i % nb], relu=True, stream=st)

        res = {}
        for key, fn in (("fused", fused), ("separate", separate)):
            ts = [time_launches(fn, args.steps, args.warmup, dev)[1] * 1e3 for _ in range(5)]
            res[key] = float(np.median(ts))
        P = B * L * J
        flops = 2 * P * sum(l.nnzb * 64 * c.H * c.K for l, c in zip(ls, cs))
        wbytes = sum(l.nnzb * 128 * c.H * c.K for l, c in zip(ls, cs))
        # one read of X (also the residual), one write of Y; separately T1 and T2 also go out and back
        by_fused = P * (I + O) * 2 + wbytes
        by_sep = P * (I + 2 * C + 2 * C + O + O) * 2 + wbytes
        floor = max(flops / (MFMA_BF16_PEAK_TFLOPS * 1e12), by_fused / (HBM_PEAK_GBS * 1e9)) * 1e6
        out.append({"block": name, "shape": f"{I}->{C}->{O} on {B}x{L}x{J}",
                    "fused_us": round(res["fused"], 2), "separate_us": round(res["separate"], 2),
                    "speedup": round(res["separate"] / res["fused"], 3),
                    "TFLOPs_nz": round(flops / res["fused"] / 1e6, 2),
                    "algorithmic_MB_fused": round(by_fused / 1e6, 2),
                    "algorithmic_MB_separate": round(by_sep / 1e6, 2),
                    "floor_us": round(floor, 2), "roofline_frac": round(floor / res["fused"], 4)})
    b1 = out[0]
    print(json.dumps({
        "metric": "effective nonzero TFLOP/s of a fused ResNet50 layer1 bottleneck (1x1 -> 3x3 -> 1x1 + residual)",
        "value": b1["TFLOPs_nz"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(b1["fused_us"] / 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ResNet50-shaped bottlenecks, batch 32, 8x8 blocks, half kept; "
                               "one launch with the intermediates in LDS against three launches"},
        "roofline": {"bound": "hbm", "achieved": round(b1["algorithmic_MB_fused"] / b1["fused_us"] * 1e3, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(b1["algorithmic_MB_fused"] / b1["fused_us"] * 1e3 / HBM_PEAK_GBS, 5),
                     "traffic": None},
        "blocks": out}))
    return 0


def union_ratio(layer):
    """Contraction units the strips of a layer run over the units in kept blocks (1.0 = work
    exactly proportional to the kept blocks), from the plan's row-band section; None without one."""
    plan = layer.plan
    off = int(plan[24])
    if off == 0:
        return None
    # kept counts every block row's units, union every strip's: a strip's units are multiplied
    # with all 16 / bo block rows of the strip
    kept, union = int(plan[off + 12]), int(plan[off + 13]) * (16 // layer.bo)
    return round(union / kept, 4) if kept > 0 else None


def bench_union(args) -> int:
    """Issued / kept contraction units of the strips for the three kinds of mask (50 % of 8x8
    blocks kept) on ResNet50-shaped layers; 16x4 blocks for comparison.  Host only."""
    import paper_2407_09453_amd as bsp
    from synthetic import draw_layer
    shapes = [("3x3 64->64", 64, 64, 3), ("3x3 256->256", 256, 256, 3), ("3x3 512->512", 512, 512, 3),
              ("1x1 256->1024", 256, 1024, 1), ("1x1 1024->256", 1024, 256, 1), ("1x1 2048->512", 2048, 512, 1)]
    rows = []
    for name, I, O, H in shapes:
        row = {"layer": name}
        for kind in ("exact", "row_balanced", "select_l2", "16x4"):
            bo, bi = (16, 4) if kind == "16x4" else (8, 8)
            c = draw_layer(name, B=1, L=3, J=3, I=I, O=O, H=H, K=H, pad=H // 2, bo=bo, bi=bi, dtype="bf16",
                           mask_kind="row_balanced" if kind == "row_balanced" else "exact", density=0.5,
                           seed=4242, draw_x=False)
            gamma = bsp.bsp_select_mask(c.W, bo, bi, 0, 0.5) if kind == "select_l2" else c.gamma
            rp, ci, pl = bsp.bsp_pack(c.W, gamma, bo, bi, bsp.BSP_BF16)
            plan = bsp.bsp_plan_build(rp, ci, pl, O, H, H, I, bo, bi)
            off = int(plan[24])
            row[kind] = round(int(plan[off + 13]) * (16 // bo) / max(1, int(plan[off + 12])), 4)
        rows.append(row)
        print(row, file=sys.stderr)
    print(json.dumps({"metric": "issued / kept contraction units of the plan's strips at 50 % density",
                      "value": rows[1]["exact"], "unit": "ratio", "n_gpus": 1, "steps": 0, "warmup": 0,
                      "ms_per_step": None, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
                      "dtype": "bf16", "data": "synthetic", "config": {"workload": "plan builder, host only"},
                      "rows": rows}))
    return 0


def network_rows(args, net: str, peaks, reps: int = 20):
    """Per-layer timing of a whole network-shaped stack: every layer on its own resident
    N(0,1) input (layers are independent: glue such as pooling is not part of the path), the
    kept-block mask and the all-ones mask through the same dispatcher.  Each layer is timed
    as `reps` back-to-back launches replayed from a HIP graph over three rotating buffer sets
    (median of five replays).  Returns one row per layer with the layer's roofline floor
    (published peaks), the fraction reached, and the ceiling on the speed-up over the
    all-ones mask that the measured sustained peaks allow."""
    import torch
    import paper_2407_09453_amd as bsp
    from synthetic import config_cases

    dev = torch.device("cuda:0")
    cfg = 3 if net == "resnet50" else 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(2407)
    F = peaks["mfma_bf16_TFLOPs"] * 1e12
    BW = peaks["hbm_copy_GBs"] * 1e9
    rows = []
    for c in config_cases(cfg, draw_x=False):
        if c.meta.get("net") != net:
            continue
        sparse = bsp.BspLayer(c.W, c.gamma, c.bo, c.bi, c.dtype, bias=c.bias)
        dense = bsp.BspLayer(c.W, np.ones_like(c.gamma), c.bo, c.bi, c.dtype, bias=c.bias)
        nb = 3
        Xs = [torch.randn((c.B, c.L, c.J, c.I), device=dev, generator=gen).to(torch.bfloat16)
              for _ in range(nb)]
        Ys = [torch.empty(sparse.out_shape(c.B, c.L, c.J, c.stride, c.pad), dtype=torch.bfloat16,
                          device=dev) for _ in range(nb)]
        res = {}
        for name, lay in (("sparse", sparse), ("dense", dense)):
            def launch(i, st, lay=lay):
                lay.conv2d(Xs[i % nb], c.stride, c.pad, out=Ys[i % nb], general=args.general, stream=st)
            ts = [time_launches(launch, reps, 2, dev)[1] * 1e3 for _ in range(5)]
            res[name] = float(np.median(ts))

        def launch_hot(i, st):   # the same buffers every time: X and Y stay in the caches
            sparse.conv2d(Xs[0], c.stride, c.pad, out=Ys[0], general=args.general, stream=st)
        res["hot"] = float(np.median([time_launches(launch_hot, reps, 2, dev)[1] * 1e3 for _ in range(3)]))
        fl = flops_nonzero(c, sparse.nnzb)
        fl_d = flops_nonzero(c, int(c.gamma.size))
        by = algorithmic_bytes(c, sparse.nnzb)
        by_d = algorithmic_bytes(c, int(c.gamma.size))
        floor_us = max(fl / (MFMA_BF16_PEAK_TFLOPS * 1e12), by / (HBM_PEAK_GBS * 1e9)) * 1e6
        bound = "mfma" if fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) > by / (HBM_PEAK_GBS * 1e9) else "hbm"
        ceiling = max(fl_d / F, by_d / BW) / max(fl / F, by / BW)
        rows.append({"layer": c.name, "I": c.I, "O": c.O, "HxK": f"{c.H}x{c.K}", "in": f"{c.L}x{c.J}",
                     "stride": c.stride[0], "nnzb": sparse.nnzb, "blocks": int(c.gamma.size),
                     "us": round(res["sparse"], 2), "us_dense_mask": round(res["dense"], 2),
                     "us_hot": round(res["hot"], 2), "issued_over_kept": union_ratio(sparse),
                     "speedup": round(res["dense"] / res["sparse"], 3),
                     "speedup_ceiling": round(ceiling, 3),
                     "TFLOPs_nz": round(fl / res["sparse"] / 1e6, 2),
                     "GBs": round(by / res["sparse"] / 1e3, 1), "bound": bound,
                     "floor_us": round(floor_us, 2), "roofline_frac": round(floor_us / res["sparse"], 4),
                     "flops_nz": fl, "bytes": by})
        del sparse, dense, Xs, Ys
    return rows


def network_summary(rows):
    tot = sum(r["us"] for r in rows)
    totd = sum(r["us_dense_mask"] for r in rows)
    fl = sum(r["flops_nz"] for r in rows)
    floor = sum(r["floor_us"] for r in rows)
    return {"layers": len(rows), "us": round(tot, 1), "us_dense_mask": round(totd, 1),
            "TFLOPs_nz": round(fl / tot / 1e6, 2), "speedup_vs_dense_mask": round(totd / tot, 4),
            "roofline_floor_us": round(floor, 1), "roofline_frac": round(floor / tot, 4)}


def bench_network(args, net: str) -> int:
    import torch
    dev = torch.device("cuda:0")
    peaks = measured_peaks(dev)
    rows = network_rows(args, net, peaks, reps=args.steps)
    print(f"{'layer':28s} {'I':>5s} {'O':>5s} {'HxK':>4s} {'in':>8s} {'us':>8s} {'dense':>8s} {'x':>6s} {'ceil':>5s} "
          f"{'TF/s':>7s} {'GB/s':>7s} {'bound':>5s} {'floor':>6s} {'frac':>6s} {'hot':>6s} {'i/k':>5s}", file=sys.stderr)
    for r in rows:
        print(f"{r['layer']:28s} {r['I']:5d} {r['O']:5d} {r['HxK']:>4s} {r['in']:>8s} {r['us']:8.1f} "
              f"{r['us_dense_mask']:8.1f} {r['speedup']:6.2f} {r['speedup_ceiling']:5.2f} {r['TFLOPs_nz']:7.1f} "
              f"{r['GBs']:7.0f} {r['bound']:>5s} {r['floor_us']:6.1f} {r['roofline_frac']:6.3f} {r['us_hot']:6.1f} "
              f"{r['issued_over_kept'] if r['issued_over_kept'] else 0:5.2f}", file=sys.stderr)
    sm = network_summary(rows)
    out = {
        "metric": "effective nonzero TFLOP/s (2*P*nnzb*bo*bi*H*K / t), 50% 8x8 block-sparse layers",
        "value": sm["TFLOPs_nz"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sm["us"] / 1e3, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{net}-shaped conv+FC stack, batch {32 if net == 'resnet50' else 16}, "
                               "8x8 blocks, half the blocks kept per layer (first conv dense)",
                   "layers": len(rows),
                   "timing": "per layer: back-to-back launches replayed from a HIP graph, median of five "
                             "replays, summed over layers"},
        "speedup_vs_dense_mask": sm["speedup_vs_dense_mask"],
        "dense_mask_ms_per_step": round(sm["us_dense_mask"] / 1e3, 6),
        "measured_peaks": peaks,
        "roofline": {"bound": "mixed", "achieved": None, "peak": None, "unit": "us",
                     "frac": sm["roofline_frac"], "traffic": None,
                     "floor_us": sm["roofline_floor_us"],
                     "note": "sum over layers of max(flops/2.5 PFLOP/s, bytes/8 TB/s) over the summed time"},
        "layers": rows,
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=3000,
                    help="untimed steps before the timed ones (default 3000, about 30 ms: the GPU "
                         "reaches its sustained state only after tens of milliseconds under load; "
                         "with 50 the same kernel reads 10-15 %% slower)")
    ap.add_argument("--workload", default="c1",
                    help="c1 (default), c0, c2:<bo>x<bi>.d<density>, c1_i8, spgemm, bottleneck, resnet50, vgg16, inception_v3, "
                         "or one layer of a stack as <net>:<layer name>")
    ap.add_argument("--sets", type=int, default=0,
                    help="distinct X/Y buffer sets cycled through (0 = enough to exceed 256 MB)")
    ap.add_argument("--mask", default="synthetic", choices=["synthetic", "l2", "l1", "var"],
                    help="synthetic: the config's seeded mask; l2/l1/var: keep the half of the "
                         "blocks with the largest importance (bsp_select_mask on the layer's W)")
    ap.add_argument("--fused", action="store_true",
                    help="time the layer with the fused residual-add + ReLU epilogue (and, for "
                         "comparison, the plain layer followed by torch's add and relu)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--general", action="store_true", help="force the general-shape kernel")
    ap.add_argument("--no-dense-mask", dest="dense_mask", action="store_false",
                    help="skip the all-ones-mask comparator (profiling runs: only the layer's own launches)")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="issue the timed launches from the Python loop instead of replaying "
                         "them from one captured HIP graph")
    ap.add_argument("--no-network-summary", dest="network_summary", action="store_false",
                    help="skip the ResNet50-shaped stack summary folded into the default line")
    ap.add_argument("--no-multi-stream", dest="multi_stream", action="store_false",
                    help="skip the extra four-stream throughput measurement")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain device copy of X (known size) a few times, so a "
                         "rocprofv3 --pmc run of this command has a reference for its byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); "
              "multi-GPU figures are not produced", file=sys.stderr)
        return 2
    if args.workload == "c1_i8":
        return bench_i8(args)
    if args.workload == "spgemm":
        if args.steps == 400:
            args.steps, args.warmup = 50, 5
        return bench_spgemm(args)
    if args.workload == "union":
        return bench_union(args)
    if args.workload == "bottleneck":
        if args.steps == 400:
            args.steps, args.warmup = 30, 5
        return bench_bottleneck(args)
    if args.workload in ("resnet50", "vgg16", "inception_v3"):
        if args.steps == 400:
            args.steps, args.warmup = 30, 5
        return bench_network(args, args.workload)

    import torch
    import paper_2407_09453_amd as bsp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    c, workload = pick_case(args.workload)
    tdt = torch.float32 if c.dtype == "f32" else torch.bfloat16

    select_ms = None
    if args.mask != "synthetic":
        t0 = time.perf_counter()
        c.gamma = bsp.bsp_select_mask(c.W, c.bo, c.bi, {"l2": 0, "l1": 1, "var": 2}[args.mask], 0.5)
        select_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    layer = bsp.BspLayer(c.W, c.gamma, c.bo, c.bi, c.dtype, bias=c.bias)
    pack_ms = (time.perf_counter() - t0) * 1e3
    dense = bsp.BspLayer(c.W, np.ones_like(c.gamma), c.bo, c.bi, c.dtype, bias=c.bias)

    nbytes = algorithmic_bytes(c, layer.nnzb)
    nsets = args.sets or max(2, int(np.ceil(300e6 / nbytes)))
    X0 = torch.from_numpy(c.X).to(tdt).to(dev)
    Xs = [X0] + [X0.clone() for _ in range(nsets - 1)]
    Ys = [torch.empty(layer.out_shape(c.B, c.L, c.J, c.stride, c.pad), dtype=tdt, device=dev)
          for _ in range(nsets)]
    stream = torch.cuda.current_stream(dev)

    Rs = [torch.randn_like(Ys[0]) for _ in range(nsets)] if args.fused else None

    def step(lay, i, st=None):
        if args.fused:
            lay.conv2d(Xs[i % nsets], c.stride, c.pad, out=Ys[i % nsets], stream=st,
                       residual=Rs[i % nsets], relu=True)
        else:
            lay.conv2d(Xs[i % nsets], c.stride, c.pad, out=Ys[i % nsets], general=args.general,
                       stream=st)

    def timed_streams(lay, steps, nstreams):
        """Same steps, issued round-robin on several default-priority streams so that
        independent batches overlap each other's launch and drain phases."""
        sts = [torch.cuda.Stream(device=dev) for _ in range(nstreams)]
        for i in range(4 * nstreams):
            step(lay, i, sts[i % nstreams].cuda_stream)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(steps):
            step(lay, i, sts[i % nstreams].cuda_stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / steps

    def timed(lay, graph):
        return time_launches(lambda i, st: step(lay, i, st), args.steps, args.warmup, dev,
                             use_graph=graph)

    def per_launch_us(lay, steps):
        """Duration of one launch from HIP events recorded on the launch stream right before
        and after it (includes the launch's own start-up and drain)."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(steps)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            a.record(stream)
            step(lay, i)
            b.record(stream)
        torch.cuda.synchronize()
        d = np.array([a.elapsed_time(b) for a, b in evs]) * 1e3
        return float(d.mean()), float(np.median(d)), float(d.min())

    # the K timed steps: replayed from a HIP graph (default) or issued from the Python loop
    ms_wall, ms_ev = timed(layer, args.graph)
    ms_wall_d, ms_ev_d = timed(dense, args.graph) if args.dense_mask else (None, None)
    ms_eager, ms_eager_ev = timed(layer, False) if args.graph else (ms_wall, ms_ev)
    k_avg, k_med, k_min = per_launch_us(layer, min(args.steps, 200))
    kd_avg = per_launch_us(dense, min(args.steps, 200))[0] if args.dense_mask else None
    peaks = measured_peaks(dev)

    ms_multi = timed_streams(layer, args.steps, 4) if args.multi_stream else None
    ms_unfused = None
    if args.fused:   # the same work as separate passes: conv, then add and relu by torch
        def unfused(i):
            y = Ys[i % nsets]
            layer.conv2d(Xs[i % nsets], c.stride, c.pad, out=y)
            y.add_(Rs[i % nsets]).relu_()
        for i in range(args.warmup):
            unfused(i)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(args.steps):
            unfused(i)
        torch.cuda.synchronize()
        ms_unfused = (time.perf_counter() - t) * 1e3 / args.steps

    fl = flops_nonzero(c, layer.nnzb)
    value = fl / (ms_wall * 1e-3) / 1e12
    # average launch duration over the timed region: HIP events on the launch stream around
    # the K back-to-back launches (what `rocprofv3 --kernel-trace --stats` reports per kernel,
    # plus the gap between consecutive launches)
    achieved = nbytes / (ms_ev * 1e-3) / 1e9
    traffic = None if args.general or args.mask != "synthetic" or args.fused \
        else MEASURED_TRAFFIC.get(args.workload)
    mfma_bound = c.dtype == "bf16" and fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) > nbytes / (HBM_PEAK_GBS * 1e9)
    if mfma_bound:   # the layer's floor is the matrix cores' (nonzero flop at the dense bf16 peak)
        ach = fl / (ms_ev * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 5), "traffic": None,
                "algorithmic_flops": fl, "algorithmic_bytes": nbytes,
                "frac_of_wall": round(fl / (ms_wall * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5),
                "frac_of_measured_mfma": round(ach / peaks["mfma_bf16_TFLOPs"], 5),
                "hbm_frac": round(achieved / HBM_PEAK_GBS, 5)}
    else:
        roof = {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": None if traffic is None else traffic["bytes"],
                "traffic_commit": None if traffic is None else traffic["commit"],
                "algorithmic_bytes": nbytes,
                "frac_of_wall": round(nbytes / (ms_wall * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
                "frac_of_measured_copy": round(achieved / peaks["hbm_copy_GBs"], 5),
                "mfma_frac_of_measured": round(fl / (ms_ev * 1e-3) / 1e12 / peaks["mfma_bf16_TFLOPs"], 5)
                if c.dtype == "bf16" else None}
    out = {
        "metric": "effective nonzero TFLOP/s (2*P*nnzb*bo*bi*H*K / t), 50% 8x8 block-sparse conv",
        "value": round(value, 4),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_wall, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": c.dtype,
        "data": "synthetic",
        "config": {"workload": workload, "block": f"{c.bo}x{c.bi}", "nnzb": layer.nnzb,
                   "density": round(layer.nnzb / c.gamma.size, 4), "buffer_sets": nsets,
                   "kernel": "general" if args.general else "dispatch"},
        "speedup_vs_dense_mask": None if ms_wall_d is None else round(ms_wall_d / ms_wall, 4),
        "dense_mask_ms_per_step": None if ms_wall_d is None else round(ms_wall_d, 6),
        "event_ms_per_step": round(ms_ev, 6),
        "timing": ("K launches captured into one HIP graph, one replay timed between synchronisations"
                   if args.graph else "K launches issued from the Python loop"),
        "eager_ms_per_step": round(ms_eager, 6),
        "event_pair_us": {"avg": round(k_avg, 3), "median": round(k_med, 3), "min": round(k_min, 3),
                          "dense_mask_avg": None if kd_avg is None else round(kd_avg, 3),
                          "note": "one launch between two events: includes launch and drain"},
        "multi_stream": None if ms_multi is None else
        {"streams": 4, "ms_per_step": round(ms_multi, 6),
         "value": round(fl / (ms_multi * 1e-3) / 1e12, 4),
         "hbm_GBs": round(nbytes / (ms_multi * 1e-3) / 1e9, 1)},
        "mfma_frac_of_peak": round(fl / (ms_ev * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5)
        if c.dtype == "bf16" else None,
        "pack_ms": round(pack_ms, 3),
        "fused_epilogue": bool(args.fused),
        "unfused_ms_per_step": None if ms_unfused is None else round(ms_unfused, 6),
        "mask": args.mask, "mask_select_ms": None if select_ms is None else round(select_ms, 3),
        "roofline": roof,
        "measured_peaks": peaks,
    }
    if args.workload == "c1" and args.network_summary and not (args.general or args.fused
                                                                or args.mask != "synthetic"):
        out["resnet50"] = network_summary(network_rows(args, "resnet50", peaks, reps=20))

    if args.copy_calibration:
        nb_copy = int(min(Xs[0].numel(), Ys[0].numel()) * Xs[0].element_size()) & ~15
        for i in range(5):   # the library's own copy kernel (bench_copy), nb_copy bytes read and written
            bsp.bsp_bench_copy(Ys[i % nsets].data_ptr(), Xs[i % nsets].data_ptr(), nb_copy, stream.cuda_stream)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = nb_copy

    if not args.no_cpu_baseline:
        import oracle
        reps, dt, used = 0, 0.0, 1
        while reps < 12 and dt * used < 12.0:   # about 10-30 s of CPU work in all
            t = time.perf_counter()
            _, used = oracle.conv2d(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                    return_threads=True)
            dt += time.perf_counter() - t
            reps += 1
        out["cpu_baseline"] = {"value": round(fl * reps / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": int(used), "kind": "oracle",
                               "sample": f"the full workload {reps} times ({dt:.2f} s wall on {used} "
                                         "threads; the oracle does the dense masked sum in fp64 "
                                         "and skips nothing)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
