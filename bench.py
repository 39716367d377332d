#!/usr/bin/env python3
"""Benchmark of the conv hot path on one MI355X.

A step is one call of dll_cnn_train_step (forward, loss, backward, SGD update) on the
large-image CNN workload (config 5: batch 128 of 3x256x256, four conv+ReLU+pool blocks,
dense 2048, dense 1000), inputs and parameters resident in HBM.  Prints ONE JSON line.

  value      GFLOP/s of the whole step (exact multiply-adds x 2: padding zeros, wasted
             MFMA lanes and split-K re-reads are not counted)
  roofline   the conv kernel instance with the longest launch, timed launch by launch with
             HIP events on the launch stream, against the fp32 MFMA peak (the FLOP it
             executes on the matrix pipe)
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample

Other workloads (--config 1..4, --mode infer/dense/rbm/crbm_pmp) exist for inspection; the default
line is config 5.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X published dense fp32 matrix peak
METRIC = "conv GFLOP/s + images/s per fwd+bwd step; % of fp32 MFMA peak"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (inspection only)")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="timed steps: replays of one step captured in a HIP graph (default), or plain launches")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the CPU oracle leg (0 = all the box gives)")
    ap.add_argument("--cpu-batch", type=int, default=128, help="batch of the CPU oracle leg (config 5 and --mode infer)")
    ap.add_argument("--mode", choices=["train", "infer", "dense", "rbm", "crbm_pmp", "fft"], default="train",
                    help="inspection lines instead of the training step of --config: infer = dll_cnn_forward on the paper's "
                         "ImageNet network (batch 128 of 3x256x256); dense = momentum step of the fully-connected 784-500-250-10 "
                         "network (batch 100); rbm = CD-1 step of a 784-500 RBM (batch 100); crbm_pmp = CD-1 step of the "
                         "config-3 CRBM with probabilistic max pooling; fft = backward-data pass of a 32-channel layer with "
                         "12x12 filters through dll_conv_full_bwd_fft (and the direct kernel's time beside it)")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also run one 256 MiB device copy, the known-size kernel that scales rocprofv3's byte counters")
    return ap.parse_args()


def event_time_ms(fn, iters, warm=5, n_groups=5):
    """Average duration of fn() in ms: HIP events on torch's current stream (the launch stream)
    around `iters` back-to-back calls, so the figure is the kernels' own time plus the gap
    between dependent launches, not the host's call overhead.  Returns (median of the groups, groups)."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    groups = []
    for _ in range(n_groups):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        b.synchronize()
        groups.append(a.elapsed_time(b) / iters)
    return float(np.median(groups)), groups


def engine_kernel_name(cs, backward: bool) -> str:
    """Name of the kernel instance the library launches for a forward or backward-data pass
    (mirrors the dispatch in csrc/conv_engine.hip; used only to group launches for the report)."""
    cin, kout, hout = (cs.K, cs.C, cs.H) if backward else (cs.C, cs.K, cs.Ho)
    same = cs.R == 3 and cs.S == 3 and cs.pad == 1
    if same and not backward and cs.C <= 3 and cs.K <= 16 and cs.act == "relu" and cs.pool == 2 and cs.W % 8 == 0:
        return "conv_fwd_fewch_kernel"   # first layer of the image networks
    # layers with 16 or 32 channels in and out, ReLU + pooling: the minimal-filtering form as a streaming kernel
    # (forward, and backward-data from the pooled gradient with the ReLU flags, as the step calls it); a 32-channel
    # source needs column segments that fill the workgroup's streams, else the tile kernel below takes the layer
    if same and cs.C in (16, 32) and cs.K in (16, 32) and cs.C + cs.K < 64 and cs.act == "relu" and cs.pool == 2 and cs.W % 8 == 0 and cs.H % 2 == 0:
        streams = 4 // ((cin // 16) * (kout // 16))
        if cin == 16 or ((cs.W + 31) // 32) % streams == 0:
            kt, ch = kout // 16, cin // 16
            return f"conv3x3_wino_stream_bwd_kernel<{kt},{ch}>" if backward else f"conv3x3_wino_stream_kernel<true,{kt},{ch}>"
    if same and cs.C == 32 and cs.K == 32 and cs.act == "relu" and cs.pool == 2 and cs.Ho % 8 == 0 and cs.Wo % 32 == 0:
        return f"conv3x3_wino_kernel<1,{'true' if backward else 'false'},2,2>"
    if same and cs.C == 16 and cs.act == "relu" and cs.pool == 2 and cs.Ho % 8 == 0 and cs.Wo % 32 == 0:
        if cs.K == 16:
            return f"conv3x3_wino_kernel<1,{'true' if backward else 'false'},1,1>"
        if cs.K == 32:   # backward-data: two chunks of 16 gradient channels; forward: two groups of 16 filters
            return "conv3x3_wino_kernel<1,true,2,1>" if backward else "conv3x3_wino_kernel<1,false,1,2>"
    chunked = cin % 16 == 0 or (cin % 8 == 0 and kout <= 16) or cin <= 12
    if same and chunked and hout > 8 and cs.W % (8 if backward and cs.pool == 2 else 4) == 0:
        src = 0 if not backward else (2 if cs.pool == 2 else 1)
        nt = 1 if kout <= 16 else 2
        cc = 8 if (nt == 1 and cin % 8 == 0) else (16 if cin % 16 == 0 else 4)
        waves = 8 if (cc == 16 and nt == 2) else 4
        pack3 = "true" if (cc == 4 and cin == 3 and not backward) else "false"
        epi = 2 if backward else (1 if (cs.act == "relu" and cs.pool == 2) else 0)
        return f"conv3x3c16_kernel<{nt},{waves},{src},{cc},{pack3},{epi}>"
    nt = 1 if kout <= 16 else (2 if kout <= 32 else 3)
    return f"conv_engine_kernel<{nt},{1 if hout <= 8 else 2}>"


def executed_flop(kernel: str, direct_flop: float) -> float:
    """FLOP a pass puts through the matrix pipe.  The minimal-filtering kernels (F(2x2,3x3) for the forward
    and backward-data passes, F(3x3,2x2) for the filter gradient) multiply 16 transformed values where
    the direct sum takes 36 products: 1/2.25 of the direct-sum FLOP; every other kernel executes the direct sum."""
    return direct_flop / 2.25 if "wino" in kernel else direct_flop


def wgrad_kernel_name(cs) -> str:
    """Name of the filter-gradient kernel instance of a layer (mirrors plan_wgrad / launch_wgrad in
    csrc/conv_wgrad.hip for aligned tensors; used only to label the pass in the report)."""
    if (cs.R == 3 and cs.S == 3 and cs.pad == 1 and cs.pool == 2 and cs.act == "relu" and cs.C in (16, 32) and cs.K in (16, 32)
            and cs.W % 8 == 0):
        # the pooled ReLU layers with 16 or 32 channels in and out: minimal-filtering form (the step passes no layer output)
        return f"wgrad_wino_kernel<{cs.K // 16},{cs.C // 16}>"
    if cs.R == 3 and cs.S == 3 and cs.pad == 1 and cs.pool == 2 and cs.act == "relu" and cs.C <= 3 and cs.K <= 16 and cs.W % 8 == 0:
        return "wgrad_fewch_kernel"   # first layer of the image networks: dz formed in registers from the pooled tensors
    taps = cs.R * cs.S
    best = None
    for cc in range(1, min(cs.C, 16) + 1):
        need = (cc * taps + 15) // 16
        ntt = next((c for c in (2, 5, 7, 9) if need <= c), 0)
        if not ntt:
            break
        cost = -(-cs.C // cc) * ntt
        if best is None or cost <= best[0]:
            best = (cost, cc, ntt)
    _, cc, ntt = best
    mtf = min(3, -(-cs.K // 16))
    lines = cc * (8 + cs.R - 1)
    fast = 2 if (ntt == 2 and lines * 8 <= 256 and lines * (cs.S - 1) <= 256) else 1
    return f"wgrad_kernel<{mtf},{ntt},{cs.pool},{fast}>"


def conv_pass_table(B, wl_cnn, dev_params, x_dev, iters):
    """Times every convolution pass of the step as its own launch: one API call = one kernel
    (forward, backward-data) or the filter-gradient kernel + its small reduction."""
    import torch
    acts, idxs = [x_dev], []
    for l, cs in enumerate(wl_cnn.conv):
        y = torch.empty(cs.y_shape, device="cuda")
        idx = torch.empty(cs.y_shape, dtype=torch.uint8, device="cuda")
        B.dll_conv_valid_fwd(cs, acts[l], dev_params[2 * l], dev_params[2 * l + 1], y, idx)
        acts.append(y)
        idxs.append(idx)
    table = []
    for l, cs in enumerate(wl_cnn.conv):
        xin, y, idx = acts[l], acts[l + 1], idxs[l]
        w, b = dev_params[2 * l], dev_params[2 * l + 1]
        dy = torch.randn(cs.y_shape, device="cuda")
        flop = 2 * cs.macs_exact()
        y2, idx2 = torch.empty_like(y), torch.empty_like(idx)
        # backward passes as the training step issues them: a pooled ReLU layer's output is not
        # passed (its activity flags sit in idx)
        yb = None if (cs.act == "relu" and cs.pool == 2) else y
        ms, _ = event_time_ms(lambda: B.dll_conv_valid_fwd(cs, xin, w, b, y2, idx2), iters)
        table.append(dict(layer=l + 1, op="fwd", kernel=engine_kernel_name(cs, False), ms=ms, flop=flop))
        if l > 0:
            dx = torch.empty(cs.x_shape, device="cuda")
            ms, _ = event_time_ms(lambda: B.dll_conv_full_bwd(cs, dy, yb, idx, w, dx), iters)
            table.append(dict(layer=l + 1, op="bwd_data", kernel=engine_kernel_name(cs, True), ms=ms, flop=flop))
        ws = B.workspace(B.dll_conv_workspace_bytes(cs))
        dw, db = torch.empty_like(w), torch.empty_like(b)
        ms, _ = event_time_ms(lambda: B.dll_conv_valid_wgrad(cs, xin, dy, yb, idx, dw, db, ws), iters)
        # the pass is the filter-gradient kernel and its small fixed-order reduction: both are in `ms`;
        # `kernel_ms` is the filter-gradient kernel alone (the first of the two launches as a call of its
        # own), which is what the training step runs per layer: its reductions ride in the closing launch
        kms, _ = event_time_ms(lambda: B.dll_conv_valid_wgrad_partial(cs, xin, dy, yb, idx, ws), iters)
        table.append(dict(layer=l + 1, op="wgrad", kernel=wgrad_kernel_name(cs), ms=ms, kernel_ms=kms, flop=flop))
        del dy
    return table


SETTLE_S = 0.1   # untimed steady-state run-in before the timed steps (see main)
N_BATCHES = 3    # input batches the timed steps of config 5 rotate through (3 x 100.7 MB: more than the 256 MB memory-side cache)

# Figures of one config-5 step (batch 128) that only profiler counter runs can give; they do not depend
# on the data, only on the kernels, and are re-taken whenever a kernel changes (the profile file
# names the commands).  MFMA wave-instructions: SQ_INSTS_VALU_MFMA_MOPS_F32-class counters summed over
# the step's kernels, each v_mfma_f32_16x16x4_f32 being 2048 FLOP.  HBM bytes: FETCH_SIZE and
# WRITE_SIZE summed over the step's kernels with the copy-kernel calibration.
RECORDED_STEP_COUNTERS = {
    ("c5_large_image_cnn", 128): {"mfma_wave_instructions": 25.95e6, "hbm_bytes": 1.837e9,
                                  "source": "profiles/c5_cnn_train_step.md (rocprofv3 --pmc runs of this bench command)"},
}


def chip_probe():
    """Runs the stand-alone probe (bench_chip_probe, built by __graft_entry__.build()) as a child
    process and returns its JSON line: the fp32 MFMA rate of a register-only loop and the HBM
    copy / read / write rates on this very box.  None when the program is not there."""
    import subprocess
    exe = os.path.join(ROOT, "bench_chip_probe")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        for line in reversed(r.stdout.splitlines()):
            if line.startswith("{"):
                return json.loads(line)
    except Exception as e:   # noqa: BLE001 - the probe is a side measurement
        print(f"bench.py: chip probe failed ({e})", file=sys.stderr)
    return None

# HBM bytes per launch of the kernels that can come out as the dominant one at config 5, batch 128,
# from the FETCH_SIZE / WRITE_SIZE counter runs summarised in profiles/c5_cnn_train_step.md
# (fetch scaled by the copy-kernel calibration, so an upper bound; averaged over the kernel's
# launches of a step like `achieved`).  Counters need profiler runs of their own, so the figure
# cannot be taken live; any other kernel or workload reports null.
MEASURED_TRAFFIC_BYTES = {
    # conv1's filter gradient: x (100.7 MB) + pooled gradient (134.2 MB) + pooling bytes (33.6 MB) in, partial sums out
    ("c5_large_image_cnn", 128, "wgrad_fewch_kernel"): (267950.7 + 2112.0) * 1024,
    # conv1's forward pass: x in; pooled output (134.2 MB) + pooling bytes (33.6 MB) out
    ("c5_large_image_cnn", 128, "conv_fwd_fewch_kernel"): (104060.4 + 164834.4) * 1024,
}


def cpu_baseline(cfg: int, cpu_batch: int, budget_s: float = 10.0, max_reps: int = 1000000, threads: int = 0):
    """The oracle as it stands on the host cores: whole steps of the same workload, repeated until
    about `budget_s` seconds of CPU work are done (at least one step)."""
    from oracle import oracle as orc
    from paper_1804_04512_amd import workloads as wl
    act = {"identity": 0, "sigmoid": 1, "relu": 2}
    if threads > 0:
        orc.set_threads(threads)
    w = wl.ALL[cfg](cpu_batch)
    if isinstance(w, wl.CnnWorkload):
        net = orc.Net([orc.conv_desc(c.N, c.C, c.H, c.W, c.K, c.R, c.S, c.pad, act[c.act], c.pool) for c in w.conv],
                      [(d.in_, d.out, act[d.act]) for d in w.dense], w.classes)
        step = lambda: orc.cnn_train_step(net, w.clone_params(), w.x, w.labels, w.lr)
        n = w.batch
    elif isinstance(w, wl.CrbmWorkload):
        c = w.conv
        d = orc.conv_desc(c.N, c.C, c.H, c.W, c.K, c.R, c.S)
        step = lambda: orc.crbm_cd1_step(d, w.v0, w.W.copy(), w.b.copy(), w.c.copy(), w.u, lr=w.lr)
        n = c.N
    else:
        c = w.conv
        d = orc.conv_desc(c.N, c.C, c.H, c.W, c.K, c.R, c.S, c.pad, act[c.act], c.pool)

        def step():
            y, idx = orc.conv_valid_fwd(d, w.x, w.w, w.bias)
            orc.conv_full_bwd(d, w.dy, y, idx, w.w)
            orc.conv_valid_wgrad(d, w.x, w.dy, y, idx)
        n = c.N
    reps, t0 = 0, time.perf_counter()
    while True:
        step()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= max_reps:
            break
    return dict(value=w.flop() * reps / dt / 1e9, unit="GFLOP/s", images_per_s=n * reps / dt, seconds=dt, cores=orc.max_threads(),
                kind="oracle", sample=f"{reps} step(s) of config {cfg} at batch {n} (same layer shapes), fp64 accumulation, plain loops")


def infer_line(args, B, wl, torch):
    """Inspection mode: one inference pass of the paper's five-block ImageNet network per step."""
    w = wl.paper_imagenet_cnn(args.batch) if args.batch else wl.paper_imagenet_cnn()
    net = B.net_desc(w.conv, w.dense, w.classes)
    params = [torch.from_numpy(p).cuda() for p in w.params]
    x = torch.from_numpy(w.x).cuda()
    prob = torch.empty((w.batch, w.classes), device="cuda")
    ws = B.workspace(B.dll_cnn_forward_workspace_bytes(net))
    step = lambda: B.dll_cnn_forward(net, params, x, None, prob, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    flop = wl.forward_flop(w)
    gflops = flop / (ms * 1e-3) / 1e9
    out = {"metric": "inference GFLOP/s + images/s per forward pass; % of fp32 MFMA peak", "value": gflops, "unit": "GFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "batch": w.batch, "flop_per_step": flop},
           "images_per_s": w.batch / (ms * 1e-3), "pct_fp32_mfma_peak": 100.0 * gflops / (PEAK_FP32_MFMA_TFLOPS * 1e3)}
    if not args.no_cpu:
        from oracle import oracle as orc
        act = {"identity": 0, "sigmoid": 1, "relu": 2}
        wc = wl.paper_imagenet_cnn(min(args.cpu_batch, w.batch))
        onet = orc.Net([orc.conv_desc(c.N, c.C, c.H, c.W, c.K, c.R, c.S, c.pad, act[c.act], c.pool) for c in wc.conv],
                       [(d.in_, d.out, act[d.act]) for d in wc.dense], wc.classes)
        t0 = time.perf_counter()
        orc.cnn_forward(onet, wc.params, wc.x)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=wl.forward_flop(wc) / dt / 1e9, unit="GFLOP/s", images_per_s=wc.batch / dt, seconds=dt,
                                   cores=orc.max_threads(), kind="oracle",
                                   sample=f"one inference pass of {wc.name} at batch {wc.batch}, fp64 accumulation, plain loops")
    print(json.dumps(out))
    return 0


def timed_ms(step, args, torch):
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / args.steps * 1e3


def timed_cpu(step, budget_s=10.0, max_reps=200):
    reps, t0 = 0, time.perf_counter()
    while True:
        step()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= max_reps:
            return reps, dt


def extra_line(args, B, wl, torch):
    """Inspection modes for the steps built around the same kernels: the fully-connected network,
    the fully-connected RBM and the CRBM with probabilistic max pooling."""
    dev = lambda a: torch.from_numpy(a).cuda()
    if args.mode == "dense":
        w = wl.paper_mnist_dense(args.batch) if args.batch else wl.paper_mnist_dense()
        net = B.net_desc(w.conv, w.dense, w.classes, w.batch)
        params = [dev(p) for p in w.params]
        vel = [torch.zeros_like(p) for p in params]
        x, labels, loss = dev(w.x), dev(w.labels), torch.zeros(1, device="cuda")
        ws = B.workspace(B.dll_cnn_workspace_bytes(net))
        step = lambda: B.dll_cnn_train_step_momentum(net, params, vel, None, x, labels, w.lr, 0.9, 0.0, loss, None, None, ws)
        batch, flop, name = w.batch, w.flop(), w.name
        what = "momentum step (lr 0.1, momentum 0.9) of the fully-connected network"
    elif args.mode == "rbm":
        w = wl.dense_rbm(args.batch) if args.batch else wl.dense_rbm()
        W, b, c, v0, u = dev(w.W), dev(w.b), dev(w.c), dev(w.v0), dev(w.u)
        dW, db, dc = torch.empty_like(W), torch.empty_like(b), torch.empty_like(c)
        ws = B.workspace(B.dll_rbm_workspace_bytes(w.batch, w.n_vis, w.n_hid))
        step = lambda: B.dll_rbm_cd1_step(w.batch, w.n_vis, w.n_hid, 0, v0, W, b, c, u, None, w.lr, dW, db, dc, ws=ws)
        batch, flop, name = w.batch, w.flop(), w.name
        what = "CD-1 step of the fully-connected RBM"
    elif args.mode == "fft":
        w = wl.large_filter_layer(args.batch) if args.batch else wl.large_filter_layer()
        cs = w.conv
        dy, wt = dev(w.dy), dev(w.w)
        dx, dx_direct = torch.empty(cs.x_shape, device="cuda"), torch.empty(cs.x_shape, device="cuda")
        ws = B.workspace(B.dll_conv_full_fft_workspace_bytes(cs))
        step = lambda: B.dll_conv_full_bwd_fft(cs, dy, None, None, wt, dx, ws)
        direct = lambda: B.dll_conv_full_bwd(cs, dy, None, None, wt, dx_direct)
        batch, flop, name = cs.N, 2 * cs.macs_exact(), w.name
        what = "backward-data pass of a 12x12-filter layer through the Fourier transform (FLOP of the direct sum)"
    else:
        cs = wl.config3(args.batch).conv if args.batch else wl.config3().conv
        w = wl.crbm_units(cs, "binary", 2)
        W, b, c, v0, u = dev(w.W), dev(w.b), dev(w.c), dev(w.v0), dev(w.u)
        dW, db, dc = torch.empty_like(W), torch.empty_like(b), torch.empty_like(c)
        ws = B.workspace(B.dll_crbm_workspace_bytes(cs))
        step = lambda: B.dll_crbm_cd1_step_units(cs, 0, 2, v0, W, b, c, u, None, w.lr, dW, db, dc, ws=ws)
        batch, flop, name = cs.N, w.flop(), "c3_crbm_probabilistic_max_pooling"
        what = "CD-1 step of the CRBM with probabilistic max pooling"
    ms = timed_ms(step, args, torch)
    gflops = flop / (ms * 1e-3) / 1e9
    out = {"metric": f"{what}: GFLOP/s + samples/s; % of fp32 MFMA peak", "value": gflops, "unit": "GFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": name, "batch": batch, "flop_per_step": flop},
           "images_per_s": batch / (ms * 1e-3), "pct_fp32_mfma_peak": 100.0 * gflops / (PEAK_FP32_MFMA_TFLOPS * 1e3)}
    if args.mode == "fft":
        out["direct_kernel_ms"] = timed_ms(direct, args, torch)
        out["max_abs_diff_over_max_abs"] = float((dx - dx_direct).abs().max() / dx_direct.abs().max())
    if not args.no_cpu:
        from oracle import oracle as orc
        act = {"identity": 0, "sigmoid": 1, "relu": 2}
        if args.mode == "fft":
            d = orc.conv_desc(cs.N, cs.C, cs.H, cs.W, cs.K, cs.R, cs.S)
            cpu_step = lambda: orc.conv_full_bwd(d, w.dy, None, None, w.w)
        elif args.mode == "dense":
            onet = orc.Net([], [(d.in_, d.out, act[d.act]) for d in w.dense], w.classes, batch=w.batch)

            def cpu_step():
                ps = w.clone_params()
                r = orc.cnn_train_step(onet, ps, w.x, w.labels, 0.0)
                for p_, g_ in zip(ps, r.grads):
                    orc.sgd_momentum(p_, np.zeros_like(p_), g_, w.lr, 0.9, 0.0)
        elif args.mode == "rbm":
            cpu_step = lambda: orc.rbm_cd1_step(w.batch, w.n_vis, w.n_hid, 0, w.v0, w.W.copy(), w.b.copy(), w.c.copy(), w.u, lr=w.lr)
        else:
            d = orc.conv_desc(cs.N, cs.C, cs.H, cs.W, cs.K, cs.R, cs.S)
            cpu_step = lambda: orc.crbm_cd1_step_units(d, 0, 2, w.v0, w.W.copy(), w.b.copy(), w.c.copy(), w.u, lr=w.lr)
        reps, dt = timed_cpu(cpu_step)
        out["cpu_baseline"] = dict(value=flop * reps / dt / 1e9, unit="GFLOP/s", images_per_s=batch * reps / dt, seconds=dt,
                                   cores=orc.max_threads(), kind="oracle",
                                   sample=f"{reps} step(s) of {name} at batch {batch}, fp64 accumulation, plain loops")
    print(json.dumps(out))
    return 0


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2
    import torch
    from paper_1804_04512_amd import binding as B
    from paper_1804_04512_amd import workloads as wl

    B.lib()  # fail loudly when the HIP library is missing
    probe = chip_probe() if args.mode == "train" else None   # before this process touches the GPU
    torch.cuda.set_device(0)
    if args.mode == "infer":
        return infer_line(args, B, wl, torch)
    if args.mode != "train":
        return extra_line(args, B, wl, torch)
    cfg = args.config
    w = wl.ALL[cfg](args.batch) if args.batch else wl.ALL[cfg]()
    dev = lambda a: torch.from_numpy(a).cuda()

    if isinstance(w, wl.CnnWorkload):
        net = B.net_desc(w.conv, w.dense, w.classes)
        params = [dev(p) for p in w.params]
        x, labels = dev(w.x), dev(w.labels)
        loss = torch.zeros(1, device="cuda")
        ws = B.workspace(B.dll_cnn_workspace_bytes(net))
        step = lambda: B.dll_cnn_train_step(net, params, None, x, labels, w.lr, loss, None, None, ws)
        batch = w.batch
        # further input batches for the timed steps to rotate through (same distribution, seeded on the device)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(18040451)
        xs, ls = [x], [labels]
        for _ in range(N_BATCHES - 1 if cfg == 5 else 0):
            xs.append(torch.randn(x.shape, device="cuda", generator=gen))
            ls.append(torch.randint(0, w.classes, labels.shape, device="cuda", generator=gen, dtype=torch.int32))
        step_on = lambda j: B.dll_cnn_train_step(net, params, None, xs[j], ls[j], w.lr, loss, None, None, ws)
    elif isinstance(w, wl.CrbmWorkload):
        cs = w.conv
        W, b, c = dev(w.W), dev(w.b), dev(w.c)
        v0, u = dev(w.v0), dev(w.u)
        dW, db, dc = torch.empty_like(W), torch.empty_like(b), torch.empty_like(c)
        ws = B.workspace(B.dll_crbm_workspace_bytes(cs))
        step = lambda: B.dll_crbm_cd1_step(cs, v0, W, b, c, u, None, w.lr, dW, db, dc, ws=ws)
        batch = cs.N
    else:
        cs = w.conv
        x, wt, bias, dy = dev(w.x), dev(w.w), dev(w.bias), dev(w.dy)
        y, dx = torch.empty(cs.y_shape, device="cuda"), torch.empty(cs.x_shape, device="cuda")
        dw, db = torch.empty_like(wt), torch.empty_like(bias)
        ws = B.workspace(B.dll_conv_workspace_bytes(cs))

        def step():
            B.dll_conv_valid_fwd(cs, x, wt, bias, y, None)
            B.dll_conv_full_bwd(cs, dy, y, None, wt, dx)
            B.dll_conv_valid_wgrad(cs, x, dy, y, None, dw, db, ws)
        batch = cs.N

    if args.pmc_calib:
        src = torch.ones(64 << 20, device="cuda")       # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Per-pass timing of the convolution kernels (the roofline measurement), at the chip's working
    # clocks: plain steps run for SETTLE_S seconds first (see below).
    table = None
    if isinstance(w, wl.CnnWorkload):
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < SETTLE_S:
            for _ in range(10):
                step()
            torch.cuda.synchronize()
        table = conv_pass_table(B, w, params, x, 20)
    # The library allocates nothing, synchronises nothing and keeps every pointer fixed from step
    # to step, so a whole step can be captured once into a HIP graph and replayed: the same
    # kernels on the same data, with the launch work done once.  Plain launches remain as
    # `--launch eager`, and as the fallback should the capture fail.
    rotating = isinstance(w, wl.CnnWorkload) and len(xs) > 1
    runs, launch = ([lambda j=j: step_on(j) for j in range(len(xs))] if rotating else [step]), "eager"
    if args.launch == "graph":
        try:
            graphs = []
            for r_ in runs:   # one graph per input batch: same kernels, same parameters and workspace, another x
                gr_ = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr_):
                    r_()
                graphs.append(gr_)
            torch.cuda.synchronize()
            for _ in range(max(1, args.warmup)):
                for gr_ in graphs:
                    gr_.replay()
            torch.cuda.synchronize()
            runs, launch = [gr_.replay for gr_ in graphs], "hip graph replay"
        except Exception as e:   # noqa: BLE001 - any capture problem means: time plain launches
            print(f"bench.py: graph capture failed ({e}); timing plain launches", file=sys.stderr)
            torch.cuda.synchronize()

    def timed(run_list):
        # The chip takes some tens of milliseconds of continuous work to reach its steady clocks after
        # an idle spell (the set-up above leaves several): steps are run, untimed, for SETTLE_S seconds
        # so that the timed steps measure the steady state a training job runs in.
        t_settle = time.perf_counter()
        k = 0
        while time.perf_counter() - t_settle < SETTLE_S:
            for _ in range(10):
                run_list[k % len(run_list)]()
                k += 1
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run_list[i % len(run_list)]()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps * 1e3

    # the timed steps: every step takes the next input batch, so that no step finds its input in the
    # memory-side cache; the same steps on ONE resident batch are timed beside them
    resident_ms = timed(runs[:1]) if rotating else None
    ms_per_step = timed(runs)
    flop = w.flop()
    gflops = flop / (ms_per_step * 1e-3) / 1e9

    # after the timed region: the state thousands of in-place updates have left must still train.
    # One more step as the timed steps ran it, and the same step from the same state as plain launches:
    # both losses must be finite and bit-equal (the kernels are deterministic).
    loss_check = None
    if isinstance(w, wl.CnnWorkload):
        saved = [p_.clone() for p_ in params]
        runs[0]()
        torch.cuda.synchronize()
        loss_timed_path = float(loss.item())
        for p_, s_ in zip(params, saved):
            p_.copy_(s_)
        (step_on(0) if rotating else step())
        torch.cuda.synchronize()
        loss_eager = float(loss.item())
        if not (np.isfinite(loss_timed_path) and loss_timed_path == loss_eager):
            print(f"bench.py: loss check failed: {loss_timed_path} (timed path) vs {loss_eager} (plain launches)", file=sys.stderr)
            return 1
        loss_check = {"loss_after_timed_steps": loss_timed_path, "equals_plain_launch_step_from_same_state": True}
        del saved

    out = {
        "metric": METRIC, "value": gflops, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": batch, "flop_per_step": flop, "launch": launch, "settle_s": SETTLE_S,
                   "input_batches_rotated": len(runs)},
        "images_per_s": batch / (ms_per_step * 1e-3),
        # value / peak with the FLOP of the direct sums (the algorithmic work), also for the passes that run in
        # the minimal-filtering form and execute fewer multiplications: an EFFECTIVE figure, not an MFMA rate
        "pct_fp32_mfma_peak": 100.0 * gflops / (PEAK_FP32_MFMA_TFLOPS * 1e3),
        "pct_fp32_mfma_peak_is": "direct-sum FLOP per second over the published peak (effective; see mfma_executed)",
    }
    if resident_ms is not None:
        out["resident_batch"] = {"ms_per_step": resident_ms, "value": flop / (resident_ms * 1e-3) / 1e9,
                                 "note": "the same steps fed ONE input batch: part of x then survives in the memory-side cache from step to step"}
    if loss_check:
        out["loss_check"] = loss_check
    if probe:
        out["measured_peaks"] = probe
        out["pct_measured_mfma_peak"] = 100.0 * gflops / (probe["mfma_f32_tflops"] * 1e3)
    rec = RECORDED_STEP_COUNTERS.get((w.name, batch))
    if rec:
        ex = rec["mfma_wave_instructions"] * 2048 / (ms_per_step * 1e-3) / 1e12
        out["mfma_executed"] = {"tflops": ex, "util_of_published_peak": ex / PEAK_FP32_MFMA_TFLOPS,
                                "util_of_measured_loop": (ex / probe["mfma_f32_tflops"]) if probe else None,
                                "wave_instructions_per_step": rec["mfma_wave_instructions"], "source": rec["source"]}
        hb = rec["hbm_bytes"] / (ms_per_step * 1e-3) / 1e9
        out["hbm"] = {"gbps": hb, "bytes_per_step": rec["hbm_bytes"], "copy_peak_gbps": probe["hbm_copy_gbps"] if probe else None,
                      "frac_of_copy_peak": (hb / probe["hbm_copy_gbps"]) if probe else None,
                      "frac_of_published_peak": hb / 8000.0, "source": rec["source"]}
    if isinstance(w, wl.CnnWorkload):
        out["config"]["conv_flop_per_step"] = w.conv_flop()
        conv_ms = sum(r["ms"] for r in table)
        out["conv_passes"] = [dict(layer=r["layer"], op=r["op"], ms=round(r["ms"], 4),
                                   tflops=round(r["flop"] / r["ms"] / 1e9, 2),
                                   **({"kernel_ms": round(r["kernel_ms"], 4)} if "kernel_ms" in r else {})) for r in table]
        out["conv_gflops"] = sum(r["flop"] for r in table) / conv_ms / 1e6
        # dominant kernel: group single-kernel launches by kernel name, take the largest total time
        groups = {}
        for r in table:
            gname = r["kernel"]
            gr = groups.setdefault(gname, dict(ms=0.0, flop=0, n=0))
            gr["ms"] += r.get("kernel_ms", r["ms"]); gr["flop"] += r["flop"]; gr["n"] += 1
        name, gr = max(groups.items(), key=lambda kv: kv[1]["ms"])
        # against the MFMA peak stands the FLOP the kernel executes on the matrix pipe: the direct sum, or
        # 1/2.25 of it for a minimal-filtering kernel (whose direct-sum rate is given beside it)
        achieved = executed_flop(name, gr["flop"]) / gr["ms"] / 1e9   # TFLOP/s
        out["roofline"] = {"bound": "mfma", "kernel": name, "launches_per_step": gr["n"],
                           "avg_launch_ms": gr["ms"] / gr["n"], "flop_per_launch": executed_flop(name, gr["flop"]) / gr["n"],
                           "direct_sum_tflops": gr["flop"] / gr["ms"] / 1e9,
                           "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                           "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, batch, name)),
                           "traffic_source": "recorded: profiles/c5_cnn_train_step.md counter runs (FETCH_SIZE, WRITE_SIZE with the "
                                             "copy-kernel calibration); counters cannot be read inside this run"}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_batch if cfg == 5 else batch, threads=args.cpu_threads)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
