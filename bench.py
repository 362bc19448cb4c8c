#!/usr/bin/env python3
"""Benchmark of the fused rotation-convolution hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: rotconv_pool_fwd, rotconv_pool_bwd_data, rotconv_pool_bwd_weight
(tap tables are built once per plan, outside the step; the filter-bank expansion and the
weight-gradient reduction kernels run inside it).  Workload: benchmark configuration 2
(N=8, 64->64 channels, 256x256, 3x3, R=4 exact quarter turns, fp32, orientation max-pool).

Prints ONE JSON line.  `value` is algorithmic TFLOP/s: per pass
F_alg = 2*P*Cin*Cout*k^2*Q + P*Cout*k^2*R  (Q = distinct first-quadrant angles; the per-tap
channel contraction is shared by the four symmetric rotations, paper Eq. 8), three passes
per step.  The dense-equivalent figure (R separate convolutions) is given beside it in
`config` for context only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3  # MI355X fp32 matrix (and vector) peak
PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0


def flops_alg(cfg, Q):
    P = cfg.N * cfg.Ho * cfg.Wo
    return 2.0 * P * cfg.Cin * cfg.Cout * cfg.k * cfg.k * Q + 1.0 * P * cfg.Cout * cfg.k * cfg.k * cfg.R


def flops_dense(cfg):
    P = cfg.N * cfg.Ho * cfg.Wo
    return 2.0 * P * cfg.Cin * cfg.Cout * cfg.k * cfg.k * cfg.R


def cpu_baseline(cfg, Q):
    """The oracle as it stands, timed on the host cores on a bounded sample (a batch slice)."""
    import dataclasses
    import numpy as np
    from oracle import rotconv_oracle as orc
    from paper_2512_08888_amd import synth

    # about 10-30 s of CPU work on the 16 host cores of the GPU machine: dense flops of the sample near 1.6e11 per pass
    n_s = max(1, min(cfg.N, int(1.6e11 / (flops_dense(cfg) / cfg.N))))
    h_s = cfg.H
    if n_s == 1 and flops_dense(cfg) / cfg.N > 3.2e11:
        h_s = max(cfg.k, int(cfg.H * 3.2e11 / (flops_dense(cfg) / cfg.N)))
    sc = dataclasses.replace(cfg, N=n_s, H=h_s)
    x, w, g = synth.make_x(sc), synth.make_w(sc), synth.make_g(sc)
    ang = None if sc.angles_deg is None else list(sc.angles_deg)
    t0 = time.perf_counter()
    _, _, idx, _ = orc.layer_fwd(x, w, sc.R, ang, sc.mode, sc.stride, sc.pad, sc.G)
    orc.layer_bwd(x, w, g, idx, sc.R, ang, sc.mode, sc.stride, sc.pad, sc.G)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {
        "value": 3.0 * flops_alg(sc, Q) / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "sample": f"{sc.name} slice N={sc.N} H={sc.H} W={sc.W} (of N={cfg.N} H={cfg.H}), fwd+bwd_data+bwd_weight, "
                  f"fp64 dense definition, {dt:.2f} s",
        "seconds": dt,
    }


def bench_unet(name, steps, warmup, dtype="f32", graph=False):
    """ms per training step of the UNet-shaped stack (benchmark configurations 4 and 5; P4 / P8 / P16: the
    paper's own block, rotation convolution then standard convolution, at 4 / 8 / 16 orientations; fp32), whole
    step timed between synchronisations; then one more step with an event pair around every library
    call for the per-call breakdown."""
    import torch
    from paper_2512_08888_amd import unet as un

    cfg = un.UNET_CONFIGS[name]
    net = un.UNet(cfg, un.make_params(cfg), dtype=dtype)
    net.load_batch(*un.make_batch(cfg))
    for _ in range(warmup):
        net.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ms_graph = None
    if graph:       # the same step recorded once into a HIP graph and replayed
        net.capture()
        net.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            net.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / steps
    net.trace = []
    net.step()
    torch.cuda.synchronize()
    by_call, by_layer = {}, {}
    for what, where, e0, e1 in net.trace:
        t = e0.elapsed_time(e1)
        by_call[what] = by_call.get(what, 0.0) + t
        if what.startswith("rotconv"):
            by_layer.setdefault(where, {})[what.replace("rotconv_pool_", "")] = round(t, 4)
    net.trace = None
    alg, dense = net.rot_flops()
    rot_ms = sum(t for k, t in by_call.items() if k.startswith("rotconv"))
    loss = float(net.loss.cpu()[0])
    out = {
        "workload": f"{cfg.name}: UNet-shaped stack, N={cfg.N} {cfg.H}x{cfg.W} widths={list(cfg.widths)} "
                    f"classes={cfg.classes} R={cfg.R} {cfg.mode} block={cfg.block}, one training step (fwd+bwd), "
                    + ("fp32" if dtype == "f32" else "bf16 parameters / activations, fp32 accumulation, fp32 dW and loss"),
        "dtype": dtype,
        "ms_per_step": ms, "ms_per_step_graph_replay": ms_graph, "steps": steps, "warmup": warmup, "loss": loss,
        "rotconv_flops_algorithmic": alg, "rotconv_flops_dense_equivalent": dense,
        "rotconv_ms": rot_ms, "glue_ms": sum(by_call.values()) - rot_ms,
        "rotconv_tflops_algorithmic": alg / (rot_ms * 1e-3) / 1e12,
        "step_tflops_algorithmic": alg / (ms * 1e-3) / 1e12,
        "frac_of_fp32_peak": alg / (ms * 1e-3) / 1e12 / PEAK_FP32_TFLOPS,
        "ms_by_call": {k: round(v, 4) for k, v in sorted(by_call.items())},
        "rotconv_ms_by_layer": by_layer,
        "kernels": {n: [net.plans[n].kernel_name(i) for i in range(3)] for n, *_ in net.layers},
    }
    del net
    torch.cuda.empty_cache()
    return out


def cpu_baseline_unet(name):
    """The oracle's whole step on a bounded sample of the stack: one image of 64x64 (R=4) or 32x32
    (R=16) pixels, the full widths."""
    import dataclasses
    import numpy as np
    from oracle import unet_oracle as uo
    from paper_2512_08888_amd import unet as un

    cfg = un.UNET_CONFIGS[name]
    side = 64 if cfg.R <= 4 else 32
    sc = dataclasses.replace(cfg, N=1, H=side, W=side)
    params = {k: v.astype(np.float64) for k, v in un.make_params(sc).items()}
    images, labels = un.make_batch(sc)
    t0 = time.perf_counter()
    uo.unet_step(images.astype(np.float64), labels, params, sc.R, sc.mode, sc.pool_group, un.oracle_layer_spec(sc))
    dt = time.perf_counter() - t0
    scale = (cfg.N * cfg.H * cfg.W) / (sc.N * sc.H * sc.W)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": dt * scale * 1e3, "unit": "ms/step (extrapolated by pixel count)", "cores": cores, "kind": "oracle",
            "sample": f"{cfg.name} stack with full widths on N=1, {side}x{side} (1/{scale:.0f} of the pixels), fwd+bwd, fp64, "
                      f"{dt:.2f} s", "seconds": dt}


def main_sweep(args):
    """Single-orientation forward (R = 1: the rotation convolution reduces to a standard convolution) over the
    shapes of the paper's appendix: square maps of 4 .. 256 pixels, 256 / 512 / 1024 input channels, 4 .. 256
    filters, batch 1, 3x3, pad 1, fp32.  One JSON line: ms per call and dense TFLOP/s of every point; `value` is
    the geometric mean of the ms over all points (a small-map / launch-latency characterisation, not the
    headline metric)."""
    import math
    import torch
    from paper_2512_08888_amd import binding as rc

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    pts = []
    for side in (4, 8, 16, 32, 64, 128, 256):
        for cin in (256, 512, 1024):
            for cout in (4, 8, 16, 32, 64, 128, 256):
                plan = rc.Plan(1, cin, side, side, cout, k=3, R=1, mode="exact90", stride=1, pad=1)
                x = torch.rand((1, cin, side, side), device="cuda")
                w = torch.randn((1, cout, cin, 3, 3), device="cuda") * (2.0 / (cin * 9)) ** 0.5
                y = torch.empty((1, cout, side, side), device="cuda")
                plan.workspace()
                for _ in range(args.warmup):
                    rc.rotconv_fwd(plan, x, w, y)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.steps):
                    rc.rotconv_fwd(plan, x, w, y)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / args.steps
                fl = 2.0 * side * side * cin * cout * 9
                pts.append({"map": side, "Cin": cin, "Cout": cout, "ms": round(ms, 5), "tflops": round(fl / ms / 1e9, 3),
                            "kernel": plan.kernel_name(0)})
                del plan, x, w, y
    gm = math.exp(sum(math.log(p["ms"]) for p in pts) / len(pts))
    print(json.dumps({
        "metric": "single_orientation_fwd_sweep_geomean_ms", "value": gm, "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": gm, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "sweep: rotconv_fwd with R=1 (standard convolution), N=1, 3x3 pad 1, maps 4..256, "
                               "Cin 256/512/1024, Cout 4..256 (the paper's appendix shapes)", "points": pts}}), flush=True)


def main_unet(args):
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    r = bench_unet(args.workload, args.steps, args.warmup, args.dtype, args.graph)
    out = {
        "metric": "unet_train_step_ms", "value": r["ms_per_step"], "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic", "config": r,
        "roofline": {"bound": "mfma",
                     "kernel": "all rotation-convolution calls of the step (fwd, bwd_data, bwd_weight; 18 layers)",
                     "achieved": r["rotconv_tflops_algorithmic"],
                     "peak": PEAK_BF16_TFLOPS if args.dtype == "bf16" else PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
                     "frac": r["rotconv_tflops_algorithmic"] / (PEAK_BF16_TFLOPS if args.dtype == "bf16" else PEAK_FP32_TFLOPS),
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_unet(args.workload)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "P4", "P8", "P16", "sweep"])
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of activations and weights (accumulation is fp32 either way)")
    ap.add_argument("--pool-op", default="max", choices=["max", "avg"],
                    help="orientation pooling of the single-layer workloads: max (Eq. 10, the benchmark) or average "
                         "(Eq. 9: one ordinary convolution with the group-averaged bank)")
    ap.add_argument("--group", default=None, choices=["p4m8"],
                    help="single-layer workloads: run the layer's shape with another orientation group; p4m8 = four "
                         "quarter turns of the filter and of its mirror image (R = 8, one pool group)")
    ap.add_argument("--ksize", type=int, default=None,
                    help="single-layer workloads: run the layer's shape with k x k filters (pad k // 2) instead of 3 x 3")
    ap.add_argument("--stride", type=int, default=None, help="single-layer workloads: convolution stride")
    ap.add_argument("--graph", action="store_true",
                    help="UNet workloads: also time the step replayed from a HIP graph (ms_per_step_graph_replay)")
    ap.add_argument("--no-unet", action="store_true", help="skip the UNet-shaped steps appended to the default line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (2 GiB of HBM traffic) so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path would shard over the batch, one process per "
              "GPU, weight gradients all-reduced); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload in ("C4", "C5", "P4", "P8", "P16"):
        return main_unet(args)
    if args.workload == "sweep":
        return main_sweep(args)

    import torch
    from paper_2512_08888_amd import binding as rc
    from paper_2512_08888_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    if args.group == "p4m8":
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "_p4m8", R=8, mode="p4m", angles_deg=None, pool_group=None)
    if args.ksize or args.stride:
        import dataclasses
        k = args.ksize or cfg.k
        cfg = dataclasses.replace(cfg, name=f"{cfg.name}_k{k}_s{args.stride or cfg.stride}", k=k, pad=k // 2,
                                  stride=args.stride or cfg.stride)
    bf = args.dtype == "bf16"
    adt = torch.bfloat16 if bf else torch.float32      # storage of x, w, g, ypool, dx; dw is fp32 either way
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16 if bf else rc.F32, pool_op=args.pool_op)
    avg = args.pool_op == "avg"
    Q = plan.orientations()[0]
    x = torch.from_numpy(synth.make_x(cfg)).cuda().to(adt)
    w = torch.from_numpy(synth.make_w(cfg)).cuda().to(adt)
    g = torch.from_numpy(synth.make_g(cfg)).cuda().to(adt)
    yp = torch.empty((cfg.N, plan.Cpooled, plan.Ho, plan.Wo), dtype=adt, device="cuda")
    idx = torch.empty((cfg.N, plan.Cpooled, plan.Ho, plan.Wo), dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(x)
    dw = torch.empty(w.shape, dtype=torch.float32, device="cuda")
    peak = PEAK_BF16_TFLOPS if bf else PEAK_FP32_TFLOPS
    plan.workspace()

    def step(ev=None):
        if ev:
            ev[0].record()
        rc.rotconv_pool_fwd(plan, x, w, yp, idx)
        if ev:
            ev[1].record()
        rc.rotconv_pool_bwd_data(plan, g, idx, w, dx)
        if ev:
            ev[2].record()
        rc.rotconv_pool_bwd_weight(plan, x, g, idx, dw)
        if ev:
            ev[3].record()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # library calls are enqueued on torch's current stream, so torch events bracket them
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    pass_ms = [sum(events[s][i].elapsed_time(events[s][i + 1]) for s in range(args.steps)) / args.steps
               for i in range(3)]
    names = ["rotconv_pool_fwd", "rotconv_pool_bwd_data", "rotconv_pool_bwd_weight"]
    # p4m: the paper's count is ONE conv-equivalent for the eight filters (the products of the base filter placed at
    # eight position maps); the kernels execute two (the mirror image is a second bank)
    fa, fd = flops_alg(cfg, 1 if args.group == "p4m8" else Q), flops_dense(cfg)
    if avg:     # the mean commutes with the convolution: one conv-equivalent per pooled channel, no placement adds
        fa = 2.0 * cfg.N * cfg.Ho * cfg.Wo * cfg.Cin * plan.Cpooled * cfg.k * cfg.k
    dom = max(range(3), key=lambda i: pass_ms[i])
    achieved = fa / (pass_ms[dom] * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and not args.group:
        try:
            traffic = json.load(open(tpath)).get(f"{args.workload}:{names[dom]}:{plan.kernel_name(dom)}")   # fp32 kernels only
        except Exception:
            traffic = None
    out = {
        "metric": "rotconv_fwd_bwd_tflops", "value": 3.0 * fa / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: N={cfg.N} Cin={cfg.Cin} Cout={cfg.Cout} {cfg.H}x{cfg.W} k={cfg.k} R={cfg.R} "
                        f"{cfg.mode} G={cfg.G} stride={cfg.stride} pad={cfg.pad} pool={args.pool_op}, "
                        f"fused fwd+bwd_data+bwd_weight",
            "flops_per_pass_algorithmic": fa, "flops_per_pass_dense_equivalent": fd,
            "dense_equivalent_tflops": 3.0 * fd / (ms_step * 1e-3) / 1e12,
            "pass_ms": dict(zip(names, pass_ms)),
            "pass_tflops_algorithmic": {n: fa / (t * 1e-3) / 1e12 for n, t in zip(names, pass_ms)},
            "kernels": {n: plan.kernel_name(i) for i, n in enumerate(names)},
        },
        "roofline": {
            "bound": "mfma", "kernel": f"{names[dom]} ({plan.kernel_name(dom)})", "achieved": achieved,
            "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
        },
    }
    if not args.no_cpu_baseline and not avg:
        out["cpu_baseline"] = cpu_baseline(cfg, Q)
    if args.workload == "C2" and not args.no_unet and not bf and not avg and not args.group and not args.ksize \
            and not args.stride:
        # the second half of the headline metric: ms per UNet-shaped training step at R=4 and R=16
        del x, w, g, yp, idx, dx, dw
        out["unet_train_step"] = {n: bench_unet(n, 5, 2) for n in ("C4", "C5")}
        out["unet_train_step"]["C5_bf16"] = bench_unet("C5", 5, 2, "bf16")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
