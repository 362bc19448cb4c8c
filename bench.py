#!/usr/bin/env python3
"""Benchmark of the fused rotation-convolution hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM: rotconv_pool_fwd, rotconv_pool_bwd_data, rotconv_pool_bwd_weight
(tap tables are built once per plan, outside the step; the filter-bank expansion and the
weight-gradient reduction kernels run inside it).  Workload of the default line: benchmark
configuration 2 (N=8, 64->64 channels, 256x256, 3x3, R=4 exact quarter turns, fp32,
orientation max-pool).

Prints ONE JSON line.  `value` is algorithmic TFLOP/s: per pass
F_alg = 2*P*Cin*Cout*k^2*Q + P*Cout*k^2*R  (Q = distinct first-quadrant angles; the per-tap
channel contraction is shared by the four symmetric rotations, paper Eq. 8), three passes
per step.  Next to it, for every pass (and every layer of the UNet-shaped steps appended to
the default line): the flops the kernel EXECUTES (the library reports the conv-equivalents
its matrix instructions perform), the algorithmic HBM bytes, and the fraction of the roof
max(executed flops / matrix peak of the dtype, bytes / 8 TB/s) that the measured time
reaches.  Fractions are computed from the executed count only, so none can exceed 1; rates
at the paper's count are given as TFLOP/s.  The default line also carries the R=16 layer
(configuration 3, fp32 and bf16), the UNet-shaped steps (configurations 4 and 5, fp32 and
bf16) layer by layer, and the measured matrix and copy peaks of the box.
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
# Vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane-instructions/s; the published 157.3 TFLOP/s fp32
# vector peak is that rate with packed two-wide multiply-adds (x 2 x 2).  A kernel on the vector ALU is priced at the
# published peak: a multiply-add counts 2 flop, an addition 1 flop at half of it (78.6e12 additions/s).  This build
# keeps the packed fp32 forms off, so what it can reach is half of that roof (`frac_of_unpacked_alu_roof`).
PEAK_VALU_LANE_OPS = 256 * 4 * 16 * 2.4e9
PASSES = ["rotconv_pool_fwd", "rotconv_pool_bwd_data", "rotconv_pool_bwd_weight"]


def flops_alg(cfg, Q):
    P = cfg.N * cfg.Ho * cfg.Wo
    return 2.0 * P * cfg.Cin * cfg.Cout * cfg.k * cfg.k * Q + 1.0 * P * cfg.Cout * cfg.k * cfg.k * cfg.R


def flops_dense(cfg):
    P = cfg.N * cfg.Ho * cfg.Wo
    return 2.0 * P * cfg.Cin * cfg.Cout * cfg.k * cfg.k * cfg.R


def source_digest():
    """sha256 over the library's sources: a stored counter reading is quoted only for the sources it was taken on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2512_08888_amd", "csrc", "*"))):
        if not f.endswith((".hip", ".h", ".cpp")):
            continue
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(key):
    """HBM bytes per launch of a pass's kernels from the committed rocprofv3 reading (profiles/hbm_traffic.json),
    or None when that reading was taken on other sources than the ones this run executes."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        d = json.load(open(path))
    except Exception:
        return None
    if d.get("source_digest") != source_digest():
        return None
    return d.get(key)


def pass_accounting(N, Cin, Cout, H, W, R, q_paper, c_pooled, k, plan, pass_ms, bf16, w_elems):
    """Per fused pass of one layer: ms, the method's flops (Eq. 8: q_paper conv-equivalents of the channel
    contraction + one add per (tap, orientation) for the placement), the flops the kernel executes, the
    algorithmic HBM bytes, the roof max(executed / matrix peak, bytes / 8 TB/s) in ms and the fraction of it that
    the measured time reaches (<= 1 by construction)."""
    Ho, Wo = plan.Ho, plan.Wo
    P = N * Ho * Wo
    ce = 2.0 * P * Cin * Cout * k * k          # one conv-equivalent
    adds = 1.0 * P * Cout * k * k * R
    e = 2 if bf16 else 4
    peak = (PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS) * 1e12
    b_in, b_out = e * N * Cin * H * W, (e + 1) * N * c_pooled * Ho * Wo
    nbytes = [b_in + b_out + e * w_elems, b_out + b_in + e * w_elems, b_in + b_out + 4 * w_elems]
    out = {}
    for i, name in enumerate(PASSES):
        if pass_ms.get(name) is None:
            continue
        ms = pass_ms[name]
        f_exec = ce * plan.conv_equivalents(i) + adds
        f_alg = ce * q_paper + adds
        t_hbm = nbytes[i] / (PEAK_HBM_GBS * 1e9)
        valu = plan.kernel_name(i) == "valu_direct"
        if valu:       # multiply-adds and placement additions as vector instructions, two per lane and clock at the peak
            lane_ops = ce * plan.conv_equivalents(i) / 2.0 + adds
            t_cmp = lane_ops / (2.0 * PEAK_VALU_LANE_OPS)
        else:
            t_cmp = f_exec / peak
        roof_ms = max(t_cmp, t_hbm) * 1e3
        out[name] = {
            "ms": round(ms, 4), "kernel": plan.kernel_name(i),
            "flops_algorithmic": f_alg, "flops_executed": f_exec,
            "conv_equivalents_paper": q_paper, "conv_equivalents_executed": plan.conv_equivalents(i),
            "bytes_algorithmic": nbytes[i],
            "tflops_paper_count": round(f_alg / (ms * 1e-3) / 1e12, 2),
            "tflops_executed": round(f_exec / (ms * 1e-3) / 1e12, 2),
            "bound": "hbm" if t_hbm > t_cmp else "alu" if valu else "mfma",
            "roof_ms": round(roof_ms, 4), "frac_of_roof": round(roof_ms / ms, 4),
        }
        if valu:
            out[name]["frac_of_unpacked_alu_roof"] = round(max(2.0 * t_cmp, t_hbm) * 1e3 / ms, 4)
    return out


def check_fractions(tree, where=""):
    """No fraction of a roof may exceed 1: that would mean the accounting credits work that was not executed."""
    bad = []
    if isinstance(tree, dict):
        for k_, v in tree.items():
            if k_ in ("frac_of_roof", "frac", "rotconv_frac_of_roof") and isinstance(v, (int, float)) and v > 1.0:
                bad.append((f"{where}/{k_}", v))
            bad += check_fractions(v, f"{where}/{k_}")
    return bad


def cpu_baseline(cfg, Q):
    """The oracle as it stands, timed on the host cores on a bounded sample (a batch slice)."""
    import dataclasses
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


def measured_peaks():
    """Sustained matrix rate of a register-resident loop of independent matrix instructions (fp32 16x16x4 and bf16
    16x16x32) and the bandwidth of a plain 1 GiB device copy, both through the library's measuring kernels."""
    import torch
    from paper_2512_08888_amd import binding as rc

    out = {}
    sink = torch.empty(rc.rotconv_diag_mfma_sink_bytes() // 4, dtype=torch.float32, device="cuda")
    for name, dt, n_iter in (("f32", rc.F32, 4000), ("bf16", rc.BF16, 8000)):
        rc.rotconv_diag_mfma(dt, 200, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = rc.rotconv_diag_mfma(dt, n_iter, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    rc.rotconv_diag_copy(dst, src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        rc.rotconv_diag_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    gbs = 5 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst, sink
    torch.cuda.empty_cache()
    return {"measured_peak_tflops": out, "measured_hbm_gbs": round(gbs, 1),
            "measured_how": "matrix: 2048 workgroups x 4 waves x 8 independent accumulator tiles, registers only; "
                            "copy: 1 GiB read + 1 GiB written, 16 bytes per lane"}


def bench_layer(cfg, steps, warmup, dtype="f32", pool_op="max", q_paper=None, calibrate_copy=False):
    """The three fused calls of one layer: step time between synchronisations, per-pass times from events on the
    launch stream, and the per-pass accounting."""
    import torch
    from paper_2512_08888_amd import binding as rc
    from paper_2512_08888_amd import synth

    bf = dtype == "bf16"
    adt = torch.bfloat16 if bf else torch.float32      # storage of x, w, g, ypool, dx; dw is fp32 either way
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16 if bf else rc.F32, pool_op=pool_op)
    Q = plan.orientations()[0]
    x = torch.from_numpy(synth.make_x(cfg)).cuda().to(adt)
    w = torch.from_numpy(synth.make_w(cfg)).cuda().to(adt)
    g = torch.from_numpy(synth.make_g(cfg)).cuda().to(adt)
    yp = torch.empty((cfg.N, plan.Cpooled, plan.Ho, plan.Wo), dtype=adt, device="cuda")
    idx = torch.empty((cfg.N, plan.Cpooled, plan.Ho, plan.Wo), dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(x)
    dw = torch.empty(w.shape, dtype=torch.float32, device="cuda")
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

    if calibrate_copy:      # a plain copy of known size in the same process, for scaling rocprofv3 byte counters
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        rc.rotconv_diag_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # library calls are enqueued on torch's current stream, so torch events bracket them
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        step(events[s])
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    pass_ms = {n: sum(events[s][i].elapsed_time(events[s][i + 1]) for s in range(steps)) / steps
               for i, n in enumerate(PASSES)}
    qp = Q if q_paper is None else q_paper
    if pool_op == "avg":     # the mean commutes with the convolution: one convolution per pooled channel
        acc = pass_accounting(cfg.N, cfg.Cin, plan.Cpooled, cfg.H, cfg.W, 0, 1, plan.Cpooled, cfg.k, plan, pass_ms, bf,
                              w.numel())
        for a in acc.values():
            a["flops_executed"] = a["flops_algorithmic"]
    else:
        acc = pass_accounting(cfg.N, cfg.Cin, cfg.Cout, cfg.H, cfg.W, cfg.R, qp, plan.Cpooled, cfg.k, plan, pass_ms, bf,
                              w.numel())
    del x, w, g, yp, idx, dx, dw
    return plan, Q, ms_step, pass_ms, acc


def layer_summary(cfg, steps, warmup, dtype):
    """Compact record of one single-layer workload for the default line's extra keys."""
    plan, Q, ms_step, pass_ms, acc = bench_layer(cfg, steps, warmup, dtype)
    f_alg = sum(a["flops_algorithmic"] for a in acc.values())
    f_exec = sum(a["flops_executed"] for a in acc.values())
    roof = sum(a["roof_ms"] for a in acc.values())
    tot = sum(a["ms"] for a in acc.values())
    return {"workload": f"{cfg.name}: N={cfg.N} Cin={cfg.Cin} Cout={cfg.Cout} {cfg.H}x{cfg.W} R={cfg.R} {cfg.mode} "
                        f"G={cfg.G}, fused fwd+bwd_data+bwd_weight", "dtype": dtype, "ms_per_step": round(ms_step, 4),
            "tflops_paper_count": round(f_alg / (ms_step * 1e-3) / 1e12, 2),
            "tflops_executed": round(f_exec / (ms_step * 1e-3) / 1e12, 2),
            "peak_tflops": PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_FP32_TFLOPS,
            "frac_of_roof": round(roof / tot, 4), "passes": acc}


def bench_unet(name, steps, warmup, dtype="f32", graph=False):
    """ms per training step of the UNet-shaped stack (benchmark configurations 4 and 5; P4 / P8 / P16: the
    paper's own block, rotation convolution then standard convolution, at 4 / 8 / 16 orientations; fp32), whole
    step timed between synchronisations; then one more step with an event pair around every library
    call for the per-call and per-layer breakdown."""
    import torch
    from paper_2512_08888_amd import unet as un

    cfg = un.UNET_CONFIGS[name]
    bf = dtype == "bf16"
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
            by_layer.setdefault(where, {})[what] = t
    net.trace = None
    alg, dense = net.rot_flops()
    rot_ms = sum(t for k, t in by_call.items() if k.startswith("rotconv"))
    loss = float(net.loss.cpu()[0])
    # per layer and pass: the paper's count, the executed count, the roof and the fraction reached
    layers = {}
    tot = {"ms": 0.0, "roof_ms": 0.0, "flops_algorithmic": 0.0, "flops_executed": 0.0}
    for sp in net.specs:
        plan = net.plans[sp["name"]]
        q_paper = plan.orientations()[0]
        w_elems = sp["B"] * sp["Cout"] * sp["Cin"] * 9
        acc = pass_accounting(cfg.N, sp["Cin"], sp["Cout"], sp["H"], sp["W"], sp["R"], q_paper, sp["width"], 3, plan,
                              by_layer.get(sp["name"], {}), bf, w_elems)
        layers[sp["name"]] = {"shape": f"{sp['Cin']}->{sp['Cout']} @{sp['H']}x{sp['W']} R={sp['R']}", "passes": acc}
        for a in acc.values():
            for k_ in tot:
                tot[k_] += a[k_]
    peak = PEAK_BF16_TFLOPS if bf else PEAK_FP32_TFLOPS
    out = {
        "workload": f"{cfg.name}: UNet-shaped stack, N={cfg.N} {cfg.H}x{cfg.W} widths={list(cfg.widths)} "
                    f"classes={cfg.classes} R={cfg.R} {cfg.mode} block={cfg.block}, one training step (fwd+bwd), "
                    + ("fp32" if dtype == "f32" else "bf16 parameters / activations, fp32 accumulation, fp32 dW and loss"),
        "dtype": dtype,
        "ms_per_step": ms, "ms_per_step_graph_replay": ms_graph, "steps": steps, "warmup": warmup, "loss": loss,
        "rotconv_flops_algorithmic": alg, "rotconv_flops_executed": tot["flops_executed"],
        "rotconv_flops_dense_equivalent": dense,
        "rotconv_ms": rot_ms, "glue_ms": sum(by_call.values()) - rot_ms,
        "rotconv_tflops_paper_count": alg / (rot_ms * 1e-3) / 1e12,
        "rotconv_tflops_executed": tot["flops_executed"] / (rot_ms * 1e-3) / 1e12,
        "rotconv_roof_ms": round(tot["roof_ms"], 3),
        "rotconv_frac_of_roof": round(tot["roof_ms"] / rot_ms, 4),
        "peak_tflops": peak,
        "ms_by_call": {k: round(v, 4) for k, v in sorted(by_call.items())},
        "layers": layers,
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
                     "kernel": "all rotation-convolution calls of the step (fwd, bwd_data, bwd_weight; 18 layers), "
                               "at the flops they execute; per layer and pass: config.layers",
                     "achieved": r["rotconv_tflops_executed"], "peak": r["peak_tflops"], "unit": "TFLOP/s",
                     "frac": r["rotconv_tflops_executed"] / r["peak_tflops"],
                     "frac_of_layerwise_roof": r["rotconv_frac_of_roof"], "traffic": None},
    }
    bad = check_fractions(out)
    if bad:
        out["accounting_error"] = [f"{w}: {v}" for w, v in bad]
        print(f"bench.py: fraction above 1: {bad}", file=sys.stderr)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_unet(args.workload)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "P4", "P8", "P16", "sweep", "C4_enc0a", "C5_enc0a", "C5_enc0b"],
                    help="C1-C3: the single layers; C4 / C5: the UNet-shaped training step; P4 / P8 / P16: the paper's own "
                         "block; C4_enc0a / C5_enc0a: the first layer (3 -> 64 channels, 512 x 512) of those stacks alone; C5_enc0b: the second one (64 -> 64)")
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
    ap.add_argument("--no-unet", action="store_true",
                    help="skip what the default line appends: configuration 3, the UNet-shaped steps, the measured peaks")
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
    from paper_2512_08888_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    q_paper = None
    if args.group == "p4m8":
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "_p4m8", R=8, mode="p4m", angles_deg=None, pool_group=None)
        q_paper = 1      # the paper's count: the products of the base filter placed at eight position maps
    if args.ksize or args.stride:
        import dataclasses
        k = args.ksize or cfg.k
        cfg = dataclasses.replace(cfg, name=f"{cfg.name}_k{k}_s{args.stride or cfg.stride}", k=k, pad=k // 2,
                                  stride=args.stride or cfg.stride)
    bf = args.dtype == "bf16"
    avg = args.pool_op == "avg"
    peak = PEAK_BF16_TFLOPS if bf else PEAK_FP32_TFLOPS
    plan, Q, ms_step, pass_ms, acc = bench_layer(cfg, args.steps, args.warmup, args.dtype, args.pool_op, q_paper,
                                                 args.calibrate_copy)
    fa = sum(a["flops_algorithmic"] for a in acc.values()) / 3.0
    fd = flops_dense(cfg)
    # the roofline object: the slowest pass, at the flops its kernel executes
    dom = max(PASSES, key=lambda n: pass_ms[n])
    a = acc[dom]
    achieved = a["flops_executed"] / (a["ms"] * 1e-3) / 1e12
    roof_unit = "TFLOP/s"
    if a["bound"] == "alu":      # vector-ALU kernel: against the published fp32 vector peak (see PEAK_VALU_LANE_OPS)
        peak, achieved = PEAK_FP32_TFLOPS, a["frac_of_roof"] * PEAK_FP32_TFLOPS
    elif a["bound"] == "hbm":
        peak, achieved, roof_unit = PEAK_HBM_GBS, a["bytes_algorithmic"] / (a["ms"] * 1e-3) / 1e9, "GB/s"
    std = args.workload in ("C2", "C3", "C4_enc0a", "C5_enc0a", "C5_enc0b") and not args.group and not args.ksize and not args.stride and not avg
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
            "passes": acc,
        },
        "roofline": {
            "bound": a["bound"], "kernel": f"{dom} ({a['kernel']})", "achieved": achieved,
            "peak": peak, "unit": roof_unit, "frac": achieved / peak,
            "flops_counted": "executed by the kernel (equal to the paper's count for this pass)"
            if a["flops_executed"] == a["flops_algorithmic"] else "executed by the kernel; the paper's count is in config.passes",
            "traffic": stored_traffic(f"{args.workload}:{dom}:{a['kernel']}") if std else None,
        },
    }
    if not args.no_cpu_baseline and not avg:
        out["cpu_baseline"] = cpu_baseline(cfg, Q)
    if args.workload == "C2" and not args.no_unet and not bf and std:
        # the rest of the headline metric: the R = 16 layer (fp32 and bf16), the R = 4 layer in bf16, ms per
        # UNet-shaped training step at R = 4 and R = 16 layer by layer, and the box's measured peaks
        out["c3_r16_layer"] = {"f32": layer_summary(synth.C3, 20, 3, "f32"), "bf16": layer_summary(synth.C3, 20, 3, "bf16")}
        out["c2_r4_layer_bf16"] = layer_summary(synth.C2, 20, 3, "bf16")
        out["unet_train_step"] = {n: bench_unet(n, 5, 2) for n in ("C4", "C5")}
        out["unet_train_step"]["C5_bf16"] = bench_unet("C5", 5, 2, "bf16")
        out.update(measured_peaks())
    bad = check_fractions(out)
    if bad:
        out["accounting_error"] = [f"{w}: {v}" for w, v in bad]
        print(f"bench.py: fraction above 1: {bad}", file=sys.stderr)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
