"""GPU parity of bfloat16 plans (include/rotconv.h, dtype ROTCONV_BF16) against the fp64 oracle fed the values
the GPU holds: the bf16-rounded inputs and base weights, and the rotated banks rounded to bf16 once more (a bf16
plan keeps its expanded banks in bf16: they are the matrix-core operand; for exact quarter turns that rounding is
the identity).  Bars: bf16 outputs within rel 1e-2 (tighter than the benchmark's 2e-2; one rounding to bf16 is
2^-9), the fp32 weight gradient within 1e-4, arg-max by the near-tie protocol of the fp32 tests; on
exact-arithmetic (dyadic) inputs everything bit for bit."""
import numpy as np
import pytest
import torch

from oracle import rotconv_oracle as orc
from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth
from parity_util import RTOL, assert_close, check_idx, round_bf16

pytestmark = pytest.mark.gpu
LC = synth.LayerConfig
BF_RTOL = 1e-2

CASES = [
    LC("b_r4", N=2, Cin=3, H=9, W=7, Cout=5, R=4, seed=51),                                   # generic kernels
    LC("b_fast", N=2, Cin=20, H=12, W=32, Cout=18, R=4, seed=52),                             # MFMA kernels
    LC("b_r16", N=1, Cin=8, H=10, W=64, Cout=6, R=16, mode="bilinear", seed=53),
    LC("b_ste_g4", N=1, Cin=4, H=8, W=16, Cout=4, R=8, mode="steerable", pool_group=4, seed=54),
    LC("b_s2k5", N=1, Cin=3, H=11, W=10, Cout=4, k=5, pad=2, stride=2, R=4, seed=55),
    # shapes of the bf16 matrix-core kernels: two chunks in flight, padded channels, ragged rows, wave chains
    # beyond the row, segmented rows, several bands, a streamed filter block
    LC("b_c64", N=2, Cin=64, H=40, W=64, Cout=32, R=4, x_dist="absnormal", seed=56),
    LC("b_c96", N=1, Cin=96, H=9, W=40, Cout=20, R=4, x_dist="absnormal", seed=57),
    LC("b_w14", N=1, Cin=33, H=7, W=14, Cout=16, R=4, seed=58),
    LC("b_c160_r16", N=1, Cin=160, H=12, W=32, Cout=24, R=16, mode="bilinear", x_dist="absnormal", seed=59),
    LC("b_w320", N=1, Cin=16, H=6, W=320, Cout=16, R=4, seed=60),
    LC("b_stream", N=1, Cin=512, H=8, W=32, Cout=16, R=4, x_dist="absnormal", seed=61),
    LC("b_stream_w96", N=1, Cin=576, H=5, W=96, Cout=8, R=8, mode="bilinear", pool_group=4, x_dist="absnormal", seed=62),
    # filter counts of the input-gradient kernel: two K-steps in flight, padded filters, streamed filter blocks
    LC("b_co64", N=2, Cin=24, H=10, W=64, Cout=64, R=4, seed=64),
    LC("b_co96", N=1, Cin=16, H=6, W=40, Cout=96, R=4, seed=65),
    LC("b_co192_r16", N=1, Cin=16, H=5, W=32, Cout=192, R=16, mode="bilinear", seed=66),
    LC("b_co576_w96", N=1, Cin=8, H=5, W=96, Cout=576, R=4, seed=67),
    LC("b_r8_fold2", N=1, Cin=40, H=9, W=64, Cout=20, R=8, mode="bilinear", seed=71),          # two banks in one wave
    LC("b_r16_fold4_w40", N=2, Cin=64, H=7, W=40, Cout=10, R=16, mode="steerable", x_dist="absnormal", seed=72),
    LC("b_r1", N=1, Cin=24, H=9, W=32, Cout=40, R=1, seed=68),                                 # a standard convolution
    # orientation sets without all four quarter turns per bank: the dense input-gradient instances
    LC("b_p4m", N=1, Cin=24, H=9, W=32, Cout=40, R=8, mode="p4m", seed=73),
    LC("b_r2", N=1, Cin=16, H=8, W=32, Cout=80, R=2, seed=74),
    # the table gradient kernels: two channel groups of 128, filters padded to a K-step, rows that end inside a lane
    # group (the weight gradient of this width runs on widened copies)
    LC("b_lut_w44", N=1, Cin=136, H=6, W=44, Cout=40, R=16, mode="bilinear", x_dist="absnormal", seed=75),
    # the weight gradient whose channel groups build a filter block's D together: two groups; five groups (two sets
    # of four, the second mostly empty) over several units; two base banks
    LC("b_lut_c128", N=1, Cin=128, H=7, W=40, Cout=24, R=16, mode="bilinear", x_dist="absnormal", seed=76),
    LC("b_lut_c320", N=2, Cin=320, H=9, W=72, Cout=40, R=16, mode="bilinear", x_dist="absnormal", seed=77),
    LC("b_lut_ste_c192", N=1, Cin=192, H=6, W=32, Cout=20, R=16, mode="steerable", x_dist="absnormal", seed=78),
    # the input gradient with shared D and its K-steps split over workgroups
    LC("b_lut_ks_c384", N=1, Cin=384, H=5, W=32, Cout=192, R=16, mode="bilinear", x_dist="absnormal", seed=79),
    # the forward with a lane per pixel column: one to four K-steps, a last K-step with idle channel groups, padded rows
    # that end inside / at a wave's 14 outputs, ragged filter blocks, several images and bands, all three modes
    LC("b_px_c8", N=2, Cin=8, H=9, W=12, Cout=5, R=4, seed=81),
    LC("b_px_c40_w26", N=1, Cin=40, H=35, W=26, Cout=20, R=8, mode="bilinear", seed=82),
    LC("b_px_c72_w27", N=2, Cin=72, H=7, W=27, Cout=33, R=16, mode="bilinear", x_dist="absnormal", seed=83),
    LC("b_px_c128_ste", N=1, Cin=128, H=40, W=70, Cout=16, R=16, mode="steerable", x_dist="absnormal", seed=84),
    LC("b_px_c104_r4", N=3, Cin=104, H=6, W=13, Cout=48, R=4, seed=85),
    # a layer on which one arg-max sat just outside the fp32 near-tie band when the rotated weights were formed in fp32
    # (one of them rounded to the neighbouring bf16 value); they are formed in fp64 now: the regression case
    LC("b_r16_bank_rounding", N=2, Cin=32, H=19, W=160, Cout=136, R=16, mode="bilinear", x_dist="absnormal", seed=9148),
]


def bf(a):
    """numpy fp32/fp64 -> (torch bf16 cuda tensor, the rounded values as fp64)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.cuda(), t.to(torch.float64).numpy()


def nan16(*shape):
    return torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")


def f64(t):
    torch.cuda.synchronize()
    return t.to(torch.float64).cpu().numpy()


def reference(cfg, x, w, ang):
    """Forward of the oracle on the banks a bf16 plan multiplies with."""
    w_rot = round_bf16(orc.expand_bank(w, cfg.R, ang, cfg.mode))
    y = orc.rotconv_fwd(x, w_rot, cfg.stride, cfg.pad)
    yp, idx = orc.orient_maxpool_fwd(y, cfg.G)
    return w_rot, y, yp, idx


def dw_rtol(plan):
    """Bar of the fp32 weight gradient of a bf16 plan.  The per-bank kernels multiply exact bf16 operands and
    accumulate in fp32: the fp32 bar.  The table kernels ("..._lut") fold the routed gradients of all orientations
    into the base taps in fp32 and round that sum to bf16 once, because it is the matrix-core operand: one bf16
    rounding (2^-9) per operand, the bar of every bf16-typed quantity."""
    return BF_RTOL if plan.kernel_name(2).endswith("_lut") else RTOL


def reference_bwd(cfg, x, w_rot, g, idx, ang):
    dy = orc.orient_maxpool_bwd(g, idx, cfg.R, cfg.G)
    dx = orc.rotconv_bwd_data(dy, w_rot, cfg.H, cfg.W, cfg.stride, cfg.pad)
    dw = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dy, cfg.k, cfg.stride, cfg.pad), ang, cfg.mode)
    return dx, dw


@pytest.mark.parametrize("cfg", CASES, ids=[c.name for c in CASES])
def test_bf16_fused_calls(cfg):
    run_bf16_fused(cfg)


def px_plan(cfg):
    """Can the pooled forward of this layer's bf16 plan take the kernel with a lane per pixel column?  (3 x 3 / stride 1
    / pad 1, 8 to 128 input channels in eights, one pool group over an evenly spaced set of 4, 8 or 16 orientations; it
    is the default for R = 16 up to 64 channels, plan option px_fwd = 1 takes it wherever it can run.)"""
    return (cfg.k == 3 and cfg.stride == 1 and cfg.pad == 1 and 8 <= cfg.Cin <= 128 and cfg.Cin % 8 == 0 and cfg.G == cfg.R
            and cfg.R in (4, 8, 16) and cfg.mode != "p4m" and cfg.angles_deg is None)


PX_CASES = [c for c in CASES if px_plan(c)]


@pytest.mark.parametrize("cfg", PX_CASES, ids=[c.name for c in PX_CASES])
def test_bf16_fused_calls_on_both_forward_kernels(cfg):
    """The layers whose forward can take the pixel-column kernel, on that kernel (plan option px_fwd = 1) and on the
    kernel with eight pixels per lane (px_fwd = -1), whichever of the two the default plan picks."""
    assert rc.Plan.from_config(cfg, dtype=rc.BF16, options=dict(px_fwd=1)).kernel_name(0) == "mfma_px_bf16"
    assert rc.Plan.from_config(cfg, dtype=rc.BF16, options=dict(px_fwd=-1)).kernel_name(0) == "mfma_p4_bf16"
    default = rc.Plan.from_config(cfg, dtype=rc.BF16).kernel_name(0)
    assert (default == "mfma_px_bf16") == (cfg.R == 16 and cfg.Cin <= 64)
    run_bf16_fused(cfg, options=dict(px_fwd=1))
    run_bf16_fused(cfg, options=dict(px_fwd=-1))


def run_bf16_fused(cfg, options=None):
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16, options=options)
    print(f"[case] bf16 fused {cfg.name} kernels {[plan.kernel_name(i) for i in range(3)]}", flush=True)
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    xd, x = bf(synth.make_x(cfg))
    wd, w = bf(synth.make_w(cfg))
    gd, g = bf(synth.make_g(cfg))
    P = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    yp, idx = nan16(*P), torch.full(P, 255, dtype=torch.uint8, device="cuda")
    rc.rotconv_pool_fwd(plan, xd, wd, yp, idx)
    w_rot, y_ref, yp_ref, idx_ref = reference(cfg, x, w, ang)
    assert_close(f64(yp), yp_ref, f"{cfg.name} ypool", rtol=BF_RTOL)
    abs_terms = orc.rotconv_fwd(np.abs(x), np.abs(w_rot), cfg.stride, cfg.pad)
    idx_h = idx.cpu().numpy()
    # no allowance for the banks' rounding: library and reference both form a rotated weight in fp64 and round it
    # to fp32, then to bf16, so they multiply with the same bf16 banks (b_r16_bank_rounding is the regression case)
    check_idx(idx_h, y_ref, abs_terms, cfg.G, f"{cfg.name} idx")
    # backward on the GPU's own idx, both sides
    dx_ref, dw_ref = reference_bwd(cfg, x, w_rot, g, idx_h, ang)
    dx = nan16(*xd.shape)
    rc.rotconv_pool_bwd_data(plan, gd, idx, wd, dx)
    assert_close(f64(dx), dx_ref, f"{cfg.name} dx", rtol=BF_RTOL)
    dw = torch.full(tuple(wd.shape), float("nan"), dtype=torch.float32, device="cuda")
    rc.rotconv_pool_bwd_weight(plan, xd, gd, idx, dw)
    assert_close(f64(dw), dw_ref, f"{cfg.name} dw (fp32)", rtol=dw_rtol(plan))


@pytest.mark.parametrize("name", ["b_r16", "b_c160_r16", "b_co192_r16", "b_r8_fold2", "b_r16_fold4_w40", "b_p4m"])
def test_bf16_gradients_per_bank_kernels(name):
    """Layers whose gradients take the routed-gradient table by default, on the per-bank bf16 gradient kernels
    (plan option bwd_lut = -1): exact bf16 operands, the fp32 bar for dW."""
    cfg = next(c for c in CASES if c.name == name)
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16, options=dict(bwd_lut=-1))
    print(f"[case] bf16 per-bank gradients {cfg.name} kernels {[plan.kernel_name(i) for i in range(3)]}", flush=True)
    assert not plan.kernel_name(1).endswith("_lut") and not plan.kernel_name(2).endswith("_lut")
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    xd, x = bf(synth.make_x(cfg))
    wd, w = bf(synth.make_w(cfg))
    gd, g = bf(synth.make_g(cfg))
    w_rot = round_bf16(orc.expand_bank(w, cfg.R, ang, cfg.mode))
    idx_h = synth.make_idx(cfg)
    idx = torch.from_numpy(idx_h).cuda()
    dx_ref, dw_ref = reference_bwd(cfg, x, w_rot, g, idx_h, ang)
    dx = nan16(*xd.shape)
    rc.rotconv_pool_bwd_data(plan, gd, idx, wd, dx)
    assert_close(f64(dx), dx_ref, f"{cfg.name} dx", rtol=BF_RTOL)
    dw = torch.full(tuple(wd.shape), float("nan"), dtype=torch.float32, device="cuda")
    rc.rotconv_pool_bwd_weight(plan, xd, gd, idx, dw)
    assert_close(f64(dw), dw_ref, f"{cfg.name} dw (fp32)", rtol=RTOL)


DYADIC = [CASES[1], CASES[5], CASES[7], next(c for c in CASES if c.name == "b_px_c8"), next(c for c in CASES if c.name == "b_px_c104_r4"), LC("b_dy_stream", N=1, Cin=512, H=6, W=64, Cout=16, R=4, seed=63),
          LC("b_dy_co64", N=1, Cin=40, H=20, W=64, Cout=64, R=4, seed=69),
          LC("b_dy_co576", N=1, Cin=8, H=5, W=64, Cout=576, R=4, seed=70)]


@pytest.mark.parametrize("cfg", DYADIC, ids=[c.name for c in DYADIC])
def test_bf16_dyadic_bit_exact(cfg):
    run_bf16_dyadic(cfg)
    if px_plan(cfg):
        run_bf16_dyadic(cfg, options=dict(px_fwd=1))
        run_bf16_dyadic(cfg, options=dict(px_fwd=-1))


def run_bf16_dyadic(cfg, options=None):
    """Inputs on the exact-arithmetic grid (all representable in bf16; every fp32 partial sum exact in any
    order): pooled output = the oracle's rounded once to bf16, arg-max and dX (rounded once) bit for bit."""
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16, options=options)
    print(f"[case] bf16 dyadic {cfg.name}", flush=True)
    xd, x = bf(synth.make_x_dyadic(cfg))
    wd, w = bf(synth.make_w_dyadic(cfg))
    gd, g = bf(synth.make_g_dyadic(cfg))
    assert np.array_equal(x, synth.make_x_dyadic(cfg)) and np.array_equal(w, synth.make_w_dyadic(cfg))
    P = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    yp, idx = nan16(*P), torch.full(P, 255, dtype=torch.uint8, device="cuda")
    rc.rotconv_pool_fwd(plan, xd, wd, yp, idx)
    w_rot, y_ref, yp_ref, idx_ref = reference(cfg, x, w, None)
    assert np.array_equal(idx.cpu().numpy(), idx_ref), f"{cfg.name}: arg-max not bit-exact"
    assert np.array_equal(f64(yp), round_bf16(yp_ref)), f"{cfg.name}: pooled output not bit-exact"
    dx_ref, dw_ref = reference_bwd(cfg, x, w_rot, g, idx_ref, None)
    dx = nan16(*xd.shape)
    rc.rotconv_pool_bwd_data(plan, gd, idx, wd, dx)
    assert np.array_equal(f64(dx), round_bf16(dx_ref)), f"{cfg.name}: dx not bit-exact"
    dw = torch.full(tuple(wd.shape), float("nan"), dtype=torch.float32, device="cuda")
    rc.rotconv_pool_bwd_weight(plan, xd, gd, idx, dw)
    if cfg.N * cfg.Ho * cfg.Wo <= (1 << 14):
        assert np.array_equal(f64(dw), dw_ref), f"{cfg.name}: dw not bit-exact"


def test_bf16_unfused_chain():
    cfg = CASES[1]
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
    xd, x = bf(synth.make_x(cfg))
    wd, w = bf(synth.make_w(cfg))
    U = (cfg.N, plan.Cunpooled, plan.Ho, plan.Wo)
    P = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    y = nan16(*U)
    rc.rotconv_fwd(plan, xd, wd, y)
    w_rot = orc.expand_bank(w, cfg.R, None, cfg.mode)
    y_ref = orc.rotconv_fwd(x, w_rot, cfg.stride, cfg.pad)
    assert_close(f64(y).reshape(y_ref.shape), y_ref, "unfused y", rtol=BF_RTOL)
    # pooling of the bf16 map is exact: the winner's bits are copied
    yp, idx = nan16(*P), torch.full(P, 255, dtype=torch.uint8, device="cuda")
    rc.orient_maxpool_fwd(plan, y, yp, idx)
    y_h = f64(y).reshape(y_ref.shape)
    yp_o, idx_o = orc.orient_maxpool_fwd(y_h, cfg.G)
    assert np.array_equal(f64(yp), yp_o) and np.array_equal(idx.cpu().numpy(), idx_o)
    gd, g = bf(synth.make_g(cfg))
    dy = nan16(*U)
    rc.orient_maxpool_bwd(plan, gd, idx, dy)
    dy_o = orc.orient_maxpool_bwd(g, idx_o, cfg.R, cfg.G)
    assert np.array_equal(f64(dy).reshape(dy_o.shape), dy_o)
    dx = nan16(*xd.shape)
    rc.rotconv_bwd_data(plan, dy, wd, dx)
    assert_close(f64(dx), orc.rotconv_bwd_data(dy_o, w_rot, cfg.H, cfg.W, cfg.stride, cfg.pad), "unfused dx", rtol=BF_RTOL)
    dw = torch.full(tuple(wd.shape), float("nan"), dtype=torch.float32, device="cuda")
    rc.rotconv_bwd_weight(plan, xd, dy, dw)
    dw_rot = orc.rotconv_bwd_weight(x, dy_o, cfg.k, cfg.stride, cfg.pad)
    assert_close(f64(dw), orc.reduce_bank_grad(dw_rot, None, cfg.mode), "unfused dw (fp32)", rtol=RTOL)


def test_bf16_workspace_too_small_is_rejected():
    cfg = CASES[0]
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
    xd, _ = bf(synth.make_x(cfg))
    wd, _ = bf(synth.make_w(cfg))
    P = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    small = torch.empty(plan.workspace_bytes - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(rc.RotconvError) as e:
        rc.rotconv_pool_fwd(plan, xd, wd, nan16(*P), torch.empty(P, dtype=torch.uint8, device="cuda"), small)
    assert e.value.status == rc.ERR_WORKSPACE


def _pts(seed, n, dims):
    return np.stack([synth.randint(seed + i, n, 0, d - 1) for i, d in enumerate(dims)], axis=1).astype(np.int32)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cfg,ns,npairs", [(synth.C2, 4096, 24), (synth.C3, 2048, 12)], ids=["C2", "C3"])
def test_bf16_config_full_size_sampled(cfg, ns, npairs):
    """Benchmark configurations 2 and 3 with bf16 tensors at full size, in the launch configuration bench.py --dtype bf16
    times: sampled pooled outputs with arg-max, sampled dX and sampled (co,ci) dW slices computed one by one by the
    oracle on the bf16 values, plus the homogeneity identities at full size."""
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
    print(f"[case] bf16 full size {cfg.name} kernels {[plan.kernel_name(i) for i in range(3)]}", flush=True)
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    xd, x = bf(synth.make_x(cfg))
    wd, w = bf(synth.make_w(cfg))
    gd, g = bf(synth.make_g(cfg))
    P = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    ypd, idxd = nan16(*P), torch.full(P, 255, dtype=torch.uint8, device="cuda")
    rc.rotconv_pool_fwd(plan, xd, wd, ypd, idxd)
    yp, idx = f64(ypd), idxd.cpu().numpy()
    w_rot = round_bf16(orc.expand_bank(w, cfg.R, ang, cfg.mode))
    ng = cfg.R // cfg.G
    pts = _pts(cfg.seed + 100, ns, (cfg.N, cfg.Cout, cfg.Ho, cfg.Wo))
    yr = orc.rotconv_fwd_at(x, w_rot, pts, cfg.stride, cfg.pad)
    ya = orc.rotconv_fwd_at(np.abs(x), np.abs(w_rot), pts, cfg.stride, cfg.pad)
    rms = float(np.sqrt(np.mean(yr.reshape(-1, cfg.G, ng).max(axis=1) ** 2)))
    for grp in range(ng):
        members = np.arange(grp, cfg.R, ng)
        best = yr[:, members].max(axis=1)
        chan = pts[:, 1] * ng + grp
        got_v = yp[pts[:, 0], chan, pts[:, 2], pts[:, 3]]
        got_i = idx[pts[:, 0], chan, pts[:, 2], pts[:, 3]].astype(np.int64)
        assert np.all(np.abs(got_v - best) <= BF_RTOL * np.abs(best) + BF_RTOL * rms), f"{cfg.name} fwd samples"
        tau = 64.0 * np.finfo(np.float32).eps * ya[:, members].max(axis=1)
        assert np.all(got_i % ng == grp) and np.all(yr[np.arange(ns), got_i] >= best - tau), f"{cfg.name} arg-max samples"
    dxd = nan16(*xd.shape)
    rc.rotconv_pool_bwd_data(plan, gd, idxd, wd, dxd)
    dwd = torch.full(tuple(wd.shape), float("nan"), dtype=torch.float32, device="cuda")
    rc.rotconv_pool_bwd_weight(plan, xd, gd, idxd, dwd)
    dx, dw = f64(dxd), f64(dwd)
    if cfg.N * cfg.Cout * cfg.R * cfg.Ho * cfg.Wo <= 160_000_000:
        dy = orc.orient_maxpool_bwd(g, idx, cfg.R, cfg.G)
        ptsx = _pts(cfg.seed + 200, ns, (cfg.N, cfg.Cin, cfg.H, cfg.W))
        ref = orc.rotconv_bwd_data_at(dy, w_rot, ptsx, cfg.H, cfg.W, cfg.stride, cfg.pad)
        assert_close(dx[ptsx[:, 0], ptsx[:, 1], ptsx[:, 2], ptsx[:, 3]], ref, f"{cfg.name} dx samples", rtol=BF_RTOL)
    pairs = _pts(cfg.seed + 300, npairs, (cfg.Cout, cfg.Cin))
    dwr = orc.rotconv_pool_bwd_weight_at(x, g, idx, pairs, cfg.R, cfg.k, cfg.G, cfg.stride, cfg.pad)
    got_dw, ref_dw = [], []
    for t, (co, ci) in enumerate(pairs):
        full = np.zeros((cfg.R, 1, 1, cfg.k, cfg.k))
        full[:, 0, 0] = dwr[t]
        ref_dw.append(orc.reduce_bank_grad(full, ang, cfg.mode)[:, 0, 0])
        got_dw.append(dw[:, co, ci])
    assert_close(np.array(got_dw), np.array(ref_dw), f"{cfg.name} dw samples (fp32)", rtol=dw_rtol(plan))
    # homogeneity through the max: <w, dW> = <x, dX> = <ypool, g>; ypool and dX carry one bf16 rounding each
    a, b, c = float((yp * g).sum()), float((x * dx).sum()), float((w * dw).sum())
    scale = float(np.abs(yp * g).sum())
    assert abs(a - b) <= 1e-4 * scale and abs(a - c) <= 1e-4 * scale, (a, b, c, scale)
