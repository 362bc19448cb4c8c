"""GPU parity of the vector-ALU kernel that runs the pooled forward of layers with at most four input channels (a
network's first layer; include/rotconv.h, plan option `direct`): every element against the oracle at sizes that span
several waves, band rows, ragged tails and padded filter blocks, in fp32 and bf16, bit for bit on the exact-arithmetic
grid, and the first layer of benchmark configurations 4 / 5 at full size element by element.  The gradient calls of
these plans run the matrix-core kernels; run_fused_parity checks them along the way."""
import dataclasses

import numpy as np
import pytest
import torch

import parity_util as pu
import test_gpu_bf16 as tb
from oracle import rotconv_oracle as orc
from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth

pytestmark = pytest.mark.gpu
LC = synth.LayerConfig


def say(msg):
    print(msg, flush=True)


# Row widths around the 62 outputs a wave holds per row (a padded row of W + 2 slots ends inside, at and behind a
# wave), several images and bands, one to four input channels, filter counts that leave the last filter block ragged,
# one / two / four first-quadrant banks in the three expansion modes.
CASES = [
    LC("d_c1", N=1, Cin=3, H=64, W=64, Cout=8, R=4, seed=1),
    LC("d_w5", N=2, Cin=3, H=7, W=5, Cout=3, R=4, seed=301),
    LC("d_w37", N=1, Cin=2, H=9, W=37, Cout=5, R=4, seed=302),
    LC("d_w60", N=3, Cin=3, H=5, W=60, Cout=9, R=4, seed=303),
    LC("d_w61", N=2, Cin=1, H=6, W=61, Cout=8, R=4, seed=304),
    LC("d_w62", N=2, Cin=4, H=6, W=62, Cout=13, R=4, seed=305),
    LC("d_w130", N=1, Cin=3, H=70, W=130, Cout=17, R=4, x_dist="absnormal", seed=306),
    LC("d_r8_bil", N=2, Cin=3, H=11, W=45, Cout=6, R=8, mode="bilinear", seed=307),
    LC("d_r8_ste", N=1, Cin=4, H=8, W=33, Cout=5, R=8, mode="steerable", seed=308),
    LC("d_r16_bil", N=1, Cin=3, H=33, W=37, Cout=5, R=16, mode="bilinear", seed=309),
    LC("d_r16_ste", N=2, Cin=2, H=9, W=66, Cout=3, R=16, mode="steerable", seed=310),
    LC("d_h1", N=1, Cin=3, H=1, W=1, Cout=2, R=4, seed=311),
    # pool groups of four quarter turns (the paper's own block): every bank pooled on its own, Q pooled channels per filter
    LC("d_r8_g4", N=2, Cin=3, H=13, W=70, Cout=7, R=8, mode="bilinear", pool_group=4, seed=312),
    LC("d_r16_g4", N=1, Cin=4, H=9, W=33, Cout=5, R=16, mode="steerable", pool_group=4, seed=313),
]


def direct_plan_check(plan):
    assert plan.kernel_name(0) == "valu_direct", plan.kernel_name(0)
    # the weight gradient of fp32 plans runs the vector-ALU kernel too when the layer has a single bank (R = 4)
    assert (plan.kernel_name(2) == "valu_direct") == (plan.R == 4 and plan.desc.dtype == rc.F32), plan.kernel_name(2)


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_direct_forward_fp32(cfg):
    say(f"[case] direct fp32 {cfg}")
    out = pu.run_fused_parity(cfg)
    direct_plan_check(out["layer"].plan)


@pytest.mark.parametrize("cfg", [c for c in CASES if c.mode == "exact90"], ids=lambda c: c.name)
def test_direct_forward_fp32_dyadic_bit_exact(cfg):
    say(f"[case] direct fp32 dyadic {cfg.name}")
    out = pu.run_fused_parity(cfg, dyadic=True)
    direct_plan_check(out["layer"].plan)


@pytest.mark.parametrize("ty", [1, 3, 8, 200])
@pytest.mark.parametrize("name", ["d_w130", "d_r16_bil"])
def test_direct_forward_band_heights(name, ty):
    """Forced band heights: one row per band, bands that do not divide H, one band for the whole image; the pooled
    output and the arg-max must not depend on the split (bit for bit against the automatic setting)."""
    cfg = next(c for c in CASES if c.name == name)
    say(f"[case] direct band height {name} ty={ty}")
    out = pu.run_fused_parity(cfg, options=dict(direct_ty=ty))
    direct_plan_check(out["layer"].plan)
    auto = pu.GpuLayer(cfg, out["x"], out["w"])
    yp, idx = auto.pool_fwd()
    assert np.array_equal(yp, out["yp"]) and np.array_equal(idx, out["idx"])


@pytest.mark.parametrize("name", ["d_c1", "d_w130", "d_r16_bil"])
def test_direct_forward_against_the_matrix_core_kernel(name):
    """The same layer with the option switched off runs the matrix-core forward: both within the bar of the oracle,
    and equal arg-max wherever the winner is clear of the near-tie band (checked through the oracle in both runs)."""
    cfg = next(c for c in CASES if c.name == name)
    say(f"[case] direct off {name}")
    out = pu.run_fused_parity(cfg, options=dict(direct=-1))
    assert out["layer"].plan.kernel_name(0) != "valu_direct"


@pytest.mark.parametrize("cfg", CASES[:3] + CASES[6:8] + CASES[9:11] + CASES[12:], ids=lambda c: c.name)
def test_direct_forward_bf16(cfg):
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
    direct_plan_check(plan)
    tb.run_bf16_fused(cfg)


@pytest.mark.parametrize("cfg", [CASES[0], CASES[5], CASES[6]], ids=lambda c: c.name)
def test_direct_forward_bf16_dyadic_bit_exact(cfg):
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
    direct_plan_check(plan)
    tb.run_bf16_dyadic(cfg)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", ["d_w130", "d_r16_bil"])
def test_direct_forward_fused_relu(name, dtype):
    """Fused ReLU: the pooled forward equals max(plain result, 0) with idx 255 exactly where that result is not
    positive."""
    cfg = next(c for c in CASES if c.name == name)
    cfg = dataclasses.replace(cfg, x_dist="normal")
    say(f"[case] direct fused ReLU {name} {dtype}")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dt = rc.BF16 if dtype == "bf16" else rc.F32
    plain, fused = rc.Plan.from_config(cfg, dtype=dt), rc.Plan.from_config(cfg, dtype=dt, relu=True)
    direct_plan_check(plain)
    direct_plan_check(fused)
    x, w = (pu.dev(a, tdt) for a in (synth.make_x(cfg), synth.make_w(cfg)))
    P = (cfg.N, plain.Cpooled, plain.Ho, plain.Wo)
    mk = lambda: (torch.full(P, float("nan"), dtype=tdt, device="cuda"), torch.full(P, 77, dtype=torch.uint8, device="cuda"))
    (y0, i0), (y1, i1) = mk(), mk()
    rc.rotconv_pool_fwd(plain, x, w, y0, i0)
    rc.rotconv_pool_fwd(fused, x, w, y1, i1)
    torch.cuda.synchronize()
    alive = y0 > 0
    assert 0.02 < float(alive.float().mean()) < 0.98
    assert torch.equal(y1, torch.where(alive, y0, torch.zeros_like(y0)))
    assert torch.equal(i1, torch.where(alive, i0, torch.full_like(i0, 255)))


def test_direct_forward_leaves_neighbours_untouched_and_is_deterministic():
    cfg = next(c for c in CASES if c.name == "d_w130")
    plan = rc.Plan.from_config(cfg)
    x, w = pu.dev(synth.make_x(cfg), torch.float32), pu.dev(synth.make_w(cfg), torch.float32)
    n = cfg.N * plan.Cpooled * plan.Ho * plan.Wo
    runs = []
    for _ in range(2):
        buf = torch.full((n + 512,), float("nan"), device="cuda")
        ib = torch.full((n + 512,), 99, dtype=torch.uint8, device="cuda")
        yp, idx = buf[256:256 + n], ib[256:256 + n]
        rc.rotconv_pool_fwd(plan, x, w, yp, idx)
        torch.cuda.synchronize()
        assert bool(torch.isnan(buf[:256]).all()) and bool(torch.isnan(buf[256 + n:]).all())
        assert bool((ib[:256] == 99).all()) and bool((ib[256 + n:] == 99).all())
        runs.append((yp.clone(), idx.clone()))
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])


FIRST_LAYERS = [
    LC("enc0a_C4", N=4, Cin=3, H=512, W=512, Cout=64, R=4, seed=401),
    LC("enc0a_C5", N=2, Cin=3, H=512, W=512, Cout=64, R=16, mode="bilinear", seed=402),
]


@pytest.mark.parametrize("cfg", FIRST_LAYERS, ids=lambda c: c.name)
def test_first_layer_full_size_forward_element_by_element(cfg):
    """The first layer of benchmark configurations 4 and 5 at full size, in the launch configuration bench.py times:
    every pooled output and arg-max against the whole oracle forward (continuous inputs, near-tie protocol)."""
    say(f"[case] first layer full size {cfg}")
    x, w = synth.make_x(cfg), synth.make_w(cfg)
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    L = pu.GpuLayer(cfg, x, w, relu=False)
    direct_plan_check(L.plan)
    yp, idx = L.pool_fwd()
    y, yp_ref, idx_ref, w_rot = orc.layer_fwd(x, w, cfg.R, ang, cfg.mode, cfg.stride, cfg.pad, cfg.G)
    pu.assert_close(yp, yp_ref, f"{cfg.name} ypool")
    abs_terms = orc.rotconv_fwd(np.abs(x), np.abs(w_rot), cfg.stride, cfg.pad)
    ties = pu.check_idx(idx, y, abs_terms, cfg.G, f"{cfg.name} idx")
    say(f"  {idx.size} outputs ok, {ties} accepted near-ties")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_direct_weight_gradient_through_fused_relu(dtype):
    """The weight gradient fed the idx of a fused-ReLU forward (255 where the pooled value was not positive) equals
    the weight gradient of the plain plan fed the masked upstream gradient, bit for bit; two runs agree bit for bit."""
    cfg = dataclasses.replace(next(c for c in CASES if c.name == "d_w130"), x_dist="normal")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dt = rc.BF16 if dtype == "bf16" else rc.F32
    plain, fused = rc.Plan.from_config(cfg, dtype=dt), rc.Plan.from_config(cfg, dtype=dt, relu=True)
    assert (plain.kernel_name(2) == "valu_direct") == (dtype == "f32")
    x, w, g = (pu.dev(a, tdt) for a in (synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)))
    P = (cfg.N, plain.Cpooled, plain.Ho, plain.Wo)
    y0, i0 = torch.empty(P, dtype=tdt, device="cuda"), torch.empty(P, dtype=torch.uint8, device="cuda")
    y1, i1 = torch.empty_like(y0), torch.empty_like(i0)
    rc.rotconv_pool_fwd(plain, x, w, y0, i0)
    rc.rotconv_pool_fwd(fused, x, w, y1, i1)
    gm = torch.where(y0 > 0, g, torch.zeros_like(g))
    dws = [torch.full(w.shape, float("nan"), device="cuda") for _ in range(3)]
    rc.rotconv_pool_bwd_weight(plain, x, gm, i0, dws[0])
    rc.rotconv_pool_bwd_weight(fused, x, g, i1, dws[1])
    rc.rotconv_pool_bwd_weight(fused, x, g, i1, dws[2])
    torch.cuda.synchronize()
    assert torch.equal(dws[0], dws[1]) and torch.equal(dws[1], dws[2])
    assert float(dws[0].abs().max()) > 0


def test_first_layer_full_size_weight_gradient():
    """The weight gradient of configuration 4's first layer at full size, in the launch configuration bench.py times:
    every (filter, channel) slice against the oracle's gradient of the rotated banks, reduced through Eq. 16."""
    cfg = FIRST_LAYERS[0]
    say(f"[case] first layer full size dW {cfg}")
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    L = pu.GpuLayer(cfg, x, w)
    assert L.plan.kernel_name(2) == "valu_direct"
    yp, idx = L.pool_fwd()
    dw = L.pool_bwd_weight(g, idx)
    dy = orc.orient_maxpool_bwd(g, idx, cfg.R, cfg.G)
    dw_ref = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dy, cfg.k, cfg.stride, cfg.pad), None, cfg.mode)
    pu.assert_close(dw, dw_ref, f"{cfg.name} dw")
