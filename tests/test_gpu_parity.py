"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle
element by element on the same seeded inputs.  Run with -m gpu on the MI355X machine."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import rotconv_oracle as orc
from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth

import parity_util as pu

pytestmark = pytest.mark.gpu

LC = synth.LayerConfig


def say(msg):
    print(msg, flush=True)


# Tiny / odd shapes: H != W, channel counts that are not multiples of any tile, N > 1,
# pad 0/1/2, k = 1/2/3/5, stride 1/2, R = 1/2/3/4/8/16, all three modes, sub-group pooling.
TINY = [
    LC("t_r4", N=2, Cin=3, H=9, W=7, Cout=5, R=4, seed=11),
    LC("t_r1", N=1, Cin=4, H=8, W=8, Cout=3, R=1, seed=12),
    LC("t_r2", N=2, Cin=2, H=6, W=10, Cout=4, R=2, angles_deg=(0.0, 180.0), seed=13),
    LC("t_r2b", N=1, Cin=2, H=6, W=6, Cout=2, R=2, angles_deg=(90.0, 270.0), seed=14),
    LC("t_k1", N=2, Cin=5, H=5, W=6, Cout=3, k=1, pad=0, R=4, seed=15),
    LC("t_k5", N=1, Cin=2, H=9, W=8, Cout=3, k=5, pad=2, R=4, seed=16),
    LC("t_k2", N=1, Cin=2, H=7, W=7, Cout=2, k=2, pad=1, R=4, seed=17),
    LC("t_pad0", N=2, Cin=3, H=8, W=9, Cout=2, pad=0, R=4, seed=18),
    LC("t_pad2", N=1, Cin=3, H=6, W=5, Cout=2, pad=2, R=4, seed=19),
    LC("t_s2", N=2, Cin=3, H=11, W=10, Cout=4, stride=2, R=4, seed=20),
    LC("t_g2", N=1, Cin=3, H=8, W=8, Cout=3, R=4, pool_group=2, seed=21),
    LC("t_g1", N=1, Cin=2, H=6, W=6, Cout=2, R=4, pool_group=1, seed=22),
    LC("t_r8bil", N=2, Cin=3, H=8, W=7, Cout=3, R=8, mode="bilinear", seed=23),
    LC("t_r16bil", N=1, Cin=4, H=10, W=10, Cout=2, R=16, mode="bilinear", seed=24),
    LC("t_r16bil_g4", N=1, Cin=4, H=10, W=9, Cout=3, R=16, mode="bilinear", pool_group=4, seed=25),
    LC("t_r16ste", N=1, Cin=3, H=8, W=8, Cout=2, R=16, mode="steerable", seed=26),
    LC("t_r8ste_g4", N=2, Cin=2, H=7, W=8, Cout=3, R=8, mode="steerable", pool_group=4, seed=27),
    LC("t_r3irr", N=1, Cin=2, H=8, W=8, Cout=2, R=3, mode="bilinear", angles_deg=(10.0, 100.0, 300.0), seed=28),
    LC("t_r5k5", N=1, Cin=2, H=9, W=9, Cout=2, k=5, pad=2, R=5, mode="bilinear",
       angles_deg=(0.0, 30.0, 120.0, 200.0, 359.0), seed=29),
    LC("t_big_tail", N=1, Cin=17, H=33, W=35, Cout=19, R=4, seed=30),
    LC("t_1px", N=1, Cin=1, H=1, W=1, Cout=1, R=4, seed=31),
    # wide rows (segmented wave chains), rows that end inside a wave chain, deep inputs (streamed filter block)
    LC("t_w512", N=1, Cin=8, H=11, W=512, Cout=20, R=4, seed=32),
    LC("t_w288", N=1, Cin=4, H=9, W=288, Cout=16, R=4, seed=33),
    LC("t_w96", N=2, Cin=4, H=9, W=96, Cout=5, R=4, seed=34),
    LC("t_w72", N=1, Cin=6, H=9, W=72, Cout=3, R=4, seed=35),
    LC("t_cin256", N=1, Cin=256, H=10, W=32, Cout=18, R=4, seed=36),
    LC("t_cin288_r16", N=1, Cin=288, H=9, W=64, Cout=16, R=16, mode="bilinear", seed=37),
    LC("t_cin288_w96", N=1, Cin=288, H=6, W=96, Cout=8, R=4, seed=42),     # streamed block, chain beyond the row
    # table weight gradient with a filter block's D built by its channel groups together: two groups and a row tail;
    # three groups and two base banks
    LC("t_lut_c136_w44", N=2, Cin=136, H=7, W=44, Cout=20, R=16, mode="bilinear", seed=43),
    LC("t_lut_ste_c192", N=1, Cin=192, H=6, W=32, Cout=20, R=16, mode="steerable", seed=46),
    LC("t_w544_cin6", N=1, Cin=6, H=6, W=544, Cout=16, R=8, mode="steerable", pool_group=4, seed=38),
    # the p4m group (rotations and reflection): the mirrored filter is a second bank of the same kernels
    LC("t_p4m", N=2, Cin=5, H=10, W=12, Cout=6, R=8, mode="p4m", seed=44),
    LC("t_p4m_r4", N=1, Cin=3, H=9, W=7, Cout=4, R=4, mode="p4m", seed=45),
    LC("t_p4m_k5_g1", N=1, Cin=2, H=8, W=8, Cout=3, k=5, pad=2, R=8, mode="p4m", pool_group=1, seed=46),
    LC("t_p4m_c40", N=1, Cin=40, H=12, W=64, Cout=24, R=8, mode="p4m", x_dist="absnormal", seed=47),
    # rows that end half way through a lane's eight pixels (W % 8 == 4), one and several strips, many rows
    LC("t_w4", N=2, Cin=5, H=10, W=4, Cout=6, R=4, seed=39),
    LC("t_w44", N=1, Cin=3, H=7, W=44, Cout=4, R=4, seed=40),
    LC("t_w20_cout72", N=1, Cin=40, H=8, W=20, Cout=72, R=4, seed=41),
    # long contraction on a small map: the input gradient shares its filter chunks out over workgroups, the parts
    # starting inside a bank (17 chunks of one bank in two parts; 2 x 13 chunks in three)
    LC("t_ksplit_q1", N=1, Cin=24, H=8, W=32, Cout=272, R=4, seed=48),
    LC("t_ksplit_q2", N=1, Cin=16, H=6, W=32, Cout=200, R=8, mode="bilinear", seed=49),
    # row widths the matrix-core kernels do not take run on rows padded to a multiple of 8 (32 beyond 256 pixels)
    LC("t_padw_r16", N=1, Cin=40, H=9, W=45, Cout=20, R=16, mode="bilinear", seed=56),
    LC("t_padw_270", N=1, Cin=4, H=6, W=270, Cout=16, R=4, seed=57),
    LC("t_padw_g2", N=2, Cin=6, H=7, W=13, Cout=5, R=8, mode="steerable", pool_group=4, seed=58),
    # small maps: one or two chunks per workgroup (three chunks of one bank; 2 x 2 chunks of two banks; six chunks in
    # threes on a map whose dX is not tiny)
    LC("t_ksplit_small", N=1, Cin=70, H=4, W=8, Cout=40, R=4, seed=54),
    LC("t_ksplit_small_q2", N=1, Cin=20, H=5, W=6, Cout=24, R=8, mode="bilinear", seed=55),
    # deep inputs on small maps: the forward splits its channel chunks over workgroups (unpooled parts, ordered sum,
    # then the pool): 17 chunks on a map narrower than a wave, R = 1; three chunks, R = 4; sub-group pooling over
    # two banks; a pool group that spans four banks
    LC("t_csplit_w8", N=1, Cin=520, H=8, W=8, Cout=20, R=1, seed=50),
    LC("t_csplit_r4", N=2, Cin=96, H=6, W=32, Cout=18, R=4, seed=51),
    LC("t_csplit_r8_g4", N=1, Cin=72, H=5, W=16, Cout=9, R=8, mode="bilinear", pool_group=4, seed=52),
    LC("t_csplit_r16", N=1, Cin=160, H=4, W=4, Cout=17, R=16, mode="bilinear", seed=53),
    # whole 64-channel groups and 16-filter chunks, one bank: the input gradient reads w itself (no packed copy): four
    # and two pixels per lane, a contraction shared out over workgroups, a single orientation
    LC("t_raw_w_px4", N=1, Cin=64, H=6, W=68, Cout=16, R=4, seed=56),
    LC("t_raw_w_px2", N=2, Cin=64, H=9, W=10, Cout=48, R=4, seed=57),
    LC("t_raw_w_r1", N=1, Cin=64, H=5, W=36, Cout=32, R=1, seed=58),
]


@pytest.mark.parametrize("cfg", TINY, ids=[c.name for c in TINY])
def test_fused_path_tiny(cfg):
    say(f"[case] fused tiny {cfg}")
    pu.run_fused_parity(cfg)


@pytest.mark.parametrize("cfg", [c for c in TINY if c.mode == "exact90"], ids=lambda c: c.name)
def test_fused_path_tiny_dyadic_bit_exact(cfg):
    say(f"[case] fused tiny dyadic {cfg.name}")
    pu.run_fused_parity(cfg, dyadic=True)


@pytest.mark.parametrize("cfg", TINY[:1] + TINY[9:12] + TINY[12:15] + TINY[16:18], ids=lambda c: c.name)
def test_unfused_chain_tiny(cfg):
    """rotconv_fwd -> orient_maxpool_fwd -> orient_maxpool_bwd -> rotconv_bwd_data / bwd_weight."""
    say(f"[case] unfused tiny {cfg.name}")
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    ref = pu.oracle_layer(cfg, x, w, g)
    L = pu.GpuLayer(cfg, x, w)
    y = L.fwd()
    N, Cout, R = cfg.N, cfg.Cout, cfg.R
    pu.assert_close(y.cpu().numpy().reshape(ref["y"].shape), ref["y"], f"{cfg.name} y")
    yp, idx = L.maxpool_fwd(y)
    pu.assert_close(yp, ref["ypool"], f"{cfg.name} ypool")
    pu.check_idx(idx, ref["y"], ref["abs_terms"], cfg.G, f"{cfg.name} idx")
    # pooling of the ORACLE's y on the GPU must reproduce the oracle's idx bit for bit
    yp2, idx2 = L.maxpool_fwd(pu.dev(ref["y"].reshape(N, Cout * R, cfg.Ho, cfg.Wo), torch.float32))
    y32 = ref["y"].astype(np.float32).astype(np.float64)
    yp_ref32, idx_ref32 = orc.orient_maxpool_fwd(y32, cfg.G)
    assert np.array_equal(idx2, idx_ref32) and np.array_equal(yp2.astype(np.float64), yp_ref32)
    dy = L.maxpool_bwd(g, ref["idx"])
    dy_ref = orc.orient_maxpool_bwd(g, ref["idx"], R, cfg.G)
    assert np.array_equal(dy.cpu().numpy().reshape(dy_ref.shape).astype(np.float64), dy_ref)
    pu.assert_close(L.bwd_data(dy), ref["dx"], f"{cfg.name} dx (unfused)")
    pu.assert_close(L.bwd_weight(dy), ref["dw"], f"{cfg.name} dw (unfused)")
    # dense (not one-hot) upstream gradient through the unfused backward calls
    dyd = synth.make_dy(cfg)
    w_rot = ref["w_rot"]
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    dyd5 = dyd.reshape(N, Cout, R, cfg.Ho, cfg.Wo)
    dx_ref = orc.rotconv_bwd_data(dyd5, w_rot, cfg.H, cfg.W, cfg.stride, cfg.pad)
    dw_ref = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dyd5, cfg.k, cfg.stride, cfg.pad), ang, cfg.mode)
    dyd_d = pu.dev(dyd, torch.float32)
    pu.assert_close(L.bwd_data(dyd_d), dx_ref, f"{cfg.name} dx (dense dy)")
    pu.assert_close(L.bwd_weight(dyd_d), dw_ref, f"{cfg.name} dw (dense dy)")


@pytest.mark.parametrize("parts", ["1", "2", "5"])
@pytest.mark.parametrize("name", ["t_cin256", "t_cin288_r16", "t_csplit_r4", "t_csplit_r16"])
def test_forward_channel_split_settings(name, parts):
    """The forward with its channel contraction kept whole (where such an instance exists) and split into a given
    number of parts: fused pooled call and the unpooled call, both against the oracle."""
    cfg = next(c for c in TINY if c.name == name)
    say(f"[case] forward channel split {name} parts={parts}")
    out = pu.run_fused_parity(cfg, options=dict(fwd_csplit=int(parts)))
    L, ref = out["layer"], out["ref"]
    y = L.fwd()
    pu.assert_close(y.cpu().numpy().reshape(ref["y"].shape), ref["y"], f"{name} y parts={parts}")


GS_CASES = [c for c in TINY if c.k != 3 or c.stride != 1 or c.pad != 1 or c.name in ("t_g2", "t_g1")] + [
    LC("t_gs_k5_r8", N=2, Cin=32, H=24, W=24, Cout=32, k=5, pad=2, R=8, mode="steerable", seed=59),
    LC("t_gs_s2_k7", N=3, Cin=5, H=21, W=18, Cout=6, k=7, pad=3, stride=2, R=4, seed=60),
    LC("t_gs_s3_p4m", N=1, Cin=4, H=17, W=16, Cout=5, k=3, pad=0, stride=3, R=8, mode="p4m", pool_group=2, seed=61),
]


@pytest.mark.parametrize("cfg", GS_CASES, ids=lambda c: c.name)
def test_gemm_scatter_family(cfg):
    """Layers outside the register-resident kernels (k, stride, pad, pool groups that cut through a bank) on the
    matrix-multiply + scatter family, forced on for every size: fused calls, then the unfused chain with a dense dy."""
    say(f"[case] gemm + scatter {cfg.name}")
    out = pu.run_fused_parity(cfg, options=dict(gs=1))
    L, ref = out["layer"], out["ref"]
    names = [L.plan.kernel_name(i) for i in range(3)]
    assert "mfma_gemm_scatter" in names, names
    y = L.fwd()
    pu.assert_close(y.cpu().numpy().reshape(ref["y"].shape), ref["y"], f"{cfg.name} y")
    x = out["x"]
    dyd = synth.make_dy(cfg)
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    dyd5 = dyd.reshape(cfg.N, cfg.Cout, cfg.R, cfg.Ho, cfg.Wo)
    dx_ref = orc.rotconv_bwd_data(dyd5, ref["w_rot"], cfg.H, cfg.W, cfg.stride, cfg.pad)
    dw_ref = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dyd5, cfg.k, cfg.stride, cfg.pad), ang, cfg.mode)
    dyd_d = pu.dev(dyd, torch.float32)
    pu.assert_close(L.bwd_data(dyd_d), dx_ref, f"{cfg.name} dx (dense dy)")
    pu.assert_close(L.bwd_weight(dyd_d), dw_ref, f"{cfg.name} dw (dense dy)")
    if cfg.mode == "exact90":
        pu.run_fused_parity(cfg, dyadic=True, label=f"{cfg.name} dyadic", options=dict(gs=1))


def test_gemm_scatter_family_one_image_at_a_time():
    """With no room for more than one image's products the family walks the batch image by image (the weight
    gradient accumulates its per-image sums in order)."""
    cfg = next(c for c in GS_CASES if c.name == "t_gs_s2_k7")
    say(f"[case] gemm + scatter, one image per chunk {cfg.name}")
    opts = dict(gs=1, gs_chunk_mb=-1)
    pu.run_fused_parity(cfg, options=opts)
    pu.run_fused_parity(cfg, dyadic=True, label=f"{cfg.name} dyadic", options=opts)


def test_gemm_scatter_family_is_the_default_for_larger_layers():
    cfg = next(c for c in GS_CASES if c.name == "t_gs_k5_r8")
    L = pu.GpuLayer(cfg, synth.make_x(cfg), synth.make_w(cfg))
    assert [L.plan.kernel_name(i) for i in range(3)] == ["mfma_gemm_scatter"] * 3


LUT_CASES = ["t_r8bil", "t_r16bil", "t_r3irr", "t_cin288_r16", "t_lut_c136_w44", "t_lut_ste_c192", "t_p4m", "t_p4m_c40", "t_ksplit_q2", "t_padw_r16", "t_csplit_r16"]


@pytest.mark.parametrize("name", LUT_CASES)
def test_gradients_per_bank_kernels(name):
    """Plans with several banks and one pool group per filter take the routed-gradient table by default (the cases
    above run it); here the same layers on the per-bank gradient kernels."""
    cfg = next(c for c in TINY if c.name == name)
    say(f"[case] per-bank gradient kernels {name}")
    pu.run_fused_parity(cfg, options=dict(bwd_lut=-1))


def test_config3_reduced_with_and_without_table():
    """Configuration 3's structure (R = 16 bilinear, one pool group) at reduced extent, both gradient variants, and
    the two must agree with each other far inside the oracle tolerance."""
    cfg = dataclasses.replace(synth.C3, name="C3r_lut", N=2, Cin=72, Cout=40, H=24, W=40)
    say(f"[case] {cfg.name}")
    a = pu.run_fused_parity(cfg)
    b = pu.run_fused_parity(cfg, options=dict(bwd_lut=-1))
    for k in ("dx", "dw"):
        scale = float(np.abs(a[k]).max())
        assert float(np.abs(a[k].astype(np.float64) - b[k]).max()) <= 2e-5 * scale, k


# Layers whose pool group spans several banks: the pooled forward multiplies with the base bank only and forms the
# banks' products on the vector ALU ("mfma_p4_base"); the TINY cases of that kind run it by default.  More of its
# branches: three row segments, a streamed filter block, a first layer (at most four channels), rows that are not
# a multiple of four or end inside a wave, several bands per workgroup, fused ReLU.
BASE_CASES = [
    LC("t_base_w288", N=1, Cin=8, H=7, W=288, Cout=20, R=16, mode="bilinear", seed=71),
    LC("t_base_w544_p4m", N=1, Cin=8, H=5, W=544, Cout=16, R=8, mode="p4m", seed=72),
    LC("t_base_stream", N=2, Cin=288, H=40, W=64, Cout=64, R=16, mode="bilinear", x_dist="absnormal", seed=73),
    LC("t_base_stream_r8", N=4, Cin=320, H=34, W=32, Cout=64, R=8, mode="bilinear", x_dist="absnormal", seed=74),
    LC("t_base_cin3", N=2, Cin=3, H=33, W=64, Cout=24, R=16, mode="bilinear", seed=75),
    LC("t_base_cin3_w46", N=1, Cin=3, H=9, W=46, Cout=8, R=8, mode="bilinear", seed=76),
    LC("t_base_w18", N=2, Cin=40, H=21, W=18, Cout=17, R=16, mode="bilinear", seed=77),
    LC("t_base_w32_bands", N=1, Cin=64, H=70, W=32, Cout=32, R=16, mode="bilinear", x_dist="absnormal", seed=78),
    LC("t_base_w100", N=1, Cin=33, H=12, W=100, Cout=16, R=8, mode="p4m", seed=79),
]


@pytest.mark.parametrize("cfg", BASE_CASES, ids=lambda c: c.name)
def test_forward_on_base_products(cfg):
    say(f"[case] forward on base products {cfg.name}")
    # layers with at most four input channels would take the vector-ALU kernel: switched off to reach this one's
    # padded-channel branch
    over = dict(options=dict(direct=-1)) if cfg.Cin <= 4 else {}
    out = pu.run_fused_parity(cfg, **over)
    assert out["layer"].plan.kernel_name(0) == "mfma_p4_base"
    if cfg.mode == "p4m":       # the mirror image is a tap permutation: exact arithmetic, ties across the two banks
        pu.run_fused_parity(cfg, dyadic=True, label=f"{cfg.name} dyadic")


# Input gradient with the D of a row built by its channel groups together, four pixels per lane (launches that still
# give every SIMD two waves): the per-bank build (R = 4, two groups) and the table build (R = 16, three groups).
SHARED_PX4 = [
    LC("t_shared_r4_px4", N=4, Cin=128, H=128, W=128, Cout=16, R=4, x_dist="absnormal", seed=81),
    LC("t_shared_r16_px4", N=2, Cin=192, H=128, W=128, Cout=16, R=16, mode="bilinear", x_dist="absnormal", seed=82),
]


@pytest.mark.parametrize("cfg", SHARED_PX4, ids=lambda c: c.name)
def test_input_gradient_shared_four_pixels_per_lane(cfg):
    say(f"[case] shared input gradient, four pixels per lane {cfg.name}")
    pu.run_fused_parity(cfg)
    pu.run_fused_parity(cfg, dyadic=True, label=f"{cfg.name} dyadic") if cfg.R == 4 else None


def test_forward_on_base_products_with_fused_relu():
    """The fused ReLU of that kernel: pooled values clamped at 0, idx 255 where the pooled value is not positive."""
    cfg = LC("t_base_relu", N=1, Cin=16, H=20, W=48, Cout=16, R=16, mode="bilinear", x_dist="normal", seed=80)
    say(f"[case] forward on base products, fused ReLU {cfg.name}")
    x, w = synth.make_x(cfg), synth.make_w(cfg)
    plain = pu.GpuLayer(cfg, x, w)
    relu = pu.GpuLayer(cfg, x, w, relu=True)
    assert relu.plan.kernel_name(0) == "mfma_p4_base"
    yp, idx = plain.pool_fwd()
    yr, ir = relu.pool_fwd()
    dead = ~(yp > 0)
    assert dead.any() and (~dead).any()
    assert np.array_equal(yr, np.where(dead, np.float32(0), yp))
    assert np.array_equal(ir, np.where(dead, np.uint8(255), idx))


@pytest.mark.parametrize("name", ["t_r8bil", "t_r16bil", "t_p4m", "t_p4m_c40", "t_ksplit_q2", "t_padw_r16",
                                  "t_ksplit_small_q2"])
def test_forward_per_bank_kernels(name):
    """The same layers with the forward kept on the per-bank kernels (plan option fwd_base = -1: the banks folded
    into a wave's filter columns, or per-bank candidates through memory)."""
    cfg = next(c for c in TINY if c.name == name)
    say(f"[case] forward per bank {name}")
    # (layers with at most four input channels: the vector-ALU kernel switched off as well)
    out = pu.run_fused_parity(cfg, options=dict(fwd_base=-1, direct=-1))
    assert out["layer"].plan.kernel_name(0) == "mfma_p4"


def test_config3_reduced_forward_both_ways():
    """Configuration 3's structure at reduced extent: the forward on base products and on the per-bank kernel must
    agree with each other far inside the oracle tolerance (and each with the oracle)."""
    cfg = dataclasses.replace(synth.C3, name="C3r_fwd", N=2, Cin=72, Cout=40, H=32, W=48)
    say(f"[case] {cfg.name}")
    a = pu.run_fused_parity(cfg)
    b = pu.run_fused_parity(cfg, options=dict(fwd_base=-1))
    assert a["layer"].plan.kernel_name(0) == "mfma_p4_base" and b["layer"].plan.kernel_name(0) == "mfma_p4"
    scale = float(np.abs(a["yp"]).max())
    diff = float(np.abs(a["yp"].astype(np.float64) - b["yp"]).max())
    assert diff <= 1e-4 * scale, (diff, scale)


@pytest.mark.parametrize("name", ["t_r4", "t_w96", "t_r16bil", "t_p4m_c40", "t_cin256", "t_padw_g2"])
def test_unfused_gradients_with_the_larger_workspace(name):
    """rotconv_bwd_data / rotconv_bwd_weight (dense dy) of plans whose fused calls run the register-resident kernels:
    with rotconv_workspace_bytes_unfused of scratch they run matrix multiply + scatter instead of the generic kernels;
    both against the oracle."""
    cfg = next(c for c in TINY if c.name == name)
    say(f"[case] unfused gradients, larger workspace {name}")
    x, w = synth.make_x(cfg), synth.make_w(cfg)
    # gs=1: the family is wanted whatever the layer's size (several of these cases lie below the automatic threshold,
    # and would run the generic kernels with either workspace)
    L = pu.GpuLayer(cfg, x, w, options=dict(gs=1))
    names = [L.plan.kernel_name(i) for i in range(5)]
    assert names[0] in ("mfma_p4", "mfma_p4_base", "valu_direct") and names[1] == "mfma_p4", names
    assert names[2] in ("mfma_p4", "valu_direct") and names[3:] == ["mfma_gemm_scatter"] * 2, names
    dyd = synth.make_dy(cfg)
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    w_rot = orc.expand_bank(w, cfg.R, ang, cfg.mode)
    dyd5 = dyd.reshape(cfg.N, cfg.Cout, cfg.R, cfg.Ho, cfg.Wo)
    dx_ref = orc.rotconv_bwd_data(dyd5, w_rot, cfg.H, cfg.W, cfg.stride, cfg.pad)
    dw_ref = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dyd5, cfg.k, cfg.stride, cfg.pad), ang, cfg.mode)
    dy_d = pu.dev(dyd, torch.float32)
    ws = torch.empty(max(L.plan.workspace_bytes_unfused, 256), dtype=torch.uint8, device="cuda")
    dx, dw = L.nan(tuple(L.x.shape)), L.nan(tuple(L.w.shape))
    rc.rotconv_bwd_data(L.plan, dy_d, L.w, dx, ws=ws)
    rc.rotconv_bwd_weight(L.plan, L.x, dy_d, dw, ws=ws)
    torch.cuda.synchronize()
    pu.assert_close(dx.cpu().numpy(), dx_ref, f"{name} dx (dense dy, larger workspace)")
    pu.assert_close(dw.cpu().numpy(), dw_ref, f"{name} dw (dense dy, larger workspace)")


def test_config1_fused_and_unfused():
    """Benchmark configuration 1 (N=1, 3->8, 64x64, R=4): both call chains, continuous and dyadic."""
    cfg = synth.C1
    say(f"[case] C1 {cfg}")
    out = pu.run_fused_parity(cfg)
    L, ref = out["layer"], out["ref"]
    y = L.fwd()
    pu.assert_close(y.cpu().numpy().reshape(ref["y"].shape), ref["y"], "C1 y")
    yp, idx = L.maxpool_fwd(y)
    assert np.array_equal(yp, out["yp"]) or np.allclose(yp, out["yp"], rtol=1e-5, atol=1e-6)
    dy = L.maxpool_bwd(out["g"], ref["idx"])
    pu.assert_close(L.bwd_data(dy), ref["dx"], "C1 dx (unfused)")
    pu.assert_close(L.bwd_weight(dy), ref["dw"], "C1 dw (unfused)")
    pu.run_fused_parity(cfg, dyadic=True, label="C1 dyadic")


def test_determinism_and_untouched_neighbours():
    """Same inputs twice -> bitwise the same outputs; guard bands around outputs stay intact."""
    cfg = LC("det", N=2, Cin=6, H=20, W=18, Cout=7, R=4, seed=77)
    say(f"[case] determinism {cfg.name}")
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    L = pu.GpuLayer(cfg, x, w)
    idx_any = synth.make_idx(cfg)
    outs = []
    for rep in range(2):
        pad = 1024
        n_p = int(np.prod(L.P))
        n_x = x.size
        buf_y = torch.full((n_p + 2 * pad,), 7.25, device="cuda")
        buf_i = torch.full((n_p + 2 * pad,), 201, dtype=torch.uint8, device="cuda")
        buf_dx = torch.full((n_x + 2 * pad,), 7.25, device="cuda")
        buf_dw = torch.full((w.size + 2 * pad,), 7.25, device="cuda")
        yp, idx = buf_y[pad:pad + n_p], buf_i[pad:pad + n_p]
        dx, dw = buf_dx[pad:pad + n_x], buf_dw[pad:pad + w.size]
        rc.rotconv_pool_fwd(L.plan, L.x, L.w, yp, idx)
        gd, idd = pu.dev(g, torch.float32), pu.dev(idx_any)
        rc.rotconv_pool_bwd_data(L.plan, gd, idd, L.w, dx)
        rc.rotconv_pool_bwd_weight(L.plan, L.x, gd, idd, dw)
        torch.cuda.synchronize()
        for b, n in ((buf_y, n_p), (buf_dx, n_x), (buf_dw, w.size)):
            assert bool((b[:pad] == 7.25).all()) and bool((b[pad + n:] == 7.25).all())
        assert bool((buf_i[:pad] == 201).all()) and bool((buf_i[pad + n_p:] == 201).all())
        outs.append([t.clone().cpu().numpy() for t in (yp, idx, dx, dw)])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_invalid_idx_values_contribute_nothing():
    cfg = LC("badidx", N=1, Cin=3, H=8, W=8, Cout=2, R=4, pool_group=2, seed=5)
    say(f"[case] invalid idx {cfg.name}")
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    L = pu.GpuLayer(cfg, x, w)
    idx = synth.make_idx(cfg)
    bad = idx.copy()
    bad[0, 0, :4] = 250          # out of range
    bad[0, 1, :4] = 0            # wrong group (channel 1 is group 1: members 1 and 3)
    g0 = g.copy()
    g0[0, 0, :4] = 0
    g0[0, 1, :4] = 0
    dx_bad, dw_bad = L.pool_bwd_data(g, bad), L.pool_bwd_weight(g, bad)
    dx_ref, dw_ref = L.pool_bwd_data(g0, idx), L.pool_bwd_weight(g0, idx)
    assert np.array_equal(dx_bad, dx_ref) and np.array_equal(dw_bad, dw_ref)


def test_workspace_too_small_is_rejected():
    cfg = TINY[0]
    L = pu.GpuLayer(cfg, synth.make_x(cfg), synth.make_w(cfg))
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    yp, idx = L.nan(L.P), L.nan(L.P, torch.uint8)
    with pytest.raises(rc.RotconvError) as e:
        rc.rotconv_pool_fwd(L.plan, L.x, L.w, yp, idx, ws=small)
    assert e.value.status == rc.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool(torch.isnan(yp).all())  # outputs untouched


def _sample_points(seed, n, dims):
    cols = [synth.randint(seed + i, n, 0, d - 1) for i, d in enumerate(dims)]
    return np.stack(cols, axis=1).astype(np.int32)


def full_size_sampled_parity(cfg, n_samples=4096, n_pairs=24):
    """Full benchmark-size layer in the launch configuration bench.py times, checked on sampled
    outputs the oracle computes one by one, plus identities that hold at any size."""
    say(f"[case] full-size sampled {cfg}")
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    L = pu.GpuLayer(cfg, x, w)
    say(f"  kernels: {[L.plan.kernel_name(i) for i in range(3)]}")
    yp, idx = L.pool_fwd()
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    w_rot = orc.expand_bank(w, cfg.R, ang, cfg.mode)
    ng = cfg.R // cfg.G
    # forward: sampled pooled outputs
    pts = _sample_points(cfg.seed + 100, n_samples, (cfg.N, cfg.Cout, cfg.Ho, cfg.Wo))
    yr = orc.rotconv_fwd_at(x, w_rot, pts, cfg.stride, cfg.pad)                   # [T,R]
    ya = orc.rotconv_fwd_at(np.abs(x), np.abs(w_rot), pts, cfg.stride, cfg.pad)
    rms = float(np.sqrt(np.mean(yr.reshape(-1, cfg.G, ng).max(axis=1) ** 2)))
    near = 0
    for t, (n, co, oy, ox) in enumerate(pts):
        for grp in range(ng):
            members = np.arange(grp, cfg.R, ng)
            vals = yr[t, members]
            got_v, got_i = float(yp[n, co * ng + grp, oy, ox]), int(idx[n, co * ng + grp, oy, ox])
            assert abs(got_v - vals.max()) <= pu.RTOL * abs(vals.max()) + pu.RTOL * rms, (t, got_v, vals.max())
            assert got_i % ng == grp
            tau = 64.0 * pu.EPS32 * ya[t, members].max()
            assert yr[t, got_i] >= vals.max() - tau, ("argmax outside near-tie band", t, got_i, vals)
            near += int(got_i != members[int(vals.argmax())])
    say(f"  fwd: {n_samples} sampled outputs ok, {near} accepted near-ties")
    # backward with the GPU's own idx given to both sides (one shared idx)
    dx = L.pool_bwd_data(g, idx)
    dw = L.pool_bwd_weight(g, idx)
    dy = None
    if cfg.N * cfg.Cout * cfg.R * cfg.Ho * cfg.Wo <= 160_000_000:
        dy = orc.orient_maxpool_bwd(g, idx, cfg.R, cfg.G)
        ptsx = _sample_points(cfg.seed + 200, n_samples, (cfg.N, cfg.Cin, cfg.H, cfg.W))
        dxr = orc.rotconv_bwd_data_at(dy, w_rot, ptsx, cfg.H, cfg.W, cfg.stride, cfg.pad)
        got = dx[ptsx[:, 0], ptsx[:, 1], ptsx[:, 2], ptsx[:, 3]]
        pu.assert_close(got, dxr, f"{cfg.name} dx samples")
        say(f"  bwd_data: {n_samples} sampled inputs ok")
    pairs = _sample_points(cfg.seed + 300, n_pairs, (cfg.Cout, cfg.Cin))
    dwr_rot = orc.rotconv_pool_bwd_weight_at(x, g, idx, pairs, cfg.R, cfg.k, cfg.G, cfg.stride, cfg.pad)  # [T,R,k,k]
    # reduce each sampled (co,ci) slice through Eq. 16 with the oracle
    got_dw, ref_dw = [], []
    for t, (co, ci) in enumerate(pairs):
        full = np.zeros((cfg.R, 1, 1, cfg.k, cfg.k))
        full[:, 0, 0] = dwr_rot[t]
        ref_dw.append(orc.reduce_bank_grad(full, ang, cfg.mode)[:, 0, 0])
        got_dw.append(dw[:, co, ci])
    pu.assert_close(np.array(got_dw), np.array(ref_dw), f"{cfg.name} dw samples", rtol=pu.RTOL)
    say(f"  bwd_weight: {n_pairs} sampled (co,ci) slices ok")
    # Euler identities through the max (the layer is positively homogeneous of degree 1 in w and in x):
    # <w, dw> = <x, dx> = <ypool, g>, at full size, no oracle needed.
    a = float((yp.astype(np.float64) * g).sum())
    b = float((x.astype(np.float64) * dx).sum())
    c = float((w.astype(np.float64) * dw).sum())
    scale = float(np.abs(yp.astype(np.float64) * g).sum())
    assert abs(a - b) <= 1e-5 * scale and abs(a - c) <= 1e-5 * scale, (a, b, c, scale)
    say(f"  homogeneity identities ok: {a:.6e} {b:.6e} {c:.6e}")
    return L


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_full_size_element_by_element(name):
    """Benchmark configurations 2 and 3 at full size, in the launch configuration bench.py times, every element of
    the pooled output, the arg-max, dX and dW against the whole oracle (continuous inputs, near-tie protocol)."""
    cfg = synth.CONFIGS[name]
    say(f"[case] full-size element by element {cfg}")
    out = pu.run_fused_parity(cfg)
    say(f"  kernels: {[out['layer'].plan.kernel_name(i) for i in range(3)]}, {out['near_ties']} accepted near-ties of "
        f"{out['idx'].size}")


def test_config2_full_size_dyadic_bit_exact():
    """Benchmark configuration 2 at full size on the exact-arithmetic grid: pooled output, arg-max and dX bit for
    bit (dW within the tolerance: its 2^19-term sums are not exact in fp32)."""
    say("[case] C2 full size, dyadic")
    pu.run_fused_parity(synth.C2, dyadic=True, label="C2 dyadic full size")


def test_config2_full_size_sampled():
    full_size_sampled_parity(synth.C2)


def test_config3_full_size_sampled():
    full_size_sampled_parity(synth.C3, n_samples=2048, n_pairs=12)


def test_odd_width_full_size_sampled():
    """Configuration 2's channels on 255 x 255 images: the matrix-core kernels on zero-padded rows."""
    cfg = dataclasses.replace(synth.C2, name="C2_255", N=4, H=255, W=255)
    L = full_size_sampled_parity(cfg, n_samples=2048, n_pairs=12)
    assert [L.plan.kernel_name(i) for i in range(3)] == ["mfma_p4"] * 3


def test_k5_full_size_sampled():
    """Configuration 2's shape with 5 x 5 filters: GEMM + scatter, several image chunks."""
    cfg = dataclasses.replace(synth.C2, name="C2_k5", N=4, k=5, pad=2)
    L = full_size_sampled_parity(cfg, n_samples=2048, n_pairs=12)
    assert [L.plan.kernel_name(i) for i in range(3)] == ["mfma_gemm_scatter"] * 3


def test_small_map_deep_channels_sampled():
    """A point of the single-orientation sweep and its R = 4 counterpart: 32 x 32 maps, 1024 -> 256 channels (the
    forward splits its channel chunks, the input gradient its weight chunks)."""
    for R in (1, 4):
        cfg = LC(f"sweep32_R{R}", N=1, Cin=1024, H=32, W=32, Cout=256, R=R, seed=62 + R)
        full_size_sampled_parity(cfg, n_samples=1024, n_pairs=8)


def test_config3_steerable_and_group4_reduced():
    """Config-3 structure (R=16, 22.5 degree steps) in steerable mode and with the paper's
    sub-group pooling (G=4), at a size the oracle finishes in seconds."""
    for mode, G in (("steerable", None), ("bilinear", 4), ("steerable", 4)):
        cfg = dataclasses.replace(synth.C3, name=f"C3r_{mode}_{G}", N=1, Cin=32, Cout=32, H=40, W=40, mode=mode,
                                  pool_group=G)
        say(f"[case] {cfg.name}")
        pu.run_fused_parity(cfg)


def test_config2_reduced_exact():
    """Config-2 structure at reduced extent: element-by-element, continuous and dyadic (bit-exact)."""
    cfg = dataclasses.replace(synth.C2, name="C2r", N=2, H=48, W=80)
    say(f"[case] {cfg.name}")
    pu.run_fused_parity(cfg)
    pu.run_fused_parity(cfg, dyadic=True, label="C2r dyadic")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unfused_forward_deep_input(dtype):
    """rotconv_fwd (every orientation written) on an input too deep for an LDS-resident filter block."""
    cfg = LC("u_deep", N=1, Cin=512, H=6, W=32, Cout=8, R=4, x_dist="absnormal", seed=43)
    say(f"[case] unfused forward, deep input, {dtype}")
    x, w = synth.make_x(cfg), synth.make_w(cfg)
    if dtype == "bf16":
        xd, wd = pu.dev(x, torch.bfloat16), pu.dev(w, torch.bfloat16)
        x, w = xd.to(torch.float64).cpu().numpy(), wd.to(torch.float64).cpu().numpy()
        plan = rc.Plan.from_config(cfg, dtype=rc.BF16)
        y = torch.full((cfg.N, plan.Cunpooled, plan.Ho, plan.Wo), float("nan"), dtype=torch.bfloat16, device="cuda")
    else:
        xd, wd = pu.dev(x), pu.dev(w)
        plan = rc.Plan.from_config(cfg)
        y = torch.full((cfg.N, plan.Cunpooled, plan.Ho, plan.Wo), float("nan"), device="cuda")
    rc.rotconv_fwd(plan, xd, wd, y)
    torch.cuda.synchronize()
    ref = orc.rotconv_fwd(x, orc.expand_bank(w, cfg.R, None, cfg.mode), cfg.stride, cfg.pad)
    pu.assert_close(y.to(torch.float64).cpu().numpy().reshape(ref.shape), ref, f"deep unfused y {dtype}",
                    rtol=1e-2 if dtype == "bf16" else pu.RTOL)


RELU_CASES = [TINY[0], TINY[10], TINY[13], TINY[18],
              LC("r_fast", N=2, Cin=20, H=12, W=32, Cout=18, R=4, x_dist="normal", seed=48),
              LC("r_r16", N=1, Cin=24, H=10, W=64, Cout=12, R=16, mode="bilinear", x_dist="normal", seed=49)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cfg", RELU_CASES, ids=lambda c: c.name)
def test_fused_relu_marks_dead_elements(cfg, dtype):
    """Plans with the fused ReLU: the pooled forward equals max(unfused result, 0) with idx 255 exactly where that
    result is not positive, and the two gradient calls fed that idx equal the gradient calls of the plain plan fed
    the ReLU-masked upstream gradient (every kernel family: generic, fp32 MFMA, bf16 MFMA, per-bank candidates)."""
    say(f"[case] fused ReLU {cfg.name} {dtype}")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dt = rc.BF16 if dtype == "bf16" else rc.F32
    plain, fused = rc.Plan.from_config(cfg, dtype=dt), rc.Plan.from_config(cfg, dtype=dt, relu=True)
    x, w, g = (pu.dev(a, tdt) for a in (synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)))
    P = (cfg.N, plain.Cpooled, plain.Ho, plain.Wo)
    mk = lambda: (torch.full(P, float("nan"), dtype=tdt, device="cuda"), torch.full(P, 77, dtype=torch.uint8, device="cuda"))
    (y0, i0), (y1, i1) = mk(), mk()
    rc.rotconv_pool_fwd(plain, x, w, y0, i0)
    rc.rotconv_pool_fwd(fused, x, w, y1, i1)
    torch.cuda.synchronize()
    alive = y0 > 0
    assert 0.02 < float(alive.float().mean()) < 0.98        # the case exercises both branches
    assert torch.equal(y1, torch.where(alive, y0, torch.zeros_like(y0)))
    assert torch.equal(i1, torch.where(alive, i0, torch.full_like(i0, 255)))
    gm = torch.where(alive, g, torch.zeros_like(g))
    dx0, dx1 = torch.full_like(x, float("nan")), torch.full_like(x, float("nan"))
    rc.rotconv_pool_bwd_data(plain, gm, i0, w, dx0)
    rc.rotconv_pool_bwd_data(fused, g, i1, w, dx1)
    dw0 = torch.full(w.shape, float("nan"), device="cuda")
    dw1 = torch.full(w.shape, float("nan"), device="cuda")
    rc.rotconv_pool_bwd_weight(plain, x, gm, i0, dw0)
    rc.rotconv_pool_bwd_weight(fused, x, g, i1, dw1)
    torch.cuda.synchronize()
    assert torch.equal(dx0, dx1) and torch.equal(dw0, dw1)
