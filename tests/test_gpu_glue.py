"""GPU parity of the network glue (include/unetglue.h) and of the UNet-shaped training step
against the CPU oracle (oracle/unet_oracle.py), called through the C-ABI binding."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import rotconv_oracle as orc
from oracle import unet_oracle as uo
from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import unet as un
from parity_util import RTOL, assert_close, check_idx, dev, layer_bwd_bf16, layer_fwd_bf16

pytestmark = pytest.mark.gpu
BF_RTOL = 1e-2      # one rounding to bfloat16 is 2^-9; the benchmark's bf16 bar is 2e-2


def nan(*shape, dtype=torch.float32):
    t = torch.empty(shape, dtype=dtype, device="cuda")
    t.fill_(float("nan") if dtype.is_floating_point else 255)
    return t


def f32(rng, *shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def test_relu_fwd_bwd():
    rng = np.random.default_rng(1)
    x = f32(rng, 3, 5, 7, 11)
    x.flat[::7] = 0.0
    dy = f32(rng, 3, 5, 7, 11)
    y = nan(*x.shape)
    rc.glue_relu_fwd(dev(x), y)
    assert np.array_equal(host(y), uo.relu_fwd(x).astype(np.float32))
    dx = nan(*x.shape)
    rc.glue_relu_bwd(y, dev(dy), dx)
    assert np.array_equal(host(dx), uo.relu_bwd(uo.relu_fwd(x), dy).astype(np.float32))
    # in place
    t = dev(x)
    rc.glue_relu_fwd(t, t)
    assert np.array_equal(host(t), host(y))


@pytest.mark.parametrize("shape", [(2, 3, 6, 10), (1, 5, 2, 2), (3, 2, 34, 18)])
def test_maxpool2(shape):
    rng = np.random.default_rng(2)
    x = rng.integers(-4, 5, size=shape).astype(np.float32)      # many ties: the first maximum must win
    N, C, H, W = shape
    y, idx = nan(N, C, H // 2, W // 2), nan(N, C, H // 2, W // 2, dtype=torch.uint8)
    rc.glue_maxpool2_fwd(dev(x), y, idx)
    yr, ir = uo.maxpool2_fwd(x)
    assert np.array_equal(host(y), yr.astype(np.float32)) and np.array_equal(host(idx), ir)
    dy = f32(rng, N, C, H // 2, W // 2)
    dx = nan(*shape)
    rc.glue_maxpool2_bwd(dev(dy), idx, dx)
    ref = uo.maxpool2_bwd(dy, ir, H, W)
    assert np.array_equal(host(dx), ref.astype(np.float32))
    base = f32(rng, *shape)
    acc = dev(base)
    rc.glue_maxpool2_bwd(dev(dy), idx, acc, accumulate=True)
    assert np.array_equal(host(acc), (base + ref.astype(np.float32)).astype(np.float32))


@pytest.mark.parametrize("N,Cin,Cout,H,W", [(2, 5, 3, 3, 5), (1, 40, 36, 9, 7), (2, 130, 70, 12, 16), (1, 256, 128, 16, 16)])
def test_upconv2(N, Cin, Cout, H, W):
    rng = np.random.default_rng(3)
    x, w = f32(rng, N, Cin, H, W), f32(rng, Cin, Cout, 2, 2, scale=Cin ** -0.5)
    dy = f32(rng, N, Cout, 2 * H, 2 * W)
    y = nan(N, Cout, 2 * H, 2 * W)
    rc.glue_upconv2_fwd(dev(x), dev(w), y)
    assert_close(host(y), uo.upconv2_fwd(x, w), "upconv2_fwd")
    dxr, dwr = uo.upconv2_bwd(x, w, dy)
    dx = nan(N, Cin, H, W)
    rc.glue_upconv2_bwd_data(dev(dy), dev(w), dx)
    assert_close(host(dx), dxr, "upconv2_bwd_data")
    dw = nan(Cin, Cout, 2, 2)
    ws = torch.empty(max(256, rc.glue_upconv2_workspace_bytes(N, Cin, Cout, H, W)), dtype=torch.uint8, device="cuda")
    rc.glue_upconv2_bwd_weight(dev(x), dev(dy), dw, ws)
    assert_close(host(dw), dwr, "upconv2_bwd_weight")
    first = host(dw).copy()
    rc.glue_upconv2_bwd_weight(dev(x), dev(dy), dw, ws)
    assert np.array_equal(first, host(dw))                      # fixed reduction order


def test_concat_split():
    rng = np.random.default_rng(4)
    a, b = f32(rng, 3, 4, 5, 6), f32(rng, 3, 7, 5, 6)
    out = nan(3, 11, 5, 6)
    rc.glue_concat2(dev(a), dev(b), out)
    cat = np.concatenate([a, b], axis=1)
    assert np.array_equal(host(out), cat)
    da, db = nan(*a.shape), nan(*b.shape)
    rc.glue_split2(out, da, db)
    assert np.array_equal(host(da), a) and np.array_equal(host(db), b)
    base = f32(rng, *a.shape)
    da = dev(base)
    rc.glue_split2(out, da, db, accumulate_a=True)
    assert np.array_equal(host(da), base + a)


@pytest.mark.parametrize("N,Cin,Cout,H,W", [(2, 7, 3, 5, 9), (1, 64, 6, 48, 40), (2, 150, 130, 6, 22),
                                           # few classes, pixel count a multiple of the vector: the streaming kernels
                                           (3, 70, 8, 16, 12), (2, 16, 1, 8, 8), (2, 64, 6, 128, 160)])
def test_conv1x1(N, Cin, Cout, H, W):
    rng = np.random.default_rng(5)
    x, w, dy = f32(rng, N, Cin, H, W), f32(rng, Cout, Cin, scale=Cin ** -0.5), f32(rng, N, Cout, H, W)
    y = nan(N, Cout, H, W)
    rc.glue_conv1x1_fwd(dev(x), dev(w), y)
    assert_close(host(y), uo.conv1x1_fwd(x, w), "conv1x1_fwd")
    dxr, dwr = uo.conv1x1_bwd(x, w, dy)
    dx = nan(N, Cin, H, W)
    rc.glue_conv1x1_bwd_data(dev(dy), dev(w), dx)
    assert_close(host(dx), dxr, "conv1x1_bwd_data")
    dw = nan(Cout, Cin)
    ws = torch.empty(max(256, rc.glue_conv1x1_workspace_bytes(N, Cin, Cout, H * W)), dtype=torch.uint8, device="cuda")
    rc.glue_conv1x1_bwd_weight(dev(x), dev(dy), dw, ws)
    assert_close(host(dw), dwr, "conv1x1_bwd_weight")


@pytest.mark.parametrize("N,K,H,W", [(1, 2, 3, 5), (2, 6, 33, 20), (3, 11, 8, 8)])
def test_softmax_ce(N, K, H, W):
    rng = np.random.default_rng(6)
    lg = f32(rng, N, K, H, W, scale=4.0)
    lab = rng.integers(0, K, size=(N, H, W)).astype(np.int32)
    loss, dl = nan(1), nan(N, K, H, W)
    ws = torch.empty(N * H * W * 4, dtype=torch.uint8, device="cuda")
    rc.glue_softmax_ce(dev(lg), dev(lab), loss, dl, ws)
    lr, dlr = uo.softmax_ce(lg, lab)
    assert abs(float(host(loss)[0]) - lr) <= RTOL * abs(lr)
    assert_close(host(dl), dlr, "softmax_ce dlogits")


def test_softmax_ce_ignores_out_of_range_labels():
    lg = np.zeros((1, 3, 2, 2), np.float32)
    lab = np.array([[[0, 7], [-1, 2]]], np.int32)
    loss, dl = nan(1), nan(1, 3, 2, 2)
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    rc.glue_softmax_ce(dev(lg), dev(lab), loss, dl, ws)
    assert np.isclose(float(host(loss)[0]), 2 * np.log(3) / 4, rtol=1e-6)
    d = host(dl)
    assert np.all(d[0, :, 0, 1] == 0) and np.all(d[0, :, 1, 0] == 0)


# ---- bfloat16 twins: same definitions on the bf16 values, one rounding of each bf16 output ----------

def _b16(a):
    """numpy -> (bf16 cuda tensor, its values as fp64)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.cuda(), t.to(torch.float64).numpy()


def _h64(t):
    torch.cuda.synchronize()
    return t.to(torch.float64).cpu().numpy()


def _rb(a):
    """fp64 reference rounded to bf16 (nearest even) -> fp64: what an exact bf16 result must equal."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).to(
        torch.float64).numpy()


@pytest.mark.parametrize("shape", [(2, 3, 6, 10), (1, 5, 2, 2), (3, 2, 34, 16), (1, 4, 8, 40)])
def test_bf16_streaming_ops(shape):
    rng = np.random.default_rng(21)
    N, C, H, W = shape
    bf = torch.bfloat16
    xd, x = _b16(rng.integers(-4, 5, size=shape))                 # ties: the first maximum must win
    y = nan(*shape, dtype=bf)
    rc.glue_relu_fwd(xd, y)
    assert np.array_equal(_h64(y), uo.relu_fwd(x))
    dyd, dy = _b16(f32(rng, *shape))
    dx = nan(*shape, dtype=bf)
    rc.glue_relu_bwd(y, dyd, dx)
    assert np.array_equal(_h64(dx), uo.relu_bwd(uo.relu_fwd(x), dy))
    yp, idx = nan(N, C, H // 2, W // 2, dtype=bf), nan(N, C, H // 2, W // 2, dtype=torch.uint8)
    rc.glue_maxpool2_fwd(xd, yp, idx)
    yr, ir = uo.maxpool2_fwd(x)
    assert np.array_equal(_h64(yp), yr) and np.array_equal(host(idx), ir)
    gd, g = _b16(f32(rng, N, C, H // 2, W // 2))
    dxp = nan(*shape, dtype=bf)
    rc.glue_maxpool2_bwd(gd, idx, dxp)
    ref = uo.maxpool2_bwd(g, ir, H, W)
    assert np.array_equal(_h64(dxp), ref)
    accd, base = _b16(f32(rng, *shape))
    rc.glue_maxpool2_bwd(gd, idx, accd, accumulate=True)
    assert np.array_equal(_h64(accd), _rb(base + ref))
    bd, b = _b16(f32(rng, N, C + 3, H, W))
    cat = nan(N, 2 * C + 3, H, W, dtype=bf)
    rc.glue_concat2(xd, bd, cat)
    assert np.array_equal(_h64(cat), np.concatenate([x, b], axis=1))
    da, db = nan(*shape, dtype=bf), nan(N, C + 3, H, W, dtype=bf)
    rc.glue_split2(cat, da, db)
    assert np.array_equal(_h64(da), x) and np.array_equal(_h64(db), b)
    rc.glue_split2(cat, accd, db, accumulate_a=True)
    assert np.array_equal(_h64(accd), _rb(_rb(base + ref) + x))


@pytest.mark.parametrize("N,Cin,Cout,H,W", [(2, 5, 3, 3, 5), (1, 40, 36, 9, 7), (2, 130, 70, 12, 16), (1, 256, 128, 16, 16),
                                           (1, 33, 65, 31, 3)])
def test_bf16_gemm_layers(N, Cin, Cout, H, W):
    rng = np.random.default_rng(22)
    bf = torch.bfloat16
    xd, x = _b16(f32(rng, N, Cin, H, W))
    wd, w = _b16(f32(rng, Cin, Cout, 2, 2, scale=Cin ** -0.5))
    dyd, dy = _b16(f32(rng, N, Cout, 2 * H, 2 * W))
    y = nan(N, Cout, 2 * H, 2 * W, dtype=bf)
    rc.glue_upconv2_fwd(xd, wd, y)
    assert_close(_h64(y), uo.upconv2_fwd(x, w), "bf16 upconv2_fwd", rtol=BF_RTOL)
    dxr, dwr = uo.upconv2_bwd(x, w, dy)
    dx = nan(N, Cin, H, W, dtype=bf)
    rc.glue_upconv2_bwd_data(dyd, wd, dx)
    assert_close(_h64(dx), dxr, "bf16 upconv2_bwd_data", rtol=BF_RTOL)
    dw = nan(Cin, Cout, 2, 2)
    ws = torch.empty(max(256, rc.glue_upconv2_workspace_bytes(N, Cin, Cout, H, W)), dtype=torch.uint8, device="cuda")
    rc.glue_upconv2_bwd_weight(xd, dyd, dw, ws)
    assert_close(host(dw), dwr, "bf16 upconv2_bwd_weight (fp32 result)")
    # 1x1 head on the same tensors, read as [N, Cin, P]
    hwd, hw = _b16(f32(rng, Cout, Cin, scale=Cin ** -0.5))
    gd, g = _b16(f32(rng, N, Cout, H, W))
    yh = nan(N, Cout, H, W, dtype=bf)
    rc.glue_conv1x1_fwd(xd, hwd, yh)
    assert_close(_h64(yh), uo.conv1x1_fwd(x, hw), "bf16 conv1x1_fwd", rtol=BF_RTOL)
    dxr, dwr = uo.conv1x1_bwd(x, hw, g)
    rc.glue_conv1x1_bwd_data(gd, hwd, dx)
    assert_close(_h64(dx), dxr, "bf16 conv1x1_bwd_data", rtol=BF_RTOL)
    dwh = nan(Cout, Cin)
    ws = torch.empty(max(256, rc.glue_conv1x1_workspace_bytes(N, Cin, Cout, H * W)), dtype=torch.uint8, device="cuda")
    rc.glue_conv1x1_bwd_weight(xd, gd, dwh, ws)
    assert_close(host(dwh), dwr, "bf16 conv1x1_bwd_weight (fp32 result)")
    # soft-max cross-entropy on bf16 logits: fp32 loss, bf16 gradient
    K = Cout
    lab = rng.integers(0, K, size=(N, H, W)).astype(np.int32)
    loss, dl = nan(1), nan(N, K, H, W, dtype=bf)
    ws = torch.empty(N * H * W * 4, dtype=torch.uint8, device="cuda")
    rc.glue_softmax_ce(gd, dev(lab), loss, dl, ws)
    lr, dlr = uo.softmax_ce(g, lab)
    assert abs(float(host(loss)[0]) - lr) <= RTOL * abs(lr)
    assert_close(_h64(dl), dlr, "bf16 softmax_ce dlogits", rtol=BF_RTOL)


@pytest.mark.parametrize("N,Cin,Cout,H,W", [(2, 64, 6, 16, 24), (1, 70, 8, 8, 8), (3, 5, 2, 4, 8), (2, 64, 6, 128, 96)])
def test_bf16_head_streaming(N, Cin, Cout, H, W):
    """1x1 head with few classes on bf16 tensors whose pixel count is a multiple of the 8-element vector."""
    rng = np.random.default_rng(23)
    bf = torch.bfloat16
    xd, x = _b16(f32(rng, N, Cin, H, W))
    wd, w = _b16(f32(rng, Cout, Cin, scale=Cin ** -0.5))
    gd, g = _b16(f32(rng, N, Cout, H, W))
    y = nan(N, Cout, H, W, dtype=bf)
    rc.glue_conv1x1_fwd(xd, wd, y)
    assert_close(_h64(y), uo.conv1x1_fwd(x, w), "bf16 head fwd", rtol=BF_RTOL)
    dxr, dwr = uo.conv1x1_bwd(x, w, g)
    dx = nan(N, Cin, H, W, dtype=bf)
    rc.glue_conv1x1_bwd_data(gd, wd, dx)
    assert_close(_h64(dx), dxr, "bf16 head bwd_data", rtol=BF_RTOL)
    dw = nan(Cout, Cin)
    ws = torch.empty(max(256, rc.glue_conv1x1_workspace_bytes(N, Cin, Cout, H * W)), dtype=torch.uint8, device="cuda")
    rc.glue_conv1x1_bwd_weight(xd, gd, dw, ws)
    assert_close(host(dw), dwr, "bf16 head bwd_weight (fp32 result)")


def test_glue_rejects_mixed_storage_types():
    a = torch.zeros(8, device="cuda")
    b = torch.zeros(8, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        rc.glue_relu_fwd(a, b)


# ---- the stack ------------------------------------------------------------------------------------

def _bf16_round(a):
    """fp32 values rounded to bfloat16 (nearest even), returned as fp32."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _run_stack(cfg, dtype="f32", fuse_relu=False):
    params = un.make_params(cfg)
    images, labels = un.make_batch(cfg)
    if dtype == "bf16":     # the values the GPU holds after its one rounding
        params = {k: _bf16_round(v) for k, v in params.items()}
        images = _bf16_round(images)
    net = un.UNet(cfg, params, dtype=dtype, fuse_relu=fuse_relu)
    net.load_batch(images, labels)
    for t in list(net.grads.values()) + [net.loss]:
        t.fill_(float("nan"))
    net.step()
    torch.cuda.synchronize()
    return net, params, images, labels


SMALL = [
    un.UNetConfig("u_r4_d2", 2, 3, 32, 64, (8, 12, 16), 4, R=4, mode="exact90", seed=11),
    un.UNetConfig("u_r4_d3", 1, 3, 64, 32, (16, 24, 40, 72), 6, R=4, mode="exact90", seed=12),
    un.UNetConfig("u_r16_d2", 1, 3, 32, 32, (8, 8, 16), 3, R=16, mode="bilinear", pool_group=16, seed=13),
    # the paper's own block: rotation convolution pooled over quarter turns, then a standard convolution
    un.UNetConfig("p_r4_d2", 2, 3, 32, 64, (8, 12, 16), 4, R=4, mode="exact90", block="rot_std", seed=14),
    un.UNetConfig("p_r8_d2", 1, 3, 32, 32, (8, 12, 16), 3, R=8, mode="bilinear", block="rot_std", seed=15),
    un.UNetConfig("p_r16_d1", 1, 3, 32, 64, (8, 16), 3, R=16, mode="steerable", block="rot_std", seed=16),
]


TEACHER = [(c, "f32") for c in SMALL] + [(SMALL[0], "bf16"), (SMALL[2], "bf16"), (SMALL[4], "bf16")]


@pytest.mark.parametrize("cfg,dtype", TEACHER, ids=[f"{c.name}-{d}" for c, d in TEACHER])
def test_unet_step_teacher_forced(cfg, dtype):
    """Every call of the step against the oracle's result for the same call, each fed the tensors the
    GPU step itself produced (so one near-tie arg-max cannot cascade), plus the loss.  bf16: the same, with
    the oracle fed the bf16 values the GPU holds; bf16 outputs to the bf16 bar, fp32 weight gradients and
    the loss to the fp32 bar."""
    net, params, images, labels = _run_stack(cfg, dtype)
    A = net.act
    H = lambda t: t.detach().to(torch.float64).cpu().numpy()
    act_close = assert_close if dtype == "f32" else (lambda got, ref, what: assert_close(got, ref, what, rtol=BF_RTOL))
    layer_fwd = orc.layer_fwd if dtype == "f32" else layer_fwd_bf16    # bf16 plans hold their rotated banks in bf16
    layer_bwd = orc.layer_bwd if dtype == "f32" else layer_bwd_bf16
    p64 = {k: v.astype(np.float64) for k, v in params.items()}
    # forward, layer by layer
    for sp in net.specs:
        name, R, mode, G = sp["name"], sp["R"], sp["mode"], sp["pool_group"]
        x = H(A[name]["x"])
        y_ref, yp_ref, idx_ref, w_rot = layer_fwd(x, p64[name], R, None, mode, 1, 1, G)
        act_close(H(A[name]["y"]), uo.relu_fwd(yp_ref), f"{name} fwd")
        abs_terms = orc.rotconv_fwd(np.abs(x), np.abs(w_rot), 1, 1)
        check_idx(H(A[name]["idx"]).astype(np.uint8), y_ref, abs_terms, G or R, f"{name} idx")
    for lvl in range(cfg.depth):
        p = A[f"pool{lvl}"]
        yr, ir = uo.maxpool2_fwd(H(A[f"enc{lvl}b"]["y"]))
        assert np.array_equal(H(p["y"]), yr) and np.array_equal(H(p["idx"]).astype(np.uint8), ir)
        u = A[f"up{lvl}"]
        act_close(H(u["y"]), uo.upconv2_fwd(H(u["x"]), p64[f"up{lvl}"]), f"up{lvl} fwd")
        assert np.array_equal(H(u["cat"]), np.concatenate([H(A[f"enc{lvl}b"]["y"]), H(u["y"])], axis=1))
    hd = A["head"]
    act_close(H(hd["y"]), uo.conv1x1_fwd(H(hd["x"]), p64["head"]), "head fwd")
    loss_ref, dl_ref = uo.softmax_ce(H(hd["y"]), labels)
    assert abs(float(net.loss.cpu()[0]) - loss_ref) <= RTOL * abs(loss_ref)
    act_close(H(hd["g"]), dl_ref, "dlogits")
    # backward, call by call, on the GPU's own upstream gradients and arg-max indices
    # (a gradient slot is masked in place by its owner's ReLU backward after it is written, so a
    # producer's dX is compared where that mask kept it)
    masked = lambda owner, ref: np.where(H(A[owner]["y"]) > 0, ref, 0.0)
    dxr, dwr = uo.conv1x1_bwd(H(hd["x"]), p64["head"], H(hd["g"]))
    assert_close(H(net.grads["head"]), dwr, "head dW")
    act_close(H(A["dec0b"]["g"]), masked("dec0b", dxr), "head dX")
    for i, sp in enumerate(net.specs):
        name = sp["name"]
        a = A[name]
        g = H(a["g"])                       # after the in-place ReLU backward: gradient of the pooled map
        assert np.all(g[H(a["y"]) <= 0] == 0), f"{name}: ReLU backward"
        dx_ref, dw_ref = layer_bwd(H(a["x"]), p64[name], g, H(a["idx"]).astype(np.uint8), sp["R"], None,
                                       sp["mode"], 1, 1, sp["pool_group"])
        # (a bf16 plan on the table kernels rounds the folded routed gradient to bf16 once: the bf16 bar)
        assert_close(H(net.grads[name]), dw_ref, f"{name} dW",
                     rtol=BF_RTOL if net.plans[name].kernel_name(2).endswith("_lut") else RTOL)
        if i == 0:
            continue
        if name.endswith("b"):              # lands in the block's first layer's slot
            act_close(H(a["gx"]), masked(name[:-1] + "a", dx_ref), f"{name} dX")
        else:                               # lands in a pool's or a concatenation's slot: not touched again
            act_close(H(a["gx"]), dx_ref, f"{name} dX")
    for lvl in range(cfg.depth):
        u = A[f"up{lvl}"]
        C = cfg.widths[lvl]
        dx_ref, dw_ref = uo.upconv2_bwd(H(u["x"]), p64[f"up{lvl}"], H(u["g"]))
        assert_close(H(net.grads[f"up{lvl}"]), dw_ref, f"up{lvl} dW")
        below = "botb" if lvl == cfg.depth - 1 else f"dec{lvl + 1}b"
        act_close(H(A[below]["g"]), masked(below, dx_ref), f"up{lvl} dX")
        assert np.array_equal(H(u["gcat"])[:, C:], H(u["g"]))
        # skip gradient + the 2x2 max-pool's routed gradient, then the encoder layer's ReLU mask
        p = A[f"pool{lvl}"]
        ref = H(u["gcat"])[:, :C] + uo.maxpool2_bwd(H(p["g"]), H(p["idx"]).astype(np.uint8), *A[f"enc{lvl}b"]["y"].shape[2:])
        act_close(H(A[f"enc{lvl}b"]["g"]), masked(f"enc{lvl}b", ref), f"enc{lvl}b upstream gradient")


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[3]], ids=lambda c: c.name)
def test_unet_step_end_to_end_loss_and_gradients(cfg):
    """The whole step against the oracle's whole step on one small stack: loss to the fp32 bar, the
    gradients in relative L2 norm (an arg-max that flips on a near-tie moves single elements, not the
    norm; the teacher-forced test above holds each call to the elementwise bar)."""
    net, params, images, labels = _run_stack(cfg)
    p64 = {k: v.astype(np.float64) for k, v in params.items()}
    loss, grads, acts = uo.unet_step(images.astype(np.float64), labels, p64, cfg.R, cfg.mode, cfg.pool_group,
                                     un.oracle_layer_spec(cfg))
    assert abs(float(net.loss.cpu()[0]) - loss) <= RTOL * abs(loss)
    for name, gref in grads.items():
        got = net.grads[name].cpu().numpy().astype(np.float64)
        rel = np.linalg.norm(got - gref) / max(np.linalg.norm(gref), 1e-30)
        assert rel < 5e-3, (name, rel)
    flips = sum(int((net.act[n]["idx"].cpu().numpy() != acts[n]["idx"]).sum()) for n, *_ in net.layers)
    total = sum(net.act[n]["idx"].numel() for n, *_ in net.layers)
    assert flips <= 1e-3 * total, (flips, total)


@pytest.mark.parametrize("cfg,dtype", [(SMALL[0], "f32"), (SMALL[2], "f32"), (SMALL[5], "f32"), (SMALL[2], "bf16")],
                         ids=lambda v: v if isinstance(v, str) else v.name)
def test_unet_step_fused_relu_equals_separate_relu(cfg, dtype):
    """The plan's fused ReLU (forward clamps the pooled value and stores idx 255 at dead elements, the gradient calls
    then skip them) against the separate ReLU passes checked call by call above: same activations, same loss, same
    parameter gradients (a dead element contributes an exact zero either way)."""
    a, *_ = _run_stack(cfg, dtype, fuse_relu=False)
    b, *_ = _run_stack(cfg, dtype, fuse_relu=True)
    assert float(a.loss.cpu()[0]) == float(b.loss.cpu()[0])
    for n, *_ in a.layers:
        ya, yb = a.act[n]["y"].float().cpu().numpy(), b.act[n]["y"].float().cpu().numpy()
        assert np.array_equal(ya, yb), n
        ia, ib = a.act[n]["idx"].cpu().numpy(), b.act[n]["idx"].cpu().numpy()
        assert np.array_equal(ib, np.where(yb > 0, ia, 255)), n
    for k in a.grads:
        assert np.array_equal(a.grads[k].cpu().numpy(), b.grads[k].cpu().numpy()), k


def test_unet_step_is_deterministic():
    cfg = SMALL[1]
    net, *_ = _run_stack(cfg)
    first = {k: v.cpu().numpy().copy() for k, v in net.grads.items()}
    l0 = float(net.loss.cpu()[0])
    net.step()
    torch.cuda.synchronize()
    assert float(net.loss.cpu()[0]) == l0
    for k, v in net.grads.items():
        assert np.array_equal(first[k], v.cpu().numpy()), k


@pytest.mark.parametrize("cfg,dtype", [(SMALL[1], "f32"), (SMALL[2], "f32"), (SMALL[2], "bf16")],
                         ids=lambda v: v if isinstance(v, str) else v.name)
def test_unet_step_replays_from_a_graph(cfg, dtype):
    """The whole training step recorded into a HIP graph: replays (with the program's own eager work and
    synchronisations between them, and a new batch in the captured buffers) give bit for bit the eager step."""
    net, *_ = _run_stack(cfg, dtype)
    net.capture()
    for rep in range(3):
        cfg2 = dataclasses.replace(cfg, seed=cfg.seed + 10 * rep) if hasattr(cfg, "seed") else cfg
        net.load_batch(*un.make_batch(cfg2))
        net.step()
        torch.cuda.synchronize()
        loss = float(net.loss.cpu()[0])
        grads = {k: v.cpu().numpy().copy() for k, v in net.grads.items()}
        for v in net.grads.values():
            v.zero_()
        net.loss.zero_()
        torch.cuda.synchronize()
        net.replay()
        torch.cuda.synchronize()
        assert float(net.loss.cpu()[0]) == loss, rep
        for k, v in net.grads.items():
            assert np.array_equal(grads[k], v.cpu().numpy()), (rep, k)


# ---- the benchmark's stacks at full size ------------------------------------------------------------

def _say(msg):
    print(msg, flush=True)


def _pts(seed, n, dims):
    from paper_2512_08888_amd import synth
    return np.stack([synth.randint(seed + i, n, 0, d - 1) for i, d in enumerate(dims)], axis=1).astype(np.int32)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg,dtype", [(un.C4, "f32"), (un.C5, "f32"), (un.P8, "f32"), (un.C5, "bf16")],
                         ids=["C4", "C5", "P8", "C5-bf16"])
def test_unet_full_size_sampled(cfg, dtype):
    """The benchmark's stacks (and the paper's own block at 8 orientations) in the launch configuration
    bench.py times.  Every rotation-convolution call is checked on sampled outputs the oracle computes one by
    one from the tensors that call read on the GPU (forward values and arg-max, input gradient, weight
    gradient), every glue call against its definition, plus the homogeneity identity <w, dW> = <y, g> per
    layer at full size.  bf16: the oracle reads the bf16 values the GPU holds (rotated banks rounded to bf16),
    bf16 outputs are held to the bf16 bar, fp32 weight gradients and the loss to the fp32 bar."""
    from parity_util import round_bf16
    net, params, images, labels = _run_stack(cfg, dtype, fuse_relu=True)     # as bench.py runs it
    A = net.act
    bf = dtype == "bf16"
    AT = BF_RTOL if bf else RTOL                    # bar of activation-typed outputs
    H = (lambda t: t.detach().to(torch.float32).cpu().numpy()) if bf else (lambda t: t.detach().cpu().numpy())
    act_close = lambda got, ref, what: assert_close(got, ref, what, rtol=AT)
    ns, npairs = 384, 4
    for li, sp in enumerate(net.specs):
        name, ci, co, h, w, R, mode = sp["name"], sp["Cin"], sp["Cout"], sp["H"], sp["W"], sp["R"], sp["mode"]
        G = sp["pool_group"] or R
        ng = R // G
        a = A[name]
        x, y, idx, g = H(a["x"]), H(a["y"]), a["idx"].cpu().numpy(), H(a["g"])
        wb = params[name].astype(np.float64)
        w_rot = orc.expand_bank(wb, R, None, mode)
        if bf:
            w_rot = round_bf16(w_rot)
        pts = _pts(1000 + li, ns, (cfg.N, co, h, w))
        yr = orc.rotconv_fwd_at(x, w_rot, pts, 1, 1)
        ya = orc.rotconv_fwd_at(np.abs(x), np.abs(w_rot), pts, 1, 1)
        rms = float(np.sqrt(np.mean(yr.reshape(ns, G, ng).max(axis=1) ** 2)))
        for grp in range(ng):
            members = np.arange(grp, R, ng)
            best = yr[:, members].max(axis=1)
            chan = pts[:, 1] * ng + grp
            got_v = y[pts[:, 0], chan, pts[:, 2], pts[:, 3]].astype(np.float64)
            got_i = idx[pts[:, 0], chan, pts[:, 2], pts[:, 3]].astype(np.int64)
            assert np.all(np.abs(got_v - np.maximum(best, 0)) <= AT * np.abs(best) + AT * rms), f"{name} fwd samples"
            tau = 64.0 * np.finfo(np.float32).eps * ya[:, members].max(axis=1)
            # fused ReLU: a dead element (pooled value not positive) carries idx 255; alive ones the arg-max
            dead = got_i == 255
            assert np.all(got_v[dead] == 0) and np.all(best[dead] <= tau[dead]), f"{name} dead elements"
            gi = np.where(dead, grp, got_i)
            assert np.all(gi % ng == grp) and np.all(gi < R), f"{name} arg-max group"
            assert np.all((yr[np.arange(ns), gi] >= best - tau) | dead), f"{name} arg-max samples"
        # weight gradient: sampled (co, ci) slices, reduced through Eq. 16 by the oracle
        pairs = _pts(2000 + li, npairs, (co, ci))
        dwr = orc.rotconv_pool_bwd_weight_at(x, g, idx, pairs, R, 3, G, 1, 1)
        dw = H(net.grads[name])
        got_dw, ref_dw = [], []
        for t, (o, c) in enumerate(pairs):
            full = np.zeros((R, 1, 1, 3, 3))
            full[:, 0, 0] = dwr[t]
            ref_dw.append(orc.reduce_bank_grad(full, None, mode)[:, 0, 0])
            got_dw.append(dw[:, o, c])
        assert_close(np.array(got_dw), np.array(ref_dw), f"{name} dW samples",
                     rtol=BF_RTOL if net.plans[name].kernel_name(2).endswith("_lut") else RTOL)
        # homogeneity through max-pool and ReLU: <w, dW> = <y, g>
        lhs = float((params[name].astype(np.float64) * dw).sum())
        rhs = float((y.astype(np.float64) * g).sum())
        scale = float(np.abs(y.astype(np.float64) * g).sum())
        # (bf16: y is the rounded output, so the identity holds to the rounding of y, about 2^-9 / sqrt(count))
        assert abs(lhs - rhs) <= (1e-4 if bf else 1e-5) * scale, (name, lhs, rhs, scale)
        # input gradient at sampled inputs of one image (slots a later in-place ReLU backward masks are
        # compared where the mask kept them)
        if li > 0 and co * R * h * w <= 300_000_000:
            n0 = li % cfg.N
            dy = orc.orient_maxpool_bwd(g[n0:n0 + 1], idx[n0:n0 + 1], R, G)
            ptx = _pts(3000 + li, ns, (1, ci, h, w))
            ref = orc.rotconv_bwd_data_at(dy, w_rot, ptx, h, w, 1, 1)
            got = H(a["gx"])[n0][ptx[:, 1], ptx[:, 2], ptx[:, 3]].astype(np.float64)
            act_close(got, ref, f"{name} dX samples")     # (fused ReLU: the slot is not masked in place afterwards)
            del dy
        _say(f"  {cfg.name} {name}: {ci}->{co} @{h}x{w} ok")
    # glue at full size
    for lvl in range(cfg.depth):
        p, e = A[f"pool{lvl}"], A[f"enc{lvl}b"]
        yr, ir = uo.maxpool2_fwd(H(e["y"]))
        assert np.array_equal(H(p["y"]), yr.astype(np.float32)) and np.array_equal(A[f"pool{lvl}"]["idx"].cpu().numpy(), ir)
        u = A[f"up{lvl}"]
        C = cfg.widths[lvl]
        xin, wu, yu = H(u["x"]).astype(np.float64), params[f"up{lvl}"].astype(np.float64), H(u["y"])
        # the whole up-convolution and its weight gradient against the glue oracle, every element
        act_close(yu, uo.upconv2_fwd(xin, wu), f"up{lvl} fwd")
        cat = H(u["cat"])
        assert np.array_equal(cat[:, :C], H(e["y"])) and np.array_equal(cat[:, C:], yu)
        gu = H(u["g"]).astype(np.float64)
        _, dwu_ref = uo.upconv2_bwd(xin, wu, gu)
        assert_close(H(net.grads[f"up{lvl}"]), dwu_ref, f"up{lvl} dW")
        del dwu_ref
        _say(f"  {cfg.name} pool{lvl}/up{lvl} ok")
    hd = A["head"]
    logits = H(hd["y"])
    act_close(logits, uo.conv1x1_fwd(H(hd["x"]), params["head"]), "head fwd")
    loss_ref, dl_ref = uo.softmax_ce(logits, labels)
    assert abs(float(net.loss.cpu()[0]) - loss_ref) <= RTOL * abs(loss_ref)
    act_close(H(hd["g"]), dl_ref, "dlogits")
    _, dwh = uo.conv1x1_bwd(H(hd["x"]), params["head"], H(hd["g"]))
    assert_close(H(net.grads["head"]), dwh, "head dW")
