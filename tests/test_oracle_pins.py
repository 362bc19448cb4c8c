"""Pins of the CPU oracle to things other than itself (CPU only).

Each test checks the oracle against a library routine, a closed form, a brute
force written here from the equations, or an invariant the mathematics fixes;
they are chosen so that a dropped term, a wrong sign or index, or a transposed
operand anywhere in oracle/rotconv_oracle.c fails at least one of them.
Equation numbers refer to the paper's Sec. III.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import rotconv_oracle as orc

RNG = np.random.default_rng(20251208)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------- rotation convention

def test_exact90_bank_is_numpy_rot90():
    """Eq. 5 with the counter-clockwise reading: W^(r) = rot90^r(W)."""
    for k in (1, 2, 3, 5):
        w = rnd(1, 3, 2, k, k)
        for R, angles in ((4, None), (2, [0.0, 180.0]), (1, None), (3, [90.0, 180.0, 270.0])):
            wr = orc.expand_bank(w, R, angles, "exact90")
            ang = orc.default_angles(R) if angles is None else angles
            for r in range(R):
                s = int(round(ang[r] / 90.0))
                assert np.array_equal(wr[r], np.rot90(w[0], s, axes=(-2, -1)))


def test_corner_tap_visits_four_corners():
    """Sec. III-B, discussion of Fig. 2: a corner weight lands in the 4 corners."""
    w = np.zeros((1, 1, 1, 3, 3))
    w[0, 0, 0, 2, 2] = 1.0
    wr = orc.expand_bank(w, 4)
    corners = {(0, 0), (0, 2), (2, 0), (2, 2)}
    seen = {tuple(np.argwhere(wr[r, 0, 0] == 1.0)[0]) for r in range(4)}
    assert seen == corners
    w[:] = 0
    w[0, 0, 0, 0, 1] = 1.0  # edge tap visits the 4 edges, centre stays
    wr = orc.expand_bank(w, 4)
    seen = {tuple(np.argwhere(wr[r, 0, 0] == 1.0)[0]) for r in range(4)}
    assert seen == {(0, 1), (1, 0), (2, 1), (1, 2)}
    w[:] = 0
    w[0, 0, 0, 1, 1] = 1.0
    wr = orc.expand_bank(w, 4)
    assert all(wr[r, 0, 0, 1, 1] == 1.0 for r in range(4))


def test_exact90_rejects_other_angles():
    with pytest.raises(ValueError):
        orc.expand_bank(rnd(1, 1, 1, 3, 3), 2, [0.0, 45.0], "exact90")


# ---------------------------------------------------------------- forward

def brute_fwd(x, w_rot, stride, pad):
    """Eq. 7 by pure-Python loops over a zero-padded copy."""
    N, Cin, H, W = x.shape
    R, Cout, _, k, _ = w_rot.shape
    xp = np.zeros((N, Cin, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (W + 2 * pad - k) // stride + 1
    y = np.zeros((N, Cout, R, Ho, Wo))
    for n, co, r, oy, ox in itertools.product(range(N), range(Cout), range(R), range(Ho), range(Wo)):
        patch = xp[n, :, oy * stride:oy * stride + k, ox * stride:ox * stride + k]
        y[n, co, r, oy, ox] = float((patch * w_rot[r, co]).sum())
    return y


@pytest.mark.parametrize("k,pad,stride", [(1, 0, 1), (3, 0, 1), (3, 1, 1), (3, 2, 1), (5, 2, 1), (3, 1, 2), (2, 1, 1)])
def test_fwd_brute_force_tiny(k, pad, stride):
    x = rnd(2, 3, 6, 7)
    w = rnd(1, 2, 3, k, k)
    wr = orc.expand_bank(w, 4)
    y = orc.rotconv_fwd(x, wr, stride, pad)
    np.testing.assert_allclose(y, brute_fwd(x, wr, stride, pad), rtol=1e-12, atol=1e-12)


def test_r1_is_plain_convolution():
    """Sec. III-A: a single orientation is the standard convolution (library: torch CPU conv2d)."""
    x = rnd(2, 5, 9, 8)
    w = rnd(1, 4, 5, 3, 3)
    for stride, pad in ((1, 0), (1, 1), (2, 1)):
        y = orc.rotconv_fwd(x, orc.expand_bank(w, 1), stride, pad)
        ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(w[0]), stride=stride, padding=pad).numpy()
        np.testing.assert_allclose(y[:, :, 0], ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("R,mode", [(4, "exact90"), (8, "bilinear"), (16, "bilinear"), (8, "steerable")])
def test_any_R_is_conv2d_with_materialised_bank(R, mode):
    x = rnd(2, 3, 8, 8)
    B = 2 if mode == "steerable" else 1
    w = rnd(B, 4, 3, 3, 3)
    wr = orc.expand_bank(w, R, None, mode)
    y = orc.rotconv_fwd(x, wr, 1, 1)
    bank = torch.from_numpy(wr.transpose(1, 0, 2, 3, 4).reshape(4 * R, 3, 3, 3))  # channel = co*R + r
    ref = F.conv2d(torch.from_numpy(x), bank, padding=1).numpy().reshape(2, 4, R, 8, 8)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,pad", [(3, 1), (3, 0), (5, 2), (1, 0), (3, 2)])
def test_scatter_form_equals_gather_form(k, pad):
    """Eq. 8 / Alg. 1 reach the same numbers as Eq. 7 (exactly, on a binary grid)."""
    x = RNG.integers(0, 16, (2, 3, 6, 5)) / 16.0
    w = RNG.integers(-16, 17, (1, 2, 3, k, k)) / 32.0
    y = orc.rotconv_fwd(x, orc.expand_bank(w, 4), 1, pad)
    ys = orc.rotconv_fwd_scatter(x, w, [0, 1, 2, 3], pad)
    assert np.array_equal(y, ys)
    y2 = orc.rotconv_fwd(x, orc.expand_bank(w, 2, [0.0, 180.0]), 1, pad)
    assert np.array_equal(y2, orc.rotconv_fwd_scatter(x, w, [0, 2], pad))


def test_fwd_at_matches_full():
    x = rnd(2, 3, 7, 6)
    wr = orc.expand_bank(rnd(1, 4, 3, 3, 3), 8, None, "bilinear")
    y = orc.rotconv_fwd(x, wr, 1, 1)
    pts = np.array([[0, 0, 0, 0], [1, 3, 6, 5], [0, 2, 3, 4], [1, 1, 0, 5]], dtype=np.int32)
    got = orc.rotconv_fwd_at(x, wr, pts, 1, 1)
    for t, (n, co, oy, ox) in enumerate(pts):
        np.testing.assert_array_equal(got[t], y[n, co, :, oy, ox])


def test_one_by_one_kernel_is_matmul():
    x = rnd(2, 5, 4, 4)
    w = rnd(1, 3, 5, 1, 1)
    y = orc.rotconv_fwd(x, orc.expand_bank(w, 4), 1, 0)
    ref = np.einsum("oc,nchw->nohw", w[0, :, :, 0, 0], x)
    for r in range(4):
        np.testing.assert_allclose(y[:, :, r], ref, rtol=1e-12, atol=1e-12)


def test_centred_delta_input_closed_form():
    """Unit impulse: the response patch of orientation r is W^(r) turned by 180 deg = W^(r+2)."""
    x = np.zeros((1, 1, 7, 7))
    x[0, 0, 3, 3] = 1.0
    w = rnd(1, 2, 1, 3, 3)
    wr = orc.expand_bank(w, 4)
    y = orc.rotconv_fwd(x, wr, 1, 1)
    for r in range(4):
        np.testing.assert_array_equal(y[0, :, r, 2:5, 2:5], wr[(r + 2) % 4, :, 0])


def test_worked_example_one_hot_corner():
    """3x3 ramp image, one-hot weight at tap (0,0), R=4, pad 1 (derived from Eq. 7, 10, 14, 16)."""
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    w = np.zeros((1, 1, 1, 3, 3))
    w[0, 0, 0, 0, 0] = 1.0
    y, yp, idx, _ = orc.layer_fwd(x, w, 4, pad=1)
    X = np.pad(x[0, 0], 2)
    sh = lambda dy, dx: X[2 + dy:5 + dy, 2 + dx:5 + dx]
    np.testing.assert_array_equal(y[0, 0, 0], sh(-1, -1))
    np.testing.assert_array_equal(y[0, 0, 1], sh(+1, -1))
    np.testing.assert_array_equal(y[0, 0, 2], sh(+1, +1))
    np.testing.assert_array_equal(y[0, 0, 3], sh(-1, +1))
    np.testing.assert_array_equal(yp[0, 0], [[5, 6, 5], [8, 9, 8], [5, 6, 5]])
    np.testing.assert_array_equal(idx[0, 0], [[2, 2, 1], [2, 2, 1], [3, 3, 0]])
    dx, dw = orc.layer_bwd(x, w, np.ones((1, 1, 3, 3)), idx, 4, pad=1)
    assert dw[0, 0, 0, 0, 0] == 57.0
    # golden file written by tests/golden/make_golden.py (oracle only) holds the same numbers
    gold = np.loadtxt(os.path.join(GOLDEN, "worked_example_onehot.txt"))
    np.testing.assert_array_equal(gold[:3], yp[0, 0])
    np.testing.assert_array_equal(gold[3:6], idx[0, 0])
    np.testing.assert_array_equal(gold[6:9], dw[0, 0, 0])
    np.testing.assert_array_equal(gold[9:12], dx[0, 0])


# ---------------------------------------------------------------- equivariance / invariance

@pytest.mark.parametrize("R,mode,G", [(4, "exact90", 4), (8, "bilinear", 8), (16, "bilinear", 4), (16, "steerable", 16)])
def test_quarter_turn_equivariance(R, mode, G):
    """Turning the input by 90 deg turns every map and shifts the orientation index by R/4."""
    B = 2 if mode == "steerable" else 1
    x = RNG.integers(0, 16, (1, 2, 6, 6)) / 16.0
    w = RNG.integers(-16, 17, (B, 3, 2, 3, 3)) / 32.0
    Q = R // 4
    y, yp, idx, _ = orc.layer_fwd(x, w, R, None, mode, 1, 1, G)
    xr = np.rot90(x, 1, axes=(-2, -1)).copy()
    y2, yp2, idx2, _ = orc.layer_fwd(xr, w, R, None, mode, 1, 1, G)
    for r in range(R):
        np.testing.assert_allclose(y2[:, :, (r + Q) % R], np.rot90(y[:, :, r], 1, axes=(-2, -1)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(yp2, np.rot90(yp, 1, axes=(-2, -1)), rtol=0, atol=1e-12)


def test_closure_under_quarter_turns():
    for mode in ("bilinear", "steerable"):
        B = 2 if mode == "steerable" else 1
        w = rnd(B, 2, 2, 3, 3)
        wr = orc.expand_bank(w, 16, None, mode)
        for q in range(4):
            for s in range(4):
                assert np.array_equal(wr[q + 4 * s], np.rot90(wr[q], s, axes=(-2, -1)))


# ---------------------------------------------------------------- first-quadrant filters

def test_steerable_rule():
    """Eq. 17 and the quadrant rule: 0 deg is f_y; 90 deg is rot90(f_y), not f_x."""
    w = rnd(2, 2, 3, 3, 3)
    wr = orc.expand_bank(w, 16, None, "steerable")
    np.testing.assert_array_equal(wr[0], w[1])
    np.testing.assert_array_equal(wr[4], np.rot90(w[1], 1, axes=(-2, -1)))
    for q in range(4):
        th = np.deg2rad(22.5 * q)
        np.testing.assert_allclose(wr[q], np.sin(th) * w[0] + np.cos(th) * w[1], rtol=1e-15, atol=1e-15)
    # linearity of the response in (f_x, f_y)
    x = rnd(1, 3, 5, 5)
    y = orc.rotconv_fwd(x, wr, 1, 1)
    yx = orc.rotconv_fwd(x, orc.expand_bank(w[0:1], 1), 1, 1)[:, :, 0]
    yy = orc.rotconv_fwd(x, orc.expand_bank(w[1:2], 1), 1, 1)[:, :, 0]
    for q in range(4):
        th = np.deg2rad(22.5 * q)
        np.testing.assert_allclose(y[:, :, q], np.sin(th) * yx + np.cos(th) * yy, rtol=1e-12, atol=1e-12)


def test_bilinear_rule_against_scipy():
    """The bilinear first-quadrant filter is scipy's order-1 rotation about the grid centre."""
    from scipy import ndimage

    for k in (3, 5):
        w = rnd(1, 1, 1, k, k)
        for phi in (22.5, 45.0, 67.5, 10.0):
            wr = orc.expand_bank(w, 1, [phi], "bilinear")[0, 0, 0]
            ref = ndimage.rotate(w[0, 0, 0], phi, reshape=False, order=1, mode="grid-constant", cval=0.0)
            np.testing.assert_allclose(wr, ref, rtol=1e-12, atol=1e-12)


def test_bilinear_identity_and_partition_of_unity():
    w = rnd(1, 2, 2, 5, 5)
    np.testing.assert_array_equal(orc.expand_bank(w, 1, [0.0], "bilinear")[0], w[0])
    ones = np.ones((1, 1, 1, 5, 5))
    f = orc.expand_bank(ones, 1, [30.0], "bilinear")[0, 0, 0]
    assert np.all(f <= 1.0 + 1e-15) and np.all(f >= 0.0)
    np.testing.assert_allclose(f[1:4, 1:4], 1.0, rtol=0, atol=1e-15)  # all four neighbours inside


# ---------------------------------------------------------------- pooling

def test_pool_is_numpy_max_argmax():
    y = RNG.integers(-3, 4, (2, 3, 8, 4, 5)).astype(np.float64)  # many exact ties
    for G in (8, 4, 2, 1):
        yp, idx = orc.orient_maxpool_fwd(y, G)
        ng = 8 // G
        # group g = orientations g, g+ng, ... ; numpy argmax returns the first maximum
        yg = y.reshape(2, 3, G, ng, 4, 5)
        np.testing.assert_array_equal(yp.reshape(2, 3, ng, 4, 5), yg.max(axis=2))
        j = yg.argmax(axis=2)
        r = j * ng + np.arange(ng).reshape(1, 1, ng, 1, 1)
        np.testing.assert_array_equal(idx.reshape(2, 3, ng, 4, 5), r)
        g = rnd(2, 3 * ng, 4, 5)
        dy = orc.orient_maxpool_bwd(g, idx, 8, G)
        np.testing.assert_array_equal(dy.reshape(2, 3, G, ng, 4, 5).sum(axis=2), g.reshape(2, 3, ng, 4, 5))
        assert np.all((dy != 0).reshape(2, 3, G, ng, 4, 5).sum(axis=2) <= 1)


# ---------------------------------------------------------------- backward

def torch_layer(x, w_rot, stride, pad, G):
    """Library cross-check: conv2d with the materialised bank, view, max over each pool group."""
    R, Cout, Cin, k, _ = w_rot.shape
    bank = w_rot.permute(1, 0, 2, 3, 4).reshape(Cout * R, Cin, k, k)
    y = F.conv2d(x, bank, stride=stride, padding=pad)
    N, _, Ho, Wo = y.shape
    ng = R // G
    return y.view(N, Cout, G, ng, Ho, Wo).max(dim=2).values.reshape(N, Cout * ng, Ho, Wo)


@pytest.mark.parametrize("R,mode,G,stride,pad,k", [
    (4, "exact90", 4, 1, 1, 3), (4, "exact90", 4, 2, 1, 3), (8, "bilinear", 4, 1, 1, 3),
    (16, "bilinear", 16, 1, 1, 3), (16, "steerable", 4, 1, 1, 3), (4, "exact90", 2, 1, 2, 5), (1, "exact90", 1, 1, 0, 3),
])
def test_backward_against_torch_autograd(R, mode, G, stride, pad, k):
    B = 2 if mode == "steerable" else 1
    x = rnd(2, 3, 7, 6)
    w = rnd(B, 2, 3, k, k)
    y, yp, idx, w_rot = orc.layer_fwd(x, w, R, None, mode, stride, pad, G)
    g = rnd(*yp.shape)
    dx, dw = orc.layer_bwd(x, w, g, idx, R, None, mode, stride, pad, G)
    # autograd through the materialised bank gives d/dW^(r); the oracle's own Eq. 14 must agree,
    # and Eq. 16's reduction is checked separately below against the chain rule.
    xt = torch.from_numpy(x).requires_grad_(True)
    wt = torch.from_numpy(w_rot).requires_grad_(True)
    out = torch_layer(xt, wt, stride, pad, G)
    np.testing.assert_allclose(out.detach().numpy(), yp, rtol=1e-12, atol=1e-12)
    out.backward(torch.from_numpy(g))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-10)
    dy = orc.orient_maxpool_bwd(g, idx, R, G)
    dw_rot = orc.rotconv_bwd_weight(x, dy, k, stride, pad)
    np.testing.assert_allclose(dw_rot, wt.grad.numpy(), rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("R,mode", [(4, "exact90"), (16, "bilinear"), (16, "steerable"), (3, "bilinear")])
def test_bank_grad_reduction_is_adjoint_of_expansion(R, mode):
    """Eq. 16: <expand(W), D> == <W, reduce(D)> for arbitrary W, D."""
    B = 2 if mode == "steerable" else 1
    angles = [10.0, 100.0, 300.0] if R == 3 else None
    w = rnd(B, 2, 3, 3, 3)
    d = rnd(R, 2, 3, 3, 3)
    lhs = float((orc.expand_bank(w, R, angles, mode) * d).sum())
    rhs = float((w * orc.reduce_bank_grad(d, angles, mode)).sum())
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_reduce_bank_grad_exact90_is_rot_back():
    d = rnd(4, 2, 2, 3, 3)
    ref = sum(np.rot90(d[r], -r, axes=(-2, -1)) for r in range(4))
    np.testing.assert_allclose(orc.reduce_bank_grad(d)[0], ref, rtol=1e-15, atol=1e-15)


def test_finite_differences_fp64():
    """Central differences of sum(G * pooled output) w.r.t. x and base weights, away from ties."""
    x = rnd(1, 2, 5, 5)
    w = rnd(1, 2, 2, 3, 3)
    R, mode, G = 8, "bilinear", 4
    y, yp, idx, _ = orc.layer_fwd(x, w, R, None, mode, 1, 1, G)
    g = rnd(*yp.shape)
    dx, dw = orc.layer_bwd(x, w, g, idx, R, None, mode, 1, 1, G)
    f = lambda xx, ww: float((orc.layer_fwd(xx, ww, R, None, mode, 1, 1, G)[1] * g).sum())
    eps = 1e-6
    for pos in [(0, 0, 0, 0), (0, 1, 2, 3), (0, 0, 4, 4)]:
        xp, xm = x.copy(), x.copy()
        xp[pos] += eps
        xm[pos] -= eps
        assert abs((f(xp, w) - f(xm, w)) / (2 * eps) - dx[pos]) < 1e-6
    for pos in [(0, 0, 0, 0, 0), (0, 1, 1, 2, 1), (0, 1, 0, 1, 1)]:
        wp, wm = w.copy(), w.copy()
        wp[pos] += eps
        wm[pos] -= eps
        assert abs((f(x, wp) - f(x, wm)) / (2 * eps) - dw[pos]) < 1e-6


def test_adjoint_identities():
    """The unpooled forward is bilinear in (x, w_base): <Y,D> = <x, bwd_data(D)> = <w, bwd_weight(x,D)>."""
    for R, mode, stride, pad in ((4, "exact90", 1, 1), (16, "bilinear", 1, 1), (8, "steerable", 2, 1)):
        B = 2 if mode == "steerable" else 1
        x = rnd(2, 3, 6, 7)
        w = rnd(B, 2, 3, 3, 3)
        wr = orc.expand_bank(w, R, None, mode)
        y = orc.rotconv_fwd(x, wr, stride, pad)
        d = rnd(*y.shape)
        a = float((y * d).sum())
        b = float((x * orc.rotconv_bwd_data(d, wr, 6, 7, stride, pad)).sum())
        c = float((w * orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, d, 3, stride, pad), None, mode)).sum())
        assert abs(a - b) < 1e-10 * max(1, abs(a)) and abs(a - c) < 1e-10 * max(1, abs(a))


def test_one_hot_delta_gives_rotated_back_patch():
    """Eq. 14 + 16: a single unit of Delta at (r,y,x) makes dW the input patch turned back by -r."""
    x = rnd(1, 1, 5, 5)
    for r in range(4):
        d = np.zeros((1, 1, 4, 5, 5))
        d[0, 0, r, 2, 3] = 1.0
        dw = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, d, 3, 1, 1))
        patch = x[0, 0, 1:4, 2:5]
        np.testing.assert_allclose(dw[0, 0, 0], np.rot90(patch, -r), rtol=0, atol=1e-15)


def test_symmetric_filter_all_orientations_equal():
    a, b, c = 0.25, -0.5, 0.125
    w = np.array([[a, b, a], [b, c, b], [a, b, a]]).reshape(1, 1, 1, 3, 3)
    x = RNG.integers(0, 16, (1, 1, 6, 6)) / 16.0
    y, yp, idx, _ = orc.layer_fwd(x, w, 4, pad=1)
    for r in range(1, 4):
        assert np.array_equal(y[:, :, r], y[:, :, 0])
    assert np.all(idx == 0)  # first maximum wins on exact ties


def test_sampled_backward_helpers_match_full():
    x = rnd(2, 3, 6, 5)
    w = rnd(1, 4, 3, 3, 3)
    R, G = 8, 4
    y, yp, idx, wr = orc.layer_fwd(x, w, R, None, "bilinear", 1, 1, G)
    g = rnd(*yp.shape)
    dy = orc.orient_maxpool_bwd(g, idx, R, G)
    dx = orc.rotconv_bwd_data(dy, wr, 6, 5, 1, 1)
    pts = np.array([[0, 0, 0, 0], [1, 2, 5, 4], [0, 1, 3, 2]], dtype=np.int32)
    got = orc.rotconv_bwd_data_at(dy, wr, pts, 6, 5, 1, 1)
    for t, p in enumerate(pts):
        assert got[t] == dx[tuple(p)]
    dwr = orc.rotconv_bwd_weight(x, dy, 3, 1, 1)
    pairs = np.array([[0, 0], [3, 2], [1, 1]], dtype=np.int32)
    got = orc.rotconv_pool_bwd_weight_at(x, g, idx, pairs, R, 3, G, 1, 1)
    for t, (co, ci) in enumerate(pairs):
        np.testing.assert_allclose(got[t], dwr[:, co, ci], rtol=1e-13, atol=1e-13)


def test_sampled_weight_gradient_routes_nothing_for_indices_outside_the_group():
    """Eq. 12's indicator: an idx that names no member of its pool group (255 = the fused ReLU's "no orientation",
    an index >= R, or an index of another group) contributes nothing.  Pinned against the two-step definition
    orient_maxpool_bwd -> rotconv_bwd_weight, whose Delta is built by the plain comparison idx == r, and against the
    same gradient with those positions' upstream gradient set to zero."""
    x = rnd(2, 3, 6, 5)
    w = rnd(1, 4, 3, 3, 3)
    R, G = 8, 4
    ng = R // G
    _, yp, idx, _ = orc.layer_fwd(x, w, R, None, "bilinear", 1, 1, G)
    g = rnd(*yp.shape)
    bad = idx.copy()
    flat = bad.reshape(-1)
    pos = RNG.permutation(flat.size)[: flat.size // 2]
    third = len(pos) // 3
    flat[pos[:third]] = 255                                   # no orientation at all
    flat[pos[third:2 * third]] = R + 3                        # beyond the orientation set
    chan_grp = (np.arange(yp.shape[1]) % ng).reshape(1, -1, 1, 1) * np.ones(idx.shape, dtype=np.int64)
    wrong = (idx.astype(np.int64) + 1) % R                    # a valid orientation, but of the other group
    assert np.all(wrong % ng != chan_grp)
    flat[pos[2 * third:]] = wrong.reshape(-1)[pos[2 * third:]]
    routed = np.zeros(idx.shape, dtype=bool)
    routed.reshape(-1)[pos] = True
    assert np.all((bad[routed] >= R) | (bad[routed] % ng != chan_grp[routed]))
    pairs = np.array([[0, 0], [3, 2], [1, 1], [2, 0]], dtype=np.int32)
    got = orc.rotconv_pool_bwd_weight_at(x, g, bad, pairs, R, 3, G, 1, 1)
    dwr = orc.rotconv_bwd_weight(x, orc.orient_maxpool_bwd(g, bad, R, G), 3, 1, 1)
    g0 = np.where(routed, 0.0, g)
    dwr0 = orc.rotconv_bwd_weight(x, orc.orient_maxpool_bwd(g0, idx, R, G), 3, 1, 1)
    for t, (co, ci) in enumerate(pairs):
        np.testing.assert_allclose(got[t], dwr[:, co, ci], rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(got[t], dwr0[:, co, ci], rtol=1e-13, atol=1e-13)
    # and the branch matters: with the valid idx the result is a different one
    full = orc.rotconv_pool_bwd_weight_at(x, g, idx, pairs, R, 3, G, 1, 1)
    assert np.abs(full - got).max() > 1e-3


# ---------------------------------------------------------------- average orientation pooling (Eq. 9, Eq. 11)

@pytest.mark.parametrize("R,mode,G,stride,pad,k", [
    (4, "exact90", 4, 1, 1, 3), (8, "bilinear", 4, 1, 1, 3), (16, "steerable", 16, 1, 1, 3), (4, "exact90", 2, 2, 2, 5),
])
def test_average_pooling_against_numpy_torch_and_linearity(R, mode, G, stride, pad, k):
    B = 2 if mode == "steerable" else 1
    x = rnd(2, 3, 7, 6)
    w = rnd(B, 2, 3, k, k)
    y, yp, w_rot = orc.layer_fwd_avg(x, w, R, None, mode, stride, pad, G)
    N, Cout, _, Ho, Wo = y.shape
    ng = R // G
    # the library definition: numpy mean over the members of each group (r = j*ng + g)
    np.testing.assert_allclose(yp, y.reshape(N, Cout, G, ng, Ho, Wo).mean(axis=2).reshape(yp.shape), rtol=1e-13, atol=1e-13)
    # linearity (Sec. IV-B: every product is divided by the number of rotations before it is added): the mean over
    # a group is ONE plain convolution with the group-averaged bank
    wavg = w_rot.reshape(G, ng, Cout, 3, k, k).mean(axis=0).transpose(1, 0, 2, 3, 4).reshape(Cout * ng, 3, k, k)
    ref = F.conv2d(torch.from_numpy(x), torch.from_numpy(np.ascontiguousarray(wavg)), stride=stride, padding=pad).numpy()
    np.testing.assert_allclose(yp, ref, rtol=1e-11, atol=1e-11)
    # gradients: torch autograd through conv2d -> view -> mean
    g = rnd(*yp.shape)
    dx, dw = orc.layer_bwd_avg(x, w, g, R, None, mode, stride, pad, G)
    dy = orc.orient_avgpool_bwd(g, R, G)
    np.testing.assert_allclose(dy.reshape(N, Cout, G, ng, Ho, Wo).sum(axis=2).reshape(g.shape), g, rtol=1e-13, atol=1e-13)
    xt = torch.from_numpy(x).requires_grad_(True)
    wt = torch.from_numpy(w_rot).requires_grad_(True)
    bank = wt.permute(1, 0, 2, 3, 4).reshape(Cout * R, 3, k, k)
    out = F.conv2d(xt, bank, stride=stride, padding=pad).view(N, Cout, G, ng, Ho, Wo).mean(dim=2).reshape(yp.shape)
    out.backward(torch.from_numpy(g))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(orc.rotconv_bwd_weight(x, dy, k, stride, pad), wt.grad.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dw, orc.reduce_bank_grad(wt.grad.numpy(), None, mode), rtol=1e-10, atol=1e-10)


def test_average_equals_max_for_a_fourfold_symmetric_filter():
    """W = rot90(W): all orientations respond alike, so mean and max coincide, and so do the gradients' sums."""
    a = rnd(1, 2, 3, 3, 3)
    w = sum(np.rot90(a, s, axes=(-2, -1)) for s in range(4))
    x = rnd(1, 3, 6, 6)
    _, yp_max, _, _ = orc.layer_fwd(x, w, 4, None, "exact90", 1, 1, 4)
    _, yp_avg, _ = orc.layer_fwd_avg(x, w, 4, None, "exact90", 1, 1, 4)
    np.testing.assert_allclose(yp_avg, yp_max, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- steerable regularisers (Eq. 19, Eq. 20)

def test_steerable_regularisers_closed_forms():
    v = rnd(5, 3, 3)
    u = rnd(5, 3, 3)
    u -= (u * v).sum() / (v * v).sum() * v                      # u orthogonal to v
    # filter 0: parallel bases of norms 2|v| and 3|v|; filter 1: orthogonal bases of equal norm
    un = u * np.sqrt((v * v).sum() / (u * u).sum())
    w = np.stack([np.stack([2 * v, v]), np.stack([3 * v, un])])  # [2 (x,y), B = 2, 5, 3, 3]
    nv = np.sqrt((v * v).sum())
    l_mag, l_orth, _, _ = orc.steerable_reg(w, eps=0.0)
    assert np.isclose(l_mag, 0.5 * (nv ** 2 + 0.0), rtol=1e-12)  # (2|v| - 3|v|)^2 / 2 + 0
    assert np.isclose(l_orth, 0.5 * (1.0 + 0.0), rtol=1e-12)     # cos^2 = 1 for the parallel pair, 0 for the other
    # homogeneity: L_mag is of degree 2, L_orth (eps = 0) of degree 0 in w
    w2 = rnd(2, 4, 3, 3, 3)
    a = orc.steerable_reg(w2, 0.0)
    b = orc.steerable_reg(3.0 * w2, 0.0)
    assert np.isclose(b[0], 9.0 * a[0], rtol=1e-12) and np.isclose(b[1], a[1], rtol=1e-12)
    # Euler: <w, dL_mag> = 2 L_mag, <w, dL_orth> = 0
    assert np.isclose((w2 * a[2]).sum(), 2.0 * a[0], rtol=1e-11) and abs((w2 * a[3]).sum()) < 1e-12


def test_steerable_regulariser_gradients_autograd_and_finite_differences():
    w = rnd(2, 3, 2, 3, 3)
    eps = 1e-3
    l_mag, l_orth, g_mag, g_orth = orc.steerable_reg(w, eps)
    wt = torch.from_numpy(w).requires_grad_(True)
    wx, wy = wt[0].reshape(3, -1), wt[1].reshape(3, -1)
    nx, ny = torch.linalg.vector_norm(wx, dim=1), torch.linalg.vector_norm(wy, dim=1)
    tm = ((nx - ny) ** 2).mean()
    to = (((wx * wy).sum(dim=1) / (nx * ny + eps)) ** 2).mean()
    assert np.isclose(l_mag, tm.item(), rtol=1e-12) and np.isclose(l_orth, to.item(), rtol=1e-12)
    gm, = torch.autograd.grad(tm, wt, retain_graph=True)
    go, = torch.autograd.grad(to, wt)
    np.testing.assert_allclose(g_mag, gm.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g_orth, go.numpy(), rtol=1e-10, atol=1e-12)
    h = 1e-6
    for _ in range(6):
        i = tuple(RNG.integers(0, s) for s in w.shape)
        wp, wm = w.copy(), w.copy()
        wp[i] += h; wm[i] -= h
        fp, fm = orc.steerable_reg(wp, eps), orc.steerable_reg(wm, eps)
        assert np.isclose((fp[0] - fm[0]) / (2 * h), g_mag[i], rtol=1e-5, atol=1e-8)
        assert np.isclose((fp[1] - fm[1]) / (2 * h), g_orth[i], rtol=1e-5, atol=1e-8)


# ---------------------------------------------------------------- p4m: rotations and reflection (Sec. II, Sec. III-B)

def test_p4m_bank_is_numpy_rot90_of_the_filter_and_of_its_mirror_image():
    for k in (2, 3, 5):
        w = rnd(1, 2, 3, k, k)
        for R in (2, 4, 8):
            half = R // 2
            wr = orc.expand_bank(w, R, None, "p4m")
            for a in range(half):
                s = a * (4 // half)
                assert np.array_equal(wr[a], np.rot90(w[0], s, axes=(-2, -1)))
                assert np.array_equal(wr[half + a], np.rot90(np.flip(w[0], axis=-1), s, axes=(-2, -1)))
    # the eight filters are closed under mirroring: flip(rot^s W) = rot^-s(flip W)
    wr = orc.expand_bank(rnd(1, 1, 1, 3, 3), 8, None, "p4m")
    for s in range(4):
        assert np.array_equal(np.flip(wr[s], axis=-1), wr[4 + (4 - s) % 4])


def test_p4m_pooled_output_is_invariant_to_mirroring_and_quarter_turns():
    x = rnd(1, 2, 6, 6)
    w = rnd(1, 3, 2, 3, 3)
    y, yp, idx, _ = orc.layer_fwd(x, w, 8, None, "p4m", 1, 1, 8)
    ym, ypm, _, _ = orc.layer_fwd(np.flip(x, axis=-1), w, 8, None, "p4m", 1, 1, 8)
    np.testing.assert_allclose(ypm, np.flip(yp, axis=-1), rtol=1e-12, atol=1e-12)
    for s in range(4):      # Y_s(flip X) = flip(Y_{4 + (-s mod 4)}(X))
        np.testing.assert_allclose(ym[:, :, s], np.flip(y[:, :, 4 + (4 - s) % 4], axis=-1), rtol=1e-12, atol=1e-12)
    _, ypr, _, _ = orc.layer_fwd(np.rot90(x, 1, axes=(-2, -1)), w, 8, None, "p4m", 1, 1, 8)
    np.testing.assert_allclose(ypr, np.rot90(yp, 1, axes=(-2, -1)), rtol=1e-12, atol=1e-12)


def test_p4m_gradient_reduction_is_the_adjoint_of_the_expansion():
    w, d = rnd(1, 2, 3, 3, 3), rnd(8, 2, 3, 3, 3)
    lhs = (orc.expand_bank(w, 8, None, "p4m") * d).sum()
    rhs = (w * orc.reduce_bank_grad(d, None, "p4m")).sum()
    assert np.isclose(lhs, rhs, rtol=1e-12)
