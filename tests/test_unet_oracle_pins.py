"""Pins of the glue oracle (oracle/unet_oracle.py) against definitions written out as loops,
closed forms and finite differences -- none of them re-calls the library routine the oracle uses."""
import numpy as np
import pytest

from oracle import unet_oracle as uo

RNG = np.random.default_rng(11)


def test_relu():
    x = np.array([-2.0, -0.0, 0.0, 0.5, 3.0])
    y = uo.relu_fwd(x)
    assert np.array_equal(y, [0, 0, 0, 0.5, 3.0])
    assert np.array_equal(uo.relu_bwd(y, np.ones(5)), [0, 0, 0, 1, 1])


def test_maxpool2_loops_and_ties():
    x = RNG.integers(-3, 4, size=(2, 3, 6, 4)).astype(np.float64)   # small integers: many ties
    y, idx = uo.maxpool2_fwd(x)
    for n in range(2):
        for c in range(3):
            for i in range(3):
                for j in range(2):
                    win = [x[n, c, 2 * i + a, 2 * j + b] for a in range(2) for b in range(2)]
                    best = 0
                    for t in range(1, 4):
                        if win[t] > win[best]:
                            best = t
                    assert y[n, c, i, j] == win[best] and idx[n, c, i, j] == best
    dy = RNG.standard_normal(y.shape)
    dx = uo.maxpool2_bwd(dy, idx, 6, 4)
    assert dx.shape == x.shape and np.count_nonzero(dx) <= dy.size
    for n in range(2):
        for c in range(3):
            for i in range(3):
                for j in range(2):
                    a, b = divmod(int(idx[n, c, i, j]), 2)
                    assert dx[n, c, 2 * i + a, 2 * j + b] == dy[n, c, i, j]
    assert np.isclose(dx.sum(), dy.sum())


def _upconv_loops(x, w):
    N, Ci, H, W = x.shape
    Co = w.shape[1]
    y = np.zeros((N, Co, 2 * H, 2 * W))
    for n in range(N):
        for co in range(Co):
            for h in range(H):
                for ww in range(W):
                    for a in range(2):
                        for b in range(2):
                            s = 0.0
                            for ci in range(Ci):
                                s += x[n, ci, h, ww] * w[ci, co, a, b]
                            y[n, co, 2 * h + a, 2 * ww + b] = s
    return y


def test_upconv2_definition_and_adjoint():
    x = RNG.standard_normal((2, 3, 3, 2))
    w = RNG.standard_normal((3, 2, 2, 2))
    y = uo.upconv2_fwd(x, w)
    np.testing.assert_allclose(y, _upconv_loops(x, w), rtol=1e-13, atol=1e-13)
    dy = RNG.standard_normal(y.shape)
    dx, dw = uo.upconv2_bwd(x, w, dy)
    # the layer is bilinear in (x, w): <dy, f(x', w)> = <dx, x'> and <dy, f(x, w')> = <dw, w'>
    x2, w2 = RNG.standard_normal(x.shape), RNG.standard_normal(w.shape)
    assert np.isclose((dy * _upconv_loops(x2, w)).sum(), (dx * x2).sum(), rtol=1e-12)
    assert np.isclose((dy * _upconv_loops(x, w2)).sum(), (dw * w2).sum(), rtol=1e-12)


def test_conv1x1_definition_and_adjoint():
    x = RNG.standard_normal((2, 5, 3, 4))
    w = RNG.standard_normal((3, 5))
    y = uo.conv1x1_fwd(x, w)
    np.testing.assert_allclose(y, np.einsum("oc,nchw->nohw", w, x), rtol=1e-13, atol=1e-13)
    dy = RNG.standard_normal(y.shape)
    dx, dw = uo.conv1x1_bwd(x, w, dy)
    np.testing.assert_allclose(dx, np.einsum("oc,nohw->nchw", w, dy), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dw, np.einsum("nohw,nchw->oc", dy, x), rtol=1e-12, atol=1e-13)


def test_softmax_ce_closed_forms_and_finite_difference():
    # uniform logits: loss = ln K; gradient (1/K - onehot)/M
    K, M = 5, 6
    lab = RNG.integers(0, K, size=(1, 2, 3))
    loss, dl = uo.softmax_ce(np.zeros((1, K, 2, 3)), lab)
    assert np.isclose(loss, np.log(K))
    onehot = np.moveaxis(np.eye(K)[lab], -1, 1)
    np.testing.assert_allclose(dl, (1.0 / K - onehot) / M, atol=1e-15)
    # written out: mean over pixels of -log softmax[label]
    lg = RNG.standard_normal((2, K, 2, 3)) * 3
    lab = RNG.integers(0, K, size=(2, 2, 3))
    loss, dl = uo.softmax_ce(lg, lab)
    tot = 0.0
    for n in range(2):
        for i in range(2):
            for j in range(3):
                z = lg[n, :, i, j]
                tot += np.log(np.exp(z).sum()) - z[lab[n, i, j]]
    assert np.isclose(loss, tot / 12, rtol=1e-13)
    assert np.allclose(dl.sum(axis=1), 0, atol=1e-15)
    # central finite differences of the loss on a few logits
    for _ in range(6):
        pos = tuple(int(RNG.integers(0, s)) for s in lg.shape)
        e = np.zeros_like(lg)
        e[pos] = 1e-6
        fd = (uo.softmax_ce(lg + e, lab)[0] - uo.softmax_ce(lg - e, lab)[0]) / 2e-6
        assert np.isclose(fd, dl[pos], rtol=1e-6, atol=1e-9)


def _tiny_params(depth, widths, cin, K, rng):
    params, c = {}, cin
    for lvl in range(depth):
        params[f"enc{lvl}a"] = rng.standard_normal((1, widths[lvl], c, 3, 3)) * (2.0 / (9 * c)) ** 0.5
        params[f"enc{lvl}b"] = rng.standard_normal((1, widths[lvl], widths[lvl], 3, 3)) * (2.0 / (9 * widths[lvl])) ** 0.5
        c = widths[lvl]
    wb = widths[depth]
    params["bota"] = rng.standard_normal((1, wb, c, 3, 3)) * (2.0 / (9 * c)) ** 0.5
    params["botb"] = rng.standard_normal((1, wb, wb, 3, 3)) * (2.0 / (9 * wb)) ** 0.5
    c = wb
    for lvl in reversed(range(depth)):
        wl = widths[lvl]
        params[f"up{lvl}"] = rng.standard_normal((c, wl, 2, 2)) * (1.0 / c) ** 0.5
        params[f"dec{lvl}a"] = rng.standard_normal((1, wl, 2 * wl, 3, 3)) * (2.0 / (18 * wl)) ** 0.5
        params[f"dec{lvl}b"] = rng.standard_normal((1, wl, wl, 3, 3)) * (2.0 / (9 * wl)) ** 0.5
        c = wl
    params["head"] = rng.standard_normal((K, c)) * (1.0 / c) ** 0.5
    return params


def test_unet_step_gradients_by_finite_differences():
    """The whole stack's backward pass against central differences of its own forward loss: pins the
    wiring of the tape (skip gradients, split order, pooling routes).  The loss is piecewise smooth
    (max-pools, ReLU); the probe is small enough that a kink is crossed only by accident, so the check
    takes the median agreement over several directions."""
    rng = np.random.default_rng(5)
    depth, widths, K = 2, [3, 4, 5], 3
    params = _tiny_params(depth, widths, 2, K, rng)
    images = rng.standard_normal((1, 2, 8, 8))
    labels = rng.integers(0, K, size=(1, 8, 8))
    loss, grads, acts = uo.unet_step(images, labels, params, R=4, mode="exact90")
    assert set(grads) == set(params)
    assert acts["head"]["y"].shape == (1, K, 8, 8)
    errs = []
    for name in ("enc0a", "enc1b", "bota", "up1", "dec0a", "dec1b", "up0", "head"):
        d = rng.standard_normal(params[name].shape)
        h = 1e-6
        pp = dict(params); pp[name] = params[name] + h * d
        pm = dict(params); pm[name] = params[name] - h * d
        fd = (uo.unet_step(images, labels, pp)[0] - uo.unet_step(images, labels, pm)[0]) / (2 * h)
        an = float((grads[name] * d).sum())
        errs.append(abs(fd - an) / max(abs(an), 1e-12))
    assert np.median(errs) < 1e-6 and max(errs) < 1e-3, errs


def test_unet_step_r16_runs_and_pools_all_orientations():
    rng = np.random.default_rng(6)
    params = _tiny_params(1, [2, 3], 2, 2, rng)
    images = rng.standard_normal((1, 2, 4, 4))
    labels = rng.integers(0, 2, size=(1, 4, 4))
    loss, grads, acts = uo.unet_step(images, labels, params, R=16, mode="bilinear", pool_group=16)
    assert np.isfinite(loss) and acts["enc0a"]["idx"].max() < 16 and acts["enc0a"]["ypool"].shape == (1, 2, 4, 4)
