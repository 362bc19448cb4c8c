"""CPU oracle of the network glue and of the UNet-shaped training step (fp64).

TEST INFRASTRUCTURE ONLY (tests, smoke, the benchmark's cpu_baseline leg).  The ordinary
layers are plain PyTorch CPU ops in float64 used as library primitives (ReLU, 2x2 max-pool,
2x2 stride-2 transposed convolution, concatenation, 1x1 convolution, mean soft-max
cross-entropy); their gradients come from torch.autograd on those same primitives.  The
rotation-convolution layers are the C oracle (rotconv_oracle).  The stack is the one the
benchmark names (paper Sec. V-A, Fig. 9, with every convolution of a block replaced by the
rotation-invariant one): Block(a->b) = rotconv_pool(a->b)+ReLU, rotconv_pool(b->b)+ReLU;
encoder widths w0..w3 with 2x2 max-pool, bottleneck w4, decoder with transposed-convolution
up-sampling and skip concatenation [skip, up], 1x1 head, mean cross-entropy.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F

from . import rotconv_oracle as orc


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))


# ---- single glue ops -----------------------------------------------------------------------

def relu_fwd(x):
    return np.maximum(np.asarray(x, dtype=np.float64), 0.0)


def relu_bwd(y, dy):
    return np.where(np.asarray(y) > 0, np.asarray(dy, dtype=np.float64), 0.0)


def maxpool2_fwd(x):
    """-> (y, idx) with idx = 2a+b of the first maximum in row-major order of the 2x2 window."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    win = x.reshape(N, C, H // 2, 2, W // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, H // 2, W // 2, 4)
    return win.max(axis=-1), win.argmax(axis=-1).astype(np.uint8)


def maxpool2_bwd(dy, idx, H, W):
    dy = np.asarray(dy, dtype=np.float64)
    N, C, Ho, Wo = dy.shape
    d = np.zeros((N, C, Ho, Wo, 4))
    np.put_along_axis(d, idx[..., None].astype(np.int64), dy[..., None], axis=-1)
    return d.reshape(N, C, Ho, Wo, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, C, H, W)


def upconv2_fwd(x, w):
    return F.conv_transpose2d(_t(x), _t(w), stride=2).numpy()


def upconv2_bwd(x, w, dy):
    xt, wt = _t(x).requires_grad_(True), _t(w).requires_grad_(True)
    y = F.conv_transpose2d(xt, wt, stride=2)
    dx, dw = torch.autograd.grad(y, (xt, wt), _t(dy))
    return dx.numpy(), dw.numpy()


def conv1x1_fwd(x, w):
    return F.conv2d(_t(x), _t(w)[:, :, None, None]).numpy()


def conv1x1_bwd(x, w, dy):
    xt, wt = _t(x).requires_grad_(True), _t(w).requires_grad_(True)
    y = F.conv2d(xt, wt[:, :, None, None])
    dx, dw = torch.autograd.grad(y, (xt, wt), _t(dy))
    return dx.numpy(), dw.numpy()


def softmax_ce(logits, labels):
    """Mean cross-entropy over all pixels -> (loss, dlogits)."""
    lt = _t(logits).requires_grad_(True)
    loss = F.cross_entropy(lt, torch.from_numpy(np.asarray(labels, dtype=np.int64)), reduction="mean")
    (dl,) = torch.autograd.grad(loss, lt)
    return float(loss.detach()), dl.numpy()


# ---- the UNet-shaped stack -------------------------------------------------------------------

def rot_layer_names(depth=4):
    names = []
    for lvl in range(depth):
        names += [f"enc{lvl}a", f"enc{lvl}b"]
    names += ["bota", "botb"]
    for lvl in reversed(range(depth)):
        names += [f"dec{lvl}a", f"dec{lvl}b"]
    return names


def unet_step(images, labels, params, R=4, mode="exact90", pool_group=None, layer_spec=None):
    """One training step (forward + backward) of the stack.  params: dict name -> array
    (rot layers [B,Cout,Cin,3,3], 'up{lvl}' [Cin,Cout,2,2], 'head' [K,C0]).  layer_spec: optional
    dict name -> (R, mode, pool_group) for layers that differ from the common setting (the paper's own
    block, Sec. V-A: rotation convolution followed by a standard convolution, R = 1).
    Returns (loss, grads dict, acts dict of every layer's forward tensors)."""
    layer_spec = layer_spec or {}
    common = (R, mode, pool_group)
    depth = sum(1 for k in params if k.startswith("enc") and k.endswith("a"))
    acts, tape = {}, []

    def rot(name, x):
        w = params[name]
        Rl, model, Gl = layer_spec.get(name, common)
        _, yp, idx, _ = orc.layer_fwd(x, w, Rl, None, model, 1, 1, Gl)
        y = relu_fwd(yp)
        acts[name] = dict(x=x, ypool=yp, idx=idx, y=y)
        tape.append(("rot", name))
        return y

    x = np.asarray(images, dtype=np.float64)
    skips = []
    for lvl in range(depth):
        x = rot(f"enc{lvl}b", rot(f"enc{lvl}a", x))
        skips.append(x)
        p, pidx = maxpool2_fwd(x)
        acts[f"pool{lvl}"] = dict(x=x, y=p, idx=pidx)
        tape.append(("pool", f"pool{lvl}"))
        x = p
    x = rot("botb", rot("bota", x))
    for lvl in reversed(range(depth)):
        up = upconv2_fwd(x, params[f"up{lvl}"])
        cat = np.concatenate([skips[lvl], up], axis=1)
        acts[f"up{lvl}"] = dict(x=x, y=up, cat=cat)
        tape.append(("up", f"up{lvl}"))
        x = rot(f"dec{lvl}b", rot(f"dec{lvl}a", cat))
    logits = conv1x1_fwd(x, params["head"])
    acts["head"] = dict(x=x, y=logits)
    loss, dl = softmax_ce(logits, labels)
    acts["loss"] = dict(dlogits=dl)

    grads = {}
    dx, grads["head"] = conv1x1_bwd(x, params["head"], dl)
    dskip = [None] * depth
    for kind, name in reversed(tape):
        a = acts[name]
        if kind == "rot":
            dyp = relu_bwd(a["y"], dx)
            a["dypool"] = dyp
            Rl, model, Gl = layer_spec.get(name, common)
            dxx, dw = orc.layer_bwd(a["x"], params[name], dyp, a["idx"], Rl, None, model, 1, 1, Gl)
            grads[name] = dw
            dx = dxx
        elif kind == "up":
            lvl = int(name[2:])
            C = a["cat"].shape[1] - a["y"].shape[1]
            dskip[lvl] = dx[:, :C]
            dxx, grads[name] = upconv2_bwd(a["x"], params[name], dx[:, C:])
            dx = dxx
        elif kind == "pool":
            lvl = int(name[4:])
            H, W = a["x"].shape[2:]
            dx = maxpool2_bwd(dx, a["idx"], H, W) + dskip[lvl]
    return loss, grads, acts
