"""One training step (forward + backward) of the UNet-shaped stack of rotation-convolution
layers (paper Sec. V-A, Fig. 9, with both convolutions of a block rotation-invariant), run
entirely through the C-ABI library: this module only owns the device buffers (torch tensors as
plain memory), the per-layer plans and the order of the calls.

    Block(a->b) = rotconv_pool(a->b) + ReLU, rotconv_pool(b->b) + ReLU        (3x3, pad 1)
    encoder: Block, 2x2 max-pool per level; bottleneck Block; decoder per level: 2x2 stride-2
    transposed convolution, concat [skip, up], Block; 1x1 head; mean soft-max cross-entropy.

No arithmetic happens here and nothing falls back to torch ops.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

from . import binding as rc
from . import synth


@dataclass(frozen=True)
class UNetConfig:
    name: str
    N: int
    Cin: int
    H: int
    W: int
    widths: Tuple[int, ...]          # encoder widths ..., last = bottleneck
    classes: int
    R: int = 4
    mode: str = "exact90"
    pool_group: Optional[int] = None  # None = pool over all R orientations
    seed: int = 2024
    # "rot_rot": both convolutions of a block rotation-invariant, pooled over pool_group (the benchmark's
    # stack).  "rot_std": the paper's own block (Sec. V-A): the first convolution rotation-invariant with
    # pooling over the 4 quarter turns of each first-quadrant angle (R/4 features per filter, so
    # width / (R/4) filters), the second a standard convolution (R = 1 through the same library).
    block: str = "rot_rot"

    @property
    def depth(self):
        return len(self.widths) - 1

    @property
    def B(self):
        return 2 if self.mode == "steerable" else 1


C4 = UNetConfig("C4", 4, 3, 512, 512, (64, 128, 256, 512, 1024), 6, R=4, mode="exact90", seed=404)
C5 = UNetConfig("C5", 2, 3, 512, 512, (64, 128, 256, 512, 1024), 6, R=16, mode="bilinear", pool_group=16, seed=505)
# the paper's own block (rotation convolution, then a standard one) at 4, 8 and 16 orientations
P4 = UNetConfig("P4", 4, 3, 512, 512, (64, 128, 256, 512, 1024), 6, R=4, mode="exact90", block="rot_std", seed=604)
P8 = UNetConfig("P8", 4, 3, 512, 512, (64, 128, 256, 512, 1024), 6, R=8, mode="bilinear", block="rot_std", seed=608)
P16 = UNetConfig("P16", 4, 3, 512, 512, (64, 128, 256, 512, 1024), 6, R=16, mode="bilinear", block="rot_std", seed=616)
UNET_CONFIGS = {"C4": C4, "C5": C5, "P4": P4, "P8": P8, "P16": P16}


def rot_layers(cfg: UNetConfig):
    """(name, Cin, Cout, H, W) of every rotation-convolution layer in forward order."""
    out, c, h, w = [], cfg.Cin, cfg.H, cfg.W
    for lvl in range(cfg.depth):
        out += [(f"enc{lvl}a", c, cfg.widths[lvl], h, w), (f"enc{lvl}b", cfg.widths[lvl], cfg.widths[lvl], h, w)]
        c, h, w = cfg.widths[lvl], h // 2, w // 2
    wb = cfg.widths[-1]
    out += [("bota", c, wb, h, w), ("botb", wb, wb, h, w)]
    for lvl in reversed(range(cfg.depth)):
        h, w = 2 * h, 2 * w
        wl = cfg.widths[lvl]
        out += [(f"dec{lvl}a", 2 * wl, wl, h, w), (f"dec{lvl}b", wl, wl, h, w)]
    return out


def layer_specs(cfg: UNetConfig):
    """Per rotation-convolution layer in forward order: dict(name, Cin, Cout (base filters), H, W, R, mode,
    pool_group, B (base banks), width (pooled output channels))."""
    out = []
    for name, ci, width, h, w in rot_layers(cfg):
        if cfg.block == "rot_std":
            if name.endswith("a"):
                per = max(1, cfg.R // 4)
                if width % per:
                    raise ValueError("layer width must be divisible by R/4 in the rot_std block")
                spec = dict(R=cfg.R, mode=cfg.mode, pool_group=min(4, cfg.R), Cout=width // per)
            else:
                spec = dict(R=1, mode="exact90", pool_group=None, Cout=width)
        else:
            spec = dict(R=cfg.R, mode=cfg.mode, pool_group=cfg.pool_group, Cout=width)
        spec.update(name=name, Cin=ci, H=h, W=w, width=width, B=2 if spec["mode"] == "steerable" else 1)
        out.append(spec)
    return out


def oracle_layer_spec(cfg: UNetConfig):
    """name -> (R, mode, pool_group) in the form the stack oracle takes."""
    return {sp["name"]: (sp["R"], sp["mode"], sp["pool_group"]) for sp in layer_specs(cfg)}


def param_shapes(cfg: UNetConfig) -> Dict[str, Tuple[int, ...]]:
    shapes = {sp["name"]: (sp["B"], sp["Cout"], sp["Cin"], 3, 3) for sp in layer_specs(cfg)}
    for lvl in range(cfg.depth):
        shapes[f"up{lvl}"] = (cfg.widths[lvl + 1], cfg.widths[lvl], 2, 2)
    shapes["head"] = (cfg.classes, cfg.widths[0])
    return shapes


def make_params(cfg: UNetConfig) -> Dict[str, np.ndarray]:
    """He-normal parameters sqrt(2 / fan_in) from the counter-based generator (fp32 values)."""
    out = {}
    for i, (name, shp) in enumerate(sorted(param_shapes(cfg).items())):
        fan_in = shp[1] if name == "head" else shp[0] if name.startswith("up") else shp[2] * 9
        n = int(np.prod(shp))
        v = synth.normal01(cfg.seed * 1000 + i, n) * np.sqrt(2.0 / fan_in)
        out[name] = v.astype(np.float32).reshape(shp)
    return out


def make_batch(cfg: UNetConfig):
    """images uniform [0,1) fp32 [N,Cin,H,W]; labels uniform ints int32 [N,H,W]."""
    n = cfg.N * cfg.Cin * cfg.H * cfg.W
    images = synth.uniform01(cfg.seed * 1000 + 900, n).astype(np.float32).reshape(cfg.N, cfg.Cin, cfg.H, cfg.W)
    labels = synth.randint(cfg.seed * 1000 + 901, cfg.N * cfg.H * cfg.W, 0, cfg.classes - 1).astype(np.int32)
    return images, labels.reshape(cfg.N, cfg.H, cfg.W)


class UNet:
    """Device state of the stack: plans, parameters, activations, gradients, one shared workspace."""

    def __init__(self, cfg: UNetConfig, params: Optional[Dict[str, np.ndarray]] = None, device="cuda",
                 dtype: str = "f32", fuse_relu: bool = True):
        """dtype "f32": everything fp32.  "bf16": images, parameters, activations and activation gradients
        are stored as bfloat16 (parameters rounded once when loaded), every call accumulates in fp32, and the
        parameter gradients and the loss are fp32.
        fuse_relu: the ReLU after every rotation convolution is the plan's fused activation (the forward writes
        max(pooled, 0) and marks dead elements in idx, so the gradient calls need no ReLU pass); False runs the
        separate glue_relu_fwd / glue_relu_bwd calls instead (same values)."""
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("the UNet-shaped step runs on the GPU only")
        rc.lib()  # fails loudly when the library is not built
        self.cfg, self.dev, self.torch = cfg, device, torch
        if dtype not in ("f32", "bf16"):
            raise ValueError("dtype must be 'f32' or 'bf16'")
        self.dtype = dtype
        self.fuse_relu = bool(fuse_relu)
        f32, u8 = torch.float32, torch.uint8
        adt = torch.bfloat16 if dtype == "bf16" else f32      # storage type of activations and parameters
        self.adt = adt
        N = cfg.N
        if cfg.H % (1 << cfg.depth) or cfg.W % (1 << cfg.depth):
            raise ValueError("H and W must be divisible by 2**depth")

        def buf(*shape, dtype=adt):
            return torch.empty(shape, dtype=dtype, device=device)

        self.layers = rot_layers(cfg)         # (name, Cin, width, H, W)
        self.specs = layer_specs(cfg)
        self.plans: Dict[str, rc.Plan] = {}
        self.act: Dict[str, Dict[str, "torch.Tensor"]] = {}
        ws_bytes = 256
        for sp in self.specs:
            name, h, w = sp["name"], sp["H"], sp["W"]
            p = rc.Plan(N, sp["Cin"], h, w, sp["Cout"], k=3, R=sp["R"], mode=sp["mode"], stride=1, pad=1,
                        pool_group=sp["pool_group"] or 0, dtype=rc.BF16 if dtype == "bf16" else rc.F32,
                        relu=self.fuse_relu)
            self.plans[name] = p
            ws_bytes = max(ws_bytes, p.workspace_bytes)
            self.act[name] = dict(y=buf(N, p.Cpooled, h, w), idx=buf(N, p.Cpooled, h, w, dtype=u8),
                                  g=buf(N, p.Cpooled, h, w))
            if p.Cpooled != sp["width"]:
                raise ValueError(f"{name}: pooled channel count {p.Cpooled} differs from the layer width {sp['width']}")
        h, w = cfg.H, cfg.W
        for lvl in range(cfg.depth):
            c = cfg.widths[lvl]
            self.act[f"pool{lvl}"] = dict(y=buf(N, c, h // 2, w // 2), idx=buf(N, c, h // 2, w // 2, dtype=u8),
                                          g=buf(N, c, h // 2, w // 2))
            cu = cfg.widths[lvl + 1]
            self.act[f"up{lvl}"] = dict(y=buf(N, c, h, w), cat=buf(N, 2 * c, h, w), gcat=buf(N, 2 * c, h, w),
                                        g=buf(N, c, h, w))
            ws_bytes = max(ws_bytes, rc.glue_upconv2_workspace_bytes(N, cu, c, h // 2, w // 2))
            h, w = h // 2, w // 2
        P = cfg.H * cfg.W
        self.act["head"] = dict(y=buf(N, cfg.classes, cfg.H, cfg.W), g=buf(N, cfg.classes, cfg.H, cfg.W))
        ws_bytes = max(ws_bytes, rc.glue_conv1x1_workspace_bytes(N, cfg.widths[0], cfg.classes, P), N * P * 4)
        self.ws = torch.empty(ws_bytes, dtype=u8, device=device)
        self.loss = buf(1, dtype=f32)
        self.trace = None         # a list turns on per-call event timing
        self._where = ""
        self.images = buf(N, cfg.Cin, cfg.H, cfg.W)
        self.labels = buf(N, cfg.H, cfg.W, dtype=torch.int32)
        self.params = {n: buf(*s) for n, s in param_shapes(cfg).items()}
        self.grads = {n: buf(*s, dtype=f32) for n, s in param_shapes(cfg).items()}
        if params is not None:
            self.load_params(params)

    def rot_flops(self):
        """(algorithmic, dense-equivalent) flops of one step's rotation convolutions: three passes per
        layer (Eq. 8 shared products over Q banks plus one add per tap and orientation), no input
        gradient for the first layer."""
        cfg = self.cfg
        alg = dense = 0.0
        for i, sp in enumerate(self.specs):
            Q = self.plans[sp["name"]].orientations()[0]
            P = cfg.N * sp["H"] * sp["W"]
            passes = 2 if i == 0 else 3
            alg += passes * (2.0 * P * sp["Cin"] * sp["Cout"] * 9 * Q * sp["B"] + P * sp["Cout"] * 9 * sp["R"])
            dense += passes * 2.0 * P * sp["Cin"] * sp["Cout"] * 9 * sp["R"]
        return alg, dense

    # ---- host <-> device plumbing -------------------------------------------------------------
    def load_params(self, params):
        for n, t in self.params.items():
            t.copy_(self.torch.from_numpy(np.ascontiguousarray(params[n], dtype=np.float32)))   # rounds if bf16

    def load_batch(self, images, labels):
        self.images.copy_(self.torch.from_numpy(np.ascontiguousarray(images, dtype=np.float32)))
        self.labels.copy_(self.torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)))

    # ---- the step -----------------------------------------------------------------------------
    def _c(self, what, fn, *args, **kw):
        """Issue one library call; with self.trace a list, bracket it with events on the current stream
        and record (call name, layer it belongs to, start, end)."""
        if self.trace is None:
            fn(*args, **kw)
            return
        ev = self.torch.cuda.Event
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        e0.record()
        fn(*args, **kw)
        e1.record()
        self.trace.append((what, self._where, e0, e1))

    def _rot_fwd(self, name, x):
        self._where = name
        a = self.act[name]
        a["x"] = x
        self._c("rotconv_pool_fwd", rc.rotconv_pool_fwd, self.plans[name], x, self.params[name], a["y"], a["idx"],
                self.ws)
        if not self.fuse_relu:
            self._c("glue_relu_fwd", rc.glue_relu_fwd, a["y"], a["y"])
        return a["y"]

    def _rot_bwd(self, name, need_dx=True):
        """a['g'] holds dL/d(ReLU output); returns nothing: dL/dx lands in the producer's 'g' slot."""
        self._where = name
        a = self.act[name]
        if not self.fuse_relu:      # fused: idx = 255 at dead elements already keeps their gradient out
            self._c("glue_relu_bwd", rc.glue_relu_bwd, a["y"], a["g"], a["g"])
        self._c("rotconv_pool_bwd_weight", rc.rotconv_pool_bwd_weight, self.plans[name], a["x"], a["g"], a["idx"],
                self.grads[name], self.ws)
        if need_dx:
            self._c("rotconv_pool_bwd_data", rc.rotconv_pool_bwd_data, self.plans[name], a["g"], a["idx"],
                    self.params[name], a["gx"], self.ws)

    def forward(self):
        cfg, act = self.cfg, self.act
        x = self.images
        for lvl in range(cfg.depth):
            x = self._rot_fwd(f"enc{lvl}a", x)
            x = self._rot_fwd(f"enc{lvl}b", x)
            p = act[f"pool{lvl}"]
            self._where = f"pool{lvl}"
            self._c("glue_maxpool2_fwd", rc.glue_maxpool2_fwd, x, p["y"], p["idx"])
            x = p["y"]
        x = self._rot_fwd("bota", x)
        x = self._rot_fwd("botb", x)
        for lvl in reversed(range(cfg.depth)):
            u = act[f"up{lvl}"]
            u["x"] = x
            self._where = f"up{lvl}"
            self._c("glue_upconv2_fwd", rc.glue_upconv2_fwd, x, self.params[f"up{lvl}"], u["y"])
            self._c("glue_concat2", rc.glue_concat2, act[f"enc{lvl}b"]["y"], u["y"], u["cat"])
            x = self._rot_fwd(f"dec{lvl}a", u["cat"])
            x = self._rot_fwd(f"dec{lvl}b", x)
        hd = act["head"]
        hd["x"] = x
        self._where = "head"
        self._c("glue_conv1x1_fwd", rc.glue_conv1x1_fwd, x, self.params["head"], hd["y"])
        self._c("glue_softmax_ce", rc.glue_softmax_ce, hd["y"], self.labels, self.loss, hd["g"], self.ws)
        return self.loss

    def backward(self):
        cfg, act = self.cfg, self.act
        hd = act["head"]
        self._where = "head"
        self._c("glue_conv1x1_bwd_weight", rc.glue_conv1x1_bwd_weight, hd["x"], hd["g"], self.grads["head"], self.ws)
        self._c("glue_conv1x1_bwd_data", rc.glue_conv1x1_bwd_data, hd["g"], self.params["head"], act["dec0b"]["g"])
        for lvl in range(cfg.depth):
            u = act[f"up{lvl}"]
            act[f"dec{lvl}b"]["gx"] = act[f"dec{lvl}a"]["g"]
            self._rot_bwd(f"dec{lvl}b")
            act[f"dec{lvl}a"]["gx"] = u["gcat"]
            self._rot_bwd(f"dec{lvl}a")
            # gradient of the concatenation: skip half into the encoder output's slot, up half on
            self._where = f"up{lvl}"
            self._c("glue_split2", rc.glue_split2, u["gcat"], act[f"enc{lvl}b"]["g"], u["g"], accumulate_a=False)
            below = act["botb"] if lvl == cfg.depth - 1 else act[f"dec{lvl + 1}b"]
            self._c("glue_upconv2_bwd_weight", rc.glue_upconv2_bwd_weight, u["x"], u["g"], self.grads[f"up{lvl}"],
                    self.ws)
            self._c("glue_upconv2_bwd_data", rc.glue_upconv2_bwd_data, u["g"], self.params[f"up{lvl}"], below["g"])
        act["botb"]["gx"] = act["bota"]["g"]
        self._rot_bwd("botb")
        act["bota"]["gx"] = act[f"pool{cfg.depth - 1}"]["g"]
        self._rot_bwd("bota")
        for lvl in reversed(range(cfg.depth)):
            p = act[f"pool{lvl}"]
            # pooled branch adds to the skip gradient already in the slot
            self._where = f"pool{lvl}"
            self._c("glue_maxpool2_bwd", rc.glue_maxpool2_bwd, p["g"], p["idx"], act[f"enc{lvl}b"]["g"],
                    accumulate=True)
            act[f"enc{lvl}b"]["gx"] = act[f"enc{lvl}a"]["g"]
            self._rot_bwd(f"enc{lvl}b")
            if lvl > 0:
                act[f"enc{lvl}a"]["gx"] = act[f"pool{lvl - 1}"]["g"]
                self._rot_bwd(f"enc{lvl}a")
            else:
                self._rot_bwd("enc0a", need_dx=False)

    def step(self):
        self.forward()
        self.backward()
        return self.loss

    def capture(self):
        """Records one step (after at least one eager step: the plans upload their tables on first use) into a HIP
        graph on the current device; `replay()` then runs the whole step with one launch from the host.  Every
        library call enqueues kernels only and every buffer of the step is preallocated, so the recorded step is
        the eager step."""
        assert self.trace is None
        self.step()
        self.torch.cuda.synchronize()
        self._graph = self.torch.cuda.CUDAGraph()
        with self.torch.cuda.graph(self._graph):
            self.step()
        return self._graph

    def replay(self):
        self._graph.replay()
        return self.loss
