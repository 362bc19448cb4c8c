"""rotconv_pool_fwd_static (the entry point that allocates nothing: its scratch is a per-GPU array inside the
library) against rotconv_pool_fwd with a caller's workspace, through the C ABI.

Both run the same kernels in the same order, so the bar is the strictest one: pooled values and arg-max bit for
bit.  The library's array keeps the last call's contents, so every case is run as two calls in a row, the
second on a smaller layer of another kernel route (other scratch layout), and the first case is run again at the end.
One case is also checked against the CPU oracle, so the pair is not merely equal to each other.
"""
import numpy as np
import pytest
import torch

from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth

pytestmark = pytest.mark.gpu


def _cases():
    L = synth.LayerConfig
    return [
        # (configuration, plan dtype) - ordered large -> small so that stale scratch would be seen
        (L("na_r4", N=2, Cin=64, H=64, W=64, Cout=64, R=4, x_dist="absnormal", seed=701), rc.F32),      # packed bank only
        (L("na_csplit", N=1, Cin=512, H=8, W=8, Cout=32, R=4, x_dist="absnormal", seed=702), rc.F32),   # channel-split parts
        (L("na_r16_fold", N=1, Cin=32, H=32, W=32, Cout=16, R=16, mode="bilinear", x_dist="absnormal", seed=703),
         rc.F32),                                                                                        # banks folded
        (L("na_r16_first", N=1, Cin=3, H=32, W=32, Cout=8, R=16, mode="bilinear", seed=704), rc.F32),   # first layer: vector ALU
        (L("na_px", N=1, Cin=64, H=20, W=32, Cout=16, R=16, mode="bilinear", x_dist="absnormal", seed=707), rc.BF16),   # bf16, a lane per pixel column
        (L("na_bf16", N=1, Cin=32, H=16, W=32, Cout=16, R=4, x_dist="absnormal", seed=705), rc.BF16),   # bf16 kernel
        (L("na_generic", N=1, Cin=2, H=7, W=5, Cout=3, R=3, mode="bilinear", pad=0, seed=706), rc.F32), # generic family
    ]


class _Layer:
    def __init__(self, cfg, dtype):
        self.cfg = cfg
        self.plan = rc.Plan.from_config(cfg, dtype=dtype)
        tdt = torch.bfloat16 if dtype == rc.BF16 else torch.float32
        self.x = torch.from_numpy(synth.make_x(cfg)).to(tdt).cuda()
        self.w = torch.from_numpy(synth.make_w(cfg)).to(tdt).cuda()
        self.shape = (cfg.N, self.plan.Cpooled, self.plan.Ho, self.plan.Wo)
        self.tdt = tdt

    def outputs(self):
        yp = torch.full(self.shape, float("nan"), dtype=self.tdt, device="cuda")
        idx = torch.full(self.shape, 254, dtype=torch.uint8, device="cuda")
        return yp, idx

    def reference(self):
        yp, idx = self.outputs()
        rc.rotconv_pool_fwd(self.plan, self.x, self.w, yp, idx)     # also the call that uploads the plan's tables
        torch.cuda.synchronize()
        return yp, idx

    def static(self):
        yp, idx = self.outputs()
        rc.rotconv_pool_fwd_static(self.plan, self.x, self.w, yp, idx)
        torch.cuda.synchronize()
        return yp, idx


def _same(a, b, what):
    ya, ia = a
    yb, ib = b
    assert torch.equal(ia, ib), f"{what}: arg-max differs"
    assert torch.equal(ya.view(torch.int16 if ya.dtype == torch.bfloat16 else torch.int32),
                       yb.view(torch.int16 if yb.dtype == torch.bfloat16 else torch.int32)), f"{what}: pooled values differ"


def test_static_scratch_forward_matches_workspace_forward():
    layers = [_Layer(cfg, dt) for cfg, dt in _cases()]
    refs = [L.reference() for L in layers]
    # two calls in a row, the second on a smaller layer of another route; then every later one; then the first again
    for i, L in enumerate(layers):
        _same(L.static(), refs[i], f"{L.cfg.name} (call {i})")
    _same(layers[0].static(), refs[0], "first case after the others")
    _same(layers[3].static(), refs[3], "candidates case after a larger one")


def test_static_scratch_forward_matches_the_oracle():
    import parity_util as pu
    cfg = synth.LayerConfig("na_oracle", N=1, Cin=8, H=12, W=16, Cout=8, R=4, seed=707)
    x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    ref = pu.oracle_layer(cfg, x, w, g)
    L = _Layer(cfg, rc.F32)
    L.reference()
    yp, idx = L.static()
    pu.assert_close(yp.cpu().numpy(), ref["ypool"], "static ypool")
    pu.check_idx(idx.cpu().numpy(), ref["y"], ref["abs_terms"], cfg.G, "static idx")


def test_static_scratch_forward_refusals():
    # a plan that has not run on the device yet: uploading its tables would allocate
    cfg = synth.LayerConfig("na_fresh", N=1, Cin=8, H=8, W=8, Cout=8, R=4, seed=708)
    L = _Layer(cfg, rc.F32)
    with pytest.raises(rc.RotconvError) as e:
        L.static()
    assert e.value.status == rc.ERR_UNSUPPORTED
    L.reference()
    L.static()          # accepted once the tables are there
    # a layer whose packed banks exceed the array (1024 x 1024 channels: 37.7 MB)
    big = rc.Plan(N=1, Cin=1024, H=32, W=32, Cout=1024, R=4)
    x = torch.zeros((1, 1024, 32, 32), device="cuda")
    w = torch.zeros((1024, 1024, 3, 3), device="cuda")
    yp = torch.zeros((1, 1024, 32, 32), device="cuda")
    idx = torch.zeros((1, 1024, 32, 32), dtype=torch.uint8, device="cuda")
    rc.rotconv_pool_fwd(big, x, w, yp, idx)
    torch.cuda.synchronize()
    with pytest.raises(rc.RotconvError) as e:
        rc.rotconv_pool_fwd_static(big, x, w, yp, idx)
    assert e.value.status == rc.ERR_WORKSPACE
    # null arguments are found first
    with pytest.raises(rc.RotconvError) as e:
        rc.rotconv_pool_fwd_static(L.plan, None, L.w, yp, idx)
    assert e.value.status == rc.ERR_NULL
