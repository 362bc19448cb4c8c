"""Helpers shared by the GPU parity tests: run a layer through the C-ABI library
(HIP path) and through the CPU oracle on the same seeded inputs, and compare
under the stated bars.

Bars
  values (fp32):  |gpu - ref| <= RTOL*|ref| + RTOL*rms(ref) elementwise and
                  ||gpu - ref||_2 <= RTOL*||ref||_2, RTOL = 1e-4 (the benchmark's
                  stated fp32 tolerance).
  arg-max idx:    bit-exact on exact-arithmetic (dyadic) inputs.  On continuous
                  inputs the two sides sum in different orders, so idx must equal
                  the oracle's wherever the oracle's winner leads every other
                  member of its pool group by more than
                  tau = 64 * eps_fp32 * sum|terms|; inside that band any member
                  within tau of the maximum is accepted (the paper's "r* in argmax").
  backward:       always fed ONE idx (the oracle's) on both sides.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import rotconv_oracle as orc
from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth

RTOL = 1e-4
EPS32 = float(np.finfo(np.float32).eps)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def assert_close(got, ref, what, rtol=RTOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values (unwritten output?)"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    bad = err > bound
    assert not bad.any(), (
        f"{what}: {int(bad.sum())}/{ref.size} elements out of tolerance; worst |err|={err.max():.3e} "
        f"at {np.unravel_index(err.argmax(), ref.shape)} ref={ref.flat[err.argmax()]:.6e} rms={rms:.3e}")
    nref = float(np.linalg.norm(ref))
    if nref > 0:
        assert float(np.linalg.norm(got - ref)) <= rtol * nref, f"{what}: relative L2 error too large"


def check_idx(idx_gpu, y_ref, abs_terms, G, what):
    """Arg-max protocol on continuous inputs.  y_ref, abs_terms: [N,Cout,R,Ho,Wo] (fp64)."""
    N, Cout, R, Ho, Wo = y_ref.shape
    ng = R // G
    yg = y_ref.reshape(N, Cout, G, ng, Ho, Wo)
    tau = 64.0 * EPS32 * abs_terms.reshape(N, Cout, G, ng, Ho, Wo).max(axis=2)  # per pooled element
    best = yg.max(axis=2)
    ig = idx_gpu.reshape(N, Cout, ng, Ho, Wo).astype(np.int64)
    grp = np.arange(ng).reshape(1, 1, ng, 1, 1)
    assert np.all(ig % ng == grp), f"{what}: idx outside its pool group"
    chosen = np.take_along_axis(yg, (ig // ng)[:, :, None], axis=2)[:, :, 0]
    bad = chosen < best - tau
    assert not bad.any(), f"{what}: {int(bad.sum())} arg-max indices differ outside the near-tie band"
    ref_idx = (yg.argmax(axis=2) * ng + grp)
    return int((ig != ref_idx).sum())  # accepted near-ties, for reporting


def round_bf16(a):
    """fp64 -> nearest-even bfloat16 -> fp64."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).to(
        torch.float64).numpy()


def layer_fwd_bf16(x, w_base, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """The oracle's layer forward on the banks a bf16 plan multiplies with: the rotated banks are rounded to
    bf16 once (the identity for exact quarter turns).  Same return values as the oracle's layer_fwd."""
    w_rot = round_bf16(orc.expand_bank(w_base, R, angles_deg, mode))
    y = orc.rotconv_fwd(x, w_rot, stride, pad)
    yp, idx = orc.orient_maxpool_fwd(y, pool_group)
    return y, yp, idx, w_rot


def layer_bwd_bf16(x, w_base, gpool, idx, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """Backward of the same: dX through the bf16-rounded banks, dW (independent of the banks) through Eq. 16."""
    x = np.asarray(x, dtype=np.float64)
    w_rot = round_bf16(orc.expand_bank(w_base, R, angles_deg, mode))
    k = w_rot.shape[-1]
    dy = orc.orient_maxpool_bwd(gpool, idx, R, pool_group)
    dx = orc.rotconv_bwd_data(dy, w_rot, x.shape[2], x.shape[3], stride, pad)
    dw = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dy, k, stride, pad), angles_deg, mode)
    return dx, dw


class GpuLayer:
    """Device tensors + plan of one layer configuration."""

    def __init__(self, cfg: synth.LayerConfig, x, w, **plan_over):
        self.cfg = cfg
        self.plan = rc.Plan.from_config(cfg, **plan_over)
        self.x = dev(x, torch.float32)
        self.w = dev(w, torch.float32)
        self.P = (cfg.N, self.plan.Cpooled, self.plan.Ho, self.plan.Wo)
        self.U = (cfg.N, self.plan.Cunpooled, self.plan.Ho, self.plan.Wo)

    def nan(self, shape, dtype=torch.float32):
        t = torch.empty(shape, dtype=dtype, device="cuda")
        if dtype.is_floating_point:
            t.fill_(float("nan"))
        else:
            t.fill_(255)
        return t

    def pool_fwd(self):
        yp, idx = self.nan(self.P), self.nan(self.P, torch.uint8)
        rc.rotconv_pool_fwd(self.plan, self.x, self.w, yp, idx)
        torch.cuda.synchronize()
        return yp.cpu().numpy(), idx.cpu().numpy()

    def fwd(self):
        y = self.nan(self.U)
        rc.rotconv_fwd(self.plan, self.x, self.w, y)
        torch.cuda.synchronize()
        return y

    def maxpool_fwd(self, y):
        yp, idx = self.nan(self.P), self.nan(self.P, torch.uint8)
        rc.orient_maxpool_fwd(self.plan, y, yp, idx)
        torch.cuda.synchronize()
        return yp.cpu().numpy(), idx.cpu().numpy()

    def maxpool_bwd(self, g, idx):
        dy = self.nan(self.U)
        rc.orient_maxpool_bwd(self.plan, dev(g, torch.float32), dev(idx), dy)
        torch.cuda.synchronize()
        return dy

    def pool_bwd_data(self, g, idx):
        dx = self.nan(tuple(self.x.shape))
        rc.rotconv_pool_bwd_data(self.plan, dev(g, torch.float32), dev(idx), self.w, dx)
        torch.cuda.synchronize()
        return dx.cpu().numpy()

    def pool_bwd_weight(self, g, idx):
        dw = self.nan(tuple(self.w.shape))
        rc.rotconv_pool_bwd_weight(self.plan, self.x, dev(g, torch.float32), dev(idx), dw)
        torch.cuda.synchronize()
        return dw.cpu().numpy()

    def bwd_data(self, dy):
        dx = self.nan(tuple(self.x.shape))
        rc.rotconv_bwd_data(self.plan, dy, self.w, dx)
        torch.cuda.synchronize()
        return dx.cpu().numpy()

    def bwd_weight(self, dy):
        dw = self.nan(tuple(self.w.shape))
        rc.rotconv_bwd_weight(self.plan, self.x, dy, dw)
        torch.cuda.synchronize()
        return dw.cpu().numpy()


def oracle_layer(cfg: synth.LayerConfig, x, w, g):
    """Full oracle pass.  Returns dict with y, ypool, idx, abs_terms, dx, dw (all fp64)."""
    ang = None if cfg.angles_deg is None else list(cfg.angles_deg)
    y, yp, idx, w_rot = orc.layer_fwd(x, w, cfg.R, ang, cfg.mode, cfg.stride, cfg.pad, cfg.G)
    abs_terms = orc.rotconv_fwd(np.abs(x), np.abs(w_rot), cfg.stride, cfg.pad)
    dx, dw = orc.layer_bwd(x, w, g, idx, cfg.R, ang, cfg.mode, cfg.stride, cfg.pad, cfg.G)
    return dict(y=y, ypool=yp, idx=idx, abs_terms=abs_terms, dx=dx, dw=dw, w_rot=w_rot)


def run_fused_parity(cfg: synth.LayerConfig, dyadic: bool = False, label: str = "", **plan_over):
    """Fused hot path (pool_fwd, pool_bwd_data, pool_bwd_weight) against the oracle.  plan_over: keyword arguments of
    the plan beyond the configuration (e.g. options=dict(gs=1), the tuning switches)."""
    what = label or cfg.name
    if dyadic:
        x, w, g = synth.make_x_dyadic(cfg), synth.make_w_dyadic(cfg), synth.make_g_dyadic(cfg)
    else:
        x, w, g = synth.make_x(cfg), synth.make_w(cfg), synth.make_g(cfg)
    ref = oracle_layer(cfg, x, w, g)
    L = GpuLayer(cfg, x, w, **plan_over)
    yp, idx = L.pool_fwd()
    dx = L.pool_bwd_data(g, ref["idx"])
    dw = L.pool_bwd_weight(g, ref["idx"])
    if dyadic:
        assert np.array_equal(yp.astype(np.float64), ref["ypool"]), f"{what}: pooled output not bit-exact"
        assert np.array_equal(idx, ref["idx"]), f"{what}: arg-max not bit-exact"
        assert np.array_equal(dx.astype(np.float64), ref["dx"]), f"{what}: dx not bit-exact"
        if cfg.N * cfg.Ho * cfg.Wo <= (1 << 14):
            assert np.array_equal(dw.astype(np.float64), ref["dw"]), f"{what}: dw not bit-exact"
        else:
            assert_close(dw, ref["dw"], f"{what} dw")
        ties = 0
    else:
        assert_close(yp, ref["ypool"], f"{what} ypool")
        ties = check_idx(idx, ref["y"], ref["abs_terms"], cfg.G, f"{what} idx")
        assert_close(dx, ref["dx"], f"{what} dx")
        assert_close(dw, ref["dw"], f"{what} dw")
    return dict(layer=L, ref=ref, yp=yp, idx=idx, dx=dx, dw=dw, near_ties=ties, x=x, w=w, g=g)
