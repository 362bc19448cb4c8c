"""The fused calls under HIP graph capture: after one eager call (which uploads the plan's tables), a captured
forward + input gradient + weight gradient replays bit-identically to the eager calls, also after the inputs
have been overwritten between replays.  The calls enqueue kernels only (no memsets, no allocations)."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2512_08888_amd import binding as rc
from paper_2512_08888_amd import synth

pytestmark = pytest.mark.gpu

LC = synth.LayerConfig
CASES = [
    LC("g_p4", N=2, Cin=24, H=12, W=32, Cout=20, R=4, seed=71),                        # register-resident kernels
    LC("g_csplit", N=1, Cin=160, H=6, W=8, Cout=18, R=8, mode="bilinear", seed=72),   # channel split + ordered sums
    LC("g_padw", N=1, Cin=8, H=9, W=13, Cout=6, R=4, seed=73),                         # staged on padded rows
    LC("g_gs", N=2, Cin=32, H=24, W=24, Cout=32, k=5, pad=2, R=8, mode="steerable", seed=74),   # GEMM + scatter
    LC("g_first", N=2, Cin=3, H=20, W=70, Cout=12, R=4, seed=75),                      # first layer: vector-ALU kernels
    LC("g_px", N=1, Cin=64, H=12, W=40, Cout=24, R=16, mode="bilinear", seed=76),      # bf16: a lane per pixel column
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_calls_replay_from_a_graph(cfg, dtype):
    print(f"[case] graph {cfg.name} {dtype}", flush=True)
    bf = dtype == "bf16"
    adt = torch.bfloat16 if bf else torch.float32
    plan = rc.Plan.from_config(cfg, dtype=rc.BF16 if bf else rc.F32)
    plan.workspace()

    def inputs(shift):
        c = dataclasses.replace(cfg, seed=cfg.seed + shift)
        return (torch.from_numpy(synth.make_x(c)).cuda().to(adt), torch.from_numpy(synth.make_w(c)).cuda().to(adt),
                torch.from_numpy(synth.make_g(c)).cuda().to(adt))

    x, w, g = inputs(0)
    shape_p = (cfg.N, plan.Cpooled, plan.Ho, plan.Wo)
    yp = torch.empty(shape_p, dtype=adt, device="cuda")
    idx = torch.empty(shape_p, dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(x)
    dw = torch.empty(w.shape, dtype=torch.float32, device="cuda")

    def step():
        rc.rotconv_pool_fwd(plan, x, w, yp, idx)
        rc.rotconv_pool_bwd_data(plan, g, idx, w, dx)
        rc.rotconv_pool_bwd_weight(plan, x, g, idx, dw)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone().cpu().view(torch.uint8).numpy() if t.dtype == torch.bfloat16 else t.clone().cpu().numpy()
                for t in (yp, idx, dx, dw)]

    step()                       # eager: uploads the tables, fixes kernel attributes
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        xn, wn, gn = inputs(rep)             # new values in the captured buffers
        x.copy_(xn); w.copy_(wn); g.copy_(gn)
        step()
        eager = snapshot()
        for t in (yp, dx, dw):
            t.zero_()
        idx.fill_(77)
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        for a, b in zip(eager, replayed):
            assert np.array_equal(a, b), f"{cfg.name} {dtype}: replay {rep} differs from the eager calls"
