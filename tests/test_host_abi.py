"""CPU-only checks of the C-ABI library: it loads, exports what include/rotconv.h
declares, rejects bad descriptors with the documented codes, and its host-built
orientation tables reproduce the oracle's materialised rotated banks."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import rotconv_oracle as orc
from paper_2512_08888_amd import binding as rc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RNG = np.random.default_rng(7)


def declared_functions(header="rotconv.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rotconv_[a-z_0-9]+|orient_maxpool_[a-z]+|glue_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = rc.lib()
    names = declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(L, n), n
    assert sorted(rc.EXPORTS) == names
    glue = declared_functions("unetglue.h")
    assert len(glue) == 28 and sorted(rc.GLUE_EXPORTS) == glue     # 15 fp32 calls + 13 bf16 twins
    for n in glue:
        assert hasattr(L, n), n


def test_library_is_not_older_than_its_sources():
    from paper_2512_08888_amd import build as b

    assert b.stale_sources() == [], "rebuild the library: python -c 'import __graft_entry__ as g; g.build()'"


def test_glue_argument_errors():
    L = rc.lib()
    assert L.glue_relu_fwd(None, 1, 4, None) == rc.ERR_NULL
    assert L.glue_maxpool2_fwd(1, 1, 1, 1, 1, 3, 4, None) == rc.ERR_SHAPE      # odd height
    assert L.glue_maxpool2_bwd(1, 1, 1, 1, 1, 4, 3, 0, None) == rc.ERR_SHAPE
    assert L.glue_upconv2_fwd(1, 1, 1, 0, 1, 1, 1, 1, None) == rc.ERR_SHAPE
    assert L.glue_upconv2_bwd_weight(1, 1, 1, 1, 4, 4, 2, 2, None, 0, None) == rc.ERR_WORKSPACE
    assert L.glue_conv1x1_bwd_weight(1, 1, 1, 1, 4, 4, 16, 1, 8, None) == rc.ERR_WORKSPACE
    assert L.glue_softmax_ce(1, 1, 1, 1, 1, 3, 16, None, 0, None) == rc.ERR_WORKSPACE
    assert L.glue_upconv2_workspace_bytes(2, 8, 4, 4, 4) >= 2 * 8 * 16 * 4


def test_status_strings():
    for s in (0, -1, -2, -3, -4, -5, -6, 17):
        assert isinstance(rc.status_string(s), str) and rc.status_string(s)


def _create(**kw):
    base = dict(N=1, Cin=2, H=8, W=8, Cout=3, k=3, R=4, angles_deg=None, mode="exact90", stride=1, pad=1, pool_group=0)
    base.update(kw)
    return rc.Plan(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(N=0), rc.ERR_SHAPE), (dict(Cin=0), rc.ERR_SHAPE), (dict(k=0), rc.ERR_SHAPE), (dict(R=0), rc.ERR_SHAPE),
    (dict(R=256, mode="bilinear"), rc.ERR_SHAPE), (dict(stride=0), rc.ERR_SHAPE), (dict(pad=-1), rc.ERR_SHAPE),
    (dict(pool_group=3), rc.ERR_SHAPE), (dict(pool_group=8), rc.ERR_SHAPE), (dict(H=1, pad=0), rc.ERR_SHAPE),
    (dict(R=8), rc.ERR_ANGLES),                                    # 45 deg in exact90 mode
    (dict(R=2, angles_deg=[0.0, 360.0]), rc.ERR_ANGLES),           # outside [0,360)
    (dict(R=2, angles_deg=[90.0, 0.0]), rc.ERR_ANGLES),            # not ascending
    (dict(R=2, angles_deg=[90.0, 90.0]), rc.ERR_ANGLES),
    (dict(mode=7), rc.ERR_UNSUPPORTED), (dict(dtype=2), rc.ERR_UNSUPPORTED),
])
def test_descriptor_errors(kw, code):
    with pytest.raises(rc.RotconvError) as e:
        _create(**kw)
    assert e.value.status == code


def test_null_arguments():
    L = rc.lib()
    h = ctypes.c_void_p()
    assert L.rotconv_plan_create(None, ctypes.byref(h)) == rc.ERR_NULL
    d = rc.Desc(1, 1, 4, 4, 1, 3, 4, None, 0, 1, 1, 0, 0)
    assert L.rotconv_plan_create(ctypes.byref(d), None) == rc.ERR_NULL
    assert L.rotconv_plan_destroy(None) == rc.OK
    assert L.rotconv_workspace_bytes(None) == 0
    p = _create()
    # NULL tensors are rejected before anything touches a device
    assert L.rotconv_pool_fwd(p.handle, None, None, None, None, None, 0, None) == rc.ERR_NULL
    assert L.rotconv_fwd(p.handle, None, 1, 1, None, 0, None) == rc.ERR_NULL
    assert L.orient_maxpool_fwd(p.handle, 1, None, 1, None) == rc.ERR_NULL
    # non-NULL tensors but no workspace
    assert L.rotconv_pool_fwd(p.handle, 1, 1, 1, 1, None, 0, None) == rc.ERR_WORKSPACE
    assert L.rotconv_pool_bwd_weight(p.handle, 1, 1, 1, 1, 1, 8, None) == rc.ERR_WORKSPACE


def test_out_shape_and_workspace():
    p = _create(N=2, H=9, W=7, stride=2, pad=1, R=4, pool_group=2)
    assert (p.Ho, p.Wo, p.Cunpooled, p.Cpooled) == (5, 4, 12, 6)
    assert p.workspace_bytes >= 4 * 4 * 3 * 2 * 9


def test_bf16_plan_adds_staging_to_the_workspace():
    a, b = _create(N=2, Cin=5, H=8, W=8, Cout=3), _create(N=2, Cin=5, H=8, W=8, Cout=3, dtype=rc.BF16)
    staging = 4 * (2 * 5 * 64 + 3 * 5 * 9 + 2 * 3 * 4 * 64)          # x, w, unpooled y in fp32
    assert b.workspace_bytes >= a.workspace_bytes + staging
    assert (b.Ho, b.Wo, b.Cpooled) == (a.Ho, a.Wo, a.Cpooled)


def test_orientation_structure():
    p = _create(R=16, mode="bilinear")
    Q, bank, quarter = p.orientations()
    assert Q == 4 and bank == [r % 4 for r in range(16)] and quarter == [r // 4 for r in range(16)]
    p = _create(R=3, mode="steerable", angles_deg=[10.0, 100.0, 300.0])
    Q, bank, quarter = p.orientations()
    assert Q == 2 and bank == [0, 0, 1] and quarter == [0, 1, 3]
    p = _create(R=2, angles_deg=[0.0, 180.0])
    assert p.orientations() == (1, [0, 0], [0, 2])


@pytest.mark.parametrize("R,mode,k,angles", [
    (4, "exact90", 3, None), (4, "exact90", 5, None), (4, "exact90", 2, None), (1, "exact90", 3, None),
    (2, "exact90", 3, [90.0, 270.0]), (16, "bilinear", 3, None), (8, "bilinear", 5, None), (16, "steerable", 3, None),
    (5, "bilinear", 3, [0.0, 30.0, 120.0, 200.0, 359.0]), (6, "steerable", 4, None),
])
def test_expansion_table_reproduces_oracle_banks(R, mode, k, angles):
    """W^(r) = E[r] . w for random base banks: the host-built tap tables against the oracle's
    explicitly rotated filters (Eq. 5, Sec. III-D, Eq. 17)."""
    p = _create(R=R, mode=mode, k=k, angles_deg=angles, pad=k // 2)
    E = p.expansion().astype(np.float64)  # [R, kk, B, kk]
    B = 2 if mode == "steerable" else 1
    w = RNG.standard_normal((B, 2, 3, k, k))
    wr = orc.expand_bank(w, R, angles, mode)
    got = np.einsum("rtbu,bocu->roct", E, w.reshape(B, 2, 3, k * k)).reshape(R, 2, 3, k, k)
    np.testing.assert_allclose(got, wr, rtol=0, atol=2e-7 * np.abs(w).max() * 4)
    if mode == "exact90":
        # pure permutation: exactly one unit entry per row
        assert np.array_equal(np.sort(E.reshape(R, k * k, -1), axis=-1)[..., -1], np.ones((R, k * k)))
        assert np.count_nonzero(E) == R * k * k


@pytest.mark.parametrize("R,mode,angles", [
    (4, "exact90", None), (16, "bilinear", None), (8, "bilinear", None), (8, "p4m", None),
    (5, "bilinear", [0.0, 30.0, 120.0, 200.0, 359.0]), (2, "exact90", [90.0, 270.0]),
])
def test_routed_gradient_table_against_the_oracle_gradients(R, mode, angles):
    """The table of the fast fp32 gradients: a single routed gradient value (one pixel, every orientation in turn)
    pushed through the table and the BASE bank must give the oracle's input gradient and weight gradient
    (Eq. 12-16 with the expansion folded in)."""
    p = rc.Plan(1, 1, 5, 5, 1, k=3, R=R, mode=mode, angles_deg=angles)
    T = p.routed_table().astype(np.float64)            # [9][R + 1][9]
    assert np.all(T[:, R] == 0)
    w = RNG.standard_normal((1, 1, 1, 3, 3))
    x = RNG.standard_normal((1, 1, 5, 5))
    w_rot = orc.expand_bank(w, R, angles, mode)
    for r in range(R):
        g = np.zeros((1, 1, 5, 5))
        g[0, 0, 2, 3] = 1.7
        idx = np.full((1, 1, 5, 5), r, dtype=np.uint8)
        dy = orc.orient_maxpool_bwd(g, idx, R, R)
        dx_ref = orc.rotconv_bwd_data(dy, w_rot, 5, 5, 1, 1)[0, 0]
        dw_ref = orc.reduce_bank_grad(orc.rotconv_bwd_weight(x, dy, 3, 1, 1), angles, mode)[0, 0, 0].reshape(9)
        # D[u][p] = G[p + delta] T[delta][r][u]: the value at (2, 3) reaches pixel (2, 3) - delta
        D = np.zeros((9, 5, 5))
        for dyy in (-1, 0, 1):
            for dxx in (-1, 0, 1):
                D[:, 2 - dyy, 3 - dxx] = 1.7 * T[(dyy + 1) * 3 + (dxx + 1), r]
        dx = np.einsum("u,uhw->hw", w.reshape(9), D)
        dw = np.einsum("uhw,hw->u", D, x[0, 0])
        np.testing.assert_allclose(dx, dx_ref, rtol=0, atol=1e-6)
        np.testing.assert_allclose(dw, dw_ref, rtol=0, atol=1e-6)
    with pytest.raises(rc.RotconvError) as e:
        rc.Plan(1, 1, 5, 5, 1, k=3, R=8, mode="steerable").routed_table()      # two base banks: no table
    assert e.value.status == rc.ERR_UNSUPPORTED


def test_extents_the_general_kernels_cannot_launch_are_refused():
    """Cout * R, Cin or N beyond a grid dimension (65535): refused when the plan is created, not at launch."""
    for kw in (dict(N=1, Cin=2, Cout=512, R=128), dict(N=1, Cin=65536, Cout=1, R=1), dict(N=65536, Cin=1, Cout=1, R=1)):
        kw = dict(dict(H=4, W=4, k=3, mode="bilinear"), **kw)
        with pytest.raises(rc.RotconvError) as e:
            rc.Plan(**kw)
        assert e.value.status == rc.ERR_UNSUPPORTED, kw
    rc.Plan(N=1, Cin=2, H=4, W=4, Cout=512, R=127, mode="bilinear", k=3).close()      # 65024 rows: accepted


def test_kernel_family_selection():
    """Which family a plan's fused calls run (host logic only): the register-resident kernels for every 3x3 / stride 1 /
    pad 1 layer whatever its row width, matrix multiply + scatter for other filter sizes and strides once the layer is
    large enough, the generic kernels for tiny ones; and the tuning switches of rotconv_plan_create_opt."""
    names = lambda p: [p.kernel_name(i) for i in range(3)]
    assert names(rc.Plan(8, 64, 256, 256, 64, k=3, R=4)) == ["mfma_p4"] * 3
    assert names(rc.Plan(2, 16, 33, 255, 8, k=3, R=4)) == ["mfma_p4"] * 3          # odd rows: padded-row plan
    # one pool group over several banks: the pooled forward multiplies with the base bank only
    assert names(rc.Plan(2, 16, 33, 270, 8, k=3, R=16, mode="bilinear")) == ["mfma_p4_base", "mfma_p4", "mfma_p4"]
    assert names(rc.Plan(2, 16, 33, 270, 8, k=3, R=16, mode="bilinear", options=dict(fwd_base=-1))) == ["mfma_p4"] * 3
    assert names(rc.Plan(1, 1024, 4, 4, 256, k=3, R=1)) == ["mfma_p4"] * 3           # small map, deep input
    assert names(rc.Plan(4, 32, 64, 64, 32, k=5, pad=2, R=8, mode="steerable")) == ["mfma_gemm_scatter"] * 3
    assert names(rc.Plan(4, 32, 64, 64, 32, k=3, stride=2, R=4)) == ["mfma_gemm_scatter"] * 3
    assert names(rc.Plan(1, 2, 9, 8, 3, k=5, pad=2, R=4)) == ["generic"] * 3       # tiny: one generic kernel
    # at most four input channels (a first layer): the pooled forward on the vector-ALU kernel, whatever the row width
    assert names(rc.Plan(4, 3, 512, 512, 64, k=3, R=4)) == ["valu_direct", "mfma_p4", "valu_direct"]
    assert names(rc.Plan(2, 3, 512, 512, 64, k=3, R=16, mode="bilinear"))[2] == "mfma_p4"      # several banks: the table kernel
    assert names(rc.Plan(1, 3, 33, 37, 5, k=3, R=16, mode="bilinear"))[0] == "valu_direct"
    assert names(rc.Plan(1, 3, 64, 64, 8, k=3, R=4, dtype=rc.BF16))[0] == "valu_direct"
    assert names(rc.Plan(4, 3, 512, 512, 64, k=3, R=4, options=dict(direct=-1))) == ["mfma_p4"] * 3
    assert names(rc.Plan(1, 3, 64, 64, 8, k=3, R=8, pool_group=4, mode="bilinear"))[0] == "valu_direct"   # every bank pooled on its own
    assert names(rc.Plan(1, 3, 64, 64, 8, k=3, R=8, pool_group=2, mode="bilinear"))[0] != "valu_direct"   # groups that cut through a bank
    assert names(rc.Plan(1, 3, 64, 64, 8, k=3, R=1))[0] != "valu_direct"            # no quarter turns to share
    # bf16 forward with a lane per pixel column: R = 16 up to 64 input channels by default, px_fwd = 1 wherever it can run
    b16 = dict(k=3, R=16, mode="bilinear", dtype=rc.BF16)
    assert names(rc.Plan(2, 64, 64, 64, 64, **b16))[0] == "mfma_px_bf16"
    assert names(rc.Plan(2, 64, 64, 64, 64, options=dict(px_fwd=-1), **b16))[0] == "mfma_p4_bf16"
    assert names(rc.Plan(2, 128, 64, 64, 64, **b16))[0] == "mfma_p4_bf16"
    assert names(rc.Plan(2, 128, 64, 64, 64, options=dict(px_fwd=1), **b16))[0] == "mfma_px_bf16"
    assert names(rc.Plan(2, 136, 64, 64, 64, options=dict(px_fwd=1), **b16))[0] == "mfma_p4_bf16"     # beyond 128 channels
    assert names(rc.Plan(2, 64, 64, 64, 64, k=3, R=4, dtype=rc.BF16))[0] == "mfma_p4_bf16"
    # a pool group that cuts through a bank: the forward pools an unpooled map, the gradients take the other family
    p = rc.Plan(4, 32, 64, 64, 32, k=3, R=4, pool_group=2)
    assert names(p) == ["mfma_p4", "mfma_gemm_scatter", "mfma_gemm_scatter"]
    assert names(rc.Plan(4, 32, 64, 64, 32, k=5, pad=2, R=8, mode="steerable", options=dict(gs=-1))) == ["generic"] * 3
    assert names(rc.Plan(1, 2, 9, 8, 3, k=5, pad=2, R=4, options=dict(gs=1))) == ["mfma_gemm_scatter"] * 3
    # the per-bank gradient kernels need more scratch than the table variant; both fit what the plan asks for
    big = dict(k=3, R=16, mode="bilinear")
    ws_lut = rc.Plan(2, 256, 64, 64, 256, **big).workspace_bytes
    ws_bank = rc.Plan(2, 256, 64, 64, 256, options=dict(bwd_lut=-1), **big).workspace_bytes
    assert 0 < ws_lut <= ws_bank
    # a forced channel split needs one unpooled part per split
    ws1 = rc.Plan(1, 256, 32, 32, 64, k=3, R=4, options=dict(fwd_csplit=1)).workspace_bytes
    ws8 = rc.Plan(1, 256, 32, 32, 64, k=3, R=4, options=dict(fwd_csplit=8)).workspace_bytes
    assert ws8 >= ws1 >= 8 * 64 * 4 * 32 * 32 * 4      # eight parts of N * Cout * R * H * W floats fit either way
    # the matrix-core input gradient addresses an image of the pooled gradient with 32-bit byte offsets: 2^30 elements and
    # more per image go to the general kernel
    assert names(rc.Plan(1, 8, 4096, 4096, 63, k=3, R=1))[1] == "mfma_p4"
    assert names(rc.Plan(1, 8, 4096, 4096, 64, k=3, R=1))[1] == "generic"
    # a non-zero reserved field is refused
    import ctypes
    bad = rc.PlanOptions()
    bad.reserved[0] = 7
    h = ctypes.c_void_p()
    d = rc.Plan(1, 2, 9, 8, 3).desc
    assert rc.lib().rotconv_plan_create_opt(ctypes.byref(d), ctypes.byref(bad), ctypes.byref(h)) == rc.ERR_UNSUPPORTED


def test_p4m_tables_reproduce_the_oracle_banks():
    """Host-built expansion of the p4m mode (two banks: the filter and its mirror image, four quarter turns each)
    against the oracle's materialised filters; and the descriptor checks of that mode."""
    for R in (2, 4, 8):
        plan = rc.Plan(1, 2, 8, 8, 3, k=3, R=R, mode="p4m")
        E = plan.expansion()                       # [R][kk][B][kk]
        w = RNG.standard_normal((1, 3, 2, 3, 3))
        ref = orc.expand_bank(w, R, None, "p4m")
        got = np.einsum("rtbu,bocu->roct", E.astype(np.float64), w.reshape(1, 3, 2, 9)).reshape(ref.shape)
        assert np.array_equal(got, ref)
        Q, bank, quarter = plan.orientations()
        assert Q == 2 and bank == [0] * (R // 2) + [1] * (R // 2)
    for bad in (dict(R=6), dict(R=8, angles_deg=[0, 45, 90, 135, 180, 225, 270, 315])):
        with pytest.raises(rc.RotconvError) as e:
            rc.Plan(1, 2, 8, 8, 3, k=3, mode="p4m", **bad)
        assert e.value.status == rc.ERR_ANGLES
