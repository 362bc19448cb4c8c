"""Thin ctypes binding of librotconv.so (the C ABI of include/rotconv.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream.  There is no
fallback of any kind: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librotconv.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ANGLES, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
MODES = {"exact90": 0, "steerable": 1, "bilinear": 2, "p4m": 3}
POOL_OPS = {"max": 0, "avg": 1}

EXPORTS = [
    "rotconv_plan_create", "rotconv_plan_create_opt", "rotconv_plan_destroy", "rotconv_workspace_bytes", "rotconv_out_shape",
    "rotconv_plan_orientations", "rotconv_plan_expansion", "rotconv_plan_routed_table",
    "rotconv_workspace_bytes_unfused",
    "rotconv_fwd", "rotconv_bwd_data", "rotconv_bwd_weight", "orient_maxpool_fwd", "orient_maxpool_bwd",
    "rotconv_pool_fwd", "rotconv_pool_bwd_data", "rotconv_pool_bwd_weight", "rotconv_pool_fwd_static",
    "rotconv_status_string", "rotconv_plan_kernel_name", "rotconv_steerable_reg", "rotconv_plan_conv_equivalents",
    "rotconv_diag_mfma_sink_bytes", "rotconv_diag_mfma", "rotconv_diag_copy",
]

# include/unetglue.h
GLUE_EXPORTS = [
    "glue_relu_fwd", "glue_relu_bwd", "glue_maxpool2_fwd", "glue_maxpool2_bwd",
    "glue_upconv2_workspace_bytes", "glue_upconv2_fwd", "glue_upconv2_bwd_data", "glue_upconv2_bwd_weight",
    "glue_concat2", "glue_split2",
    "glue_conv1x1_workspace_bytes", "glue_conv1x1_fwd", "glue_conv1x1_bwd_data", "glue_conv1x1_bwd_weight",
    "glue_softmax_ce",
]
# the bfloat16 twins: every call above except the two workspace-size queries
GLUE_EXPORTS += [n + "_bf16" for n in GLUE_EXPORTS if not n.endswith("_workspace_bytes")]


class Desc(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_int32), ("Cin", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
        ("Cout", ctypes.c_int32), ("k", ctypes.c_int32), ("R", ctypes.c_int32),
        ("angles_deg", ctypes.POINTER(ctypes.c_double)),
        ("mode", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32),
        ("pool_group", ctypes.c_int32), ("dtype", ctypes.c_int32), ("pool_op", ctypes.c_int32),
        ("activation", ctypes.c_int32),
    ]


class PlanOptions(ctypes.Structure):
    """rotconv_plan_options: tuning switches of a plan's kernel choice (all zero: automatic)."""
    _fields_ = [
        ("fwd_csplit", ctypes.c_int32), ("gs", ctypes.c_int32), ("gs_chunk_mb", ctypes.c_int32),
        ("bwd_lut", ctypes.c_int32), ("fwd_base", ctypes.c_int32), ("direct", ctypes.c_int32),
        ("direct_ty", ctypes.c_int32), ("px_fwd", ctypes.c_int32), ("reserved", ctypes.c_int32 * 4),
    ]


class RotconvError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def lib():
    """Loads librotconv.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2512_08888_amd.build` "
                "(or __graft_entry__.build()); there is no non-HIP fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32p = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int32)
        L.rotconv_plan_create.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(vp)]
        L.rotconv_plan_create_opt.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(PlanOptions), ctypes.POINTER(vp)]
        L.rotconv_plan_destroy.argtypes = [vp]
        L.rotconv_workspace_bytes.argtypes = [vp]
        L.rotconv_workspace_bytes.restype = sz
        L.rotconv_workspace_bytes_unfused.argtypes = [vp]
        L.rotconv_workspace_bytes_unfused.restype = sz
        L.rotconv_out_shape.argtypes = [vp, i32p, i32p, i32p, i32p]
        L.rotconv_plan_orientations.argtypes = [vp, i32p, i32p, i32p]
        L.rotconv_plan_expansion.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
        L.rotconv_plan_routed_table.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
        L.rotconv_fwd.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.rotconv_bwd_data.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.rotconv_bwd_weight.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.orient_maxpool_fwd.argtypes = [vp, vp, vp, vp, vp]
        L.orient_maxpool_bwd.argtypes = [vp, vp, vp, vp, vp]
        L.rotconv_pool_fwd.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        L.rotconv_pool_fwd_static.argtypes = [vp, vp, vp, vp, vp, vp]
        L.rotconv_pool_bwd_data.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        L.rotconv_pool_bwd_weight.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        L.rotconv_status_string.argtypes = [ctypes.c_int]
        L.rotconv_status_string.restype = ctypes.c_char_p
        L.rotconv_plan_kernel_name.argtypes = [vp, ctypes.c_int]
        L.rotconv_plan_kernel_name.restype = ctypes.c_char_p
        L.rotconv_diag_mfma_sink_bytes.restype = sz
        L.rotconv_diag_mfma.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, ctypes.POINTER(ctypes.c_double)]
        L.rotconv_diag_copy.argtypes = [vp, vp, sz, vp]
        L.rotconv_plan_conv_equivalents.argtypes = [vp, ctypes.c_int]
        L.rotconv_plan_conv_equivalents.restype = ctypes.c_double
        L.rotconv_steerable_reg.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                            ctypes.c_float, vp, vp, ctypes.c_int32, vp, sz, vp]
        ci = ctypes.c_int
        L.glue_relu_fwd.argtypes = [vp, vp, sz, vp]
        L.glue_relu_bwd.argtypes = [vp, vp, vp, sz, vp]
        L.glue_maxpool2_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp]
        L.glue_maxpool2_bwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.glue_upconv2_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.glue_upconv2_workspace_bytes.restype = sz
        L.glue_upconv2_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.glue_upconv2_bwd_data.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.glue_upconv2_bwd_weight.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.glue_concat2.argtypes = [vp, vp, vp, ci, ci, ci, sz, vp]
        L.glue_split2.argtypes = [vp, vp, vp, ci, ci, ci, sz, ci, vp]
        L.glue_conv1x1_workspace_bytes.argtypes = [ci, ci, ci, sz]
        L.glue_conv1x1_workspace_bytes.restype = sz
        L.glue_conv1x1_fwd.argtypes = [vp, vp, vp, ci, ci, ci, sz, vp]
        L.glue_conv1x1_bwd_data.argtypes = [vp, vp, vp, ci, ci, ci, sz, vp]
        L.glue_conv1x1_bwd_weight.argtypes = [vp, vp, vp, ci, ci, ci, sz, vp, sz, vp]
        L.glue_softmax_ce.argtypes = [vp, vp, vp, vp, ci, ci, sz, vp, sz, vp]
        for name in GLUE_EXPORTS:
            if name.endswith("_bf16"):
                getattr(L, name).argtypes = getattr(L, name[:-5]).argtypes
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().rotconv_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != OK:
        raise RotconvError(status, what)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor; None stays NULL."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr()


def _stream() -> Optional[int]:
    import torch

    return torch.cuda.current_stream().cuda_stream or None


class Plan:
    """Owns a rotconv_plan*.  Mirrors rotconv_plan_create / destroy and the host-side queries."""

    def __init__(self, N, Cin, H, W, Cout, k=3, R=4, angles_deg: Optional[Sequence[float]] = None, mode="exact90",
                 stride=1, pad=1, pool_group=0, dtype=F32, pool_op="max", relu=False, options=None):
        """options: dict of rotconv_plan_options fields (fwd_csplit, gs, gs_chunk_mb, bwd_lut, fwd_base, direct,
        direct_ty, px_fwd) or None."""
        self._h = ctypes.c_void_p()
        self._angles = None
        ang = None
        if angles_deg is not None:
            self._angles = (ctypes.c_double * len(angles_deg))(*[float(a) for a in angles_deg])
            ang = ctypes.cast(self._angles, ctypes.POINTER(ctypes.c_double))
        m = MODES[mode] if isinstance(mode, str) else int(mode)
        po = POOL_OPS[pool_op] if isinstance(pool_op, str) else int(pool_op)
        self.desc = Desc(N, Cin, H, W, Cout, k, R, ang, m, stride, pad, pool_group or 0, dtype, po, 1 if relu else 0)
        if options:
            self.options = PlanOptions(**{k: int(v) for k, v in options.items()})
            _check(lib().rotconv_plan_create_opt(ctypes.byref(self.desc), ctypes.byref(self.options),
                                                 ctypes.byref(self._h)), "rotconv_plan_create_opt")
        else:
            self.options = None
            _check(lib().rotconv_plan_create(ctypes.byref(self.desc), ctypes.byref(self._h)), "rotconv_plan_create")
        ho, wo, cu, cp = (ctypes.c_int32() for _ in range(4))
        lib().rotconv_out_shape(self._h, ctypes.byref(ho), ctypes.byref(wo), ctypes.byref(cu), ctypes.byref(cp))
        self.Ho, self.Wo, self.Cunpooled, self.Cpooled = ho.value, wo.value, cu.value, cp.value
        self.N, self.Cin, self.H, self.W, self.Cout, self.k, self.R = N, Cin, H, W, Cout, k, R
        self.B = 2 if m == MODES["steerable"] else 1
        self.workspace_bytes = int(lib().rotconv_workspace_bytes(self._h))
        self.workspace_bytes_unfused = int(lib().rotconv_workspace_bytes_unfused(self._h))
        self._ws = None

    @classmethod
    def from_config(cls, cfg, **over):
        kw = dict(N=cfg.N, Cin=cfg.Cin, H=cfg.H, W=cfg.W, Cout=cfg.Cout, k=cfg.k, R=cfg.R, angles_deg=cfg.angles_deg,
                  mode=cfg.mode, stride=cfg.stride, pad=cfg.pad, pool_group=cfg.pool_group or 0)
        kw.update(over)
        return cls(**kw)

    def close(self):
        if self._h:
            lib().rotconv_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def orientations(self):
        q = ctypes.c_int32()
        bank = (ctypes.c_int32 * self.R)()
        quarter = (ctypes.c_int32 * self.R)()
        _check(lib().rotconv_plan_orientations(self._h, ctypes.byref(q), bank, quarter), "rotconv_plan_orientations")
        return q.value, list(bank), list(quarter)

    def expansion(self):
        import numpy as np

        kk = self.k * self.k
        E = np.zeros((self.R, kk, self.B, kk), dtype=np.float32)
        _check(lib().rotconv_plan_expansion(self._h, E.ctypes.data_as(ctypes.POINTER(ctypes.c_float))),
               "rotconv_plan_expansion")
        return E

    def routed_table(self):
        import numpy as np

        T = np.zeros((9, self.R + 1, 9), dtype=np.float32)
        _check(lib().rotconv_plan_routed_table(self._h, T.ctypes.data_as(ctypes.POINTER(ctypes.c_float))),
               "rotconv_plan_routed_table")
        return T

    def conv_equivalents(self, which: int) -> float:
        """Conv-equivalents of matrix work fused call `which` (0 fwd, 1 bwd_data, 2 bwd_weight) executes."""
        return float(lib().rotconv_plan_conv_equivalents(self._h, which))

    def kernel_name(self, which: int) -> str:
        return lib().rotconv_plan_kernel_name(self._h, which).decode()

    def workspace(self, device="cuda"):
        """A torch byte tensor of workspace_bytes on the device (allocated once per plan)."""
        import torch

        if self._ws is None:
            self._ws = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8, device=device)
        return self._ws


def _ws_args(plan: Plan, ws):
    if ws is None:
        ws = plan.workspace()
    return _ptr(ws), ws.numel() * ws.element_size()


def rotconv_fwd(plan: Plan, x, w, y, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_fwd(plan.handle, _ptr(x), _ptr(w), _ptr(y), p, n, _stream()), "rotconv_fwd")


def rotconv_bwd_data(plan: Plan, dy, w, dx, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_bwd_data(plan.handle, _ptr(dy), _ptr(w), _ptr(dx), p, n, _stream()), "rotconv_bwd_data")


def rotconv_bwd_weight(plan: Plan, x, dy, dw, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_bwd_weight(plan.handle, _ptr(x), _ptr(dy), _ptr(dw), p, n, _stream()), "rotconv_bwd_weight")


def orient_maxpool_fwd(plan: Plan, y, ypool, idx):
    _check(lib().orient_maxpool_fwd(plan.handle, _ptr(y), _ptr(ypool), _ptr(idx), _stream()), "orient_maxpool_fwd")


def orient_maxpool_bwd(plan: Plan, gpool, idx, dy):
    _check(lib().orient_maxpool_bwd(plan.handle, _ptr(gpool), _ptr(idx), _ptr(dy), _stream()), "orient_maxpool_bwd")


def rotconv_pool_fwd(plan: Plan, x, w, ypool, idx, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_pool_fwd(plan.handle, _ptr(x), _ptr(w), _ptr(ypool), _ptr(idx), p, n, _stream()),
           "rotconv_pool_fwd")


def rotconv_pool_fwd_static(plan: Plan, x, w, ypool, idx):
    """rotconv_pool_fwd on the library's own per-GPU scratch array: no workspace, no allocation."""
    _check(lib().rotconv_pool_fwd_static(plan.handle, _ptr(x), _ptr(w), _ptr(ypool), _ptr(idx), _stream()),
           "rotconv_pool_fwd_static")


def rotconv_pool_bwd_data(plan: Plan, gpool, idx, w, dx, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_pool_bwd_data(plan.handle, _ptr(gpool), _ptr(idx), _ptr(w), _ptr(dx), p, n, _stream()),
           "rotconv_pool_bwd_data")


def rotconv_pool_bwd_weight(plan: Plan, x, gpool, idx, dw, ws=None):
    p, n = _ws_args(plan, ws)
    _check(lib().rotconv_pool_bwd_weight(plan.handle, _ptr(x), _ptr(gpool), _ptr(idx), _ptr(dw), p, n, _stream()),
           "rotconv_pool_bwd_weight")


def rotconv_diag_mfma(dtype: int, n_iter: int, sink) -> float:
    """Enqueues the matrix-instruction loop; returns the floating-point operations it executes."""
    fl = ctypes.c_double()
    _check(lib().rotconv_diag_mfma(int(dtype), int(n_iter), _ptr(sink), _stream(), ctypes.byref(fl)), "rotconv_diag_mfma")
    return fl.value


def rotconv_diag_mfma_sink_bytes() -> int:
    return int(lib().rotconv_diag_mfma_sink_bytes())


def rotconv_diag_copy(dst, src):
    _check(lib().rotconv_diag_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream()), "rotconv_diag_copy")


def rotconv_steerable_reg(w, lambda_mag, lambda_orth, eps, losses, dw=None, accumulate=False, ws=None):
    """w [2,Cout,Cin,k,k] fp32; losses [2] fp32; dw like w or None; ws: at least Cout*2 floats (allocated if None)."""
    import torch

    Cout = w.shape[1]
    per = w.numel() // (2 * Cout)
    if ws is None:
        ws = torch.empty(max(256, Cout * 8), dtype=torch.uint8, device=w.device)
    _check(lib().rotconv_steerable_reg(_ptr(w), Cout, per, float(lambda_mag), float(lambda_orth), float(eps),
                                       _ptr(losses), _ptr(dw), int(bool(accumulate)), _ptr(ws),
                                       ws.numel() * ws.element_size(), _stream()), "rotconv_steerable_reg")


# ---- network glue (include/unetglue.h): same names, argument marshalling only -------------------

def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _glue(name, *tensors):
    """The library entry point for the tensors' storage type: `name` for fp32, `name`_bf16 for bfloat16
    (all activation tensors of one call share the type)."""
    import torch

    kinds = {t.dtype for t in tensors}
    if kinds == {torch.bfloat16}:
        return getattr(lib(), name + "_bf16")
    if kinds == {torch.float32}:
        return getattr(lib(), name)
    raise TypeError(f"{name}: tensors must be all float32 or all bfloat16, got {sorted(map(str, kinds))}")


def glue_relu_fwd(x, y):
    _check(_glue("glue_relu_fwd", x, y)(_ptr(x), _ptr(y), x.numel(), _stream()), "glue_relu_fwd")


def glue_relu_bwd(y, dy, dx):
    _check(_glue("glue_relu_bwd", y, dy, dx)(_ptr(y), _ptr(dy), _ptr(dx), y.numel(), _stream()), "glue_relu_bwd")


def glue_maxpool2_fwd(x, y, idx):
    N, C, H, W = x.shape
    _check(_glue("glue_maxpool2_fwd", x, y)(_ptr(x), _ptr(y), _ptr(idx), N, C, H, W, _stream()), "glue_maxpool2_fwd")


def glue_maxpool2_bwd(dy, idx, dx, accumulate=False):
    N, C, H, W = dx.shape
    _check(_glue("glue_maxpool2_bwd", dy, dx)(_ptr(dy), _ptr(idx), _ptr(dx), N, C, H, W, int(bool(accumulate)), _stream()),
           "glue_maxpool2_bwd")


def glue_upconv2_workspace_bytes(N, Cin, Cout, H, W):
    return int(lib().glue_upconv2_workspace_bytes(N, Cin, Cout, H, W))


def glue_upconv2_fwd(x, w, y):
    N, Cin, H, W = x.shape
    _check(_glue("glue_upconv2_fwd", x, w, y)(_ptr(x), _ptr(w), _ptr(y), N, Cin, w.shape[1], H, W, _stream()), "glue_upconv2_fwd")


def glue_upconv2_bwd_data(dy, w, dx):
    N, Cin, H, W = dx.shape
    _check(_glue("glue_upconv2_bwd_data", dy, w, dx)(_ptr(dy), _ptr(w), _ptr(dx), N, Cin, w.shape[1], H, W, _stream()),
           "glue_upconv2_bwd_data")


def glue_upconv2_bwd_weight(x, dy, dw, ws):
    N, Cin, H, W = x.shape
    _check(_glue("glue_upconv2_bwd_weight", x, dy)(_ptr(x), _ptr(dy), _ptr(dw), N, Cin, dw.shape[1], H, W, _ptr(ws), _nbytes(ws),
                                         _stream()), "glue_upconv2_bwd_weight")


def glue_concat2(a, b, out):
    N, Ca = a.shape[0], a.shape[1]
    P = a.numel() // (N * Ca)
    _check(_glue("glue_concat2", a, b, out)(_ptr(a), _ptr(b), _ptr(out), N, Ca, b.shape[1], P, _stream()), "glue_concat2")


def glue_split2(dcat, da, db, accumulate_a=False):
    N, Ca = da.shape[0], da.shape[1]
    P = da.numel() // (N * Ca)
    _check(_glue("glue_split2", dcat, da, db)(_ptr(dcat), _ptr(da), _ptr(db), N, Ca, db.shape[1], P, int(bool(accumulate_a)), _stream()),
           "glue_split2")


def glue_conv1x1_workspace_bytes(N, Cin, Cout, P):
    return int(lib().glue_conv1x1_workspace_bytes(N, Cin, Cout, P))


def glue_conv1x1_fwd(x, w, y):
    N, Cin = x.shape[0], x.shape[1]
    P = x.numel() // (N * Cin)
    _check(_glue("glue_conv1x1_fwd", x, w, y)(_ptr(x), _ptr(w), _ptr(y), N, Cin, w.shape[0], P, _stream()), "glue_conv1x1_fwd")


def glue_conv1x1_bwd_data(dy, w, dx):
    N, Cin = dx.shape[0], dx.shape[1]
    P = dx.numel() // (N * Cin)
    _check(_glue("glue_conv1x1_bwd_data", dy, w, dx)(_ptr(dy), _ptr(w), _ptr(dx), N, Cin, w.shape[0], P, _stream()),
           "glue_conv1x1_bwd_data")


def glue_conv1x1_bwd_weight(x, dy, dw, ws):
    N, Cin = x.shape[0], x.shape[1]
    P = x.numel() // (N * Cin)
    _check(_glue("glue_conv1x1_bwd_weight", x, dy)(_ptr(x), _ptr(dy), _ptr(dw), N, Cin, dw.shape[0], P, _ptr(ws), _nbytes(ws),
                                         _stream()), "glue_conv1x1_bwd_weight")


def glue_softmax_ce(logits, labels, loss, dlogits, ws):
    N, K = logits.shape[0], logits.shape[1]
    P = logits.numel() // (N * K)
    _check(_glue("glue_softmax_ce", logits, dlogits)(_ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits), N, K, P, _ptr(ws), _nbytes(ws),
                                 _stream()), "glue_softmax_ce")
