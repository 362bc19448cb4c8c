"""ctypes front end of the CPU oracle (oracle/rotconv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  Every function
takes and returns plain numpy arrays, computes in fp64 and follows the
definition cited in the C source (paper Sec. III, Eq. 1-17).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rotconv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

MODES = {"exact90": 0, "steerable": 1, "bilinear": 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _bp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def default_angles(R: int) -> np.ndarray:
    """Evenly spaced orientations (Sec. III-D): theta_r = r * 360 / R."""
    return np.arange(R, dtype=np.float64) * (360.0 / R)


def out_extent(H: int, k: int, stride: int, pad: int) -> int:
    return (H + 2 * pad - k) // stride + 1


def expand_bank(w_base, R: int, angles_deg: Optional[Sequence[float]] = None, mode: str = "exact90") -> np.ndarray:
    """[B,Cout,Cin,k,k] -> [R,Cout,Cin,k,k] rotated banks (Eq. 5, Sec. III-D, Eq. 17)."""
    w = _f64(w_base)
    if w.ndim == 4:
        w = w[None]
    if mode == "p4m":
        # the p4m group (Sec. II, Sec. III-B): R/2 quarter-turn rotations of the filter, then the same rotations
        # of its left-right mirror image M[i][j] = W[i][k-1-j]
        assert R % 2 == 0 and angles_deg is None
        plain = expand_bank(w, R // 2, None, "exact90")
        mirrored = expand_bank(np.flip(w, axis=-1), R // 2, None, "exact90")
        return np.concatenate([plain, mirrored], axis=0)
    B, Cout, Cin, k, k2 = w.shape
    assert k == k2 and B == (2 if mode == "steerable" else 1)
    ang = default_angles(R) if angles_deg is None else _f64(angles_deg)
    assert ang.shape == (R,)
    out = np.empty((R, Cout, Cin, k, k), dtype=np.float64)
    rc = _load().orc_expand_bank(MODES[mode], R, _dp(ang), k, Cout, Cin, _dp(w), _dp(out))
    if rc != 0:
        raise ValueError("exact90 mode needs angles that are multiples of 90 degrees")
    return out


def reduce_bank_grad(dw_rot, angles_deg: Optional[Sequence[float]] = None, mode: str = "exact90") -> np.ndarray:
    """[R,Cout,Cin,k,k] -> [B,Cout,Cin,k,k]: inverse-rotate and accumulate (Eq. 16)."""
    d = _f64(dw_rot)
    R, Cout, Cin, k, _ = d.shape
    if mode == "p4m":   # adjoint of the expansion above: rotate back both halves, mirror the second back, add
        assert R % 2 == 0 and angles_deg is None
        return reduce_bank_grad(d[:R // 2], None, "exact90") + np.flip(reduce_bank_grad(d[R // 2:], None, "exact90"), axis=-1)
    ang = default_angles(R) if angles_deg is None else _f64(angles_deg)
    B = 2 if mode == "steerable" else 1
    out = np.empty((B, Cout, Cin, k, k), dtype=np.float64)
    rc = _load().orc_reduce_bank_grad(MODES[mode], R, _dp(ang), k, Cout, Cin, _dp(d), _dp(out))
    if rc != 0:
        raise ValueError("exact90 mode needs angles that are multiples of 90 degrees")
    return out


def rotconv_fwd(x, w_rot, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 7 with zero padding/stride.  Returns y [N,Cout,R,Ho,Wo]."""
    x = _f64(x)
    w = _f64(w_rot)
    N, Cin, H, W = x.shape
    R, Cout, Cin2, k, _ = w.shape
    assert Cin == Cin2
    Ho, Wo = out_extent(H, k, stride, pad), out_extent(W, k, stride, pad)
    y = np.empty((N, Cout, R, Ho, Wo), dtype=np.float64)
    _load().orc_rotconv_fwd(_dp(x), _dp(w), _dp(y), N, Cin, H, W, Cout, R, k, stride, pad)
    return y


def rotconv_fwd_at(x, w_rot, pts, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 7 at sampled outputs.  pts [T,4] = (n, co, oy, ox) -> [T,R]."""
    x = _f64(x)
    w = _f64(w_rot)
    pts = np.ascontiguousarray(pts, dtype=np.int32)
    N, Cin, H, W = x.shape
    R, Cout, _, k, _ = w.shape
    out = np.empty((pts.shape[0], R), dtype=np.float64)
    _load().orc_rotconv_fwd_at(_dp(x), _dp(w), _ip(pts), pts.shape[0], _dp(out), N, Cin, H, W, Cout, R, k, stride, pad)
    return out


def rotconv_fwd_scatter(x, w_base, quarter_turns: Sequence[int], pad: int) -> np.ndarray:
    """Alg. 1 / Eq. 8: scatter form, symmetric rotations, stride 1.  w_base [Cout,Cin,k,k]."""
    x = _f64(x)
    w = _f64(w_base)
    if w.ndim == 5:
        w = w[0]
    q = np.ascontiguousarray(quarter_turns, dtype=np.int32)
    N, Cin, H, W = x.shape
    Cout, _, k, _ = w.shape
    R = q.shape[0]
    Ho, Wo = out_extent(H, k, 1, pad), out_extent(W, k, 1, pad)
    y = np.empty((N, Cout, R, Ho, Wo), dtype=np.float64)
    _load().orc_rotconv_fwd_scatter(_dp(x), _dp(w), _ip(q), _dp(y), N, Cin, H, W, Cout, R, k, pad)
    return y


def orient_maxpool_fwd(y, pool_group: Optional[int] = None):
    """Eq. 10 over pool groups.  y [N,Cout,R,Ho,Wo] -> (ypool [N,Cout*(R/G),Ho,Wo], idx uint8)."""
    y = _f64(y)
    N, Cout, R, Ho, Wo = y.shape
    G = R if pool_group is None else pool_group
    assert R % G == 0
    ng = R // G
    yp = np.empty((N, Cout * ng, Ho, Wo), dtype=np.float64)
    idx = np.empty((N, Cout * ng, Ho, Wo), dtype=np.uint8)
    _load().orc_orient_maxpool_fwd(_dp(y), _dp(yp), _bp(idx), N, Cout, R, G, Ho, Wo)
    return yp, idx


def orient_maxpool_bwd(gpool, idx, R: int, pool_group: Optional[int] = None) -> np.ndarray:
    """Eq. 12.  -> Delta [N,Cout,R,Ho,Wo]."""
    g = _f64(gpool)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    G = R if pool_group is None else pool_group
    ng = R // G
    N, Cp, Ho, Wo = g.shape
    Cout = Cp // ng
    dy = np.empty((N, Cout, R, Ho, Wo), dtype=np.float64)
    _load().orc_orient_maxpool_bwd(_dp(g), _bp(idx), _dp(dy), N, Cout, R, G, Ho, Wo)
    return dy


def orient_avgpool_fwd(y, pool_group: Optional[int] = None) -> np.ndarray:
    """Eq. 9 over pool groups: the point-wise mean of the group's orientations.
    y [N,Cout,R,Ho,Wo] -> ypool [N,Cout*(R/G),Ho,Wo]; group g holds the orientations r with r mod (R/G) == g."""
    y = _f64(y)
    N, Cout, R, Ho, Wo = y.shape
    G = R if pool_group is None else pool_group
    assert R % G == 0
    ng = R // G
    yp = np.zeros((N, Cout, ng, Ho, Wo), dtype=np.float64)
    for r in range(R):                      # plain loop over orientations, in order
        yp[:, :, r % ng] += y[:, :, r]
    return (yp / G).reshape(N, Cout * ng, Ho, Wo)


def orient_avgpool_bwd(gpool, R: int, pool_group: Optional[int] = None) -> np.ndarray:
    """Eq. 11: the upstream gradient is shared equally by the group's members.  -> Delta [N,Cout,R,Ho,Wo]."""
    g = _f64(gpool)
    G = R if pool_group is None else pool_group
    ng = R // G
    N, Cp, Ho, Wo = g.shape
    Cout = Cp // ng
    g = g.reshape(N, Cout, ng, Ho, Wo)
    dy = np.empty((N, Cout, R, Ho, Wo), dtype=np.float64)
    for r in range(R):
        dy[:, :, r] = g[:, :, r % ng] / G
    return dy


def rotconv_bwd_data(dy, w_rot, H: int, W: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 13 + 15.  dy [N,Cout,R,Ho,Wo] -> dx [N,Cin,H,W]."""
    dy = _f64(dy)
    w = _f64(w_rot)
    N, Cout, R, Ho, Wo = dy.shape
    _, _, Cin, k, _ = w.shape
    assert Ho == out_extent(H, k, stride, pad) and Wo == out_extent(W, k, stride, pad)
    dx = np.empty((N, Cin, H, W), dtype=np.float64)
    _load().orc_rotconv_bwd_data(_dp(dy), _dp(w), _dp(dx), N, Cin, H, W, Cout, R, k, stride, pad)
    return dx


def rotconv_bwd_data_at(dy, w_rot, pts, H: int, W: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 13 + 15 at sampled inputs.  pts [T,4] = (n, ci, h, w) -> [T]."""
    dy = _f64(dy)
    w = _f64(w_rot)
    pts = np.ascontiguousarray(pts, dtype=np.int32)
    N, Cout, R, Ho, Wo = dy.shape
    _, _, Cin, k, _ = w.shape
    out = np.empty(pts.shape[0], dtype=np.float64)
    _load().orc_rotconv_bwd_data_at(_dp(dy), _dp(w), _ip(pts), pts.shape[0], _dp(out), N, Cin, H, W, Cout, R, k, stride, pad)
    return out


def rotconv_bwd_weight(x, dy, k: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 14 summed over the batch.  -> dw_rot [R,Cout,Cin,k,k]."""
    x = _f64(x)
    dy = _f64(dy)
    N, Cin, H, W = x.shape
    _, Cout, R, Ho, Wo = dy.shape
    dw = np.empty((R, Cout, Cin, k, k), dtype=np.float64)
    _load().orc_rotconv_bwd_weight(_dp(x), _dp(dy), _dp(dw), N, Cin, H, W, Cout, R, k, stride, pad)
    return dw


def rotconv_pool_bwd_weight_at(x, gpool, idx, pairs, R: int, k: int, pool_group: Optional[int] = None,
                               stride: int = 1, pad: int = 0) -> np.ndarray:
    """Eq. 12 + 14 at sampled (co,ci) pairs.  pairs [T,2] -> dw_rot samples [T,R,k,k]."""
    x = _f64(x)
    g = _f64(gpool)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    pairs = np.ascontiguousarray(pairs, dtype=np.int32)
    G = R if pool_group is None else pool_group
    N, Cin, H, W = x.shape
    Cout = g.shape[1] // (R // G)
    out = np.empty((pairs.shape[0], R, k, k), dtype=np.float64)
    _load().orc_rotconv_pool_bwd_weight_at(_dp(x), _dp(g), _bp(idx), _ip(pairs), pairs.shape[0], _dp(out), N, Cin, H, W,
                                           Cout, R, G, k, stride, pad)
    return out


# ---- the whole layer, composed from the definitions above ------------------

def layer_fwd(x, w_base, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """Rotated banks -> Eq. 7 -> Eq. 10.  Returns (y, ypool, idx, w_rot)."""
    w_rot = expand_bank(w_base, R, angles_deg, mode)
    y = rotconv_fwd(x, w_rot, stride, pad)
    yp, idx = orient_maxpool_fwd(y, pool_group)
    return y, yp, idx, w_rot


def layer_bwd(x, w_base, gpool, idx, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """Eq. 12 -> Eq. 13/15 and Eq. 14/16.  Returns (dx, dw_base [B,Cout,Cin,k,k])."""
    x = _f64(x)
    w_rot = expand_bank(w_base, R, angles_deg, mode)
    k = w_rot.shape[-1]
    dy = orient_maxpool_bwd(gpool, idx, R, pool_group)
    dx = rotconv_bwd_data(dy, w_rot, x.shape[2], x.shape[3], stride, pad)
    dw_rot = rotconv_bwd_weight(x, dy, k, stride, pad)
    dw = reduce_bank_grad(dw_rot, angles_deg, mode)
    return dx, dw


def layer_fwd_avg(x, w_base, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """Rotated banks -> Eq. 7 -> Eq. 9.  Returns (y, ypool, w_rot)."""
    w_rot = expand_bank(w_base, R, angles_deg, mode)
    y = rotconv_fwd(x, w_rot, stride, pad)
    return y, orient_avgpool_fwd(y, pool_group), w_rot


def layer_bwd_avg(x, w_base, gpool, R, angles_deg=None, mode="exact90", stride=1, pad=0, pool_group=None):
    """Eq. 11 -> Eq. 13/15 and Eq. 14/16.  Returns (dx, dw_base [B,Cout,Cin,k,k])."""
    x = _f64(x)
    w_rot = expand_bank(w_base, R, angles_deg, mode)
    k = w_rot.shape[-1]
    dy = orient_avgpool_bwd(gpool, R, pool_group)
    dx = rotconv_bwd_data(dy, w_rot, x.shape[2], x.shape[3], stride, pad)
    dw = reduce_bank_grad(rotconv_bwd_weight(x, dy, k, stride, pad), angles_deg, mode)
    return dx, dw


def steerable_reg(w, eps: float = 1e-8):
    """Regularisers of the steerable pair (Sec. III-D, Eq. 19 and Eq. 20) and their gradients.
    w [2,Cout,Cin,k,k] (f_x then f_y); filter b = output filter b flattened over (Cin,k,k), B = Cout.
    Returns (L_mag, L_orth, dL_mag/dw, dL_orth/dw).  A zero-norm filter gets a zero gradient for the terms that
    divide by that norm."""
    w = _f64(w)
    B = w.shape[1]
    wx, wy = w[0].reshape(B, -1), w[1].reshape(B, -1)
    l_mag = l_orth = 0.0
    g_mag, g_orth = np.zeros((2,) + wx.shape), np.zeros((2,) + wx.shape)
    for b in range(B):
        nx, ny = np.sqrt(np.sum(wx[b] ** 2)), np.sqrt(np.sum(wy[b] ** 2))
        dot = float(np.sum(wx[b] * wy[b]))
        diff = nx - ny
        l_mag += diff ** 2 / B
        ux = wx[b] / nx if nx > 0 else 0.0 * wx[b]
        uy = wy[b] / ny if ny > 0 else 0.0 * wy[b]
        g_mag[0, b] = 2.0 * diff * ux / B
        g_mag[1, b] = -2.0 * diff * uy / B
        den = nx * ny + eps
        c = dot / den
        l_orth += c ** 2 / B
        g_orth[0, b] = 2.0 * c * (wy[b] / den - dot * ny * ux / den ** 2) / B
        g_orth[1, b] = 2.0 * c * (wx[b] / den - dot * nx * uy / den ** 2) / B
    return l_mag, l_orth, g_mag.reshape(w.shape), g_orth.reshape(w.shape)
