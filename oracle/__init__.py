"""CPU oracle for RIB window attention -- TEST INFRASTRUCTURE, not product code.

Thin numpy/ctypes front end of oracle/rib_oracle.c (see that file's header for
the definition it implements and the paper passages it follows: Sec. 2.2,
Sec. 3.1 Eq. 5-6).  Only tests/, the smoke check and bench.py's cpu_baseline leg
may import this package; nothing here imports the GPU package.

All inputs are float32 numpy arrays (bf16 workloads pass their bf16 values
widened to float32); all results are float64.
"""
import ctypes
from typing import NamedTuple, Sequence

import numpy as np

from .build import build as _build

_lib = None


class Geometry(NamedTuple):
    """Problem shape in the paper's notation: grid B x H x W, `heads` heads of
    dim d, RIB rank r, window side M, cyclic shift s, and the two logit scales
    of Eq. 5 (content, positional)."""
    B: int
    H: int
    W: int
    heads: int
    d: int
    r: int
    M: int
    s: int
    scale_c: float
    scale_p: float

    @property
    def N(self):
        return self.M * self.M

    @property
    def C(self):
        return self.heads * self.d

    @property
    def n_windows(self):
        return self.B * (self.H // self.M) * (self.W // self.M)

    @property
    def n_units(self):
        return self.n_windows * self.heads


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build())
        _lib.rib_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().rib_oracle_num_threads())


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _head(g: Geometry):
    return (ctypes.c_int(g.B), ctypes.c_int(g.H), ctypes.c_int(g.W), ctypes.c_int(g.heads),
            ctypes.c_int(g.d), ctypes.c_int(g.r), ctypes.c_int(g.M), ctypes.c_int(g.s),
            ctypes.c_double(g.scale_c), ctypes.c_double(g.scale_p))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (rc={rc})")


def _grids(g, *arrs):
    return [_f32(a, (g.B, g.H, g.W, g.C)) for a in arrs]


def fwd(g: Geometry, q, k, v, f_q, f_k):
    """Full forward.  Returns (O [B,H,W,C], LSE [B*nW, heads, N]) in float64."""
    q, k, v = _grids(g, q, k, v)
    f_q, f_k = _f32(f_q, (g.heads, g.N, g.r)), _f32(f_k, (g.heads, g.N, g.r))
    O = np.zeros((g.B, g.H, g.W, g.C), np.float64)
    lse = np.zeros((g.n_windows, g.heads, g.N), np.float64)
    rc = _load().rib_oracle_fwd(*_head(g), _p(q), _p(k), _p(v), _p(f_q), _p(f_k), _p(O), _p(lse))
    _check(rc, "fwd")
    return O, lse


def fwd_units(g: Geometry, q, k, v, f_q, f_k, units: Sequence[int]):
    """Forward of selected (window, head) units u = w*heads + hd.
    Returns (O_units [n, N, d], LSE_units [n, N]) in window-local token order."""
    q, k, v = _grids(g, q, k, v)
    f_q, f_k = _f32(f_q, (g.heads, g.N, g.r)), _f32(f_k, (g.heads, g.N, g.r))
    u = np.ascontiguousarray(units, dtype=np.int64)
    O = np.zeros((len(u), g.N, g.d), np.float64)
    lse = np.zeros((len(u), g.N), np.float64)
    rc = _load().rib_oracle_fwd_units(*_head(g), _p(q), _p(k), _p(v), _p(f_q), _p(f_k),
                                      ctypes.c_int64(len(u)), _p(u), _p(O), _p(lse))
    _check(rc, "fwd_units")
    return O, lse


def bwd(g: Geometry, q, k, v, f_q, f_k, d_out):
    """Full backward.  Returns (dQ, dK, dV [B,H,W,C], dF_q, dF_k [heads,N,r])."""
    q, k, v, d_out = _grids(g, q, k, v, d_out)
    f_q, f_k = _f32(f_q, (g.heads, g.N, g.r)), _f32(f_k, (g.heads, g.N, g.r))
    dQ = np.zeros((g.B, g.H, g.W, g.C), np.float64)
    dK, dV = np.zeros_like(dQ), np.zeros_like(dQ)
    dFq = np.zeros((g.heads, g.N, g.r), np.float64)
    dFk = np.zeros_like(dFq)
    rc = _load().rib_oracle_bwd(*_head(g), _p(q), _p(k), _p(v), _p(f_q), _p(f_k), _p(d_out),
                                _p(dQ), _p(dK), _p(dV), _p(dFq), _p(dFk))
    _check(rc, "bwd")
    return dQ, dK, dV, dFq, dFk


def bwd_units(g: Geometry, q, k, v, f_q, f_k, d_out, units: Sequence[int]):
    """Backward of selected units, un-scattered: (dq, dk, dv [n,N,d], and the
    units' own contributions to dF_q, dF_k [n,N,r])."""
    q, k, v, d_out = _grids(g, q, k, v, d_out)
    f_q, f_k = _f32(f_q, (g.heads, g.N, g.r)), _f32(f_k, (g.heads, g.N, g.r))
    u = np.ascontiguousarray(units, dtype=np.int64)
    dq = np.zeros((len(u), g.N, g.d), np.float64)
    dk, dv = np.zeros_like(dq), np.zeros_like(dq)
    dfq = np.zeros((len(u), g.N, g.r), np.float64)
    dfk = np.zeros_like(dfq)
    rc = _load().rib_oracle_bwd_units(*_head(g), _p(q), _p(k), _p(v), _p(f_q), _p(f_k), _p(d_out),
                                      ctypes.c_int64(len(u)), _p(u),
                                      _p(dq), _p(dk), _p(dv), _p(dfq), _p(dfk))
    _check(rc, "bwd_units")
    return dq, dk, dv, dfq, dfk


def unit_token_index(g: Geometry, unit: int):
    """Grid coordinates (b, y[N], x[N], hd) of a unit's tokens in window-local
    order, following the same map as the C file: token n = iy*M + ix of window
    (wy, wx) sits at ((wy*M + iy + s) mod H, (wx*M + ix + s) mod W)."""
    hd = unit % g.heads
    w = unit // g.heads
    nwx, nwy = g.W // g.M, g.H // g.M
    wx, wy, b = w % nwx, (w // nwx) % nwy, w // (nwx * nwy)
    n = np.arange(g.N)
    y = (wy * g.M + n // g.M + g.s) % g.H
    x = (wx * g.M + n % g.M + g.s) % g.W
    return b, y, x, hd


def gated_fwd(g: Geometry, q, k, v, f_q, f_k, gate):
    """Forward with the convolutional-local-attention gate of the paper's Eq. 9 applied to the
    result: returns (O' = O * G, O, LSE), all float64; `gate` is a [B,H,W,C] grid."""
    O, lse = fwd(g, q, k, v, f_q, f_k)
    return O * np.asarray(gate, np.float64), O, lse


def gated_bwd(g: Geometry, q, k, v, f_q, f_k, gate, d_out_gated):
    """Backward of gated_fwd for the upstream gradient of O': product rule through Eq. 9
    (dO = dO' * G, dG = dO' * O), then the plain backward.  Returns
    (dQ, dK, dV, dF_q, dF_k, dG)."""
    O, _ = fwd(g, q, k, v, f_q, f_k)
    up = np.asarray(d_out_gated, np.float64)
    d_out = up * np.asarray(gate, np.float64)
    return (*bwd(g, q, k, v, f_q, f_k, d_out.astype(np.float32)), up * O)
