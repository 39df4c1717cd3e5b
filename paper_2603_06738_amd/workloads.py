"""Seeded synthetic inputs for RIB window attention.

This module only draws random numbers and describes shapes.  It contains none
of the method's arithmetic and imports neither the CPU oracle nor the GPU
library, so both sides can be fed the same tensors.

The five named workloads follow the shapes of the paper's SST network
(Appendix "Network implementation details": 180 channels, 6 heads, windows
16/32/64; training patches of 96x96): channel-last token grids q, k, v of
N(0, 1) values and per-head RIB features f_q, f_k of shape [heads, M*M, r] with
standard deviation 0.5.  They stand in for activations of the paper's trained
network, which are not available; attention cost does not depend on the values.

Tensors are always drawn in the order q, k, v, f_q, f_k, d_out from one Philox
stream keyed by the workload's seed.  For a bf16 workload every value is rounded
to the nearest bf16 (ties to even) and returned widened to float32, so that the
oracle and the GPU library start from bit-identical numbers.
"""
from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # "f32" or "bf16": storage type of q,k,v,f_q,f_k,O and gradients
    B: int
    H: int
    W: int
    heads: int
    d: int              # head dim; C = heads*d
    r: int              # RIB rank
    M: int              # window side; N = M*M tokens per window
    s: int              # cyclic shift
    scale_c: float      # scale of the content term q.k
    scale_p: float      # scale of the positional term f_q.f_k
    seed: int
    backward: bool = False

    @property
    def C(self):
        return self.heads * self.d

    @property
    def N(self):
        return self.M * self.M

    @property
    def n_windows(self):
        return self.B * (self.H // self.M) * (self.W // self.M)

    @property
    def n_units(self):
        return self.n_windows * self.heads

    @property
    def tokens(self):
        return self.B * self.H * self.W

    # Algorithmic work, counted on the unpadded dims (exp/max/sum not counted).
    @property
    def fwd_flop(self):
        return 2.0 * self.N * self.N * (2 * self.d + self.r) * self.n_units

    @property
    def bwd_flop(self):
        return 2.0 * self.N * self.N * (5 * self.d + 3 * self.r) * self.n_units

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def fwd_bytes(self):
        """q, k, v read once and O written once."""
        return 4.0 * self.tokens * self.C * self.elem_bytes


def _uniform_scale(d, r):
    return 1.0 / float(np.sqrt(d + r))


def _w(name, dtype, B, HW, heads, d, r, M, s, seed, backward=False):
    sc = _uniform_scale(d, r)
    return Workload(name, dtype, B, HW, HW, heads, d, r, M, s, sc, sc, seed, backward)


_SEED0 = 0x51570000

WORKLOADS: Dict[str, Workload] = {
    "c1": _w("c1", "f32", 1, 48, 2, 30, 8, 16, 0, _SEED0 + 1),
    "c2": _w("c2", "bf16", 4, 64, 6, 30, 16, 16, 8, _SEED0 + 2),
    "c3": _w("c3", "bf16", 8, 96, 6, 30, 16, 32, 0, _SEED0 + 3),
    "c3s": _w("c3s", "bf16", 8, 96, 6, 30, 16, 32, 16, _SEED0 + 3),
    "c4": _w("c4", "bf16", 1, 512, 6, 30, 16, 64, 32, _SEED0 + 4),
    "c5": _w("c5", "bf16", 16, 96, 6, 30, 16, 32, 16, _SEED0 + 5, backward=True),
}


def _eq5(name, B, HW, heads, d, r, M, seed):
    return Workload(name, "bf16", B, HW, HW, heads, d, r, M, 0, 1.0 / float(np.sqrt(d)), 1.0 / float(np.sqrt(r)),
                    seed, True)


# The attention layers of the paper's own networks (Appendix, table "Network implementation
# details"): window sides cycle per layer and the RIB rank grows in the second cycle.  One
# entry per distinct (head dim, rank, window) of the "+" variants trained on 96x96 patches,
# plus the 64-windows of the base variants; no shift (the paper's networks use none), the
# paper's two scales (Eq. 5), forward + backward, batch 16.
SCHEDULE: Dict[str, Workload] = {
    w.name: w for w in [
        _eq5("sst-m16-r18", 16, 96, 6, 30, 18, 16, _SEED0 + 101),
        _eq5("sst-m32-r18", 16, 96, 6, 30, 18, 32, _SEED0 + 102),
        _eq5("sst-m48-r18", 16, 96, 6, 30, 18, 48, _SEED0 + 103),
        _eq5("sst-m32-r34", 16, 96, 6, 30, 34, 32, _SEED0 + 104),
        _eq5("sst-m48-r34", 16, 96, 6, 30, 34, 48, _SEED0 + 105),
        _eq5("sst-m96-r34", 16, 96, 6, 30, 34, 96, _SEED0 + 106),
        _eq5("sst-m64-r34", 16, 128, 6, 30, 34, 64, _SEED0 + 107),
        _eq5("sstl-m32-r16", 16, 96, 6, 32, 16, 32, _SEED0 + 111),
        _eq5("sstl-m48-r32", 16, 96, 6, 32, 32, 48, _SEED0 + 112),
        _eq5("sstl-m96-r32", 16, 96, 6, 32, 32, 96, _SEED0 + 113),
        _eq5("light-m48-r16", 16, 96, 3, 16, 16, 48, _SEED0 + 121),
        _eq5("light-m96-r24", 16, 96, 3, 16, 24, 96, _SEED0 + 122),
    ]
}


def paper_scales(wl: Workload) -> Workload:
    """Same workload with the paper's own two scales (Eq. 5): 1/sqrt(d) on the
    content part and 1/sqrt(r) on the positional part."""
    return replace(wl, name=wl.name + "-eq5", scale_c=1.0 / float(np.sqrt(wl.d)),
                   scale_p=1.0 / float(np.sqrt(max(wl.r, 1))))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); float32 result."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of bf16-representable float32 values (int16 array)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).view(np.int16).reshape(a.shape)


def make_inputs(wl: Workload, with_dout: bool = None) -> Dict[str, np.ndarray]:
    """Draw q, k, v [B,H,W,C], f_q, f_k [heads,N,r] (and d_out [B,H,W,C]) as
    float32 arrays; bf16 workloads are already rounded to bf16 values."""
    if with_dout is None:
        with_dout = wl.backward
    rng = np.random.Generator(np.random.Philox(key=wl.seed))
    grid = (wl.B, wl.H, wl.W, wl.C)
    feat = (wl.heads, wl.N, wl.r)
    out = {}
    for name in ("q", "k", "v"):
        out[name] = rng.standard_normal(grid, dtype=np.float32)
    for name in ("f_q", "f_k"):
        out[name] = 0.5 * rng.standard_normal(feat, dtype=np.float32)
    if with_dout:
        out["d_out"] = rng.standard_normal(grid, dtype=np.float32)
    if wl.dtype == "bf16":
        out = {n: round_to_bf16(a) for n, a in out.items()}
    return out


def custom(name, dtype, B, H, W, heads, d, r, M, s, seed, scale_c=None, scale_p=None,
           backward=False) -> Workload:
    """A free-form workload for parity tests (ragged sizes, tiny windows, ...)."""
    sc = _uniform_scale(d, r)
    return Workload(name, dtype, B, H, W, heads, d, r, M, s,
                    sc if scale_c is None else scale_c,
                    sc if scale_p is None else scale_p, seed, backward)


def make_generator_params(heads: int, r: int, L: int = 10, d_h: int = 32, seed: int = _SEED0 + 900) -> Dict[str, np.ndarray]:
    """Random parameters of the RIB feature generator (paper Sec. 3.1 Eq. 2-3; L = 10 and
    d_h = 32 are the paper's settings): W_h [2+4L, d_h], b_h [d_h], W_pq, W_pk [heads, d_h, r],
    float32, drawn in that order from one Philox stream; the standard deviations only keep
    the generated features at the size of the attention workloads' (about 0.5)."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    n_in = 2 + 4 * L
    out = {
        "W_h": rng.standard_normal((n_in, d_h), dtype=np.float32) * np.float32(1.0 / np.sqrt(n_in)),
        "b_h": rng.standard_normal((d_h,), dtype=np.float32) * np.float32(0.1),
        "W_pq": rng.standard_normal((heads, d_h, r), dtype=np.float32) * np.float32(0.25),
        "W_pk": rng.standard_normal((heads, d_h, r), dtype=np.float32) * np.float32(0.25),
    }
    return out


def make_feature_grads(heads: int, M: int, r: int, seed: int = _SEED0 + 901) -> Dict[str, np.ndarray]:
    """Upstream gradients df_q, df_k [heads, M*M, r] (float32, N(0,1)) for generator tests."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    shape = (heads, M * M, r)
    return {"df_q": rng.standard_normal(shape, dtype=np.float32), "df_k": rng.standard_normal(shape, dtype=np.float32)}


def make_gate(wl: Workload, seed_offset: int = 0x4000) -> np.ndarray:
    """A synthetic CLA gate G [B,H,W,C] (paper Eq. 8-9): uniform in (0, 1), the range of the
    sigmoid that produces it; rounded to bf16 for bf16 workloads.  Its own Philox stream, so the
    other tensors of the workload do not change."""
    rng = np.random.Generator(np.random.Philox(key=wl.seed + seed_offset))
    g = rng.random((wl.B, wl.H, wl.W, wl.C), dtype=np.float32)
    return round_to_bf16(g) if wl.dtype == "bf16" else g
