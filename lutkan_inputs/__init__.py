"""Seeded synthetic inputs for LUT-KAN layers (shared by the CPU oracle's tests and the HIP path).

This module only draws random numbers and lays out knot grids. It contains none of the
method's arithmetic (no spline evaluation, no quantisation, no lookup), so that the oracle
and the HIP library, which share no code, can still be fed bit-identical inputs.

The workloads mirror the shapes the paper measures on (Sec. 6.2 "Models and Experimental
Cases": randomly initialised KAN layers, grid G, cubic splines, batches of fp32 rows), scaled
up to GPU-sized layers.  Everything is synthetic: the paper's CICIDS2017 case study (Sec. 8)
is represented by its tabular *shape* only (78 standardised features, heavy tails).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

SYM_INT8 = 0      # symmetric int8 scheme, Sec. 4.4
ASYM_UINT8 = 1    # asymmetric uint8 scheme, Sec. 4.4
HALF_OPEN = 0     # boundary_mode, Sec. 5.2
CLOSED = 1
CLIP_X = 0        # oob_policy, Sec. 5.4
ZERO_SPLINE = 1


def uniform_ext_knots(a: float, b: float, G: int, p: int = 3) -> np.ndarray:
    """Extended uniform knot vector tau[0..G+2p] (fp32) whose interior grid tau[p..p+G] spans [a,b].

    Each entry is computed in fp64 as a + (r-p)*(b-a)/G and rounded once to fp32, so the
    PyKAN-style extension by p intervals on both sides shares the spacing of the domain grid.
    """
    r = np.arange(G + 2 * p + 1, dtype=np.float64)
    return (np.float64(a) + (r - p) * (np.float64(b) - np.float64(a)) / np.float64(G)).astype(np.float32)


def nonuniform_ext_knots(rng: np.random.Generator, a: float, b: float, G: int, p: int = 3) -> np.ndarray:
    """Strictly increasing, non-uniform extended knot vector with tau[p]=a, tau[p+G]=b (fp32)."""
    gaps = rng.uniform(0.5, 1.5, size=G + 2 * p)
    pos = np.concatenate([[0.0], np.cumsum(gaps)])
    lo, hi = pos[p], pos[p + G]
    tau = (a + (pos - lo) * (b - a) / (hi - lo)).astype(np.float32)
    tau[p] = np.float32(a)
    tau[p + G] = np.float32(b)
    assert np.all(np.diff(tau) > 0)
    return tau


@dataclass
class LayerSpec:
    d: int
    m: int
    G: int
    p: int
    ext_knots: np.ndarray      # [G+2p+1] fp32, or [d][G+2p+1] with per_input
    coef: np.ndarray           # [d][m][G+p] fp32
    L: int
    scheme: int
    boundary: int
    oob: int
    edge_scales: object = None    # None (value_repr = phi) or (s_base, s_spline, s_out), each [d][m] fp32 (Eq. 2)
    per_input: bool = False       # one knot vector per input dimension (Sec. 6.2 "shared per input dimension")


@dataclass
class Workload:
    name: str
    layers: List[LayerSpec]
    x: np.ndarray              # [B][d0] fp32
    note: str = ""
    meta: dict = field(default_factory=dict)


def _layers(rng, widths, G, lo, hi, coef_std, L, scheme, boundary, oob, p=3):
    out = []
    for d, m in zip(widths[:-1], widths[1:]):
        std = coef_std(d) if callable(coef_std) else coef_std
        coef = rng.normal(0.0, std, size=(d, m, G + p)).astype(np.float32)
        out.append(LayerSpec(d, m, G, p, uniform_ext_knots(lo, hi, G, p), coef, L, scheme, boundary, oob))
    return out


def cfg1(seed: int = 0, B: int = 1024) -> Workload:
    """4->3, G=5 on [-1,1], coef~N(0,1), L=16 symmetric int8, x~U(-1.2,1.2), closed+clip_x."""
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = _layers(rng, [4, 3], 5, -1.0, 1.0, 1.0, 16, SYM_INT8, CLOSED, CLIP_X)
    x = rng.uniform(-1.2, 1.2, size=(B, 4)).astype(np.float32)
    return Workload("cfg1_4x3_G5_L16_sym", layers, x)


def cfg2(seed: int = 0, B: int = 65536) -> Workload:
    """[78,16,2] tabular shape, G=5 on [-3,3], coef~N(0,sd 0.5), L=64 asymmetric uint8.

    x: per element N(0,1) with probability 0.9, Student-t(nu=3) with probability 0.1.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = _layers(rng, [78, 16, 2], 5, -3.0, 3.0, 0.5, 64, ASYM_UINT8, CLOSED, CLIP_X)
    g = rng.normal(0.0, 1.0, size=(B, 78))
    t = rng.standard_t(3.0, size=(B, 78))
    pick = rng.random(size=(B, 78)) < 0.1
    x = np.where(pick, t, g).astype(np.float32)
    return Workload("cfg2_78x16x2_G5_L64_asym", layers, x)


def cfg3(seed: int = 0, L: int = 64, scheme: int = SYM_INT8, B: int = 16384, d: int = 256, m: int = 256) -> Workload:
    """256->256, G=8 on [-1,1], coef~N(0,1), x~U(-1,1); one point of the L x scheme sweep."""
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = _layers(rng, [d, m], 8, -1.0, 1.0, 1.0, L, scheme, CLOSED, CLIP_X)
    x = rng.uniform(-1.0, 1.0, size=(B, d)).astype(np.float32)
    return Workload(f"cfg3_{d}x{m}_G8_L{L}_{'sym' if scheme == SYM_INT8 else 'asym'}", layers, x)


def cfg4(seed: int = 0, B: int = 32768, d: int = 1024, m: int = 1024) -> Workload:
    """1024->1024, G=10 on [-1,1], coef~N(0,1), L=64 symmetric int8; x~N(0,sd 0.5) clipped to [-1.2,1.2]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = _layers(rng, [d, m], 10, -1.0, 1.0, 1.0, 64, SYM_INT8, CLOSED, CLIP_X)
    x = np.clip(rng.normal(0.0, 0.5, size=(B, d)), -1.2, 1.2).astype(np.float32)
    return Workload(f"cfg4_{d}x{m}_G10_L64_sym_B{B}", layers, x)


def cfg5(seed: int = 0, B: int = 131072, boundary: int = CLOSED, oob: int = CLIP_X,
         widths: Tuple[int, ...] = (64, 128, 128, 64, 8)) -> Workload:
    """Deep [64,128,128,64,8], G=5 on [-1,1], coef~N(0,1/sqrt(d_l)), L=32 asymmetric uint8.

    x: with probability 0.7 U(-1,1); with probability 0.3 a Student-t(nu=2) draw redrawn until |x|>1.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = _layers(rng, list(widths), 5, -1.0, 1.0, lambda d: 1.0 / np.sqrt(d), 32, ASYM_UINT8, boundary, oob)
    d0 = widths[0]
    u = rng.uniform(-1.0, 1.0, size=(B, d0))
    t = rng.standard_t(2.0, size=(B, d0))
    bad = np.abs(t) <= 1.0
    while bad.any():
        t[bad] = rng.standard_t(2.0, size=int(bad.sum()))
        bad = np.abs(t) <= 1.0
    pick = rng.random(size=(B, d0)) < 0.3
    x = np.where(pick, t, u).astype(np.float32)
    bn = "closed" if boundary == CLOSED else "half_open"
    on = "clip_x" if oob == CLIP_X else "zero_spline"
    return Workload(f"cfg5_deep_G5_L32_asym_{bn}_{on}", layers, x)


def draw_edge_scales(rng: np.random.Generator, d: int, m: int):
    """PyKAN-style per-edge scalars of Eq. 2: s_base ~ N(0,1), s_spline ~ N(1,0.1), s_out ~ N(1,0.2)."""
    return (rng.normal(0.0, 1.0, size=(d, m)).astype(np.float32), rng.normal(1.0, 0.1, size=(d, m)).astype(np.float32),
            rng.normal(1.0, 0.2, size=(d, m)).astype(np.float32))


def case_a(seed: int = 0, L: int = 64, scheme: int = SYM_INT8, boundary: int = CLOSED, oob: int = CLIP_X,
           B: int = 1024, clip_inputs: bool = True) -> Workload:
    """The paper's controlled-sweep shape (Sec. 6.2 Case A): one layer 10->8, grid 8, cubic, value_repr =
    spline_component with SiLU; inputs N(0,1) clipped to the knot domain [-1,1] (so some sit exactly on t_K)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    layer = _layers(rng, [10, 8], 8, -1.0, 1.0, 1.0, L, scheme, boundary, oob)[0]
    layer.edge_scales = draw_edge_scales(rng, 10, 8)
    x = rng.normal(0.0, 1.0, size=(B, 10))
    x = (np.clip(x, -1.0, 1.0) if clip_inputs else x).astype(np.float32)
    return Workload(f"caseA_10x8_G8_L{L}_s{scheme}_b{boundary}_o{oob}", [layer], x)


def random_layer(seed: int, d: int, m: int, G: int, L: int, scheme: int, boundary: int, oob: int,
                 B: int, lo: float = -1.0, hi: float = 1.0, uniform: bool = True,
                 oob_frac: float = 0.15, p: int = 3, with_base: bool = False) -> Workload:
    """Property-test layer: optional non-uniform knots; x covers the domain, its exact knots and both tails."""
    rng = np.random.Generator(np.random.PCG64(seed))
    tau = uniform_ext_knots(lo, hi, G, p) if uniform else nonuniform_ext_knots(rng, lo, hi, G, p)
    coef = rng.normal(0.0, 1.0, size=(d, m, G + p)).astype(np.float32)
    span = hi - lo
    x = rng.uniform(lo - oob_frac * span, hi + oob_frac * span, size=(B, d)).astype(np.float32)
    # sprinkle exact knot values (including t_0 and t_K) and their fp32 neighbours
    grid = tau[p:p + G + 1]
    n_special = max(1, (B * d) // 16)
    idx = rng.integers(0, B * d, size=n_special)
    vals = grid[rng.integers(0, G + 1, size=n_special)]
    nudge = rng.integers(-1, 2, size=n_special)
    vals = np.where(nudge < 0, np.nextafter(vals, np.float32(-np.inf)),
                    np.where(nudge > 0, np.nextafter(vals, np.float32(np.inf)), vals)).astype(np.float32)
    x.reshape(-1)[idx] = vals
    layer = LayerSpec(d, m, G, p, tau, coef, L, scheme, boundary, oob)
    if with_base:
        layer.edge_scales = draw_edge_scales(rng, d, m)
    return Workload(f"rand_{d}x{m}_G{G}_L{L}_s{scheme}_b{boundary}_o{oob}_seed{seed}{'_sc' if with_base else ''}", [layer], x)


def per_input_layer(seed: int, d: int, m: int, G: int, L: int, scheme: int, boundary: int, oob: int, B: int,
                    oob_frac: float = 0.15, p: int = 3, with_base: bool = False) -> Workload:
    """Layer whose inputs each have their own knot vector, as after a per-feature grid update: input i has the domain
    [lo_i, hi_i] with lo_i ~ U(-3,-0.5) and width ~ U(0.5,4), uniform or (every other input) non-uniform knots; x_i
    covers that domain and both tails, with exact knot values and their fp32 neighbours sprinkled in."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = G + 2 * p + 1
    tau = np.zeros((d, n), dtype=np.float32)
    x = np.zeros((B, d), dtype=np.float32)
    for i in range(d):
        lo = float(rng.uniform(-3.0, -0.5))
        hi = lo + float(rng.uniform(0.5, 4.0))
        tau[i] = uniform_ext_knots(lo, hi, G, p) if i % 2 == 0 else nonuniform_ext_knots(rng, lo, hi, G, p)
        assert np.all(np.diff(tau[i]) > 0)
        span = hi - lo
        col = rng.uniform(lo - oob_frac * span, hi + oob_frac * span, size=B).astype(np.float32)
        n_special = max(1, B // 16)
        idx = rng.integers(0, B, size=n_special)
        vals = tau[i, p:p + G + 1][rng.integers(0, G + 1, size=n_special)]
        nudge = rng.integers(-1, 2, size=n_special)
        col[idx] = np.where(nudge < 0, np.nextafter(vals, np.float32(-np.inf)),
                            np.where(nudge > 0, np.nextafter(vals, np.float32(np.inf)), vals)).astype(np.float32)
        x[:, i] = col
    coef = rng.normal(0.0, 1.0, size=(d, m, G + p)).astype(np.float32)
    layer = LayerSpec(d, m, G, p, tau, coef, L, scheme, boundary, oob, per_input=True)
    if with_base:
        layer.edge_scales = draw_edge_scales(rng, d, m)
    return Workload(f"perinput_{d}x{m}_G{G}_L{L}_s{scheme}_b{boundary}_o{oob}_seed{seed}{'_sc' if with_base else ''}", [layer], x)
