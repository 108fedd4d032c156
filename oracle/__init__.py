"""ctypes front-end of the CPU oracle (oracle/lutkan_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline leg
of the benchmark.  Nothing in the product package imports this module, and this module imports
nothing from the product package.  It only marshals numpy arrays into the C functions; all of
the method's arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# The two overrides exist for tests/test_oracle_mutations.py, which builds deliberately broken copies of
# the C file and checks that the pin tests reject them.
_SRC = os.environ.get("LUTKAN_ORACLE_SRC", os.path.join(_HERE, "lutkan_oracle.c"))
_LIB = os.environ.get("LUTKAN_ORACLE_LIB", os.path.join(_HERE, "liblutkan_oracle.so"))

SYM_INT8, ASYM_UINT8 = 0, 1
HALF_OPEN, CLOSED = 0, 1
CLIP_X, ZERO_SPLINE = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction: every fp32 step rounds once."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=gnu11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.lko_bspline_basis.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_void_p]
        L.lko_bspline_basis.restype = None
        L.lko_spline_value.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_double]
        L.lko_spline_value.restype = C.c_double
        L.lko_sample_x.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.lko_sample_x.restype = C.c_double
        L.lko_quantize_segment.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.lko_quantize_segment.restype = None
        L.lko_compile.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 5 + [C.c_int]
        L.lko_compile.restype = C.c_int
        L.lko_lut_forward.argtypes = ([C.c_int] * 7 + [C.c_void_p, C.c_int] + [C.c_void_p] * 7 + [C.c_long] + [C.c_void_p] * 8 + [C.c_int])
        L.lko_lut_forward.restype = C.c_int
        L.lko_bspline_forward.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_int] + [C.c_void_p] * 4 + [C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                                           C.c_long, C.c_void_p, C.c_void_p, C.c_int]
        L.lko_silu.argtypes = [C.c_float]
        L.lko_silu.restype = C.c_float
        L.lko_bspline_forward.restype = C.c_int
        L.lko_artifact_bytes.argtypes = [C.c_long, C.c_int, C.c_int, C.c_int]
        L.lko_artifact_bytes.restype = C.c_long
        L.lko_max_threads.restype = C.c_int
        L.lko_round_to_fp16.argtypes = [C.c_float]
        L.lko_round_to_fp16.restype = C.c_float
        L.lko_round_params_fp16.argtypes = [C.c_void_p, C.c_long]
        L.lko_round_params_fp16.restype = C.c_long
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def default_threads() -> int:
    return max(1, min(lib().lko_max_threads(), os.cpu_count() or 1))


def bspline_basis(tau, p: int, x: float) -> np.ndarray:
    """All B_{r,p}(x), r = 0..n-2-p, for knot vector tau (Eq. 4-5)."""
    tau = np.ascontiguousarray(tau, dtype=np.float64)
    n = tau.size
    N = np.zeros(n - 1, dtype=np.float64)
    lib().lko_bspline_basis(_p(tau), n, p, float(x), _p(N))
    return N[: n - 1 - p].copy()


def spline_value(ext_knots, p: int, coef, x: float) -> float:
    """s(x) of Eq. 3 for one edge; ext_knots fp32 [G+2p+1], coef fp32 [G+p]."""
    tau = _f32(ext_knots)
    c = _f32(coef)
    G = tau.size - 2 * p - 1
    assert c.size == G + p
    return float(lib().lko_spline_value(_p(tau), G, p, _p(c), float(x)))


def sample_x(knots, L: int, k: int, l: int) -> float:
    T = _f32(knots)
    return float(lib().lko_sample_x(_p(T), L, k, l))


def quantize_segment(v, scheme: int):
    v = _f32(v)
    q = np.zeros(v.size, dtype=np.int8 if scheme == SYM_INT8 else np.uint8)
    a = np.zeros(1, dtype=np.float32)
    y0 = np.zeros(1, dtype=np.float32)
    lib().lko_quantize_segment(_p(v), v.size, scheme, _p(q), _p(a), _p(y0))
    return q, np.float32(a[0]), np.float32(y0[0])


def round_to_fp16(x: float) -> float:
    return float(lib().lko_round_to_fp16(float(np.float32(x))))


def compile_layer(d, m, G, p, ext_knots, coef, L, scheme, want_v=False, nthreads=None, param_fp16=False, extended=False,
                  per_input=False):
    """Artifact arrays of Sec. 4.6: knots [K+1], q [E,K,L] (e=i*m+j), scale [E,K], y_min [E,K].
    param_fp16: scale and y_min are stored rounded to binary16 (held here as fp32 arrays of those values).
    extended: the LUT covers every interval of the extended knot vector, K = G + 2p (else the domain grid, K = G).
    per_input: ext_knots is [d, G+2p+1], one knot vector per input dimension, and knots comes back as [d, K+1]."""
    tau = _f32(ext_knots)
    coef = _f32(coef)
    assert tau.size == (d if per_input else 1) * (G + 2 * p + 1) and coef.size == d * m * (G + p)
    E, K = d * m, (G + 2 * p if extended else G)
    q = np.zeros((E, K, L), dtype=np.int8 if scheme == SYM_INT8 else np.uint8)
    scale = np.zeros((E, K), dtype=np.float32)
    y_min = np.zeros((E, K), dtype=np.float32)
    knots = np.zeros((d, K + 1) if per_input else K + 1, dtype=np.float32)
    v = np.zeros((E, K, L), dtype=np.float32) if want_v else None
    rc = lib().lko_compile(d, m, G, p, _p(tau), _p(coef), L, scheme, int(bool(extended)), int(bool(per_input)), _p(q), _p(scale), _p(y_min), _p(knots), _p(v),
                           nthreads or default_threads())
    if rc != 0:
        raise ValueError(f"lko_compile failed: {rc}")
    if param_fp16:
        lost = lib().lko_round_params_fp16(_p(scale), scale.size) + lib().lko_round_params_fp16(_p(y_min), y_min.size)
        if lost:
            raise ValueError(f"{lost} dequantisation parameters do not fit binary16")
    return SimpleNamespace(d=d, m=m, K=K, L=L, scheme=scheme, knots=knots, q=q, scale=scale, y_min=y_min, v=v,
                           param_fp16=bool(param_fp16), per_input=bool(per_input))


def _edge_scalars(edge_scalars, E):
    """None (value_repr = phi) or the three per-edge fp32 arrays (s_base, s_spline, s_out) of Eq. 2, each [E]."""
    if edge_scalars is None:
        return None, None, None
    sb, ss, so = (_f32(a).reshape(-1) for a in edge_scalars)
    assert sb.size == E and ss.size == E and so.size == E
    return sb, ss, so


def silu(x: float) -> float:
    return float(lib().lko_silu(float(np.float32(x))))


def lut_forward(art, boundary, oob, x, trace=False, codes=False, nthreads=None, edge_scalars=None):
    """Layer forward on the artifact.  Returns y fp32 [B,m], A fp64 [B,m], and optionally the trace.
    edge_scalars = (s_base, s_spline, s_out) switches to value_repr = spline_component."""
    x = _f32(x)
    B = x.shape[0]
    d, m = art.d, art.m
    assert x.shape == (B, d)
    y = np.zeros((B, m), dtype=np.float32)
    A = np.zeros((B, m), dtype=np.float64)
    k = l0 = inn = w = q01 = None
    if trace:
        k = np.zeros((B, d), dtype=np.int32)
        l0 = np.zeros((B, d), dtype=np.int32)
        inn = np.zeros((B, d), dtype=np.uint8)
        w = np.zeros((B, d), dtype=np.float32)
    if codes:
        q01 = np.zeros((B, d, m, 2), dtype=np.int16)
    stats = np.zeros(2, dtype=np.uint64)
    sb, ss, so = _edge_scalars(edge_scalars, d * m)
    rc = lib().lko_lut_forward(d, m, art.K, art.L, art.scheme, boundary, oob,
                               _p(art.knots), int(getattr(art, "per_input", False)), _p(art.q), _p(art.scale), _p(art.y_min), _p(sb), _p(ss), _p(so), _p(x), B,
                               _p(y), _p(A), _p(k), _p(l0), _p(inn), _p(w), _p(q01), _p(stats),
                               nthreads or default_threads())
    if rc != 0:
        raise ValueError(f"lko_lut_forward failed: {rc}")
    return SimpleNamespace(y=y, A=A, k=k, l0=l0, inside=inn, w=w, q01=q01,
                           oob_count=int(stats[0]), oob_any_rows=int(stats[1]))


def bspline_forward(d, m, G, p, ext_knots, coef, boundary, oob, x, nthreads=None, edge_scalars=None, extended=False,
                    per_input=False):
    tau = _f32(ext_knots)
    assert tau.size == (d if per_input else 1) * (G + 2 * p + 1)
    coef = _f32(coef)
    x = _f32(x)
    B = x.shape[0]
    y = np.zeros((B, m), dtype=np.float32)
    A = np.zeros((B, m), dtype=np.float64)
    sb, ss, so = _edge_scalars(edge_scalars, d * m)
    rc = lib().lko_bspline_forward(d, m, G, p, _p(tau), int(bool(per_input)), _p(coef), _p(sb), _p(ss), _p(so), boundary, oob, int(bool(extended)), _p(x), B, _p(y), _p(A),
                                   nthreads or default_threads())
    if rc != 0:
        raise ValueError(f"lko_bspline_forward failed: {rc}")
    return SimpleNamespace(y=y, A=A)


def artifact_bytes(E: int, K: int, L: int, param_bytes_per_segment: int) -> int:
    return int(lib().lko_artifact_bytes(E, K, L, param_bytes_per_segment))


def error_stats(y, y_ref, x, t0, tK, boundary):
    """OOB evaluation protocol of Sec. 5.6 written out: a sample (row) is in-range when every input satisfies the
    domain predicate In(x) of Sec. 5.2 (half_open: t0 <= x < tK, closed: t0 <= x <= tK; NaN is outside), else it is
    in the OOB-only subset; OOB_any_frac is the share of rows in the second subset.  t0 and tK are scalars, or [d]
    arrays when every input has its own domain.  Per subset: number of rows, and over the outputs of its rows, in fp64,
    the sum, the maximum and the mean (MAE, Sec. 6.5) of |y - y_ref|.  A difference that is NaN is counted (nan_in,
    nan_oob) and left out of all three, so MAE = sum / (rows * m - nan): the mean of the differences that exist, NaN
    when there is none."""
    x = _f32(x)
    y = np.asarray(y, dtype=np.float32).astype(np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float32).astype(np.float64)
    t0, tK = np.asarray(t0, dtype=np.float32), np.asarray(tK, dtype=np.float32)
    inside = (x >= t0) & ((x <= tK) if boundary == CLOSED else (x < tK))
    row_in = inside.all(axis=1)
    err = np.abs(y - y_ref)
    out = {"rows_in": int(row_in.sum()), "rows_oob": int((~row_in).sum()), "oob_any_frac": float((~row_in).sum() / x.shape[0])}
    nan = np.isnan(err)
    for name, rows in (("in", row_in), ("oob", ~row_in)):
        e = err[rows][~nan[rows]]                       # the subset's differences that exist
        out["nan_" + name] = int(nan[rows].sum())
        out["sum_abs_" + name] = float(e.sum()) if e.size else 0.0
        out["max_abs_" + name] = float(e.max()) if e.size else 0.0
        out["mae_" + name] = float(e.sum() / e.size) if e.size else float("nan")
    return out
