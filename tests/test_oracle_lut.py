"""Pins for the oracle's LUT compile + forward (Sec. 4.2-4.5, Sec. 5) against facts the paper and
the arithmetic fix: sampling positions, code-range invariants, the boundary special cases stated in
the text, numpy.searchsorted, closed forms for constant and linear edge functions, brute force on a
tiny layer, and the trend in L of Table 1.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import ASYM_UINT8, CLIP_X, CLOSED, HALF_OPEN, SYM_INT8, ZERO_SPLINE
from lutkan_inputs import cfg1, nonuniform_ext_knots, random_layer, uniform_ext_knots

P = 3
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _greville(tau):
    t = tau.astype(np.float64)
    return np.array([(t[r + 1] + t[r + 2] + t[r + 3]) / 3.0 for r in range(tau.size - P - 1)])


def _compile_spec(s, want_v=False):
    return oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, want_v=want_v)


# ---------------------------------------------------------------- sampling (Eq. 7)
def test_sampling_positions():
    T = uniform_ext_knots(-1.0, 1.0, 5)[P:P + 6]
    for L in (2, 16, 64):
        for k in range(5):
            assert oracle.sample_x(T, L, k, 0) == float(T[k])                      # x_{k,0} = t_k exactly
            delta = (float(T[k + 1]) - float(T[k])) / L
            last = oracle.sample_x(T, L, k, L - 1)
            assert abs(last - (float(T[k + 1]) - delta)) <= 1e-15                  # x_{k,L-1} = t_{k+1} - Delta_k
            assert last < float(T[k + 1])                                          # right end never sampled


def test_compiled_samples_are_the_spline_at_the_sampling_positions():
    w = random_layer(3, 2, 3, 6, 8, SYM_INT8, CLOSED, CLIP_X, B=4, uniform=False)
    s = w.layers[0]
    art = _compile_spec(s, want_v=True)
    np.testing.assert_array_equal(art.knots, s.ext_knots[P:P + s.G + 1])
    for e in range(s.d * s.m):
        i, j = divmod(e, s.m)
        for k in range(s.G):
            for l in range(s.L):
                xs = oracle.sample_x(art.knots, s.L, k, l)
                assert art.v[e, k, l] == np.float32(oracle.spline_value(s.ext_knots, P, s.coef[i, j], xs))


# ---------------------------------------------------------------- quantisation (Eq. 10-12)
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_quantisation_invariants(scheme):
    rng = np.random.Generator(np.random.PCG64(21))
    for trial in range(200):
        L = int(rng.choice([2, 3, 16, 64, 128]))
        v = (rng.normal(size=L) * 10.0 ** rng.uniform(-3, 2) + rng.normal() * (trial % 3)).astype(np.float32)
        q, a, y0 = oracle.quantize_segment(v, scheme)
        deq = (np.float32(y0) + np.float32(a) * q.astype(np.float32)).astype(np.float32)
        assert a > 0
        # each dequantised sample is within half a step (plus a rounding) of the float sample
        assert np.all(np.abs(deq.astype(np.float64) - v) <= 0.5 * float(a) * (1 + 1e-5) + 1e-30)
        if scheme == SYM_INT8:
            assert y0 == 0.0 and q.dtype == np.int8
            assert q.min() >= -127 and q.max() <= 127                       # -128 is never produced
            assert abs(int(q[np.argmax(np.abs(v))])) == 127                 # the arg-max |v| sample saturates
            np.testing.assert_allclose(float(a), float(np.abs(v).max()) / 127.0, rtol=1e-6)
        else:
            assert q.dtype == np.uint8
            assert y0 == v.min()                                            # y_min = min_l v exactly
            assert q[np.argmin(v)] == 0 and q[np.argmax(v)] == 255
            np.testing.assert_allclose(float(a), (float(v.max()) - float(v.min())) / 255.0, rtol=1e-6)


def test_symmetric_codes_negate_with_the_values():
    rng = np.random.Generator(np.random.PCG64(22))
    v = rng.normal(size=64).astype(np.float32)
    q, a, _ = oracle.quantize_segment(v, SYM_INT8)
    qn, an, _ = oracle.quantize_segment(-v, SYM_INT8)
    np.testing.assert_array_equal(qn, -q)
    assert a == an


@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_zero_range_segment(scheme):
    for c in (0.0, 1.25, -3.0):
        v = np.full(16, c, dtype=np.float32)
        q, a, y0 = oracle.quantize_segment(v, scheme)
        deq = np.float32(y0) + np.float32(a) * q.astype(np.float32)
        if scheme == ASYM_UINT8 or c == 0.0:
            assert a == 1.0 and np.all(q == 0)                              # degenerate range: alpha = 1, codes 0
            assert np.all(deq == np.float32(c))
        else:
            assert np.all(np.abs(q) == 127)                                 # symmetric constant: +-127 * (|c|/127)
            assert np.all(np.abs(deq - np.float32(c)) <= np.spacing(np.float32(abs(c))))


def test_round_half_to_even():
    # values at exactly k + 0.5 steps of alpha = 1 (max = 255): codes go to the even neighbour
    v = np.array([0.0, 0.5, 1.5, 2.5, 3.5, 255.0], dtype=np.float32)
    q, a, y0 = oracle.quantize_segment(v, ASYM_UINT8)
    assert a == 1.0 and y0 == 0.0
    np.testing.assert_array_equal(q, [0, 0, 2, 2, 4, 255])
    v = np.array([0.5, -0.5, 1.5, -2.5, 127.0], dtype=np.float32)
    q, a, _ = oracle.quantize_segment(v, SYM_INT8)
    assert a == 1.0
    np.testing.assert_array_equal(q, [0, 0, 2, -2, 127])


def test_artifact_bytes_matches_table9():
    rows = [l.split() for l in open(os.path.join(GOLD, "table9_artifact_bytes.txt")) if l[0] != "#"]
    total = 0
    for E, K, L, nbytes in rows:
        got = oracle.artifact_bytes(int(E), int(K), int(L), 4)
        assert got == int(nbytes)
        total += got
    assert total == 2262096                                                   # "LUT Total" row of Table 9
    art = _compile_spec(cfg1().layers[0])
    assert art.q.nbytes + art.scale.nbytes + art.y_min.nbytes + art.knots.nbytes == oracle.artifact_bytes(12, 5, 16, 8)


# ---------------------------------------------------------------- indexing (Eq. 13-16, Sec. 5.2-5.3)
def _one_edge_art(tau, L, scheme, coef=None):
    G = tau.size - 2 * P - 1
    if coef is None:
        coef = np.random.Generator(np.random.PCG64(31)).normal(size=G + P)
    return oracle.compile_layer(1, 1, G, P, tau, np.asarray(coef, dtype=np.float32), L, scheme)


@pytest.mark.parametrize("uniform", [True, False])
@pytest.mark.parametrize("L", [2, 16, 33, 64])
def test_special_points(uniform, L):
    rng = np.random.Generator(np.random.PCG64(5))
    tau = uniform_ext_knots(-1.0, 1.0, 5) if uniform else nonuniform_ext_knots(rng, -1.0, 1.0, 5)
    art = _one_edge_art(tau, L, SYM_INT8)
    T, K = art.knots, art.K
    for boundary in (HALF_OPEN, CLOSED):
        x = T[:K].reshape(-1, 1)
        r = oracle.lut_forward(art, boundary, CLIP_X, x, trace=True)
        np.testing.assert_array_equal(r.k[:, 0], np.arange(K))                 # x = t_k -> (k, 0, w=0)
        assert np.all(r.l0 == 0) and np.all(r.w == 0) and np.all(r.inside == 1)
        lo = np.array([[T[0] - 1.0], [np.nextafter(T[0], np.float32(-np.inf))], [-np.inf]], dtype=np.float32)
        r = oracle.lut_forward(art, boundary, CLIP_X, lo, trace=True)
        assert np.all(r.k == 0) and np.all(r.l0 == 0) and np.all(r.w == 0) and np.all(r.inside == 0)
    tK = np.array([[T[K]]], dtype=np.float32)
    r = oracle.lut_forward(art, CLOSED, CLIP_X, tK, trace=True)                  # Sec. 4.2: last index, last segment
    assert (r.k[0, 0], r.l0[0, 0], r.w[0, 0], r.inside[0, 0]) == (K - 1, L - 1, 0.0, 1)
    r = oracle.lut_forward(art, HALF_OPEN, CLIP_X, tK, trace=True)               # Sec. 5.5: OOB yet safely indexed
    assert r.inside[0, 0] == 0 and r.k[0, 0] == K - 1 and r.l0[0, 0] <= L - 1 and r.oob_count == 1
    below = np.nextafter(T[K], np.float32(-np.inf)).reshape(1, 1)
    r2 = oracle.lut_forward(art, HALF_OPEN, CLIP_X, below, trace=True)
    assert r2.inside[0, 0] == 1 and r2.y[0, 0] == r.y[0, 0] and r2.l0[0, 0] == r.l0[0, 0] and r2.w[0, 0] == r.w[0, 0]
    hi = np.array([[T[K] + 0.5], [np.inf]], dtype=np.float32)
    for boundary in (HALF_OPEN, CLOSED):
        r = oracle.lut_forward(art, boundary, CLIP_X, hi, trace=True)
        assert np.all(r.k == K - 1) and np.all(r.inside == 0)


def _neighbourhood(v, n):
    out = [np.float32(v)]
    a = b = np.float32(v)
    for _ in range(n):
        a = np.nextafter(a, np.float32(-np.inf))
        b = np.nextafter(b, np.float32(np.inf))
        out += [a, b]
    return np.array(sorted(out), dtype=np.float32)


@pytest.mark.parametrize("uniform", [True, False])
def test_segment_index_every_float_near_every_knot_vs_numpy_searchsorted(uniform):
    rng = np.random.Generator(np.random.PCG64(6))
    tau = uniform_ext_knots(-1.0, 1.0, 10) if uniform else nonuniform_ext_knots(rng, -2.0, 3.0, 7)
    L = 64
    art = _one_edge_art(tau, L, ASYM_UINT8)
    T, K = art.knots, art.K
    xs = np.concatenate([_neighbourhood(t, 300) for t in T] + [rng.uniform(T[0] - 1, T[K] + 1, 5000).astype(np.float32)])
    for boundary in (HALF_OPEN, CLOSED):
        r = oracle.lut_forward(art, boundary, CLIP_X, xs.reshape(-1, 1), trace=True)
        tKs = T[K] if boundary == CLOSED else np.nextafter(T[K], np.float32(-np.inf))
        xc = np.minimum(np.maximum(xs, T[0]), tKs)
        k_ref = np.clip(np.searchsorted(T, xc, side="right") - 1, 0, K - 1)       # Eq. 14 via the library routine
        np.testing.assert_array_equal(r.k[:, 0], k_ref)
        inside_ref = (xs >= T[0]) & ((xs <= T[K]) if boundary == CLOSED else (xs < T[K]))
        np.testing.assert_array_equal(r.inside[:, 0].astype(bool), inside_ref)
        # the located segment really contains x' and (l0, w) reassemble z = u (L-1) within [0, L-1]
        assert np.all(T[r.k[:, 0]] <= xc) and np.all((xc < T[r.k[:, 0] + 1]) | ((xc == T[K]) & (r.k[:, 0] == K - 1)))
        z = r.l0[:, 0] + r.w[:, 0].astype(np.float64)
        u = (xc.astype(np.float64) - T[r.k[:, 0]]) / (T[r.k[:, 0] + 1].astype(np.float64) - T[r.k[:, 0]])
        assert np.all(np.abs(z - u * (L - 1)) <= 1e-4)
        assert np.all((r.l0 >= 0) & (r.l0 <= L - 1) & (r.w >= 0) & (r.w < 1))
        assert r.oob_count == int((~inside_ref).sum())


def test_boundary_modes_differ_only_at_tK():
    w = random_layer(9, 3, 2, 5, 16, SYM_INT8, CLOSED, CLIP_X, B=4096)
    art = _compile_spec(w.layers[0])
    tK = art.knots[-1]
    a = oracle.lut_forward(art, CLOSED, CLIP_X, w.x, trace=True)
    b = oracle.lut_forward(art, HALF_OPEN, CLIP_X, w.x, trace=True)
    differs = a.inside != b.inside
    assert differs.any()                                   # the generator plants exact t_K values
    assert np.all(w.x[differs] == tK) and np.all((w.x == tK) == differs)


# ---------------------------------------------------------------- interpolation + dequantisation (Eq. 10, 17)
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_w_zero_returns_the_dequantised_code_exactly(scheme):
    tau = uniform_ext_knots(-1.0, 1.0, 4)            # h = 0.5: sample lookups with w = 0 are exact in fp32
    L = 17                                            # L-1 = 16 so that u = l/16 is exact
    art = _one_edge_art(tau, L, scheme)
    T = art.knots
    for k in range(4):
        for l in range(L - 1):
            x = np.float32(T[k] + np.float32(0.5) * np.float32(l / 16.0)).reshape(1, 1)
            r = oracle.lut_forward(art, CLOSED, CLIP_X, x, trace=True, codes=True)
            assert (r.k[0, 0], r.l0[0, 0], r.w[0, 0]) == (k, l, 0.0)
            code = art.q[0, k, l]
            assert r.q01[0, 0, 0, 0] == int(code)
            assert r.y[0, 0] == np.float32(art.y_min[0, k] + np.float32(art.scale[0, k] * np.float32(code)))


@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_output_lies_between_the_two_dequantised_neighbours(scheme):
    w = random_layer(12, 1, 1, 6, 32, scheme, CLOSED, CLIP_X, B=3000, uniform=False)
    art = _compile_spec(w.layers[0])
    r = oracle.lut_forward(art, CLOSED, CLIP_X, w.x, trace=True, codes=True)
    k = r.k[:, 0]
    v0 = art.y_min[0, k] + art.scale[0, k] * r.q01[:, 0, 0, 0].astype(np.float32)
    v1 = art.y_min[0, k] + art.scale[0, k] * r.q01[:, 0, 0, 1].astype(np.float32)
    lo, hi = np.minimum(v0, v1), np.maximum(v0, v1)
    tol = 2 * np.spacing(np.maximum(np.abs(lo), np.abs(hi)).astype(np.float32))
    assert np.all(r.y[:, 0] >= lo - tol) and np.all(r.y[:, 0] <= hi + tol)
    l1 = np.minimum(r.l0[:, 0] + 1, 31)
    np.testing.assert_array_equal(r.q01[:, 0, 0, 0], art.q[0, k, r.l0[:, 0]].astype(np.int16))
    np.testing.assert_array_equal(r.q01[:, 0, 0, 1], art.q[0, k, l1].astype(np.int16))


@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_constant_edge_function(scheme):
    tau = uniform_ext_knots(-1.0, 1.0, 5)
    art = _one_edge_art(tau, 16, scheme, coef=np.full(8, 0.7))
    x = np.linspace(-1.3, 1.3, 777, dtype=np.float32).reshape(-1, 1)
    r = oracle.lut_forward(art, CLOSED, CLIP_X, x)
    if scheme == ASYM_UINT8:
        # partition of unity in fp64 may leave the samples a few ulp apart; the LUT is then exact to one code step
        assert np.all(np.abs(r.y - np.float32(0.7)) <= 2 * np.spacing(np.float32(0.7)))
    else:
        assert np.all(np.abs(r.y - np.float32(0.7)) <= 4 * np.spacing(np.float32(0.7)))


@pytest.mark.parametrize("uniform", [True, False])
@pytest.mark.parametrize("L", [16, 64])
def test_linear_edge_function_closed_form(uniform, L):
    """Samples sit at u = l/L (Eq. 7) but are looked up at u = l/(L-1) (Eq. 16): on a linear edge function
    f(x) = a x + c the table therefore returns f(t_k + u h_k (L-1)/L), up to the quantisation step."""
    rng = np.random.Generator(np.random.PCG64(8))
    tau = uniform_ext_knots(-1.0, 1.0, 5) if uniform else nonuniform_ext_knots(rng, -1.0, 1.0, 5)
    a_, c_ = 1.75, -0.25
    art = _one_edge_art(tau, L, ASYM_UINT8, coef=a_ * _greville(tau) + c_)
    T = art.knots.astype(np.float64)
    x = rng.uniform(-1.0, 1.0, 4000).astype(np.float32)
    r = oracle.lut_forward(art, CLOSED, CLIP_X, x.reshape(-1, 1), trace=True)
    k = r.k[:, 0]
    h = T[k + 1] - T[k]
    u = (x.astype(np.float64) - T[k]) / h
    want = a_ * (T[k] + u * h * (L - 1) / L) + c_
    step = art.scale[0, k].astype(np.float64)
    assert np.all(np.abs(r.y[:, 0] - want) <= 0.5 * step + 1e-6)
    # ... which is NOT f(x): the deviation is a u h_k / L (zero at the left knot, one sampling step at the right)
    dev = np.abs(r.y[:, 0] - (a_ * x.astype(np.float64) + c_))
    assert np.all(np.abs(dev - a_ * u * h / L) <= 0.5 * step + 1e-6)
    assert dev.max() > 0.5 * a_ * h.min() / L


def test_error_halves_per_doubling_of_L_like_table1():
    w = random_layer(2, 10, 8, 8, 16, ASYM_UINT8, CLOSED, CLIP_X, B=4096, oob_frac=0.0)
    s = w.layers[0]
    x = np.clip(w.x, -1.0, 1.0)
    exact = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, CLOSED, CLIP_X, x).y.astype(np.float64)
    for scheme, name in ((ASYM_UINT8, "asym"), (SYM_INT8, "sym")):
        mae = []
        for L in (16, 32, 64, 128):
            art = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, L, scheme)
            mae.append(np.abs(oracle.lut_forward(art, CLOSED, CLIP_X, x).y - exact).mean())
        ours = np.array(mae[:-1]) / np.array(mae[1:])
        rows = [l.split() for l in open(os.path.join(GOLD, "table1_mae_vs_L.txt")) if l[0] != "#" and l.startswith(name)]
        paper = np.array([float(r[2]) for r in rows])
        paper_ratio = paper[:-1] / paper[1:]
        assert np.all(np.abs(paper_ratio - 2.0) < 0.15)                        # Table 1: ~2x per doubling
        assert np.all(ours[:2] > 1.7) and np.all(ours[:2] < 2.3), ours          # same O(1/L) trend here
        assert ours[2] > 1.4                                                    # quantisation floor starts to show


# ---------------------------------------------------------------- OOB policies (Sec. 5.4)
@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_oob_policies(scheme):
    w = random_layer(4, 3, 4, 5, 16, scheme, CLOSED, CLIP_X, B=2000, oob_frac=0.3)
    s = w.layers[0]
    art = _compile_spec(s)
    res = {(b, o): oracle.lut_forward(art, b, o, w.x, trace=True) for b in (HALF_OPEN, CLOSED) for o in (CLIP_X, ZERO_SPLINE)}
    # rows whose inputs are all strictly inside: identical outputs under all four contracts
    inside_all = np.all((w.x >= art.knots[0]) & (w.x < art.knots[-1]), axis=1)
    assert inside_all.sum() > 50
    base = res[(CLOSED, CLIP_X)].y[inside_all]
    for r in res.values():
        np.testing.assert_array_equal(r.y[inside_all], base)
    # zero_spline: an OOB input contributes exactly 0; clip_x: x < t_0 contributes the dequantised code [k=0][l=0]
    for b in (HALF_OPEN, CLOSED):
        r = res[(b, ZERO_SPLINE)]
        all_out = np.all(r.inside == 0, axis=1)
        x_out = np.full((3, s.d), 7.5, dtype=np.float32)
        x_out[1] = -7.5
        x_out[2, ::2] = -np.inf
        rz = oracle.lut_forward(art, b, ZERO_SPLINE, x_out)
        assert np.all(rz.y == 0.0) and np.all(rz.A == 0.0) and rz.oob_any_rows == 3 and rz.oob_count == 3 * s.d
        rc = oracle.lut_forward(art, b, CLIP_X, x_out[1:2])
        want = np.zeros(s.m)
        for i in range(s.d):
            for j in range(s.m):
                e = i * s.m + j
                want[j] += float(np.float32(art.y_min[e, 0] + np.float32(art.scale[e, 0] * np.float32(art.q[e, 0, 0]))))
        np.testing.assert_allclose(rc.y[0], want.astype(np.float32), rtol=1e-6)
        assert r.oob_any_rows == int(np.any(r.inside == 0, axis=1).sum()) and all_out.sum() >= 0


def test_nan_input_poisons_its_row_only():
    w = random_layer(4, 3, 2, 5, 16, ASYM_UINT8, CLOSED, ZERO_SPLINE, B=8, oob_frac=0.0)
    art = _compile_spec(w.layers[0])
    x = w.x.copy()
    x[2, 1] = np.nan
    for oob in (CLIP_X, ZERO_SPLINE):
        r = oracle.lut_forward(art, CLOSED, oob, x, trace=True)
        assert np.isnan(r.y[2]).all() and np.isfinite(np.delete(r.y, 2, axis=0)).all()
        assert (r.inside[2, 1], r.k[2, 1], r.l0[2, 1]) == (0, 0, 0)


# ---------------------------------------------------------------- layer sum (Eq. 1)
def test_tiny_layer_brute_force_from_single_edges():
    """cfg-1-sized layer: y[b][j] must equal the fp64 sum over i of the single-edge (d=m=1) outputs."""
    w = cfg1(seed=0, B=64)
    s = w.layers[0]
    art = _compile_spec(s)
    full = oracle.lut_forward(art, s.boundary, s.oob, w.x)
    want = np.zeros((64, s.m))
    wantA = np.zeros((64, s.m))
    for i in range(s.d):
        for j in range(s.m):
            e = i * s.m + j
            one = oracle.compile_layer(1, 1, s.G, s.p, s.ext_knots, s.coef[i, j], s.L, s.scheme)
            np.testing.assert_array_equal(one.q[0], art.q[e])
            assert np.array_equal(one.scale[0], art.scale[e]) and np.array_equal(one.y_min[0], art.y_min[e])
            ye = oracle.lut_forward(one, s.boundary, s.oob, w.x[:, i:i + 1]).y[:, 0].astype(np.float64)
            want[:, j] += ye
            wantA[:, j] += np.abs(ye)
    np.testing.assert_array_equal(full.y, want.astype(np.float32))
    np.testing.assert_allclose(full.A, wantA, rtol=1e-15)


def test_rows_are_independent_and_threads_do_not_matter():
    w = random_layer(15, 5, 7, 6, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, B=257)
    art = _compile_spec(w.layers[0])
    a = oracle.lut_forward(art, HALF_OPEN, ZERO_SPLINE, w.x, nthreads=1)
    perm = np.random.Generator(np.random.PCG64(1)).permutation(257)
    b = oracle.lut_forward(art, HALF_OPEN, ZERO_SPLINE, w.x[perm], nthreads=4)
    np.testing.assert_array_equal(a.y[perm], b.y)
    assert a.oob_count == b.oob_count and a.oob_any_rows == b.oob_any_rows


def test_lut_tracks_the_exact_spline_layer():
    """End-to-end sanity: LUT layer vs the fp64 B-spline layer differ by O(h |f'| / L) + quantisation only."""
    w = random_layer(17, 6, 5, 8, 128, ASYM_UINT8, CLOSED, CLIP_X, B=512, oob_frac=0.1)
    s = w.layers[0]
    art = _compile_spec(s)
    lut = oracle.lut_forward(art, CLOSED, CLIP_X, w.x)
    ref = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, CLOSED, CLIP_X, w.x)
    assert np.abs(lut.y - ref.y).max() < 6 * 0.02 and np.abs(lut.y - ref.y).mean() < 0.01
    # zero_spline on the B-spline layer masks the same inputs
    z_lut = oracle.lut_forward(art, CLOSED, ZERO_SPLINE, w.x)
    z_ref = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, CLOSED, ZERO_SPLINE, w.x)
    assert np.abs(z_lut.y - z_ref.y).max() < 6 * 0.02
    far = np.full((2, s.d), 9.0, dtype=np.float32)
    assert np.all(oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, CLOSED, ZERO_SPLINE, far).y == 0)


# ---------------------------------------------------------------- value_repr = spline_component (Eq. 2, Sec. 4.3 B, Sec. 5.4)
from scipy.special import expit  # noqa: E402


def _scalars(rng, E):
    return (rng.normal(0.0, 1.0, E).astype(np.float32), rng.normal(1.0, 0.3, E).astype(np.float32),
            rng.normal(1.0, 0.2, E).astype(np.float32))


def test_silu_values_and_identities():
    assert oracle.silu(0.0) == 0.0
    for x in (0.25, 1.0, 3.5, 17.0):
        assert abs((oracle.silu(x) - oracle.silu(-x)) - x) <= 2e-7 * max(1.0, x)          # x*s(x) - (-x)*s(-x) = x
    assert abs(oracle.silu(30.0) - 30.0) < 1e-5 and abs(oracle.silu(-30.0)) < 1e-11
    xs = np.linspace(-6, 6, 2401)
    v = np.array([oracle.silu(x) for x in xs])
    np.testing.assert_allclose(v, xs * expit(xs), rtol=2e-7, atol=1e-9)                     # library routine
    imin = int(np.argmin(v))
    assert abs(xs[imin] + 1.2785) < 0.006 and abs(v[imin] + 0.27846) < 1e-5                 # the SiLU minimum


def test_spline_component_reduces_to_phi_when_base_is_off():
    w = random_layer(31, 5, 4, 6, 32, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, B=500, oob_frac=0.3)
    art = _compile_spec(w.layers[0])
    E = 20
    ones, zeros = np.ones(E, np.float32), np.zeros(E, np.float32)
    for b in (HALF_OPEN, CLOSED):
        for o in (CLIP_X, ZERO_SPLINE):
            phi = oracle.lut_forward(art, b, o, w.x)
            sc = oracle.lut_forward(art, b, o, w.x, edge_scalars=(zeros, ones, ones))
            np.testing.assert_array_equal(phi.y, sc.y)
            np.testing.assert_allclose(phi.A, sc.A, rtol=1e-12)


def test_spline_component_base_branch_only_matches_closed_form_at_raw_x():
    rng = np.random.Generator(np.random.PCG64(32))
    w = random_layer(32, 6, 3, 5, 16, SYM_INT8, CLOSED, CLIP_X, B=300, oob_frac=1.5)    # many inputs far outside [-1,1]
    art = _compile_spec(w.layers[0])
    sb, ss, so = _scalars(rng, 18)
    r = oracle.lut_forward(art, CLOSED, CLIP_X, w.x, edge_scalars=(sb, np.zeros(18, np.float32), so))
    x64 = w.x.astype(np.float64)
    want = (x64 * expit(x64)) @ (so.astype(np.float64) * sb.astype(np.float64)).reshape(6, 3)   # base at RAW x
    np.testing.assert_allclose(r.y, want, rtol=3e-6, atol=3e-6)
    clipped = np.clip(x64, -1, 1)
    wrong = (clipped * expit(clipped)) @ (so.astype(np.float64) * sb.astype(np.float64)).reshape(6, 3)
    assert np.abs(r.y - wrong).max() > 0.1


def test_spline_component_zero_spline_masks_the_spline_branch_only():
    rng = np.random.Generator(np.random.PCG64(33))
    w = random_layer(33, 4, 2, 5, 16, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, B=64)
    art = _compile_spec(w.layers[0])
    sb, ss, so = _scalars(rng, 8)
    x = np.full((3, 4), 2.5, dtype=np.float32)
    x[1] = -4.0
    x[2, :2] = 0.3                                                     # a row with two inputs inside, two outside
    full = oracle.lut_forward(art, HALF_OPEN, ZERO_SPLINE, x, edge_scalars=(sb, ss, so))
    base = oracle.lut_forward(art, HALF_OPEN, ZERO_SPLINE, x, edge_scalars=(sb, np.zeros(8, np.float32), so))
    np.testing.assert_array_equal(full.y[:2], base.y[:2])              # all inputs OOB: only the base branch is left
    assert np.abs(full.y[2] - base.y[2]).max() > 1e-3                  # in-range inputs keep their spline branch
    clip = oracle.lut_forward(art, HALF_OPEN, CLIP_X, x, edge_scalars=(sb, ss, so))
    assert np.abs(clip.y[:2] - base.y[:2]).max() > 1e-3                # clip_x keeps the saturated spline value


def test_spline_component_single_edge_composition_and_output_scale():
    rng = np.random.Generator(np.random.PCG64(34))
    tau = uniform_ext_knots(-1.0, 1.0, 5)
    art = _one_edge_art(tau, 32, SYM_INT8)
    x = rng.uniform(-1.5, 1.5, 400).astype(np.float32).reshape(-1, 1)
    v = oracle.lut_forward(art, CLOSED, ZERO_SPLINE, x).y[:, 0]        # m(x) * s^(x')
    sb, ss, so = np.float32(0.7), np.float32(-1.3), np.float32(0.9)
    r = oracle.lut_forward(art, CLOSED, ZERO_SPLINE, x, edge_scalars=([sb], [ss], [so]))
    b = np.array([oracle.silu(t) for t in x[:, 0]], dtype=np.float32)
    want = (so * ((sb * b).astype(np.float32) + (ss * v).astype(np.float32)).astype(np.float32)).astype(np.float32)
    np.testing.assert_array_equal(r.y[:, 0], want)
    r2 = oracle.lut_forward(art, CLOSED, ZERO_SPLINE, x, edge_scalars=([sb], [ss], [np.float32(2) * so]))
    np.testing.assert_array_equal(r2.y, np.float32(2) * r.y)           # s_out scales the whole edge (Eq. 2)


def test_bspline_layer_spline_component_matches_fp64_closed_form():
    from scipy.interpolate import BSpline
    rng = np.random.Generator(np.random.PCG64(35))
    w = random_layer(35, 3, 2, 6, 16, SYM_INT8, CLOSED, ZERO_SPLINE, B=200, uniform=False, oob_frac=0.4)
    s = w.layers[0]
    sb, ss, so = _scalars(rng, 6)
    r = oracle.bspline_forward(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, CLOSED, ZERO_SPLINE, w.x, edge_scalars=(sb, ss, so))
    x64 = w.x.astype(np.float64)
    t64 = s.ext_knots.astype(np.float64)
    lo, hi = t64[3], t64[3 + s.G]
    inside = (x64 >= lo) & (x64 <= hi)
    want = np.zeros((200, s.m))
    for i in range(s.d):
        for j in range(s.m):
            e = i * s.m + j
            sp = BSpline(t64, s.coef[i, j].astype(np.float64), 3, extrapolate=False)(np.clip(x64[:, i], lo, np.nextafter(hi, -np.inf)))
            want[:, j] += float(so[e]) * (float(sb[e]) * x64[:, i] * expit(x64[:, i]) + float(ss[e]) * np.where(inside[:, i], sp, 0.0))
    np.testing.assert_allclose(r.y, want, rtol=2e-6, atol=2e-6)


# ---------------------------------------------------------------------------------------------------
# float16 dequantisation parameters (Sec. 4.6: scale and y_min "float16 or float32")
# ---------------------------------------------------------------------------------------------------
def test_round_to_fp16_is_the_library_cast():
    """Pin: numpy's float32 -> float16 cast (IEEE round-to-nearest-even) on random values, exact ties, the
    subnormal range and both sides of the overflow threshold."""
    rng = np.random.default_rng(11)
    ties = [1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2048 + 1, 2048 + 3, 2.0 ** -14 * (1 + 2.0 ** -11), 2.0 ** -25, 3 * 2.0 ** -25,
            5 * 2.0 ** -25, 2.0 ** -24, 2.0 ** -26, 65504.0, 65519.996, 65520.0, 65535.0, 1e30, 0.0]
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-6, 10000), rng.uniform(-70000, 70000, 10000),
                        ties, [-t for t in ties]]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float32)
    got = np.array([oracle.round_to_fp16(v) for v in x], dtype=np.float32)
    assert np.array_equal(want, got)
    assert np.array_equal(np.signbit(want), np.signbit(got))


@pytest.mark.parametrize("scheme", [SYM_INT8, ASYM_UINT8])
def test_fp16_params_keep_the_codes_and_round_the_parameters(scheme):
    w = random_layer(61, 5, 6, 7, 16, scheme, CLOSED, CLIP_X, 8)
    s = w.layers[0]
    a32 = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme)
    a16 = oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, scheme, param_fp16=True)
    assert np.array_equal(a32.q, a16.q)
    assert np.array_equal(a16.scale, a32.scale.astype(np.float16).astype(np.float32))
    assert np.array_equal(a16.y_min, a32.y_min.astype(np.float16).astype(np.float32))
    assert not np.array_equal(a16.scale, a32.scale)


def test_fp16_params_forward_dequantises_with_the_stored_values():
    """d = m = 1, x on a knot: w = 0 and the output is fl(y_min16 + fl(alpha16 * q)) of that segment's first code."""
    w = random_layer(62, 1, 1, 6, 8, ASYM_UINT8, CLOSED, CLIP_X, 4)
    s = w.layers[0]
    art = oracle.compile_layer(1, 1, s.G, s.p, s.ext_knots, s.coef, s.L, ASYM_UINT8, param_fp16=True)
    x = art.knots[:-1].reshape(-1, 1).copy()
    out = oracle.lut_forward(art, CLOSED, CLIP_X, x)
    for k in range(s.G):
        a16, y16 = np.float32(np.float16(art.scale[0, k])), np.float32(np.float16(art.y_min[0, k]))
        assert a16 == art.scale[0, k] and y16 == art.y_min[0, k]
        want = np.float32(y16 + np.float32(a16 * np.float32(art.q[0, k, 0])))
        assert out.y[k, 0] == want


def test_fp16_params_that_do_not_fit_are_refused():
    w = random_layer(63, 2, 2, 5, 8, SYM_INT8, CLOSED, CLIP_X, 4)
    s = w.layers[0]
    with pytest.raises(ValueError):
        oracle.compile_layer(s.d, s.m, s.G, s.p, s.ext_knots, s.coef * np.float32(1e8), s.L, SYM_INT8, param_fp16=True)


# ---------------------------------------------------------------------------------------------------
# OOB evaluation protocol (Sec. 5.6): in-range / OOB-only error statistics
# ---------------------------------------------------------------------------------------------------
def test_error_stats_on_a_hand_made_example():
    """Three rows on the domain [-1, 1]: all inside; one input at t_K; one input beyond.  Values by hand."""
    x = np.array([[0.0, 0.5], [1.0, -1.0], [0.2, 1.5]], dtype=np.float32)
    y = np.array([[1.0, 2.0], [3.0, 5.0], [0.0, 0.0]], dtype=np.float32)
    r = np.array([[1.5, 2.0], [2.0, 5.5], [4.0, -1.0]], dtype=np.float32)
    c = oracle.error_stats(y, r, x, -1.0, 1.0, CLOSED)            # t_K belongs to the domain: rows 0, 1 in-range
    assert (c["rows_in"], c["rows_oob"], c["nan_in"], c["nan_oob"]) == (2, 1, 0, 0)
    assert c["sum_abs_in"] == 0.5 + 0.0 + 1.0 + 0.5 and c["max_abs_in"] == 1.0 and c["mae_in"] == 2.0 / 4
    assert c["sum_abs_oob"] == 5.0 and c["max_abs_oob"] == 4.0 and c["mae_oob"] == 2.5 and c["oob_any_frac"] == 1 / 3
    h = oracle.error_stats(y, r, x, -1.0, 1.0, HALF_OPEN)         # x = t_K is outside (Sec. 5.5): row 1 moves over
    assert (h["rows_in"], h["rows_oob"]) == (1, 2)
    assert h["sum_abs_in"] == 0.5 and h["sum_abs_oob"] == 6.5 and h["max_abs_oob"] == 4.0 and h["mae_oob"] == 6.5 / 4


def test_error_stats_mean_leaves_nan_differences_out_of_the_count():
    """A NaN output inside each subset: it is counted per subset and left out of that subset's sum, maximum AND of the
    number the sum is divided by, so the mean is the mean of the differences that exist.  Dividing by rows * m instead
    (the NaN output still counted as a term) would give 1.5 / 4 and 5.0 / 4 below.  Values by hand."""
    nan = np.float32(np.nan)
    x = np.array([[0.0, 0.5], [0.9, -1.0], [0.2, 1.5], [3.0, 0.0]], dtype=np.float32)     # rows 0, 1 inside [-1, 1]
    y = np.array([[1.0, nan], [3.0, 5.0], [0.0, 0.0], [nan, 2.0]], dtype=np.float32)
    r = np.array([[1.5, 2.0], [2.5, 5.5], [4.0, -1.0], [1.0, 2.0]], dtype=np.float32)
    c = oracle.error_stats(y, r, x, -1.0, 1.0, CLOSED)
    assert (c["rows_in"], c["rows_oob"], c["nan_in"], c["nan_oob"]) == (2, 2, 1, 1)
    assert c["sum_abs_in"] == 1.5 and c["max_abs_in"] == 0.5 and c["mae_in"] == 1.5 / 3
    assert c["sum_abs_oob"] == 5.0 and c["max_abs_oob"] == 4.0 and c["mae_oob"] == 5.0 / 3
    assert c["oob_any_frac"] == 0.5
    # the library routine for "mean of what is not NaN" on each subset
    e = np.abs(y.astype(np.float64) - r.astype(np.float64))
    assert c["mae_in"] == np.nanmean(e[:2]) and c["mae_oob"] == np.nanmean(e[2:])
    # a subset whose every difference is NaN has no mean
    allnan = oracle.error_stats(np.full((1, 2), nan), r[:1], x[:1], -1.0, 1.0, CLOSED)
    assert (allnan["rows_in"], allnan["nan_in"], allnan["sum_abs_in"]) == (1, 2, 0.0) and np.isnan(allnan["mae_in"])
    assert np.isnan(allnan["mae_oob"]) and allnan["oob_any_frac"] == 0.0


def test_error_stats_against_plain_loops_and_nan_rules():
    rng = np.random.default_rng(5)
    B, d, m = 37, 5, 3
    x = rng.uniform(-1.4, 1.4, size=(B, d)).astype(np.float32)
    x[3, 2] = np.nan                                              # NaN input: the row is OOB
    y = rng.normal(size=(B, m)).astype(np.float32)
    r = rng.normal(size=(B, m)).astype(np.float32)
    y[7, 1] = np.nan                                              # NaN difference: counted, left out
    for boundary in (HALF_OPEN, CLOSED):
        got = oracle.error_stats(y, r, x, -1.0, 1.0, boundary)
        rows = {"in": 0, "oob": 0}
        sums = {"in": 0.0, "oob": 0.0}
        maxs = {"in": 0.0, "oob": 0.0}
        nans = {"in": 0, "oob": 0}
        for b in range(B):
            inside = True
            for i in range(d):
                v = float(x[b, i])
                ok = (v >= -1.0) and ((v <= 1.0) if boundary == CLOSED else (v < 1.0))
                inside = inside and ok
            key = "in" if inside else "oob"
            rows[key] += 1
            for j in range(m):
                e = abs(float(y[b, j]) - float(r[b, j]))
                if e != e:
                    nans[key] += 1
                    continue
                sums[key] += e
                maxs[key] = max(maxs[key], e)
        assert (got["rows_in"], got["rows_oob"]) == (rows["in"], rows["oob"])
        assert (got["nan_in"], got["nan_oob"]) == (nans["in"], nans["oob"]) and nans["in"] + nans["oob"] == 1
        assert got["oob_any_frac"] == rows["oob"] / B
        for key in ("in", "oob"):
            assert abs(got["sum_abs_" + key] - sums[key]) <= 1e-12 * sums[key]
            assert got["max_abs_" + key] == maxs[key]
            assert abs(got["mae_" + key] - sums[key] / (rows[key] * m - nans[key])) <= 1e-15


# ---------------------------------------------------------------------------------------------------
# LUT over the whole extended knot vector (the reading that the byte counts of Table 9 imply)
# ---------------------------------------------------------------------------------------------------
def _basis_sum(tau, coef, x):
    """sum_r c_r B_{r,3}(x) with SciPy's basis elements (each is zero outside its own support)."""
    from scipy.interpolate import BSpline
    total = np.zeros_like(x, dtype=np.float64)
    for r in range(coef.size):
        b = BSpline.basis_element(tau[r:r + 5].astype(np.float64), extrapolate=False)(x)
        total += float(coef[r]) * np.nan_to_num(b, nan=0.0)
    return total


@pytest.mark.parametrize("uniform", [True, False])
def test_extended_lut_covers_every_extended_interval(uniform):
    G, L = 5, 16
    w = random_layer(71, 2, 3, G, L, ASYM_UINT8, CLOSED, CLIP_X, 4, uniform=uniform)
    s = w.layers[0]
    dom = oracle.compile_layer(s.d, s.m, G, P, s.ext_knots, s.coef, L, ASYM_UINT8, want_v=True)
    ext = oracle.compile_layer(s.d, s.m, G, P, s.ext_knots, s.coef, L, ASYM_UINT8, want_v=True, extended=True)
    assert ext.K == G + 2 * P == 11 and np.array_equal(ext.knots, s.ext_knots)
    # the G inner segments are the domain artifact, bit for bit
    assert np.array_equal(ext.q[:, P:P + G], dom.q) and np.array_equal(ext.scale[:, P:P + G], dom.scale)
    assert np.array_equal(ext.y_min[:, P:P + G], dom.y_min) and np.array_equal(ext.v[:, P:P + G], dom.v)
    # on the outer intervals fewer than p+1 basis functions exist; the samples are still the sum of Eq. 3
    tau = s.ext_knots
    for k in list(range(P)) + list(range(P + G, G + 2 * P)):
        xs = np.array([oracle.sample_x(tau, L, k, l) for l in range(L)])
        for e in range(s.d * s.m):
            want = _basis_sum(tau, s.coef.reshape(-1, G + P)[e], xs)
            np.testing.assert_allclose(ext.v[e, k], want, rtol=0, atol=2e-6)
    assert np.abs(ext.v[:, 0, 0]).max() == 0.0                      # at tau_0 itself nothing is non-zero yet


def test_extended_bspline_layer_and_the_last_knot():
    G = 4
    w = random_layer(72, 3, 2, G, 8, SYM_INT8, CLOSED, CLIP_X, 4, uniform=False)
    s = w.layers[0]
    tau = s.ext_knots
    x = np.random.Generator(np.random.PCG64(3)).uniform(tau[0], tau[-1], size=(40, 3)).astype(np.float32)
    x[0, :] = tau[-1]                                               # closed mode: in the domain, but every basis function is 0 there
    x[1, :] = np.float32(tau[-1] + 1.0)                             # clipped onto the last knot
    x[2, :] = tau[0]
    out = oracle.bspline_forward(s.d, s.m, G, P, tau, s.coef, CLOSED, CLIP_X, x, extended=True)
    assert np.all(out.y[0] == 0.0) and np.all(out.y[1] == 0.0) and np.all(out.y[2] == 0.0)
    want = np.zeros((40, 2))
    for i in range(3):
        for j in range(2):
            want[:, j] += _basis_sum(tau, s.coef[i, j], x[:, i].astype(np.float64))
    np.testing.assert_allclose(out.y[3:], want[3:], rtol=0, atol=5e-6)
    # the same inputs in domain mode are clipped to the inner grid instead
    inner = oracle.bspline_forward(s.d, s.m, G, P, tau, s.coef, CLOSED, CLIP_X, x)
    far = np.any((x < tau[P]) | (x > tau[P + G]), axis=1)
    assert far.any() and not np.allclose(inner.y[far], out.y[far])
    # zero_spline in half_open mode: the last knot is out of the domain
    z = oracle.bspline_forward(s.d, s.m, G, P, tau, s.coef, HALF_OPEN, ZERO_SPLINE, x[:3], extended=True)
    assert np.all(z.y[:2] == 0.0)


def test_extended_lut_forward_tracks_the_extended_spline():
    G, L = 6, 64
    w = random_layer(73, 4, 3, G, L, SYM_INT8, HALF_OPEN, CLIP_X, 4)
    s = w.layers[0]
    tau = s.ext_knots
    art = oracle.compile_layer(s.d, s.m, G, P, tau, s.coef, L, SYM_INT8, extended=True)
    x = np.random.Generator(np.random.PCG64(9)).uniform(tau[0], tau[-2], size=(300, 4)).astype(np.float32)
    lut = oracle.lut_forward(art, HALF_OPEN, CLIP_X, x, trace=True)
    ref = oracle.bspline_forward(s.d, s.m, G, P, tau, s.coef, HALF_OPEN, CLIP_X, x, extended=True)
    assert lut.inside.all() and lut.k.max() == G + 2 * P - 2 and lut.k.min() == 0
    assert np.abs(lut.y - ref.y).max() < 0.5 and np.abs(lut.y - ref.y).mean() < 0.08     # O(1/L) table error, d = 4 edges per output


def test_table9_segment_count_is_the_extended_reading():
    """Table 9's byte counts fit K = 11 = G + 2p for the case study's grid 5, cubic: the extended artifact's K."""
    s = random_layer(74, 1, 1, 5, 64, ASYM_UINT8, CLOSED, CLIP_X, 4).layers[0]
    art = oracle.compile_layer(1, 1, 5, P, s.ext_knots, s.coef, 64, ASYM_UINT8, param_fp16=True, extended=True)
    rows = [l.split() for l in open(os.path.join(GOLD, "table9_artifact_bytes.txt")) if l[0] != "#"]
    for E, K, L, nbytes in rows:
        assert int(K) == art.K and int(L) == art.L
        per_edge = art.q[0].nbytes + art.scale[0].size * 2 + art.y_min[0].size * 2      # float16 scale and y_min
        assert int(E) * per_edge + art.knots.nbytes == int(nbytes)


# ---- one knot vector per input dimension (Sec. 6.2 "knot grid shared per input dimension") ----

from lutkan_inputs import per_input_layer  # noqa: E402


def test_per_input_knots_equal_rows_are_the_shared_layer():
    """d copies of one knot vector must give the shared-vector layer bit for bit (artifact, outputs, trace)."""
    w = random_layer(81, 4, 3, 6, 16, ASYM_UINT8, HALF_OPEN, ZERO_SPLINE, 200, uniform=False, with_base=True)
    s = w.layers[0]
    tiled = np.tile(s.ext_knots, (s.d, 1))
    one = oracle.compile_layer(s.d, s.m, s.G, P, s.ext_knots, s.coef, s.L, s.scheme)
    per = oracle.compile_layer(s.d, s.m, s.G, P, tiled, s.coef, s.L, s.scheme, per_input=True)
    assert per.knots.shape == (s.d, s.G + 1) and all(np.array_equal(per.knots[i], one.knots) for i in range(s.d))
    assert np.array_equal(per.q, one.q) and np.array_equal(per.scale, one.scale) and np.array_equal(per.y_min, one.y_min)
    a = oracle.lut_forward(one, s.boundary, s.oob, w.x, trace=True, edge_scalars=s.edge_scales)
    b = oracle.lut_forward(per, s.boundary, s.oob, w.x, trace=True, edge_scalars=s.edge_scales)
    for f in ("y", "A", "k", "l0", "inside", "w"):
        np.testing.assert_array_equal(getattr(a, f), getattr(b, f), err_msg=f)
    assert (a.oob_count, a.oob_any_rows) == (b.oob_count, b.oob_any_rows)
    ya = oracle.bspline_forward(s.d, s.m, s.G, P, s.ext_knots, s.coef, s.boundary, s.oob, w.x, edge_scalars=s.edge_scales)
    yb = oracle.bspline_forward(s.d, s.m, s.G, P, tiled, s.coef, s.boundary, s.oob, w.x, edge_scalars=s.edge_scales, per_input=True)
    np.testing.assert_array_equal(ya.y, yb.y)


@pytest.mark.parametrize("scheme,boundary,oob", [(SYM_INT8, CLOSED, CLIP_X), (ASYM_UINT8, HALF_OPEN, ZERO_SPLINE)])
def test_per_input_knots_layer_is_the_sum_of_its_single_input_layers(scheme, boundary, oob):
    """Each input's edges form a shared-vector layer of their own (d = 1) on that input's knots: artifact rows, trace
    columns and counters must be theirs, and the outputs the fp64 sum of theirs."""
    w = per_input_layer(82, 5, 3, 6, 16, scheme, boundary, oob, 300)
    s = w.layers[0]
    per = oracle.compile_layer(s.d, s.m, s.G, P, s.ext_knots, s.coef, s.L, scheme, per_input=True)
    full = oracle.lut_forward(per, boundary, oob, w.x, trace=True)
    spl = oracle.bspline_forward(s.d, s.m, s.G, P, s.ext_knots, s.coef, boundary, oob, w.x, per_input=True)
    want, want_spl, oob_count = np.zeros((300, s.m)), np.zeros((300, s.m)), 0
    any_oob = np.zeros(300, dtype=bool)
    for i in range(s.d):
        one = oracle.compile_layer(1, s.m, s.G, P, s.ext_knots[i], s.coef[i], s.L, scheme)
        rows = slice(i * s.m, (i + 1) * s.m)
        assert np.array_equal(per.knots[i], one.knots) and np.array_equal(per.q[rows], one.q)
        assert np.array_equal(per.scale[rows], one.scale) and np.array_equal(per.y_min[rows], one.y_min)
        r = oracle.lut_forward(one, boundary, oob, w.x[:, i:i + 1], trace=True)
        for f in ("k", "l0", "inside", "w"):
            np.testing.assert_array_equal(getattr(full, f)[:, i], getattr(r, f)[:, 0], err_msg=f"{f} of input {i}")
        # numpy's searchsorted on this input's own knots (Eq. 14) and its own domain (Sec. 5.2)
        T = per.knots[i]
        xc = np.clip(w.x[:, i], T[0], T[-1] if boundary == CLOSED else np.nextafter(T[-1], np.float32(-np.inf)))
        np.testing.assert_array_equal(full.k[:, i], np.clip(np.searchsorted(T, xc, side="right") - 1, 0, s.G - 1))
        inside = (w.x[:, i] >= T[0]) & ((w.x[:, i] <= T[-1]) if boundary == CLOSED else (w.x[:, i] < T[-1]))
        np.testing.assert_array_equal(full.inside[:, i], inside.astype(np.uint8))
        oob_count += int((~inside).sum())
        any_oob |= ~inside
        want += r.y.astype(np.float64)     # a single-input layer's fp32 output is its one edge value exactly
        want_spl += oracle.bspline_forward(1, s.m, s.G, P, s.ext_knots[i], s.coef[i], boundary, oob, w.x[:, i:i + 1]).y
    assert (full.oob_count, full.oob_any_rows) == (oob_count, int(any_oob.sum()))
    np.testing.assert_array_equal(full.y, want.astype(np.float32))
    np.testing.assert_allclose(spl.y, want_spl, rtol=0, atol=1e-5)


def test_per_input_knots_domains_decide_the_mask_closed_form():
    """All coefficients 1: every spline is 1 on its domain (partition of unity), so with zero_spline the output
    counts the inputs that lie in THEIR OWN domain; mixing up the vectors changes the count."""
    G, L, d, m = 4, 8, 3, 2
    tau = np.stack([uniform_ext_knots(-1, 1, G), uniform_ext_knots(2, 3, G), uniform_ext_knots(-5, -4, G)])
    coef = np.ones((d, m, G + P), dtype=np.float32)
    x = np.array([[0.0, 2.5, -4.5],      # all three inside their own domain
                  [0.0, 0.0, 0.0],       # only input 0
                  [2.5, 2.5, 2.5],       # only input 1
                  [-4.5, -4.5, 2.5],     # none
                  [1.0, 3.0, -4.0]],     # the right ends: inside when closed, outside when half-open
                 dtype=np.float32)
    per = oracle.compile_layer(d, m, G, P, tau, coef, L, ASYM_UINT8, per_input=True)
    assert np.all(per.q == 0) and np.all(per.y_min == 1.0)           # a constant segment: alpha = 0, y_min = the value
    yc = oracle.lut_forward(per, CLOSED, ZERO_SPLINE, x).y
    yh = oracle.lut_forward(per, HALF_OPEN, ZERO_SPLINE, x).y
    np.testing.assert_array_equal(yc[:, 0], [3, 1, 1, 0, 3])
    np.testing.assert_array_equal(yh[:, 0], [3, 1, 1, 0, 0])
    np.testing.assert_array_equal(yc[:, 1], yc[:, 0])
    bs = oracle.bspline_forward(d, m, G, P, tau, coef, HALF_OPEN, ZERO_SPLINE, x, per_input=True).y
    np.testing.assert_allclose(bs[:, 0], [3, 1, 1, 0, 0], atol=1e-6)
    # clip_x: every input saturates at its own domain end, where its spline is still 1
    np.testing.assert_allclose(oracle.bspline_forward(d, m, G, P, tau, coef, CLOSED, CLIP_X, x, per_input=True).y, 3.0, atol=1e-6)


def test_per_input_knots_linear_functions_closed_form():
    """Greville coefficients c_r = mean of the r-th knot triple reproduce f(x) = x on every knot vector; on per-input
    knots the exact layer output is sum_i clip(x_i) and the LUT tracks it to O(range/L) + quantisation."""
    G, L, d = 6, 128, 4
    w = per_input_layer(83, d, 1, G, L, ASYM_UINT8, CLOSED, CLIP_X, 400)
    s = w.layers[0]
    coef = np.zeros((d, 1, G + P), dtype=np.float32)
    for i in range(d):
        t = s.ext_knots[i].astype(np.float64)
        coef[i, 0] = [(t[r + 1] + t[r + 2] + t[r + 3]) / 3.0 for r in range(G + P)]
    lo, hi = s.ext_knots[:, P], s.ext_knots[:, P + G]
    want = np.clip(w.x, lo, hi).astype(np.float64).sum(axis=1)
    bs = oracle.bspline_forward(d, 1, G, P, s.ext_knots, coef, CLOSED, CLIP_X, w.x, per_input=True).y[:, 0]
    np.testing.assert_allclose(bs, want, rtol=0, atol=5e-6)
    per = oracle.compile_layer(d, 1, G, P, s.ext_knots, coef, L, ASYM_UINT8, per_input=True)
    lut = oracle.lut_forward(per, CLOSED, CLIP_X, w.x).y[:, 0]
    widths = (hi - lo).astype(np.float64) / G
    assert np.abs(lut - want).max() <= float((widths / L + widths / 255.0).sum()) * 1.01
