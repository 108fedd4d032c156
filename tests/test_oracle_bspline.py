"""Pins for the oracle's B-spline evaluation (Sec. 3.2, Eq. 3-5) against textbook identities and SciPy.

None of these re-types the recursion: they check facts that any correct Cox--de Boor evaluation
must satisfy, and a library routine (scipy.interpolate.BSpline) evaluated on the same knots/coefs.
"""
import numpy as np
import pytest
from scipy.interpolate import BSpline

import oracle
from lutkan_inputs import nonuniform_ext_knots, uniform_ext_knots

P = 3


def _grids():
    rng = np.random.Generator(np.random.PCG64(7))
    yield "uniform5", uniform_ext_knots(-1.0, 1.0, 5)
    yield "uniform8", uniform_ext_knots(-1.0, 1.0, 8)
    yield "uniform10_wide", uniform_ext_knots(-3.0, 3.0, 10)
    yield "nonuniform6", nonuniform_ext_knots(rng, -1.0, 1.0, 6)
    yield "nonuniform9", nonuniform_ext_knots(rng, -2.0, 5.0, 9)


GRIDS = list(_grids())


def _domain_points(tau, n=401):
    a, b = float(tau[P]), float(tau[-P - 1])
    xs = np.linspace(a, b, n)[:-1]                       # half-open domain [t_0, t_K)
    return np.concatenate([xs, tau[P:-P - 1].astype(np.float64)])   # plus every left breakpoint


@pytest.mark.parametrize("name,tau", GRIDS)
def test_partition_of_unity_nonneg_local_support(name, tau):
    G = tau.size - 2 * P - 1
    for x in _domain_points(tau):
        N = oracle.bspline_basis(tau, P, x)
        assert N.size == G + P
        assert abs(N.sum() - 1.0) <= 1e-14
        assert (N >= 0.0).all()
        nz = np.nonzero(N)[0]
        assert 1 <= nz.size <= P + 1
        # support of B_{r,3} is [tau_r, tau_{r+4}): the non-zero ones are r = mu-3..mu for the span mu
        mu = np.searchsorted(tau.astype(np.float64), x, side="right") - 1
        assert nz.min() >= mu - P and nz.max() <= mu


def test_uniform_knot_values_one_sixth_four_sixths():
    tau = uniform_ext_knots(-1.0, 1.0, 4)                 # spacing 0.5: exactly representable
    for kappa in range(0, 5):
        x = float(tau[P + kappa])
        N = oracle.bspline_basis(tau, P, x)
        mu = P + kappa
        np.testing.assert_allclose(N[mu - 3:mu], [1 / 6, 4 / 6, 1 / 6], rtol=0, atol=1e-15)
        if mu < N.size:
            assert N[mu] == 0.0


@pytest.mark.parametrize("name,tau", GRIDS)
def test_constant_and_greville_linear_reproduction(name, tau):
    G = tau.size - 2 * P - 1
    R = G + P
    t64 = tau.astype(np.float64)
    grev = np.array([(t64[r + 1] + t64[r + 2] + t64[r + 3]) / 3.0 for r in range(R)])
    for x in _domain_points(tau, 97):
        N = oracle.bspline_basis(tau, P, x)
        assert abs(float(N @ np.full(R, 2.5)) - 2.5) <= 1e-14          # all c_r = c  =>  s == c
        assert abs(float(N @ grev) - x) <= 1e-14 * max(1.0, abs(x))     # Greville abscissae => s(x) = x
    # and through the fp32-coefficient entry point (coefficients rounded to fp32 first)
    c32 = (1.75 * grev - 0.25).astype(np.float32)
    for x in _domain_points(tau, 31):
        want = float(oracle.bspline_basis(tau, P, x) @ c32.astype(np.float64))
        assert abs(oracle.spline_value(tau, P, c32, x) - want) <= 1e-15 * max(1.0, abs(want))
        assert abs(oracle.spline_value(tau, P, c32, x) - (1.75 * x - 0.25)) <= 5e-7


@pytest.mark.parametrize("name,tau", GRIDS)
def test_against_scipy_bspline(name, tau):
    rng = np.random.Generator(np.random.PCG64(11))
    G = tau.size - 2 * P - 1
    R = G + P
    for _ in range(4):
        c = rng.normal(size=R).astype(np.float32)
        ref = BSpline(tau.astype(np.float64), c.astype(np.float64), P, extrapolate=False)
        for x in _domain_points(tau, 57):
            got = oracle.spline_value(tau, P, c, x)
            want = float(ref(x))
            assert abs(got - want) <= 1e-13 * max(1.0, np.abs(c).max())


def test_scipy_basis_elementwise_nonuniform():
    rng = np.random.Generator(np.random.PCG64(3))
    tau = nonuniform_ext_knots(rng, 0.0, 1.0, 7)
    t64 = tau.astype(np.float64)
    R = tau.size - P - 1
    for x in np.linspace(0.0, 1.0, 50)[:-1]:
        N = oracle.bspline_basis(tau, P, x)
        for r in range(R):
            e = np.zeros(R)
            e[r] = 1.0
            want = float(BSpline(t64, e, P, extrapolate=False)(x))
            assert abs(N[r] - want) <= 1e-13


def test_right_end_of_domain_is_continuous():
    # closed boundary mode evaluates at x' = t_K: the extended knot vector keeps that point inside a
    # regular span, so the value equals the limit from the left.
    tau = uniform_ext_knots(-1.0, 1.0, 5)
    rng = np.random.Generator(np.random.PCG64(5))
    c = rng.normal(size=8).astype(np.float32)
    tK = float(tau[-P - 1])
    at = oracle.spline_value(tau, P, c, tK)
    left = oracle.spline_value(tau, P, c, np.nextafter(tK, -np.inf))
    assert abs(at - left) <= 1e-12
    N = oracle.bspline_basis(tau, P, tK)
    np.testing.assert_allclose(N[5:8], [1 / 6, 4 / 6, 1 / 6], atol=1e-7)   # fp32-rounded uniform knots
    assert N[:5].sum() == 0.0


def test_zero_over_zero_convention_repeated_knots():
    # clamped knot vector with repeated end knots exercises the 0/0 = 0 rule (Eq. 5)
    tau = np.array([0, 0, 0, 0, 1, 2, 3, 3, 3, 3], dtype=np.float64)
    for x in [0.0, 0.3, 1.0, 2.999]:
        N = oracle.bspline_basis(tau, P, x)
        assert np.isfinite(N).all() and abs(N.sum() - 1.0) <= 1e-14
        want = [float(BSpline(tau, np.eye(6)[r], P, extrapolate=False)(x)) for r in range(6)]
        np.testing.assert_allclose(N, want, atol=1e-14)
