"""Pins for the skew-normal prune-possibility schedule (Section 5.3, Eq. 4-6) and the library's host
implementation of it."""
import ctypes as C
import math

import numpy as np
import pytest
from scipy import integrate, stats

from oracle import schedule as S
from paper_2203_05705_amd import binding as ard

CASES = [(0.5, 0.04, 0.0), (0.45, 0.05, 3.0), (0.6, 0.02, -2.0), (0.3, 0.01, 8.0), (0.5, 0.09, 0.7)]


@pytest.mark.parametrize("mean,var,lam", CASES)
def test_density_is_the_library_skew_normal(mean, var, lam):
    """Eq. (4) against scipy's skew-normal (shape a = lambda, loc = mu, scale = sigma)."""
    mu, sigma = S.skew_normal_params(mean, var, lam)
    for y in np.linspace(mu - 4 * sigma, mu + 4 * sigma, 41):
        assert S.skew_normal_pdf(y, mu, sigma, lam) == pytest.approx(stats.skewnorm.pdf(y, lam, loc=mu, scale=sigma), rel=1e-11, abs=1e-300)


@pytest.mark.parametrize("mean,var,lam", CASES)
def test_moments_by_numerical_integration(mean, var, lam):
    """Eq. (5), (6): the density built from (mu, sigma) integrates to 1 and has the requested mean and
    variance (quadrature, not the formulas)."""
    mu, sigma = S.skew_normal_params(mean, var, lam)
    f = lambda y: S.skew_normal_pdf(y, mu, sigma, lam)
    lo, hi = mu - 12 * sigma, mu + 12 * sigma
    m0 = integrate.quad(f, lo, hi, epsabs=1e-13)[0]
    m1 = integrate.quad(lambda y: y * f(y), lo, hi, epsabs=1e-13)[0]
    m2 = integrate.quad(lambda y: (y - mean) ** 2 * f(y), lo, hi, epsabs=1e-13)[0]
    assert m0 == pytest.approx(1.0, abs=1e-9)
    assert m1 == pytest.approx(mean, abs=1e-9)
    assert m2 == pytest.approx(var, abs=1e-9)


def test_constants_of_eq_5_and_6():
    assert S.mu0(0.0) == 0.0 and S.sigma0_sq(0.0) == 1.0
    assert S.mu0(1e9) == pytest.approx(math.sqrt(2 / math.pi), rel=1e-12)          # half-normal limit
    assert S.sigma0_sq(1e9) == pytest.approx(1 - 2 / math.pi, rel=1e-12)
    assert S.mu0(-3.0) == -S.mu0(3.0)
    # lambda = 0: the plain normal density with the requested mean and variance
    mu, sigma = S.skew_normal_params(0.4, 0.09, 0.0)
    assert (mu, sigma) == (0.4, pytest.approx(0.3))
    assert S.skew_normal_pdf(0.1, mu, sigma, 0.0) == pytest.approx(stats.norm.pdf(0.1, 0.4, 0.3), rel=1e-12)


def test_schedule_shape_and_average():
    """Low at the start, rising, low again at the end (Section 5.3), average = total prune possibility."""
    p = S.prune_schedule(100, 0.4, 0.5, 0.05, 2.0)
    assert p.mean() == pytest.approx(0.4, rel=1e-12)
    k = int(np.argmax(p))
    assert 0 < k < 99 and np.all(np.diff(p[:k + 1]) > 0) and np.all(np.diff(p[k:]) < 0)    # one hump
    assert p[0] < 0.4 and p[-1] < 0.4
    assert k < 50                                            # positive skew: the hump sits before the mean time
    q = S.prune_schedule(100, 0.4, 0.5, 0.05, -2.0)
    assert np.allclose(q, p[::-1], rtol=1e-12)               # mirrored skew mirrors the curve
    c = S.prune_schedule(50, 0.6, 0.5, 0.01, 0.0, p_max=0.9)
    assert c.max() == 0.9 and c.min() >= 0.0                 # clipped


@pytest.mark.parametrize("mean,var,lam", CASES)
def test_library_schedule_matches_the_oracle(mean, var, lam):
    lib = ard.lib()
    mu, sigma = C.c_double(), C.c_double()
    assert lib.ard_skew_normal_params(mean, var, lam, C.byref(mu), C.byref(sigma)) == 0
    omu, osig = S.skew_normal_params(mean, var, lam)
    assert mu.value == pytest.approx(omu, rel=1e-13) and sigma.value == pytest.approx(osig, rel=1e-13)
    for y in (0.0, 0.2, 0.5, 0.9, 1.3):
        assert lib.ard_skew_normal_pdf(y, omu, osig, lam) == pytest.approx(S.skew_normal_pdf(y, omu, osig, lam), rel=1e-12, abs=1e-300)
        # ... and against the library routine directly
        assert lib.ard_skew_normal_pdf(y, omu, osig, lam) == pytest.approx(stats.skewnorm.pdf(y, lam, loc=omu, scale=osig), rel=1e-10, abs=1e-300)
    for n, total, pmax in ((100, 0.4, 1.0), (7, 0.55, 0.8), (1, 0.3, 1.0)):
        out = (C.c_double * n)()
        assert lib.ard_prune_schedule(n, total, mean, var, lam, pmax, out) == 0
        assert np.allclose(np.array(out), S.prune_schedule(n, total, mean, var, lam, pmax), rtol=1e-12, atol=1e-15)


def test_library_schedule_argument_errors():
    lib = ard.lib()
    out = (C.c_double * 4)()
    assert lib.ard_prune_schedule(0, 0.4, 0.5, 0.05, 1.0, 1.0, out) == -2
    assert lib.ard_prune_schedule(4, 1.4, 0.5, 0.05, 1.0, 1.0, out) == -1
    assert lib.ard_prune_schedule(4, 0.4, 0.5, -0.05, 1.0, 1.0, out) == -1
    assert lib.ard_prune_schedule(4, 0.4, 0.5, 0.05, 1.0, 1.0, None) == -1
    assert lib.ard_skew_normal_params(0.5, 0.0, 1.0, None, None) == -1
