"""Pins for the distribution search (Section 3.3) and the pattern sampler (Section 3.4)."""
import json
import os

import numpy as np
import pytest

from oracle import patterns as P
from oracle import sampler as S
from oracle import search as K


def _closed_form(p, N, lam_p, lam_e):
    """Stationary point of (d.pu - p)^2*lam_p + lam_e*sum d ln d on the simplex:
    d_i ~ exp(theta*pu_i), theta solving pg(theta) - p + theta*lam_e/(2 lam_p) = 0
    (monotone in theta) -- solved here by bisection, no gradient descent."""
    i = np.arange(1, N + 1)
    pu = (i - 1) / i

    def d_of(th):
        w = np.exp(th * pu - np.max(th * pu))
        return w / w.sum()

    def f(th):
        return float(d_of(th) @ pu) - p + th * lam_e / (2 * lam_p)
    lo, hi = -1e4, 1e4
    for _ in range(400):
        mid = 0.5 * (lo + hi)
        if f(mid) > 0:
            hi = mid
        else:
            lo = mid
    th = 0.5 * (lo + hi)
    return d_of(th), th


def test_rate_vector_from_paper(golden_dir):
    with open(os.path.join(golden_dir, "paper_examples.json")) as f:
        g = json.load(f)["rate_vector"]
    assert np.allclose(K.rate_vector(g["N"]), g["p_u"], rtol=0, atol=1e-16)


@pytest.mark.parametrize("p", [0.3, 0.5, 0.7])
@pytest.mark.parametrize("N", [4, 8])
def test_search_matches_closed_form(p, N):
    if N == 4 and p > 0.7:
        pytest.skip("unreachable")
    d, info = K.search_k(p, N)
    ref, th = _closed_form(p, N, 1.0, 1e-3)
    assert abs(d.sum() - 1.0) < 1e-12 and np.all(d > 0)
    assert np.max(np.abs(d - ref)) < 2e-5, (d, ref, info)
    pu = K.rate_vector(N)
    # expected global rate hits the target up to the entropy term's pull (Eq. 3: p_g ~= p)
    assert abs(float(d @ pu) - p) <= abs(th) * 1e-3 / 2 + 1e-6
    # E[kept fraction] = E[1/dp] = 1 - p_g
    assert abs(float(d @ (1.0 / np.arange(1, N + 1))) - (1 - float(d @ pu))) < 1e-12


def test_search_entropy_term_prefers_uniform():
    # when the uniform distribution already meets the rate, both loss terms are minimal there
    N = 8
    p = 1.0 - sum(1.0 / i for i in range(1, N + 1)) / N          # = 0.66027...
    assert abs(p - 0.66027) < 1e-5
    d, _ = K.search_k(p, N, v0=np.linspace(-1, 1, N))
    assert np.max(np.abs(d - 1.0 / N)) < 1e-5


def test_search_is_independent_of_start():
    d0, _ = K.search_k(0.5, 8)
    d1, _ = K.search_k(0.5, 8, v0=np.array([2.0, -1, 0.5, 0, 0, 1, -2, 0.3]))
    assert np.max(np.abs(d0 - d1)) < 5e-5


def test_fixed_point_cdf():
    d, _ = K.search_k(0.5, 8)
    cdf = K.fixed_point_cdf(d)
    assert cdf.dtype == np.uint64 and int(cdf[-1]) == 1 << 32
    assert np.all(np.diff(cdf.astype(np.int64)) >= 0)
    steps = np.diff(np.concatenate([[0], cdf.astype(np.float64)])) / 2.0**32
    assert np.max(np.abs(steps - d)) < 2.0**-31
    assert K.fixed_point_cdf(np.array([1.0])).tolist() == [1 << 32]


def test_mixer_is_splitmix64():
    # published first outputs of SplitMix64 seeded with 0
    assert S.mix64(S.GOLDEN) == 0xE220A8397B1DCDAF
    assert S.mix64((2 * S.GOLDEN) & S.M64) == 0x6E789E6AA1B965F4
    assert S.mix64((3 * S.GOLDEN) & S.M64) == 0x06C45D188009454F


def test_sampler_boundaries_exhaustive():
    cdf = [1000, 1000, 5000, 1 << 32]                  # second pattern has probability zero
    for r1, dp in [(0, 1), (999, 1), (1000, 3), (4999, 3), (5000, 4), ((1 << 32) - 1, 4)]:
        got, b = S.pattern_from_words(cdf, r1, 0)
        assert got == dp and b == 1
    for dp_target, r1 in [(1, 0), (3, 1000), (4, 5000)]:
        seen = set()
        for r2 in [0, (1 << 32) // dp_target - 1, min((1 << 32) // dp_target + 1, (1 << 32) - 1), (1 << 31), (1 << 32) - 1]:
            dp, b = S.pattern_from_words(cdf, r1, r2)
            assert dp == dp_target and 1 <= b <= dp and b == 1 + (r2 * dp) // (1 << 32)
            seen.add(b)
        assert max(seen) == dp_target


def test_sampler_is_stateless_and_streams_differ():
    d, _ = K.search_k(0.5, 8)
    cdf = K.fixed_point_cdf(d)
    a = [S.sample_pattern(cdf, 2, it, 1) for it in range(50)]
    assert a == [S.sample_pattern(cdf, 2, it, 1) for it in range(50)]
    assert a != [S.sample_pattern(cdf, 2, it, 2) for it in range(50)]
    assert a != [S.sample_pattern(cdf, 3, it, 1) for it in range(50)]


@pytest.mark.parametrize("p", [0.3, 0.7])
def test_per_neuron_drop_frequency_matches_global_rate(p):
    """Eq. (2)-(3): every neuron's drop probability equals sum_i k_i (i-1)/i = p_g ~= p."""
    N, n, T = 8, 24, 100000
    d, _ = K.search_k(p, N)
    cdf = K.fixed_point_cdf(d)
    pu = K.rate_vector(N)
    pg = float(d @ pu)
    # exact marginal: each neuron is kept by exactly one of the dp biases
    for r in range(n):
        exact = sum(d[dp - 1] * sum(1 for b in range(1, dp + 1) if P.row_mask(n, dp, b)[r] == 0) / dp
                    for dp in range(1, N + 1))
        assert abs(exact - pg) < 1e-12
    masks = {(dp, b): P.row_mask(n, dp, b) for dp in range(1, N + 1) for b in range(1, dp + 1)}
    dropped = np.zeros(n)
    dp_hist = np.zeros(N)
    b_hist = {dp: np.zeros(dp) for dp in range(1, N + 1)}
    for it in range(T):
        dp, b = S.sample_pattern(cdf, 11, it, 0)
        dropped += 1 - masks[(dp, b)]
        dp_hist[dp - 1] += 1
        b_hist[dp][b - 1] += 1
    # sampling noise of the (dependent) indicator is below Bernoulli's, 5 sigma bound
    assert np.max(np.abs(dropped / T - pg)) < 5 * np.sqrt(pg * (1 - pg) / T)
    assert abs(pg - p) < 2.5e-3
    assert np.max(np.abs(dp_hist / T - d)) < 5 * np.sqrt(0.25 / T)
    for dp in range(2, N + 1):
        tot = b_hist[dp].sum()
        assert np.max(np.abs(b_hist[dp] / tot - 1.0 / dp)) < 5 * np.sqrt(0.25 / tot)
