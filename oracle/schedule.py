"""Dynamic dropout-ratio tuning (Section 5.3, Eq. 4-6): the prune possibility over the training
epochs follows a skew-normal curve (test oracle, CPU only, fp64).

Eq. (4): f_Y(y) = (2 / sigma) * phi((y - mu) / sigma) * Phi(lambda * (y - mu) / sigma)
Eq. (5): E(Y) = mu + mu0(lambda) * sigma,   mu0(lambda) = sqrt(2 / pi) * lambda / sqrt(1 + lambda^2)
Eq. (6): D(Y) = sigma0^2(lambda) * sigma^2, sigma0^2 = 1 - mu0^2

The paper gives the curve and how mu and sigma follow from E(Y) and D(Y); it does not say how the curve
is turned into a per-epoch possibility.  Reading taken here: epochs e = 0..n-1 sit at the normalised
times y_e = (e + 1/2) / n; E(Y) and D(Y) are the mean and the variance of the curve in that normalised
time; the possibility of epoch e is proportional to f_Y(y_e), scaled so that the average over the run
equals the total prune possibility, then clipped to [0, p_max].
"""
import math

import numpy as np


def mu0(lam: float) -> float:
    return math.sqrt(2.0 / math.pi) * lam / math.sqrt(1.0 + lam * lam)


def sigma0_sq(lam: float) -> float:
    return 1.0 - mu0(lam) ** 2


def skew_normal_params(mean: float, var: float, lam: float):
    """(mu, sigma) of Eq. (4) from E(Y) = mean and D(Y) = var (Eq. 5 and 6 solved for mu, sigma)."""
    sigma = math.sqrt(var / sigma0_sq(lam))
    return mean - mu0(lam) * sigma, sigma


def std_normal_pdf(z: float) -> float:
    return math.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def std_normal_cdf(z: float) -> float:
    return 0.5 * math.erfc(-z / math.sqrt(2.0))   # (erfc keeps the lower tail: 1 + erf cancels there)


def skew_normal_pdf(y: float, mu: float, sigma: float, lam: float) -> float:
    z = (y - mu) / sigma
    return 2.0 / sigma * std_normal_pdf(z) * std_normal_cdf(lam * z)


def prune_schedule(n_epochs: int, total: float, mean: float, var: float, lam: float, p_max: float = 1.0) -> np.ndarray:
    mu, sigma = skew_normal_params(mean, var, lam)
    f = np.array([skew_normal_pdf((e + 0.5) / n_epochs, mu, sigma, lam) for e in range(n_epochs)], dtype=np.float64)
    p = total * f / f.mean()
    return np.clip(p, 0.0, p_max)
