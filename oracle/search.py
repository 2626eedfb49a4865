"""Search for the pattern distribution K (test oracle, CPU only).

Section 3.3 (the algorithm float is missing from the text; this follows the
prose): v in R^N, d = softmax(v), p_u = {(i-1)/i}, loss = distance between the
expected global rate d.p_u and the target p, plus the negative entropy of d;
descend on v until the loss stops moving; return d.

Readings where the paper is silent: squared distance, weights lam_p=1 and
lam_e=1e-3, v0 = 0, full-gradient steps with backtracking, fp64.
"""
import numpy as np


def rate_vector(N: int) -> np.ndarray:
    """p_u[i-1] = (i-1)/i: fraction dropped by a pattern of period dp=i (Section 3.3)."""
    i = np.arange(1, N + 1, dtype=np.float64)
    return (i - 1.0) / i


def softmax(v: np.ndarray) -> np.ndarray:
    e = np.exp(v - np.max(v))
    return e / e.sum()


def loss_terms(d: np.ndarray, p: float, pu: np.ndarray):
    e_p = (float(d @ pu) - p) ** 2                        # rate mismatch
    e_n = float(np.sum(d * np.log(np.maximum(d, 1e-300))))  # negative entropy
    return e_p, e_n


def search_k(p: float, N: int, lam_p: float = 1.0, lam_e: float = 1e-3,
             v0=None, max_steps: int = 200000, tol: float = 1e-15):
    """Returns (d, info).  d sums to 1; d.p_u ~= p."""
    if not (0.0 <= p < 1.0) or N < 1:
        raise ValueError("need 0 <= p < 1 and N >= 1")
    pu = rate_vector(N)
    v = np.zeros(N) if v0 is None else np.array(v0, dtype=np.float64)

    def loss_of(vv):
        d = softmax(vv)
        e_p, e_n = loss_terms(d, p, pu)
        return lam_p * e_p + lam_e * e_n, d

    lr = 1.0
    cur, d = loss_of(v)
    steps = 0
    for steps in range(1, max_steps + 1):
        # dL/dd, then through the softmax Jacobian: dL/dv = d * (g - d.g)
        g = lam_p * 2.0 * (float(d @ pu) - p) * pu + lam_e * (np.log(np.maximum(d, 1e-300)) + 1.0)
        gv = d * (g - float(d @ g))
        while True:
            nxt, dn = loss_of(v - lr * gv)
            if nxt <= cur or lr < 1e-12:
                break
            lr *= 0.5
        v = v - lr * gv
        delta = cur - nxt
        cur, d = nxt, dn
        lr = min(lr * 2.0, 1e6)
        if delta < tol and np.max(np.abs(gv)) < 1e-10:
            break
    return d, dict(steps=steps, loss=cur, rate=float(d @ pu))


def fixed_point_cdf(k: np.ndarray) -> np.ndarray:
    """Quantised cumulative table used by the integer sampler:
    cdf[i] = round(2^32 * sum_{j<=i} k_j), kept non-decreasing, last entry 2^32.
    uint64[N]."""
    c = np.cumsum(np.asarray(k, dtype=np.float64))
    q = np.floor(c * 4294967296.0 + 0.5)
    q = np.minimum(np.maximum(q, 0.0), 4294967296.0).astype(np.uint64)
    q = np.maximum.accumulate(q)
    q[-1] = np.uint64(4294967296)
    return q
