"""Oracle of the cache-provisioning model (Sec. 4.2, Eq. 1-4, Algorithm 1), fp64.

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the product path.  Plain and slow: it
takes the algorithm's steps in the paper's order and notation, one candidate M at a time, one
adapter i at a time, with the dynamic programme over the Poisson-binomial distribution written
out as stated.  Library primitives used as steps: scipy's regularized incomplete gamma function
(the Poisson tail of Eq. 2) and numpy array arithmetic.

Reading taken where the paper is silent: Eq. 2 defines Q(lambda, tau) = Pr[Poisson(lambda) > tau]
with tau as the upper limit of a sum, i.e. for integer tau, while Eq. 3 asks for the tau* at which
the q_i sum to M exactly, which needs a continuous tau.  Q is therefore extended to real
tau >= -1 by Q(lambda, tau) = P(tau + 1, lambda), the regularized lower incomplete gamma
function, which equals the sum of Eq. 2 at every integer tau.  Adapters with p_i = 0 are never
resident (q_i = 0).  If M is at least the number of adapters with p_i > 0, all of those are
resident (tau* = -1, q_i = 1).
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import gammainc


def poisson_tail(lam, tau):
    """Q(lambda, tau) = Pr[Poisson(lambda) > tau] (Eq. 2), continuous in tau >= -1."""
    lam = np.asarray(lam, dtype=np.float64)
    out = np.zeros_like(lam)
    pos = lam > 0
    if tau <= -1.0:
        out[pos] = 1.0
    else:
        out[pos] = gammainc(tau + 1.0, lam[pos])
    return out


def poisson_tail_by_sum(lam: float, tau: int) -> float:
    """Eq. 2 as printed, for integer tau: 1 - sum_{k=0}^{tau} lambda^k exp(-lambda) / k!."""
    if lam <= 0:
        return 0.0
    s = 0.0
    for k in range(0, tau + 1):
        s += math.exp(k * math.log(lam) - lam - math.lgamma(k + 1))
    return 1.0 - s


def solve_threshold(lam, M: int, iters: int = 200) -> float:
    """tau* with sum_i Q(lambda_i, tau*) = M (Eq. 3), by bisection; the sum decreases in tau."""
    lam = np.asarray(lam, dtype=np.float64)
    n_pos = int((lam > 0).sum())
    if M >= n_pos:
        return -1.0
    lo, hi = -1.0, 1.0
    while poisson_tail(lam, hi).sum() > M:
        hi = 2.0 * hi + 1.0
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if poisson_tail(lam, mid).sum() > M:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def slots_distribution_without(q, i: int) -> np.ndarray:
    """dp[k] = Pr[exactly k of the adapters j != i are resident], each independently with
    probability q_j: the dynamic programme of Algorithm 1."""
    N = len(q)
    dp = np.zeros(N + 1, dtype=np.float64)
    dp[0] = 1.0
    for j in range(N):
        if j == i:
            continue
        # for k = N-1 down to 1: dp[k] = dp[k] (1 - q_j) + dp[k-1] q_j; then dp[0] *= (1 - q_j).
        # The descending order makes every right-hand side use the values from before this j,
        # which is what one array expression over the old dp does.
        dp[1:N] = dp[1:N] * (1.0 - q[j]) + dp[0:N - 1] * q[j]
        dp[0] = dp[0] * (1.0 - q[j])
    return dp


def iar(p, LB: float, M: int):
    """IAR(M) of Eq. 4 together with tau* and the q_i it was computed from."""
    p = np.asarray(p, dtype=np.float64)
    lam = LB * p
    tau = solve_threshold(lam, M)
    q = poisson_tail(lam, tau)
    total = 0.0
    for i in range(len(p)):
        dp = slots_distribution_without(q, i)
        p_free = dp[:M].sum()                       # at most M - 1 of the others resident
        total += p[i] * (q[i] + (1.0 - q[i]) * p_free)
    return total, tau, q


def min_cache(p, LB: float, alpha: float):
    """M* of Eq. 1: the first M = 1, 2, ... with IAR(M) >= alpha (Algorithm 1)."""
    N = len(p)
    for M in range(1, N + 1):
        value, _, _ = iar(p, LB, M)
        if value >= alpha:
            return M, value
    return N, iar(p, LB, N)[0]
