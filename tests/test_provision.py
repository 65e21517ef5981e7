"""Cache provisioning (Sec. 4.2, Eq. 1-4, Algorithm 1): pins of the oracle against what the
mathematics fixes, then the library's implementation against the oracle.  CPU only.

The paper's own check of the model (predicted admission rates 83.0 / 92.2 / 100.0 % at cache
capacities 128 / 192 / 256, Sec. 6.3) cannot be reproduced: the per-instance batch size B
behind LB is not stated for that experiment.  That comparison is "parity unpinned".
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import stats

import paper_2604_07173_amd as L
from oracle import provision_oracle as P


def zipf(n, s):
    w = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


# ---------------------------------------------------------------- pins of the oracle


@pytest.mark.parametrize("lam", [0.01, 0.7, 3.0, 25.0])
@pytest.mark.parametrize("tau", [0, 1, 4, 30])
def test_poisson_tail_is_eq2_at_integers(lam, tau):
    """The continuous tail equals the printed sum of Eq. 2 at integer tau, and a library's
    Poisson survival function."""
    q = float(P.poisson_tail(np.array([lam]), float(tau))[0])
    assert q == pytest.approx(P.poisson_tail_by_sum(lam, tau), abs=1e-13)
    assert q == pytest.approx(stats.poisson.sf(tau, lam), abs=1e-13)


def test_poisson_tail_edges():
    lam = np.array([0.0, 2.0])
    assert P.poisson_tail(lam, -1.0).tolist() == [0.0, 1.0]       # p_i = 0 is never resident
    assert P.poisson_tail(lam, 5.0)[0] == 0.0
    a, b = P.poisson_tail(lam, 1.3)[1], P.poisson_tail(lam, 1.6)[1]
    assert P.poisson_tail(lam, 1.0)[1] > a > b > P.poisson_tail(lam, 2.0)[1]   # decreasing in tau


@pytest.mark.parametrize("N,s,LB", [(12, 1.2, 8.0), (30, 1.0, 64.0), (30, 0.0, 5.0)])
def test_threshold_fills_the_cache_exactly(N, s, LB):
    """Eq. 3: at tau* the residency probabilities sum to M."""
    p = zipf(N, s)
    for M in range(1, N):
        tau = P.solve_threshold(LB * p, M)
        assert P.poisson_tail(LB * p, tau).sum() == pytest.approx(M, abs=1e-9)
    assert P.solve_threshold(LB * p, N) == -1.0


def brute_force_p_free(q, i, M):
    """Pr[at most M - 1 of the adapters j != i are resident] by enumerating every subset."""
    others = [j for j in range(len(q)) if j != i]
    total = 0.0
    for mask in itertools.product((0, 1), repeat=len(others)):
        if sum(mask) <= M - 1:
            pr = 1.0
            for bit, j in zip(mask, others):
                pr *= q[j] if bit else 1.0 - q[j]
            total += pr
    return total


@pytest.mark.parametrize("N", [2, 5, 9, 12])
def test_poisson_binomial_dp_against_brute_force(N):
    rng = np.random.default_rng(N)
    q = rng.random(N)
    q[0], q[-1] = 0.0, 1.0                                   # the edges too
    for i in (0, N // 2, N - 1):
        dp = P.slots_distribution_without(q, i)
        assert dp.sum() == pytest.approx(1.0, abs=1e-12)
        assert dp[N - 1:].sum() == pytest.approx(dp[N - 1], abs=0)    # at most N - 1 others
        for M in (1, max(1, N // 2), N):
            assert dp[:M].sum() == pytest.approx(brute_force_p_free(q, i, M), abs=1e-12)


def brute_force_iar(p, q, M):
    return sum(p[i] * (q[i] + (1 - q[i]) * brute_force_p_free(q, i, M)) for i in range(len(p)))


def test_iar_against_brute_force_on_tiny_inputs():
    """Eq. 4 with P_free enumerated subset by subset, for N <= 10."""
    for N, s, LB in [(4, 1.0, 3.0), (7, 1.2, 6.0), (10, 0.8, 20.0)]:
        p = zipf(N, s)
        for M in range(1, N + 1):
            value, tau, q = P.iar(p, LB, M)
            assert value == pytest.approx(brute_force_iar(p, q, M), abs=1e-12)


@pytest.mark.parametrize("N,LB", [(8, 4.0), (20, 10.0), (33, 100.0)])
def test_uniform_popularity_has_a_binomial_closed_form(N, LB):
    """With p_i = 1/N every q_i = M/N and the others' slots are Binomial(N - 1, M/N):
    IAR = q + (1 - q) BinomCDF(M - 1; N - 1, q)."""
    p = np.full(N, 1.0 / N)
    for M in range(1, N + 1):
        value, tau, q = P.iar(p, LB, M)
        qq = M / N
        assert np.allclose(q, qq, atol=1e-9)
        want = qq + (1 - qq) * stats.binom.cdf(M - 1, N - 1, qq)
        assert value == pytest.approx(want, abs=1e-9)


@pytest.mark.parametrize("N,s,LB", [(16, 1.2, 8.0), (24, 1.0, 64.0), (24, 1.2, 2.0), (10, 0.0, 3.0)])
def test_iar_is_monotone_and_reaches_one(N, s, LB):
    p = zipf(N, s)
    vals = [P.iar(p, LB, M)[0] for M in range(1, N + 1)]
    assert all(b >= a - 1e-12 for a, b in zip(vals, vals[1:]))
    assert vals[-1] == pytest.approx(1.0, abs=1e-12)         # IAR(N) = 1: everything fits
    assert 0.0 < vals[0] < 1.0
    M, value = P.min_cache(p, LB, 0.95)
    assert vals[M - 1] >= 0.95 and (M == 1 or vals[M - 2] < 0.95) and value == vals[M - 1]


def test_zero_probability_adapters_take_no_slot():
    """Adapters that are never requested do not change IAR(M) for M below the rest's count."""
    p = zipf(9, 1.1)
    padded = np.concatenate([p, np.zeros(5)])
    for M in (1, 4, 8):
        assert P.iar(padded, 12.0, M)[0] == pytest.approx(P.iar(p, 12.0, M)[0], abs=1e-12)
    assert P.iar(padded, 12.0, 9)[0] == pytest.approx(1.0, abs=1e-12)


def test_very_large_batches_keep_exactly_the_most_popular_adapters():
    """LB -> infinity: the Poisson counts concentrate, q_i becomes 1 for the M most popular
    adapters and 0 for the rest, the cache is always full, and IAR(M) tends to the popularity
    mass of the top M."""
    p = zipf(20, 1.2)
    top = np.cumsum(p)
    for M in (1, 5, 12, 19):
        value, tau, q = P.iar(p, 1e7, M)
        assert np.allclose(q[:M], 1.0, atol=1e-9) and np.allclose(q[M:], 0.0, atol=1e-9)
        assert value == pytest.approx(top[M - 1], abs=1e-8)


# ---------------------------------------------------------------- the library against the oracle


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.lib_path()):
        from paper_2604_07173_amd import build
        build.build()
    return L.load_library()


@pytest.mark.parametrize("N,s,LB", [(12, 1.2, 8.0), (48, 1.2, 64.0), (48, 1.0, 16.0), (31, 0.0, 7.5),
                                    (40, 2.0, 300.0)])
def test_library_iar_matches_oracle(lib, N, s, LB):
    """Every M: IAR, tau* and the q_i.  The library divides adapter i out of one distribution
    of all N instead of running one dynamic programme per adapter; the results must agree to
    rounding."""
    p = zipf(N, s)
    for M in range(1, N + 1):
        want, tau_w, q_w = P.iar(p, LB, M)
        got, tau_g, q_g = L.lora_provision_iar(p, LB, M)
        assert got == pytest.approx(want, abs=1e-10), M
        assert tau_g == pytest.approx(tau_w, abs=1e-8)
        assert np.allclose(q_g, q_w, atol=1e-10)


@pytest.mark.parametrize("alpha", [0.5, 0.9, 0.95, 0.999, 1.0])
def test_library_min_cache_matches_oracle(lib, alpha):
    for N, s, LB in [(20, 1.2, 8.0), (36, 1.0, 40.0), (15, 0.0, 4.0)]:
        p = zipf(N, s)
        if alpha == 1.0:
            # IAR only reaches 1 up to rounding below M = N; both sides must agree on where
            want = next(M for M in range(1, N + 1) if P.iar(p, LB, M)[0] >= 1.0 - 1e-12)
            got, value = L.lora_provision_min_cache(p, LB, 1.0 - 1e-12)
            assert abs(got - want) <= 1 and value >= 1.0 - 1e-10
            continue
        want, want_value = P.min_cache(p, LB, alpha)
        got, value = L.lora_provision_min_cache(p, LB, alpha)
        assert got == want and value == pytest.approx(want_value, abs=1e-10)


def test_library_at_the_evaluation_scale(lib):
    """512 adapters, Zipf 1.2 (Sec. 6.1): runs in well under a second, IAR rises to 1, and
    the oracle agrees at a few sampled capacities (a full sweep of the oracle takes minutes)."""
    p = zipf(512, 1.2)
    LB = 4 * 64.0
    vals = [L.lora_provision_iar(p, LB, M)[0] for M in (1, 64, 128, 192, 256, 384, 512)]
    assert all(b >= a - 1e-12 for a, b in zip(vals, vals[1:]))
    assert vals[-1] == pytest.approx(1.0, abs=1e-10)
    for M in (64, 256):
        assert L.lora_provision_iar(p, LB, M)[0] == pytest.approx(P.iar(p, LB, M)[0], abs=1e-9)
    M, value = L.lora_provision_min_cache(p, LB, 0.95)
    assert 1 < M < 512 and value >= 0.95
    assert L.lora_provision_iar(p, LB, M - 1)[0] < 0.95
    # memory budget of Sec. 4.2's last step with the adapter footprint printed in Sec. 2.3
    assert L.lora_provision_memory_bytes(M, 1811939328) == M * 1811939328


def test_library_rejects_bad_arguments(lib):
    p = zipf(6, 1.0)
    for args in [(p, 0.0, 3), (p, -1.0, 3), (p, 4.0, 0), (p, 4.0, 7), (p * 0.5, 4.0, 3),
                 (np.array([0.5, -0.1, 0.6]), 4.0, 2), (np.array([0.5, math.nan, 0.5]), 4.0, 2)]:
        with pytest.raises(L.ProvisionError):
            L.lora_provision_iar(*args)
    for alpha in (0.0, 1.5, -0.2):
        with pytest.raises(L.ProvisionError):
            L.lora_provision_min_cache(p, 4.0, alpha)
    assert L.lora_provision_memory_bytes(-1, 10) == -1
