"""Pins of oracle.smc (exact SMC-induced policies on an enumerable space) and of oracle.subsample as the
selection rule of that definition. CPU only."""
import math

import numpy as np
import pytest
from scipy import integrate

import oracle
from oracle import smc
import workload as W


def toy(K=4, seed=3):
    g = np.random.default_rng(seed)
    pt = g.dirichlet(np.ones(K) * 2)
    pd = g.dirichlet(np.ones(K) * 2)
    r = g.uniform(0, 1, K)
    return pt.tolist(), pd.tolist(), r.tolist()


def test_single_draw_returns_the_generator_and_constant_score_changes_nothing():
    pt, pd, r = toy()
    phi = smc.exponentiated_score(pt, pd, r, 2.0)
    assert np.allclose(smc.smc_policy(pd, phi, 1), pd, atol=1e-15)
    for N in (2, 5, 9):
        assert np.allclose(smc.smc_policy(pd, [3.7] * 4, N), pd, atol=1e-14)
        assert abs(sum(smc.smc_policy(pd, phi, N)) - 1) < 1e-13


def test_importance_identity_and_convergence_to_the_tilted_policy():
    """sum_y pi_gen(y) phi(y) = sum_y pi_target(y) exp(beta r(y)) (Eqs. 3-4), and pi_N -> pi*_beta."""
    pt, pd, r = toy()
    beta = 1.5
    phi = smc.exponentiated_score(pt, pd, r, beta)
    assert math.isclose(sum(g * f for g, f in zip(pd, phi)), sum(t * math.exp(beta * x) for t, x in zip(pt, r)),
                        rel_tol=1e-13)
    star = smc.tilted_policy(pt, r, beta)
    kls = [smc.kl(smc.smc_policy(pd, phi, N), star) for N in (1, 2, 4, 8, 16, 32)]
    assert all(a > b for a, b in zip(kls, kls[1:]))
    assert kls[-1] < 2e-3 and kls[-1] < kls[0] / 50


def test_two_point_instance_matches_the_papers_integral():
    """Lower-bound instance (appendix, proof of the lower-bound theorem): Y = {y0, y1}, r = (0, R),
    pi_target(y1) = 1/(1+theta), theta = exp(beta R), generator = target. The paper gives the Poissonised policy as
    theta/(1+theta) * n/(1-exp(-n)) * int_0^1 exp(n((theta t + t^theta)/(1+theta) - 1)) dt; the enumeration over
    count vectors must reproduce it, and the tilted policy is (1/2, 1/2)."""
    for line in open(__file__.replace("test_oracle_smc.py", "golden/two_point_instance.txt")):
        if line.startswith("#") or not line.strip():
            continue
        beta, R, p0, p1 = map(float, line.split())
        if beta * R > 5:
            continue                                             # theta beyond what a short Poisson sum resolves
        theta = math.exp(beta * R)
        pt = [theta / (1 + theta), 1 / (1 + theta)]
        r = [0.0, R]
        assert np.allclose(smc.tilted_policy(pt, r, beta), [p0, p1], atol=1e-14)
        phi = smc.exponentiated_score(pt, pt, r, beta)
        for n in (3, 10, 25):
            val, _ = integrate.quad(lambda t: math.exp(n * ((theta * t + t ** theta) / (1 + theta) - 1)), 0, 1,
                                    epsabs=1e-13, epsrel=1e-13)
            want = theta / (1 + theta) * n / (1 - math.exp(-n)) * val
            got = smc.poissonised_policy(pt, phi, n)[0]
            assert abs(got - want) < 1e-10, (beta, R, n, got, want)


def test_poissonised_kl_decays_like_theta_squared_over_n_squared():
    """Upper bound O~(exp(2 beta R) / n^2) (target-sampling corollary) and matching lower bound on the two-point
    instance for n >= exp(beta R): n^2 E[KL] / theta^2 stays within constants as n grows fourfold."""
    beta, R = 1.0, 1.0
    theta = math.exp(beta * R)
    pt = [theta / (1 + theta), 1 / (1 + theta)]
    phi = smc.exponentiated_score(pt, pt, [0.0, R], beta)
    star = [0.5, 0.5]
    c = [n * n * smc.poissonised_kl(pt, phi, star, n) / theta ** 2 for n in (8, 16, 32)]
    assert all(0.005 < x < 5 for x in c), c
    assert max(c) / min(c) < 4 * (math.log(32) / math.log(8)) ** 2, c
    # and for a fixed n the divergence shrinks at least like n^-3/2 between n and 4n
    k8, k32 = (smc.kl(smc.smc_policy(pt, phi, n), star) for n in (8, 32))
    assert k32 < k8 / 4 ** 1.5 * (math.log(32) / math.log(8)) ** 2


def test_best_of_n_is_the_large_beta_limit():
    pt, _, r = toy(K=3, seed=5)
    for N in (2, 6):
        hard = smc.best_of_n_policy(pt, r, N)
        assert abs(sum(hard) - 1) < 1e-14
        soft = smc.smc_policy(pt, smc.exponentiated_score(pt, pt, r, 400.0), N)
        assert np.allclose(hard, soft, atol=1e-12)


def test_subsample_rule_realises_the_smc_policy_in_monte_carlo():
    """Seeded draws from pi_gen pushed through oracle.subsample (Alg. 2 with given uniforms) reproduce the exact
    induced policy within five binomial standard deviations."""
    pt, pd, r = toy(K=4, seed=11)
    beta, N, trials = 2.0, 6, 40000
    phi = smc.exponentiated_score(pt, pd, r, beta)
    exact = smc.smc_policy(pd, phi, N)
    cdf = np.cumsum(pd)
    draws = np.minimum(np.searchsorted(cdf, W.rng.uniform_f64(5, "smc/draws", trials * N), side="right"), 3)
    draws = draws.reshape(trials, N)
    u = W.rng.uniform_f64(5, "smc/u", trials)
    lt, ld, rr = np.log(pt)[draws], np.log(pd)[draws], np.asarray(r)[draws]
    hist = np.zeros(4)
    for t in range(trials):
        hist[draws[t, oracle.subsample(lt[t], ld[t], rr[t], beta, float(u[t]))]] += 1
    for k in range(4):
        sd = math.sqrt(exact[k] * (1 - exact[k]) / trials)
        assert abs(hist[k] / trials - exact[k]) < 5 * sd, (k, hist[k] / trials, exact[k])
