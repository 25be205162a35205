"""Exact induced policies of sequential Monte Carlo selection on a finite response space. Test infrastructure.

Definition (SMC, appendix "Sampling by approximating the partition function"): draw N responses i.i.d. from
pi_gen, then return the i-th with probability proportional to phi(Y_i) = exp(S(Y_i)), where
phi(y) = pi_target(y) / pi_gen(y) * exp(beta * r(y)) is the exponentiated score (Eq. 1). The induced policy
pi_N averages over the draws. On a response space small enough to enumerate, that average is a finite sum over
the possible count vectors (how many of the N draws equal each response), which is what this module writes out.
The optimal tilted policy is pi*_beta(y) proportional to pi_target(y) exp(beta r(y)) (Eqs. 3-4).
Poissonisation: the theory states its rates for N ~ Poisson(n) conditioned on N > 0.
"""
import math


def exponentiated_score(pi_target, pi_gen, reward, beta):
    return [pt / pg * math.exp(beta * r) for pt, pg, r in zip(pi_target, pi_gen, reward)]


def tilted_policy(pi_target, reward, beta):
    w = [pt * math.exp(beta * r) for pt, r in zip(pi_target, reward)]
    z = math.fsum(w)
    return [x / z for x in w]


def _count_vectors(total, parts):
    """All tuples of `parts` non-negative integers that sum to `total`."""
    if parts == 1:
        yield (total,)
        return
    for k in range(total + 1):
        for rest in _count_vectors(total - k, parts - 1):
            yield (k,) + rest


def smc_policy(pi_gen, phi, N):
    """P(Y* = y) for a fixed number N >= 1 of draws: sum over count vectors c (multinomial probability) of
    c_y phi_y / sum_z c_z phi_z."""
    K = len(pi_gen)
    out = [0.0] * K
    logp = [math.log(p) if p > 0 else -math.inf for p in pi_gen]
    for c in _count_vectors(N, K):
        lp = math.lgamma(N + 1)
        for k in range(K):
            if c[k]:
                lp += c[k] * logp[k] - math.lgamma(c[k] + 1)
        if lp == -math.inf:
            continue
        pr = math.exp(lp)
        z = math.fsum(c[k] * phi[k] for k in range(K))
        for k in range(K):
            out[k] += pr * c[k] * phi[k] / z
    return out


def best_of_n_policy(pi_gen, reward, N):
    """Hard selection (the beta -> infinity limit with pi_gen = pi_target): the draw of largest reward wins.
    Rewards must be distinct. P(y) = F(y)^N - F(y-)^N with F the distribution function of the reward under pi_gen."""
    order = sorted(range(len(pi_gen)), key=lambda k: reward[k])
    out, below = [0.0] * len(pi_gen), 0.0
    for k in order:
        out[k] = (below + pi_gen[k]) ** N - below ** N
        below += pi_gen[k]
    return out


def kl(p, q):
    return math.fsum(a * math.log(a / b) for a, b in zip(p, q) if a > 0)


def poisson_positive(n, tail=1e-16):
    """[(N, P(N))] of Poisson(n) conditioned on N > 0, truncated where single terms drop below `tail`."""
    out, N = [], 1
    norm = 1.0 - math.exp(-n)
    while True:
        p = math.exp(-n + N * math.log(n) - math.lgamma(N + 1)) / norm
        out.append((N, p))
        if N > 2 * n and p < tail:                     # past the mode the terms fall faster than geometrically
            return out
        N += 1


def poissonised_policy(pi_gen, phi, n):
    """Mixture of pi_N over N ~ Poisson(n) | N > 0."""
    K = len(pi_gen)
    out = [0.0] * K
    for N, w in poisson_positive(n):
        pN = smc_policy(pi_gen, phi, N)
        for k in range(K):
            out[k] += w * pN[k]
    return out


def poissonised_kl(pi_gen, phi, target, n):
    """E_{N ~ Poisson(n) | N > 0} KL(pi_N || target)."""
    return math.fsum(w * kl(smc_policy(pi_gen, phi, N), target) for N, w in poisson_positive(n))
