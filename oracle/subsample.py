"""SubSample (Alg. 2) and the score of Eq. 1 in sequential float64. Test infrastructure.

S_i = log(pi_target(Y_i|tr) / pi_gen(Y_i|tr)) + beta * r(Y_i|tr)            (Eq. 1)
P(i* = i) proportional to exp(S_i) * 1[i in L], L = all candidates unless masked (Alg. 2)

The random choice is made deterministic by a given uniform u in [0,1): inverse CDF in index
order with a strict comparison, i* = min{k : c_k > u * c_n}, c_k = sum_{i<=k} w_i,
w_i = exp(S_i - max S). If rounding leaves no such k, the last live index with w > 0.
"""
import math


def scores(logp_target, logp_gen, reward, beta):
    return [float(lt) - float(lg) + float(beta) * float(r) for lt, lg, r in zip(logp_target, logp_gen, reward)]


def selection_probs(logp_target, logp_gen, reward, beta, mask=None):
    S = scores(logp_target, logp_gen, reward, beta)
    live = [True] * len(S) if mask is None else [bool(m) for m in mask]
    m = max(s for s, l in zip(S, live) if l)
    w = [math.exp(s - m) if l else 0.0 for s, l in zip(S, live)]
    tot = 0.0
    for x in w:
        tot += x
    return [x / tot for x in w]


def subsample(logp_target, logp_gen, reward, beta, u, mask=None):
    """Index chosen by Alg. 2 for the uniform u; -1 if no candidate is live."""
    if not (0.0 <= u < 1.0):
        raise ValueError("u must lie in [0,1)")
    S = scores(logp_target, logp_gen, reward, beta)
    n = len(S)
    live = [True] * n if mask is None else [bool(m) for m in mask]
    if not any(live):
        return -1
    m = -math.inf
    for s, l in zip(S, live):
        if l and s > m:
            m = s
    w = [math.exp(s - m) if l else 0.0 for s, l in zip(S, live)]
    c, run = [], 0.0
    for x in w:
        run += x
        c.append(run)
    thr = u * c[-1]
    for k in range(n):
        if c[k] > thr:
            return k
    for k in range(n - 1, -1, -1):
        if w[k] > 0.0:
            return k
    return -1


def subsample_batch(lt, ld, r, betas, u, mask=None):
    """lt, ld, r: [B][n]; betas: [nb]; u: [B][nb] -> idx [B][nb]; also max reward per prefix."""
    B = len(lt)
    idx = [[subsample(lt[b], ld[b], r[b], betas[j], float(u[b][j]), None if mask is None else mask[b])
            for j in range(len(betas))] for b in range(B)]
    maxr = [max(float(x) for x in r[b]) for b in range(B)]
    return idx, maxr
