"""Step I of Alg. 1: the generator draws n candidate blocks of L tokens each from pi_gen(.|tr), one token at a
time, and the block log-likelihood log pi_gen(Y_i|tr) falls out of the same pass. TEST INFRASTRUCTURE ONLY.

Ancestral sampling written out: for t = 1..L the next-token distribution is the full softmax (temperature 1) of
the model's logits at the preceding position, and the token is read off the inverse distribution function in
vocabulary-id order from a given uniform u in [0,1): y = min{k : c_k > u * c_V}, c_k = sum_{v<=k} exp(z_v - max z)
accumulated sequentially in float64 (the same convention as the candidate selection of Alg. 2; if rounding leaves
no such k, the last id of positive weight). The random numbers are inputs, so the procedure is deterministic.

Every new token is pushed through the trunk with `forward_sequences` against a per-candidate cache (the shared
prefix cache extended by the candidate's own earlier tokens): nothing here re-implements the transformer.
"""
import numpy as np
from .rounding import operand
from .transformer import PrefixCache, forward_sequences, rms_norm, _f64


def sample_token(z, u, with_interval=False):
    """(token id, log softmax(z)[token]) for one row of logits z and one uniform u; with_interval adds the
    interval [c_{k-1}/c_V, c_k/c_V) of uniforms that map to the token."""
    if not (0.0 <= u < 1.0):
        raise ValueError("u must lie in [0,1)")
    m = float(np.max(z))
    w = np.exp(z - m)
    c = np.cumsum(w)                      # sequential, in id order
    thr = u * c[-1]
    k = int(np.searchsorted(c, thr, side="right"))        # first index with c_k > thr
    if k >= len(z):
        k = int(np.nonzero(w > 0)[0][-1])
    lp = float(z[k]) - m - float(np.log(c[-1]))
    if with_interval:
        return k, lp, ((float(c[k - 1]) if k else 0.0) / float(c[-1]), float(c[k]) / float(c[-1]))
    return k, lp


def generate_blocks(desc, weights, cache: PrefixCache, n, L, u, vocab_limit=None, p_max=None):
    """u [n, L] uniforms; vocab_limit: only the first vocab_limit ids may be drawn (softmax restricted to them).
    p_max: optional float array [n, L] that receives the largest single-id probability of every sampled distribution
    (a test that accepts an id other than the drawn one bounds the probability mass between the two with it).
    Returns (tokens [n, L] int64, token log-probs [n, L], block log-probs [n],
    caches: per candidate the prefix cache extended by its block, whose h_last is the state at its last token,
    bounds [n, L, 2]: the interval of uniforms that maps to each drawn token)."""
    u = np.asarray(u, dtype=np.float64).reshape(n, L)
    head = _f64(weights.head())
    gain = weights.gains()["final"]
    caches = [PrefixCache(cache.length, list(cache.K), list(cache.V), cache.h_last.copy()) for _ in range(n)]
    tokens = np.zeros((n, L), dtype=np.int64)
    logp = np.zeros((n, L))
    bounds = np.zeros((n, L, 2))
    for t in range(L):
        H = np.stack([c.h_last for c in caches])
        z = operand(rms_norm(H, gain, desc.rms_eps), desc.dtype) @ head.T
        if vocab_limit:
            z = z[:, :vocab_limit]
        for i in range(n):
            tokens[i, t], logp[i, t], bounds[i, t] = sample_token(z[i], float(u[i, t]), with_interval=True)
            if p_max is not None:
                p_max[i, t] = 1.0 / float(np.exp(z[i] - np.max(z[i])).sum())
        xs, kv = forward_sequences(desc, weights, [tokens[i:i + 1, t:t + 1] for i in range(n)], prefixes=caches,
                                   collect_kv=True)
        caches = [PrefixCache(c.length + 1,
                              [np.concatenate([c.K[l], kv[i][l][0]], axis=0) for l in range(desc.n_layers)],
                              [np.concatenate([c.V[l], kv[i][l][1]], axis=0) for l in range(desc.n_layers)],
                              xs[i][0, -1, :].copy()) for i, c in enumerate(caches)]
    block = np.array([sum(float(v) for v in row) for row in logp])
    return tokens, logp, block, caches, bounds
