"""Block scoring under a decoder-only transformer, written out from the definitions.
TEST INFRASTRUCTURE ONLY (float64 numpy; slow on purpose; no blocking or fusion).

What is computed (Sec. 2.2, Eq. 1; Alg. 2): for a trace tr of P tokens and a candidate block
Y = (y_1..y_L), log pi(Y|tr) = sum_t log softmax(z_{P+t-2})[y_t], where z_p are the model's
logits at 0-based position p of the sequence [tr, Y] (the chain rule over the block's tokens,
natural log, temperature 1, full vocabulary), and the PRM reward r(Y|tr) = sigmoid(w_r . h),
h being the final-normalised hidden state at the last block token. The paper fixes none of the
transformer's internals (it serves stock Qwen/Llama models); the workload statement does:
pre-norm residual blocks, RMSNorm (eps 1e-6), rotary embedding (rotate-half pairing, base
10000, absolute 0-based positions), grouped-query attention with scale 1/sqrt(head_dim),
SwiGLU feed-forward, no biases, untied vocabulary head.

Two modes. `block_logprobs_full` / `reward_full` recompute every candidate over all P+L
positions with plain causal attention: that is the definition. `prefill` + `score_cached`
keep the prefix keys/values and the last prefix hidden state and run only the L block
positions (the appendix's engineering notes ask for log-probabilities of the last step's tokens
only); tests prove the two modes equal before the second is trusted at large sizes.

`weights` is any object with embed_rows(ids) -> [len(ids), d], layer(l) -> dict with
wqkv [(Hq+2Hkv)*hd, d] (q heads, then k heads, then v heads), wo [d, Hq*hd], wg [F, d],
wu [F, d], wd [d, F], head() -> [V, d] or [1, d], gains() -> dict(attn, ffn, final) of [d].
`desc` carries n_layers, d_model, n_q_heads, n_kv_heads, head_dim, rope_base, rms_eps, dtype.
"""
from dataclasses import dataclass
from typing import List, Optional
import numpy as np
from .rounding import operand


def log_softmax(z):
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def rms_norm(x, gain, eps):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * gain


def rope(x, pos, base):
    """x [T, H, hd], pos [T]: pair (i, i + hd/2) rotated by angle pos * base**(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def linear(a, w):
    """y = a W^T for W stored [out_features, in_features]."""
    return np.asarray(a, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def token_logprob(a, w_head, targets):
    """log softmax(a W^T)[target] per row: the chain-rule term of one token."""
    lp = log_softmax(linear(a, w_head))
    return lp[np.arange(len(targets)), np.asarray(targets)]


def swiglu_ffn(a, wg, wu, wd, dtype):
    act = operand(silu(a @ wg.T) * (a @ wu.T), dtype)
    return act @ wd.T


def attention(q, k, v, mask, dtype):
    """q [T, Hq, hd]; k, v [S, Hkv, hd]; mask [T, S] (True = may attend) -> [T, Hq*hd].

    Query head h reads key/value head h // (Hq/Hkv). out = softmax(q k^T / sqrt(hd)) v. The softmax weights
    are rounded as a matrix operand in un-normalised form relative to a power-of-two reference:
    w = 2^(s' - ceil(max s')) with s' = s log2(e), i.e. the row's weights divided by the smallest power of two
    that is not below the largest of them. Rounding to bf16 commutes with scaling by a power of two, so ANY
    power-of-two reference yields the same rounded operand up to that scale: an evaluation that walks the keys in
    tiles and only knows a running maximum rounds the same values as this one, which knows the global maximum.
    The normaliser sums the unrounded weights.
    """
    T, Hq, hd = q.shape
    S, Hkv, _ = k.shape
    g = Hq // Hkv
    scale = 1.0 / np.sqrt(float(hd))
    log2e = 1.0 / np.log(2.0)
    out = np.empty((T, Hq, hd), dtype=np.float64)
    step = max(1, (1 << 25) // max(S, 1))
    for h in range(Hq):
        kh, vh = k[:, h // g, :], v[:, h // g, :]
        for t0 in range(0, T, step):
            t1 = min(T, t0 + step)
            s2 = (q[t0:t1, h, :] @ kh.T) * (scale * log2e)
            s2 = np.where(mask[t0:t1], s2, -np.inf)
            w = np.exp2(s2 - np.ceil(s2.max(axis=-1, keepdims=True)))
            out[t0:t1, h, :] = (operand(w, dtype) @ vh) / w.sum(axis=-1, keepdims=True)
    return out.reshape(T, Hq * hd)


@dataclass
class PrefixCache:
    length: int
    K: List[np.ndarray]            # per layer [P, Hkv, hd], operand-rounded, after RoPE
    V: List[np.ndarray]
    h_last: np.ndarray             # [d] residual-stream output of the last layer at position P-1


def _f64(w):
    return np.asarray(w, dtype=np.float64)


def forward_sequences(desc, weights, tokens, prefixes: Optional[List[Optional[PrefixCache]]] = None,
                      collect_kv=False):
    """Run the trunk over groups of sequences, layer by layer.

    tokens: list of int arrays [Bt, T_j] (group j); prefixes[j]: PrefixCache shared by all the
    sequences of group j, or None (sequence starts at position 0).
    Returns (hidden: list of [Bt, T_j, d] final residual streams, kv: per group per layer (K, V)
    of sequence 0 of the group if collect_kv).
    """
    d, Hq, Hkv, hd = desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    dt = desc.dtype
    gains = weights.gains()
    groups = [np.asarray(t) for t in tokens]
    if prefixes is None:
        prefixes = [None] * len(groups)
    xs = [_f64(weights.embed_rows(t.reshape(-1))).reshape(t.shape[0], t.shape[1], d) for t in groups]
    kv = [[] for _ in groups]
    for l in range(desc.n_layers):
        w = {k: _f64(v) for k, v in weights.layer(l).items()}
        for j, x in enumerate(xs):
            Bt, T, _ = x.shape
            pc = prefixes[j]
            P = 0 if pc is None else pc.length
            pos = P + np.arange(T)
            a = operand(rms_norm(x, gains["attn"], desc.rms_eps), dt)
            qkv = a.reshape(Bt * T, d) @ w["wqkv"].T
            qkv = qkv.reshape(Bt, T, Hq + 2 * Hkv, hd)
            mask = np.concatenate([np.ones((T, P), dtype=bool), np.tril(np.ones((T, T), dtype=bool))], axis=1)
            o = np.empty((Bt, T, Hq * hd))
            for b in range(Bt):
                q = operand(rope(qkv[b, :, :Hq], pos, desc.rope_base), dt)
                k = operand(rope(qkv[b, :, Hq:Hq + Hkv], pos, desc.rope_base), dt)
                v = operand(qkv[b, :, Hq + Hkv:], dt)
                if collect_kv and b == 0:
                    kv[j].append((k, v))
                if pc is not None:
                    k = np.concatenate([pc.K[l], k], axis=0)
                    v = np.concatenate([pc.V[l], v], axis=0)
                o[b] = operand(attention(q, k, v, mask, dt), dt)
            x = x + (o.reshape(Bt * T, Hq * hd) @ w["wo"].T).reshape(Bt, T, d)
            a2 = operand(rms_norm(x, gains["ffn"], desc.rms_eps), dt)
            x = x + swiglu_ffn(a2.reshape(Bt * T, d), w["wg"], w["wu"], w["wd"], dt).reshape(Bt, T, d)
            xs[j] = x
        del w
    return xs, kv


def _token_logprobs(desc, weights, h_prev, targets):
    """h_prev [R, d]: residual stream at the position preceding each scored token; targets [R]."""
    a = operand(rms_norm(h_prev, weights.gains()["final"], desc.rms_eps), desc.dtype)
    z = a @ _f64(weights.head()).T
    lp = log_softmax(z)
    return lp[np.arange(len(targets)), targets]


def _reward(desc, weights, h):
    """h [R, d] at the last block token -> sigmoid(w_r . RMSNorm(h)); the normalised state is not rounded."""
    a = rms_norm(h, weights.gains()["final"], desc.rms_eps)
    s = a @ _f64(weights.head()).reshape(-1)
    return 1.0 / (1.0 + np.exp(-s))


def block_logprobs_full(desc, weights, prefix_tokens, cand):
    """Definition: every candidate recomputed over [tr, Y_i]. cand [n, L] -> (block [n], token [n, L])."""
    cand = np.asarray(cand)
    n, L = cand.shape
    P = len(prefix_tokens)
    seqs = np.concatenate([np.tile(np.asarray(prefix_tokens)[None, :], (n, 1)), cand], axis=1)
    (x,), _ = forward_sequences(desc, weights, [seqs])
    tok = _token_logprobs(desc, weights, x[:, P - 1:P + L - 1, :].reshape(n * L, -1), cand.reshape(-1)).reshape(n, L)
    block = np.array([sum(float(v) for v in row) for row in tok])
    return block, tok


def reward_full(desc, weights, prefix_tokens, cand):
    cand = np.asarray(cand)
    n, L = cand.shape
    seqs = np.concatenate([np.tile(np.asarray(prefix_tokens)[None, :], (n, 1)), cand], axis=1)
    (x,), _ = forward_sequences(desc, weights, [seqs])
    return _reward(desc, weights, x[:, -1, :])


def prefill(desc, weights, prefix_tokens_list):
    """Keys/values and last hidden state of each prefix (list of token arrays) -> list of PrefixCache."""
    toks = [np.asarray(t)[None, :] for t in prefix_tokens_list]
    xs, kv = forward_sequences(desc, weights, toks, collect_kv=True)
    return [PrefixCache(t.shape[1], [k for k, _ in kvj], [v for _, v in kvj], x[0, -1, :].copy())
            for t, x, kvj in zip(toks, xs, kv)]


def score_cached(desc, weights, caches, cand):
    """cand [B, n, L] scored against caches[b]. LM head: (block [B,n], token [B,n,L]); PRM head: reward [B,n]."""
    cand = np.asarray(cand)
    B, n, L = cand.shape
    xs, _ = forward_sequences(desc, weights, [cand[b] for b in range(B)], prefixes=list(caches))
    if getattr(desc, "head", "lm") == "prm":
        return np.stack([_reward(desc, weights, x[:, -1, :]) for x in xs])
    tok = np.empty((B, n, L))
    for b, x in enumerate(xs):
        h_prev = np.concatenate([np.tile(caches[b].h_last[None, None, :], (n, 1, 1)), x[:, :L - 1, :]], axis=1)
        tok[b] = _token_logprobs(desc, weights, h_prev.reshape(n * L, -1), cand[b].reshape(-1)).reshape(n, L)
    block = np.array([[sum(float(v) for v in tok[b, i]) for i in range(n)] for b in range(B)])
    return block, tok
