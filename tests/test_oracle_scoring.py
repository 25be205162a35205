"""Pins of the oracle's block scoring: library second opinion, brute-force normalisation,
cache = recompute, shared prefix = independent runs, causality, importance-weight identity."""
import itertools
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workload as W
from workload.configs import HostWeights, ModelDesc


def toy(role, V=4, nl=2, d=16, hq=4, hkv=2, hd=4, f=24, dtype="f32", head="lm"):
    return ModelDesc(role, nl, d, hq, hkv, hd, f, V, dtype, head)


class BigWeights(HostWeights):
    """Same streams, but a larger std so that toy models are far from uniform."""
    def _gen(self, name, shape, rows=None):
        return super()._gen(name, shape, rows) * 25.0


def torch_library_logprobs(desc, hw, seq, P, L):
    """The same model from torch library ops (sdpa with is_causal, rms_norm, silu, cross_entropy)
    and a complex-number RoPE: an independent formulation, float64, no cache, no rounding."""
    d, Hq, Hkv, hd = desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    seq = torch.as_tensor(np.asarray(seq), dtype=torch.long)
    Tn = len(seq)
    x = torch.from_numpy(hw.embed_rows(seq.numpy())).double()
    ang = torch.arange(Tn).double()[:, None] * desc.rope_base ** (-torch.arange(hd // 2).double() * 2 / hd)
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]

    def rope(t):
        c = torch.complex(t[..., :hd // 2], t[..., hd // 2:]) * rot
        return torch.cat([c.real, c.imag], -1)

    for l in range(desc.n_layers):
        w = {k: torch.from_numpy(v).double() for k, v in hw.layer(l).items()}
        a = F.rms_norm(x, (d,), None, desc.rms_eps)
        qkv = (a @ w["wqkv"].T).view(Tn, Hq + 2 * Hkv, hd)
        q, k, v = rope(qkv[:, :Hq]), rope(qkv[:, Hq:Hq + Hkv]), qkv[:, Hq + Hkv:]
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)[0].transpose(0, 1).reshape(Tn, Hq * hd)
        x = x + o @ w["wo"].T
        a = F.rms_norm(x, (d,), None, desc.rms_eps)
        x = x + (F.silu(a @ w["wg"].T) * (a @ w["wu"].T)) @ w["wd"].T
    if desc.head == "prm":
        return None, x
    z = F.rms_norm(x, (d,), None, desc.rms_eps) @ torch.from_numpy(hw.head()).double().T
    nll = F.cross_entropy(z[P - 1:P + L - 1], seq[P:P + L], reduction="none")
    return (-nll).numpy(), x


def test_full_mode_matches_library_formulation_on_tiny_config():
    c = W.get_config("c1_tiny")
    pt, cand = c.prefix_tokens()[0], c.candidates()[0]
    for desc in (c.target, c.draft):
        hw = BigWeights(desc)
        blk, tok = oracle.block_logprobs_full(desc, hw, pt, cand)
        for i in range(c.n):
            want, _ = torch_library_logprobs(desc, hw, np.concatenate([pt, cand[i]]), len(pt), c.L)
            assert np.allclose(tok[i], want, atol=1e-10)
            assert abs(blk[i] - want.sum()) < 1e-10
    assert np.ptp(blk) > 1.0      # the comparison is not vacuous: candidates differ


def test_reward_matches_library_formulation():
    c = W.get_config("c1_tiny")
    pt, cand = c.prefix_tokens()[0], c.candidates()[0]
    hw = BigWeights(c.prm)
    r = oracle.reward_full(c.prm, hw, pt, cand)
    for i in range(c.n):
        _, x = torch_library_logprobs(c.prm, hw, np.concatenate([pt, cand[i]]), len(pt), c.L)
        h = F.rms_norm(x[-1], (c.prm.d_model,), None, c.prm.rms_eps)
        want = torch.sigmoid(h @ torch.from_numpy(hw.head()).double()[0]).item()
        assert abs(r[i] - want) < 1e-12
    assert np.ptp(r) > 1e-3


@pytest.mark.parametrize("V,L", [(3, 3), (4, 2)])
def test_block_probabilities_sum_to_one_over_all_blocks(V, L):
    desc = toy("target", V=V)
    hw = BigWeights(desc)
    prefix = np.array([1, 0, 2])
    blocks = np.array(list(itertools.product(range(V), repeat=L)))
    blk, tok = oracle.block_logprobs_full(desc, hw, prefix, blocks)
    assert abs(np.exp(blk).sum() - 1.0) < 1e-12
    assert np.exp(blk).max() > 2.0 / len(blocks)     # far from uniform, so the sum is a real check
    # marginal of the first token equals the next-token distribution after the prefix
    p1 = np.array([np.exp(blk[blocks[:, 0] == a]).sum() for a in range(V)])
    assert np.allclose(p1, np.exp([tok[np.argmax(blocks[:, 0] == a), 0] for a in range(V)]), atol=1e-12)


def test_importance_weight_identity_on_enumerable_space():
    """sum_y pi_gen(y) e^{S(y)} = sum_y pi_target(y) e^{beta r(y)}  (Eqs. 3-4; Z under either sampler)."""
    V, L, beta = 3, 2, 1.7
    tgt, drf, prm = toy("target", V=V), toy("draft", V=V, nl=1), toy("prm", V=V, head="prm")
    prefix = np.array([2, 1])
    blocks = np.array(list(itertools.product(range(V), repeat=L)))
    lt, _ = oracle.block_logprobs_full(tgt, BigWeights(tgt), prefix, blocks)
    ld, _ = oracle.block_logprobs_full(drf, BigWeights(drf), prefix, blocks)
    r = oracle.reward_full(prm, BigWeights(prm), prefix, blocks)
    S = np.array(oracle.scores(lt, ld, r, beta))
    z_gen = (np.exp(ld) * np.exp(S)).sum()
    z_tgt = (np.exp(lt) * np.exp(beta * r)).sum()
    assert abs(z_gen - z_tgt) < 1e-12 * z_tgt
    # and the tilted policy is the same distribution in both forms
    assert np.allclose(np.exp(ld + S) / z_gen, np.exp(lt + beta * r) / z_tgt, atol=1e-14)
    assert np.abs(lt - ld).max() > 0.1


def small_gqa(dtype):
    t = ModelDesc("target", 2, 128, 4, 2, 32, 320, 257, dtype, "lm")
    return t, ModelDesc("prm", 2, 128, 4, 2, 32, 320, 257, dtype, "prm")


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-9), ("bf16", 2e-3)])
def test_cached_mode_equals_full_recompute(dtype, tol):
    c = W.get_config("c1_tiny")
    cases = [(c.target, c.prm, c.prefix_tokens()[0], c.candidates()[0])] if dtype == "f32" else []
    t, p = small_gqa(dtype)
    toks = W.rng.uniform_tokens(3, "t", 40 + 3 * 9, 257)
    cases.append((t, p, toks[:40], toks[40:].reshape(3, 9)))
    for lm, prm, pt, cand in cases:
        hw, hp = HostWeights(lm), HostWeights(prm)
        blk, tok = oracle.block_logprobs_full(lm, hw, pt, cand)
        blk2, tok2 = oracle.score_cached(lm, hw, oracle.prefill(lm, hw, [pt]), cand[None])
        assert np.abs(tok2[0] - tok).max() < tol and np.abs(blk2[0] - blk).max() < tol * 10
        r = oracle.reward_full(prm, hp, pt, cand)
        r2 = oracle.score_cached(prm, hp, oracle.prefill(prm, hp, [pt]), cand[None])
        assert np.abs(r2[0] - r).max() < tol


def test_shared_prefix_equals_independent_runs_and_candidates_do_not_interact():
    t, _ = small_gqa("f32")
    hw = HostWeights(t)
    toks = W.rng.uniform_tokens(5, "t", 24 + 4 * 6, 257)
    pt, cand = toks[:24], toks[24:].reshape(4, 6)
    caches = oracle.prefill(t, hw, [pt])
    blk, tok = oracle.score_cached(t, hw, caches, cand[None])
    for i in range(4):
        b1, t1 = oracle.score_cached(t, hw, caches, cand[None, i:i + 1])
        assert np.allclose(t1[0, 0], tok[0, i], atol=1e-12)
    perm = np.array([2, 0, 3, 1])
    bp, _ = oracle.score_cached(t, hw, caches, cand[None, perm])
    assert np.allclose(bp[0], blk[0, perm], atol=1e-12)
    c2 = cand.copy(); c2[1] = (c2[1] + 1) % 257
    b2, _ = oracle.score_cached(t, hw, caches, c2[None])
    assert np.allclose(np.delete(b2[0], 1), np.delete(blk[0], 1), atol=1e-12) and abs(b2[0, 1] - blk[0, 1]) > 1e-6
    # two prefixes in one call = two calls
    pt2 = toks[3:20]
    both = oracle.prefill(t, hw, [pt, pt2])
    bb, _ = oracle.score_cached(t, hw, both, np.stack([cand, cand]))
    b_alone, _ = oracle.score_cached(t, hw, oracle.prefill(t, hw, [pt2]), cand[None])
    assert np.allclose(bb[0], blk[0], atol=1e-12) and np.allclose(bb[1], b_alone[0], atol=1e-12)
    assert np.abs(bb[1] - bb[0]).max() > 1e-6


def test_causality_within_the_block():
    t, _ = small_gqa("f32")
    hw = HostWeights(t)
    toks = W.rng.uniform_tokens(6, "t", 16 + 2 * 8, 257)
    pt, cand = toks[:16], toks[16:].reshape(2, 8)
    cand[1, 0] = cand[0, 0]                       # same first token => same first log-prob
    caches = oracle.prefill(t, hw, [pt])
    _, tok = oracle.score_cached(t, hw, caches, cand[None])
    assert abs(tok[0, 0, 0] - tok[0, 1, 0]) < 1e-13
    c2 = cand.copy(); c2[0, 5] = (c2[0, 5] + 7) % 257
    _, tok2 = oracle.score_cached(t, hw, caches, c2[None])
    assert np.allclose(tok2[0, 0, :5], tok[0, 0, :5], atol=1e-13)       # earlier tokens unaffected
    assert np.all(np.abs(tok2[0, 0, 5:] - tok[0, 0, 5:]) > 1e-9)        # token 5 and everything after it change


def test_gqa_equals_mha_with_repeated_kv_weights():
    g = ModelDesc("target", 1, 32, 4, 2, 8, 48, 50, "f32", "lm")
    m = ModelDesc("target", 1, 32, 4, 4, 8, 48, 50, "f32", "lm")
    hw = HostWeights(g)

    class Rep(HostWeights):
        def layer(self, l):
            w = hw.layer(l)
            q, k, v = w["wqkv"][:32], w["wqkv"][32:48].reshape(2, 8, 32), w["wqkv"][48:].reshape(2, 8, 32)
            w["wqkv"] = np.concatenate([q, np.repeat(k, 2, 0).reshape(32, 32), np.repeat(v, 2, 0).reshape(32, 32)])
            return w
        def embed_rows(self, ids): return hw.embed_rows(ids)
        def head(self): return hw.head()

    toks = W.rng.uniform_tokens(8, "t", 20, 50)
    a, _ = oracle.block_logprobs_full(g, hw, toks[:12], toks[12:].reshape(2, 4))
    b, _ = oracle.block_logprobs_full(m, Rep(m), toks[:12], toks[12:].reshape(2, 4))
    assert np.allclose(a, b, atol=1e-12)
