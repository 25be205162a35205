"""Pins of the oracle's building blocks against library routines, closed forms and invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F
import scipy.special as sps

import oracle
from oracle import transformer as T

RNG = np.random.default_rng(1234)


def test_round_bf16_matches_library_conversion():
    x32 = (RNG.standard_normal(200000) * np.exp(RNG.uniform(-20, 20, 200000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_bf16(x32.astype(np.float64))
    assert np.array_equal(got, want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert oracle.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # a float64 just above a tie must round up although its float32 image is the tie itself
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    assert np.array_equal(oracle.operand(np.array([1.0 + 2.0 ** -8]), "f32"), np.array([1.0 + 2.0 ** -8]))


def test_log_softmax_rows_normalise_and_match_library():
    z = RNG.standard_normal((7, 513)) * 30.0
    lp = oracle.log_softmax(z)
    assert np.allclose(np.exp(lp).sum(-1), 1.0, atol=1e-12)
    assert np.allclose(lp, sps.log_softmax(z, axis=-1), atol=1e-12)
    # shift invariance and no overflow at huge logits
    assert np.allclose(oracle.log_softmax(z + 1e4), lp, atol=1e-9)


def test_rms_norm():
    x = RNG.standard_normal((5, 64))
    g = RNG.standard_normal(64)
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(oracle.rms_norm(x, g, 1e-6), want, atol=1e-13)
    u = np.sign(RNG.standard_normal((3, 64)))          # rows of +-1 have unit mean square
    assert np.allclose(oracle.rms_norm(u, np.ones(64), 0.0), u, atol=1e-15)


def test_rope_closed_forms():
    x = RNG.standard_normal((6, 3, 16))
    pos = np.array([0, 1, 2, 5, 100, 4095])
    y = oracle.rope(x, pos, 10000.0)
    assert np.allclose(y[0], x[0], atol=0)                              # position 0: identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))   # a rotation
    # complex form: pair (i, i+hd/2) as a complex number times exp(j * pos * base^(-2i/hd))
    zc = (x[..., :8] + 1j * x[..., 8:]) * np.exp(1j * pos[:, None, None] * 10000.0 ** (-np.arange(8) / 8.0))
    assert np.allclose(y[..., :8], zc.real) and np.allclose(y[..., 8:], zc.imag)
    # head_dim 2: a plain planar rotation by angle pos
    v = np.array([[[1.0, 0.0]]])
    r = oracle.rope(v, np.array([0.5]), 10000.0)
    assert np.allclose(r[0, 0], [np.cos(0.5), np.sin(0.5)])
    # scores depend on the position difference only
    q, k = RNG.standard_normal((1, 1, 16)), RNG.standard_normal((1, 1, 16))
    s1 = (oracle.rope(q, [7], 1e4) * oracle.rope(k, [3], 1e4)).sum()
    s2 = (oracle.rope(q, [1007], 1e4) * oracle.rope(k, [1003], 1e4)).sum()
    assert abs(s1 - s2) < 1e-9
    # base -> infinity leaves all but the first pair untouched
    yb = oracle.rope(x, pos, 1e300)
    assert np.allclose(yb[..., 1:8], x[..., 1:8]) and np.allclose(yb[..., 9:], x[..., 9:])


def test_swiglu():
    a = RNG.standard_normal((4, 8))
    wg, wu, wd = RNG.standard_normal((12, 8)), RNG.standard_normal((12, 8)), RNG.standard_normal((8, 12))
    ta, tg, tu, td = map(torch.from_numpy, (a, wg, wu, wd))
    want = ((F.silu(ta @ tg.T) * (ta @ tu.T)) @ td.T).numpy()
    assert np.allclose(oracle.swiglu_ffn(a, wg, wu, wd, "f32"), want, atol=1e-12)
    assert np.all(oracle.swiglu_ffn(a, np.zeros_like(wg), wu, wd, "f32") == 0.0)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_attention_matches_library_sdpa_and_gqa_mapping(Hq, Hkv):
    Tq, S, hd = 5, 9, 8
    q = RNG.standard_normal((Tq, Hq, hd))
    k = RNG.standard_normal((S, Hkv, hd))
    v = RNG.standard_normal((S, Hkv, hd))
    mask = np.concatenate([np.ones((Tq, S - Tq), bool), np.tril(np.ones((Tq, Tq), bool))], 1)
    got = oracle.attention(q, k, v, mask, "f32").reshape(Tq, Hq, hd)
    g = Hq // Hkv
    # library routine, with K/V heads repeated per group by hand (h -> h // g)
    kr, vr = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)
    want = F.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2)[None], torch.from_numpy(kr).permute(1, 0, 2)[None],
        torch.from_numpy(vr).permute(1, 0, 2)[None], attn_mask=torch.from_numpy(mask))[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, atol=1e-12)
    # MHA on the repeated heads is the same thing
    assert np.allclose(oracle.attention(q, kr, vr, mask, "f32").reshape(Tq, Hq, hd), got, atol=1e-14)


def test_attention_zero_query_averages_values():
    S, hd = 7, 4
    v = RNG.standard_normal((S, 1, hd))
    out = oracle.attention(np.zeros((1, 2, hd)), RNG.standard_normal((S, 1, hd)), v, np.ones((1, S), bool), "f32")
    assert np.allclose(out.reshape(2, hd), v[:, 0].mean(0)[None].repeat(2, 0))


def test_attention_bf16_rounds_only_the_softmax_weights():
    """The rounded operand is the un-normalised weight relative to a power-of-two reference, 2^(s' - ceil(max s'));
    any other power-of-two reference gives the same output, and so does a tile-by-tile evaluation that only knows
    a running maximum, as long as its reference exponents are integers."""
    Tq, S, hd = 3, 33, 8
    q, k, v = RNG.standard_normal((Tq, 1, hd)), RNG.standard_normal((S, 1, hd)), RNG.standard_normal((S, 1, hd))
    mask = np.ones((Tq, S), bool)
    s2 = (q[:, 0] @ k[:, 0].T) / np.sqrt(hd) / np.log(2.0)
    ref = np.ceil(s2.max(-1, keepdims=True))
    got = oracle.attention(q, k, v, mask, "bf16")
    for shift in (0, -3, 5):
        w = np.exp2(s2 - ref - shift)
        assert np.allclose(got, (oracle.round_bf16(w) @ v[:, 0]) / w.sum(-1, keepdims=True), atol=1e-15)
    # weights lie in (1/2, 1] at the row maximum, and the unrounded evaluation is the plain softmax
    assert np.all(np.exp2(s2 - ref).max(-1) > 0.5) and np.all(np.exp2(s2 - ref).max(-1) <= 1.0)
    p = np.exp(s2 * np.log(2.0) - (s2 * np.log(2.0)).max(-1, keepdims=True))
    assert np.allclose(oracle.attention(q, k, v, mask, "f32"), (p @ v[:, 0]) / p.sum(-1, keepdims=True), atol=1e-14)
    # streaming evaluation: tiles of 8 keys, integer reference that follows the running maximum
    for t in range(Tq):
        m, l, o = -np.inf, 0.0, np.zeros(hd)
        for k0 in range(0, S, 8):
            st = s2[t, k0:k0 + 8]
            m_new = max(m, np.ceil(st.max()))
            alpha = 0.0 if m == -np.inf else np.exp2(m - m_new)
            w = np.exp2(st - m_new)
            l = l * alpha + w.sum()
            o = o * alpha + oracle.round_bf16(w) @ v[k0:k0 + 8, 0]
            m = m_new
        assert np.allclose(o / l, got[t], atol=1e-14)
    # a non-power-of-two reference (the plain maximum) rounds different values: the reading matters
    w_max = np.exp2(s2 - s2.max(-1, keepdims=True))
    other = (oracle.round_bf16(w_max) @ v[:, 0]) / w_max.sum(-1, keepdims=True)
    assert np.abs(other - got).max() > 1e-6


def test_reward_head_is_a_logistic_of_the_normalised_state():
    class W:
        def gains(self): return {"final": np.ones(4)}
        def head(self): return np.array([[1.0, -2.0, 0.5, 0.0]])
    class D: rms_eps = 0.0; dtype = "f32"
    h = np.array([[2.0, 2.0, -2.0, 2.0], [0.0, 0.0, 0.0, 4.0]])       # rms = 2 for both rows
    r = T._reward(D, W(), h)
    assert np.allclose(r, [1 / (1 + np.exp(1.5)), 0.5])
    assert np.all((r > 0) & (r < 1))


def test_linear_is_the_row_by_row_dot_product_with_stored_rows():
    """y = a W^T for W stored [out, in]: pinned by hand-set operands (a transposed or mis-indexed operand
    gives a different matrix), by explicit dot products, and by the library routine in a different formulation."""
    a = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 0.5]])
    w = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 1.0], [2.0, 2.0, 2.0], [-1.0, 0.5, 0.0]])     # [out=4, in=3]
    want = np.array([[1.0, 5.0, 12.0, 0.0], [0.0, -0.5, -1.0, -0.5]])
    assert np.array_equal(oracle.linear(a, w), want)
    A, Wm = RNG.standard_normal((9, 33)), RNG.standard_normal((17, 33))
    y = oracle.linear(A, Wm)
    assert y.shape == (9, 17)
    for m in (0, 4, 8):
        for n in (0, 7, 16):
            assert abs(y[m, n] - sum(A[m, k] * Wm[n, k] for k in range(33))) < 1e-12
    assert np.allclose(y, F.linear(torch.from_numpy(A), torch.from_numpy(Wm)).numpy(), atol=1e-12)
    # float32 inputs are promoted, not multiplied in float32
    a32, w32 = A.astype(np.float32), Wm.astype(np.float32)
    assert oracle.linear(a32, w32).dtype == np.float64
    assert np.allclose(oracle.linear(a32, w32), a32.astype(np.float64) @ w32.astype(np.float64).T, atol=1e-14)


def test_token_logprob_is_minus_cross_entropy_and_picks_the_right_column():
    """log softmax(a W^T)[target] per row: equals minus the library's per-row cross entropy, sums to one over
    all targets, and on a hand-set case with logits (0, ln 2, ln 3) gives ln(1/6), ln(2/6), ln(3/6)."""
    Wm = np.eye(3)
    a = np.array([[0.0, np.log(2.0), np.log(3.0)]] * 3)
    got = oracle.token_logprob(a, Wm, [0, 1, 2])
    assert np.allclose(got, np.log([1 / 6, 2 / 6, 3 / 6]), atol=1e-15)
    A, Wh = RNG.standard_normal((11, 24)), RNG.standard_normal((50, 24))
    tg = RNG.integers(0, 50, 11)
    z = torch.from_numpy(A) @ torch.from_numpy(Wh).T
    want = -F.cross_entropy(z, torch.from_numpy(tg), reduction="none").numpy()
    assert np.allclose(oracle.token_logprob(A, Wh, tg), want, atol=1e-12)
    # each row is a distribution over targets, and rows do not mix: row r with every target
    for r in (0, 10):
        allp = oracle.token_logprob(np.repeat(A[r:r + 1], 50, axis=0), Wh, np.arange(50))
        assert abs(np.exp(allp).sum() - 1.0) < 1e-12
        assert abs(allp[tg[r]] - want[r]) < 1e-12
    # the model's own vocabulary-head path (final norm with unit gains on unit-mean-square rows = identity)
    class _W:
        def gains(self): return {"final": np.ones(24)}
        def head(self): return Wh
    class _D:
        rms_eps, dtype = 0.0, "f32"
    unit = np.sign(A)
    assert np.allclose(T._token_logprobs(_D, _W(), unit, tg), oracle.token_logprob(unit, Wh, tg), atol=1e-12)


def test_float_accumulation_jitter_is_off_by_default_and_only_moves_rounding_decisions():
    """The tolerance-derivation tool of oracle/rounding.py: outside its context operand() rounds exact values; inside,
    values are perturbed by ~2e-7 relative BEFORE rounding, so an operand either stays the same bf16 value or moves
    by exactly one bf16 unit, and only for the few values that sit next to a rounding boundary. Float operands are
    never touched. With amplitude 0 the context is the identity."""
    x = RNG.standard_normal(400000) * np.exp(RNG.uniform(-8, 8, 400000))
    base = oracle.operand(x, "bf16")
    assert np.array_equal(base, oracle.round_bf16(x))
    with oracle.float_accumulation_jitter(0.0):
        assert np.array_equal(oracle.operand(x, "bf16"), base)
    with oracle.float_accumulation_jitter(2.0e-7, seed=3):
        jit = oracle.operand(x, "bf16")
        assert np.array_equal(oracle.operand(x, "f32"), x)
    assert np.array_equal(oracle.operand(x, "bf16"), base)              # switched off again
    moved = jit != base
    frac = moved.mean()
    # a relative jitter of 2e-7 against a rounding grid of 2^-8 .. 2^-7 relative: about 1e-4 of the values flip
    assert 1e-5 < frac < 1e-3, frac
    ulp = 2.0 ** (np.floor(np.log2(np.abs(base[moved]))) - 7)
    assert np.allclose(np.abs(jit[moved] - base[moved]), ulp, rtol=0, atol=0) or \
        np.all(np.isin(np.abs(jit[moved] - base[moved]) / ulp, (0.5, 1.0, 2.0)))
    # the same seed gives the same perturbation (stored figures are reproducible)
    with oracle.float_accumulation_jitter(2.0e-7, seed=3):
        assert np.array_equal(oracle.operand(x, "bf16"), jit)
