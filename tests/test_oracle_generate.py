"""Pins of the oracle's block generator (Alg. 1, Step I): the inverse-CDF rule against closed forms, the joint law
of a generated block against the block likelihood computed by full recompute, and the incremental cache against
block-parallel scoring of the generated tokens. CPU only."""
import itertools
import math

import numpy as np
import pytest

import oracle
import workload as W
from workload.configs import HostWeights, ModelDesc


class BigWeights(HostWeights):
    def _gen(self, name, shape, rows=None):
        return super()._gen(name, shape, rows) * 25.0


def toy(V=3, dtype="f32"):
    return ModelDesc("draft", 2, 16, 4, 2, 4, 24, V, dtype, "lm")


def test_inverse_cdf_closed_forms():
    z = np.log(np.array([1.0, 2.0, 3.0, 0.0]) + 1e-300)          # weights 1, 2, 3, (0): boundaries 1/6, 1/2
    picks = [oracle.sample_token(z, u)[0] for u in (0.0, 0.1, 1 / 6 + 1e-12, 0.3, 0.5 - 1e-12, 0.5, 0.999999)]
    assert picks == [0, 0, 1, 1, 1, 2, 2]
    k, lp = oracle.sample_token(z, 0.3)
    assert math.isclose(lp, math.log(2 / 6), rel_tol=1e-12)
    assert oracle.sample_token(np.array([-np.inf, 0.0, -np.inf]), 0.0)[0] == 1          # zero-weight ids are never drawn
    assert np.allclose(oracle.sample_token(z, 0.3, with_interval=True)[2], (1 / 6, 1 / 2), atol=1e-15)
    with pytest.raises(ValueError):
        oracle.sample_token(z, 1.0)
    grid = (np.arange(1 << 12) + 0.5) / (1 << 12)
    zz = np.array([0.3, -1.2, 2.0, 0.0, 0.7])
    hist = np.bincount([oracle.sample_token(zz, float(u))[0] for u in grid], minlength=5) / len(grid)
    assert np.allclose(hist, np.exp(zz) / np.exp(zz).sum(), atol=2.0 / len(grid))


def test_joint_law_of_a_generated_block_is_the_block_likelihood():
    """V = 3, L = 2: sweeping (u_1, u_2) over a 96 x 96 midpoint grid, the fraction of the unit square that yields
    block (a, b) must equal exp(log pi(a, b | tr)) from the full-recompute scorer (the definition), and the
    log-probability the generator reports for a block must be that same number."""
    desc = toy()
    hw = BigWeights(desc, 4)
    tr = np.array([2, 0, 1, 1, 2])
    cache = oracle.prefill(desc, hw, [tr])[0]
    blocks = np.array(list(itertools.product(range(3), repeat=2)))
    want, _ = oracle.block_logprobs_full(desc, hw, tr, blocks)
    G = 96
    g = (np.arange(G) + 0.5) / G
    u = np.stack(np.meshgrid(g, g, indexing="ij"), -1).reshape(-1, 2)
    tokens, tok_lp, blk, _, _ = oracle.generate_blocks(desc, hw, cache, len(u), 2, u)
    area = np.zeros(9)
    for (a, b), lp in zip(tokens, blk):
        area[a * 3 + b] += 1.0 / len(u)
        assert abs(lp - want[a * 3 + b]) < 1e-10
    assert np.abs(area - np.exp(want)).max() < 2.5 / G
    assert 0.2 < np.exp(want).max() < 0.98                      # the toy law is neither uniform nor degenerate


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_generated_blocks_rescore_to_the_same_log_probabilities(dtype):
    """Incremental decoding against a growing cache equals block-parallel scoring of the same tokens against the
    prefix cache, and the caches it returns equal a prefill of [tr, Y_i]."""
    wl = W.get_config("c1_tiny")
    desc = W.configs.ModelDesc("draft", 2, 64, 4, 2, 16, 128, 97, dtype, "lm")
    hw = BigWeights(desc, 9)
    tr = wl.prefix_tokens()[0] % 97
    cache = oracle.prefill(desc, hw, [tr])[0]
    n, L = 3, 6
    u = W.rng.uniform_f64(3, "gen/u", n * L).reshape(n, L)
    tokens, tok_lp, blk, caches, bounds = oracle.generate_blocks(desc, hw, cache, n, L, u)
    assert np.all((bounds[..., 0] <= u) & (u < bounds[..., 1]))
    blk2, tok2 = oracle.score_cached(desc, hw, [cache], tokens[None])
    tol = 1e-9 if dtype == "f32" else 1e-9        # same rounding points, same operands: the two paths agree
    assert np.abs(tok2[0] - tok_lp).max() < tol and np.abs(blk2[0] - blk).max() < tol * L
    assert len({tuple(t) for t in tokens}) > 1
    ext = oracle.prefill(desc, hw, [np.concatenate([tr, tokens[1]])])[0]
    assert ext.length == caches[1].length
    assert np.abs(ext.h_last - caches[1].h_last).max() < 1e-9
    assert np.abs(ext.K[1] - caches[1].K[1]).max() < 1e-12 and np.abs(ext.V[0] - caches[1].V[0]).max() < 1e-12
