"""Pins of the oracle's SubSample (Alg. 2) and score (Eq. 1)."""
import math
import os
import numpy as np
import pytest
import scipy.special as sps

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_worked_weights_one_two_three():
    # lt - ld = (0, ln 2, 0), r = (0, 0, ln 3), beta = 1 -> weights (1, 2, 3); boundaries 1/6 and 1/2
    lt, ld, r = [0.0, math.log(2.0), 0.0], [0.0, 0.0, 0.0], [0.0, 0.0, math.log(3.0)]
    assert np.allclose(oracle.selection_probs(lt, ld, r, 1.0), [1 / 6, 2 / 6, 3 / 6], atol=1e-15)
    picks = {0.0: 0, 0.1: 0, 0.3: 1, 0.4999: 1, 0.5: 2, 0.999: 2}
    for u, want in picks.items():
        assert oracle.subsample(lt, ld, r, 1.0, u) == want
    # the log-ratio enters with weight 1 and only the reward is scaled by beta (Eq. 1)
    assert np.allclose(oracle.scores([1.0], [3.0], [0.5], 10.0), [1.0 - 3.0 + 5.0])


def test_two_point_instance_from_the_lower_bound_proof():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "two_point_instance.txt")) if l.strip() and l[0] != "#"]
    for beta, R, p0, p1 in [[float(x) for x in r] for r in rows]:
        theta = math.exp(beta * R)
        lt = [math.log(theta / (1 + theta)), math.log(1 / (1 + theta))]
        # candidates enumerate the space once each under a uniform generator: selection law = tilted policy
        p = oracle.selection_probs(lt, [math.log(0.5)] * 2, [0.0, R], beta)
        assert np.allclose(p, [p0, p1], atol=1e-12)
        assert oracle.subsample(lt, [math.log(0.5)] * 2, [0.0, R], beta, 0.5 - 1e-9) == 0
        assert oracle.subsample(lt, [math.log(0.5)] * 2, [0.0, R], beta, 0.5 + 1e-9) == 1


@pytest.mark.parametrize("beta", [0.0, 0.5, 4.0])
def test_selection_frequencies_over_a_uniform_grid_equal_softmax_of_scores(beta):
    rng = np.random.default_rng(7)
    n = 6
    lt, ld, r = rng.normal(-40, 3, n), rng.normal(-42, 3, n), rng.uniform(0, 1, n)
    want = sps.softmax(lt - ld + beta * r)
    assert np.allclose(oracle.selection_probs(lt, ld, r, beta), want, atol=1e-14)
    G = 1 << 14
    idx = np.array([oracle.subsample(lt, ld, r, beta, (k + 0.5) / G) for k in range(G)])
    assert np.all(np.diff(idx) >= 0)                               # inverse CDF is monotone in u
    freq = np.bincount(idx, minlength=n) / G
    assert np.abs(freq - want).max() <= 1.0 / G + 1e-12


def test_beta_limits_when_generator_equals_target():
    rng = np.random.default_rng(3)
    n = 8
    l, r = rng.normal(-30, 2, n), rng.uniform(0, 1, n)
    assert np.allclose(oracle.selection_probs(l, l, r, 0.0), 1.0 / n)            # beta = 0: uniform
    for u in np.linspace(0, 0.999, 50):
        assert oracle.subsample(l, l, r, 0.0, u) == int(u * n)
        assert oracle.subsample(l, l, r, 1e4, u) == int(np.argmax(r))            # beta -> inf: argmax r
    # general case at beta = 0: pure importance resampling, P ~ pi_target / pi_gen
    ld = rng.normal(-30, 2, n)
    assert np.allclose(oracle.selection_probs(l, ld, r, 0.0), sps.softmax(l - ld), atol=1e-14)


def test_no_overflow_at_tuned_magnitudes():
    lt, ld, r = [-1000.0, 0.0, -10.0], [0.0, -1000.0, -10.0], [0.2, 0.1, 0.9]
    for beta in (1e2, 1e3, 1e4):
        p = oracle.selection_probs(lt, ld, r, beta)
        assert all(math.isfinite(x) for x in p) and abs(sum(p) - 1) < 1e-12
    assert oracle.subsample(lt, ld, r, 1e2, 0.7) == 1            # log-ratio +1000 beats beta*r = 90
    assert oracle.subsample(lt, ld, r, 1e4, 0.7) == 2            # 9000 beats 1000 + 1000


def test_mask_and_edges():
    lt, ld, r = [0.0, 0.0, 0.0, 0.0], [0.0] * 4, [0.0] * 4
    assert oracle.subsample(lt, ld, r, 1.0, 0.0) == 0
    assert oracle.subsample(lt, ld, r, 1.0, 0.25) == 1           # strict '>' at an exact boundary
    assert oracle.subsample(lt, ld, r, 1.0, 0.0, mask=[0, 0, 1, 1]) == 2
    assert oracle.selection_probs(lt, ld, r, 1.0, mask=[0, 1, 0, 1]) == [0.0, 0.5, 0.0, 0.5]
    assert oracle.subsample(lt, ld, r, 1.0, 0.3, mask=[0, 0, 0, 0]) == -1
    assert oracle.subsample([0.0], [0.0], [0.3], 2.0, 0.99) == 0
    with pytest.raises(ValueError):
        oracle.subsample(lt, ld, r, 1.0, 1.0)
    idx, maxr = oracle.subsample_batch([lt, lt], [ld, ld], [[0.1, 0.9, 0.2, 0.3], r], [0.0, 1e4], [[0.6, 0.6], [0.6, 0.6]])
    assert idx == [[2, 1], [2, 2]] and maxr == [0.9, 0.0]
