"""SubSample kernel against the sequential float64 oracle: indices must be bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import workload as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2506_15733_amd import binding as B
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    c = B.specs_ctx_create(0, torch.cuda.current_stream().cuda_stream, ws)
    yield c
    B.specs_ctx_destroy(c)


def run(ctx, lt, ld, r, betas, u, mask=None):
    from paper_2506_15733_amd import binding as B
    dev = "cuda:0"
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)
    idx = torch.full((lt.shape[0], len(betas)), -7, dtype=torch.int32, device=dev)
    mr = torch.zeros(lt.shape[0], dtype=torch.float32, device=dev)
    B.specs_subsample(ctx, t(lt, torch.float32), t(ld, torch.float32), t(r, torch.float32), betas, t(u, torch.float64),
                      idx, None if mask is None else t(mask, torch.uint8), mr)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), mr.cpu().numpy(), B.specs_ctx_status(ctx)


@pytest.mark.parametrize("n", [1, 4, 16, 64, 100, 1024])
def test_indices_bit_exact_on_synthetic_scores(ctx, n):
    wl = W.get_config("c5_7b_batched")
    Bn = 64
    lt, ld, r = wl.synthetic_scores(Bn, n)
    betas = (0.0, 0.25, 1.0, 4.0, 16.0, 100.0, 1e4)
    u = W.rng.uniform_f64(1, f"u{n}", Bn * len(betas)).reshape(Bn, -1)
    idx, mr, st = run(ctx, lt, ld, r, betas, u)
    want, want_mr = oracle.subsample_batch(lt, ld, r, betas, u)
    assert st == 0
    assert np.array_equal(idx, np.asarray(want))
    assert np.array_equal(mr, np.asarray(want_mr, dtype=np.float32))
    if n >= 16:
        assert len(np.unique(idx[:, 1])) > 3          # low beta spreads the picks: the test is not vacuous


def test_boundaries_masks_and_edge_uniforms(ctx):
    lt = np.zeros((3, 4), np.float32); ld = np.zeros((3, 4), np.float32); r = np.zeros((3, 4), np.float32)
    u = np.array([[0.0, 0.25], [0.5, 0.75 - 1e-12], [np.nextafter(1.0, 0), 0.2499999]])
    idx, _, st = run(ctx, lt, ld, r, (1.0, 3.0), u)
    assert st == 0 and idx.tolist() == [[0, 1], [2, 2], [3, 0]]
    mask = np.array([[0, 0, 1, 1], [1, 0, 0, 0], [0, 1, 0, 1]], np.uint8)
    idx, _, st = run(ctx, lt, ld, r, (1.0, 3.0), u, mask)
    want, _ = oracle.subsample_batch(lt, ld, r, (1.0, 3.0), u, mask)
    assert st == 0 and idx.tolist() == want


def test_overflow_safe_at_tuned_beta(ctx):
    lt = np.array([[-1000.0, 0.0, -10.0]], np.float32); ld = np.array([[0.0, -1000.0, -10.0]], np.float32)
    r = np.array([[0.2, 0.1, 0.9]], np.float32)
    idx, _, st = run(ctx, lt, ld, r, (1e2, 1e4), np.array([[0.7, 0.7]]))
    assert st == 0 and idx.tolist() == [[1, 2]]


def test_device_side_errors_are_reported_not_fatal(ctx):
    from paper_2506_15733_amd import binding as B
    z = np.zeros((1, 4), np.float32)
    idx, _, st = run(ctx, z, z, z, (1.0,), np.array([[1.0]]))
    assert st == 4 and idx.tolist() == [[-1]]                                  # u outside [0,1)
    bad = z.copy(); bad[0, 2] = np.nan
    idx, _, st = run(ctx, bad, z, z, (1.0,), np.array([[0.3]]))
    assert st == 5 and idx.tolist() == [[-1]]                                  # NaN score
    idx, _, st = run(ctx, z, z, z, (1.0,), np.array([[0.3]]), np.zeros((1, 4), np.uint8))
    assert st == 5 and idx.tolist() == [[-1]]                                  # nobody live
    with pytest.raises(B.SpecsError) as e:
        run(ctx, z, z, z, (-1.0,), np.array([[0.3]]))
    assert e.value.code == 4
    idx, _, st = run(ctx, z, z, z, (1.0,), np.array([[0.3]]))
    assert st == 0 and idx.tolist() == [[1]]                                   # the context is still usable


def test_monte_carlo_marginal_matches_the_exact_smc_policy(ctx):
    """Statistical check of the kernel as a sampler: 2^18 independent SMC trials on a four-response space (draws
    from pi_gen and uniforms from the seeded generator, scores from the toy tables) selected by the GPU kernel;
    the histogram of returned responses must match the exact induced policy (enumeration over count vectors in
    oracle.smc) within five binomial standard deviations, for soft selection, and for hard best-of-n at beta = 1e4
    with generator = target."""
    import math
    from oracle import smc
    g = np.random.default_rng(11)
    pt, pd, r = g.dirichlet(np.ones(4) * 2), g.dirichlet(np.ones(4) * 2), g.uniform(0, 1, 4)
    N, trials = 8, 1 << 18
    draws = np.minimum(np.searchsorted(np.cumsum(pd), W.rng.uniform_f64(7, "mc/draws", trials * N), side="right"), 3)
    draws = draws.reshape(trials, N)
    u = W.rng.uniform_f64(7, "mc/u", trials * 2).reshape(trials, 2)
    lt, ld, rr = np.log(pt)[draws], np.log(pd)[draws], r[draws]
    idx, _, st = run(ctx, lt, ld, rr, (2.0,), u[:, :1])
    assert st == 0
    picked = draws[np.arange(trials), idx[:, 0]]
    exact = smc.smc_policy(pd.tolist(), smc.exponentiated_score(pt.tolist(), pd.tolist(), r.tolist(), 2.0), N)
    for k in range(4):
        sd = math.sqrt(exact[k] * (1 - exact[k]) / trials)
        assert abs(np.mean(picked == k) - exact[k]) < 5 * sd, (k, np.mean(picked == k), exact[k])
    # hard selection: generator = target (log-ratio zero), beta = 1e4 -> the draw with the largest reward
    idx, _, st = run(ctx, ld, ld, rr, (1e4,), u[:, 1:])
    assert st == 0
    picked = draws[np.arange(trials), idx[:, 0]]
    assert np.array_equal(rr[np.arange(trials), idx[:, 0]], rr.max(axis=1))
    hard = smc.best_of_n_policy(pd.tolist(), r.tolist(), N)
    for k in range(4):
        sd = math.sqrt(max(hard[k] * (1 - hard[k]), 1e-9) / trials)
        assert abs(np.mean(picked == k) - hard[k]) < 5 * sd, (k, np.mean(picked == k), hard[k])


def test_select_and_switch_is_eq1_with_the_current_generator_then_step_three():
    """Alg. 1 Steps II-III behind the ABI: beams whose flag is 0 (target generates) select with S = beta r, beams
    whose flag is 1 with the full score of Eq. 1; afterwards a beam with max r > tau (strictly) has its flag set and
    set flags stay set. Indices are bit-exact against the sequential float64 rule; the threshold test uses exact
    float comparisons, including a reward equal to tau (no switch)."""
    from paper_2506_15733_amd import binding as B
    wl = W.get_config("c5_7b_batched")
    Bn, n = 64, 8
    lt, ld, r = wl.synthetic_scores(Bn, n)
    tau = np.float32(0.9)
    r[5, :] = np.minimum(r[5, :], tau)
    r[5, 3] = tau                                        # equal to the threshold: must NOT switch
    r[6, 2] = np.nextafter(tau, np.float32(2.0))         # one float above: must switch
    flags0 = (W.rng.raw_u32(3, "flags", 0, Bn) & 1).astype(np.uint8)
    flags0[5] = flags0[6] = 0
    u = W.rng.uniform_f64(3, "sel/u", Bn)
    dev = "cuda:0"
    ws = torch.zeros(4096, dtype=torch.uint8, device=dev)
    ctx = B.specs_ctx_create(0, torch.cuda.current_stream().cuda_stream, ws)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    gen, idx, maxr = t(flags0), torch.full((Bn,), -7, dtype=torch.int32, device=dev), torch.zeros(Bn, device=dev)
    beta = 2.0
    B.specs_select_and_switch(ctx, t(lt), t(ld), t(r), beta, float(tau), t(u), gen, idx, None, maxr)
    torch.cuda.synchronize()
    assert B.specs_ctx_status(ctx) == 0
    got_idx, got_gen = idx.cpu().numpy(), gen.cpu().numpy()
    for b in range(Bn):
        lg = ld[b] if flags0[b] else lt[b]               # pi_gen = pi_target while the target generates
        assert got_idx[b] == oracle.subsample(lt[b], lg, r[b], beta, float(u[b])), b
        want_flag = 1 if (flags0[b] or float(r[b].max()) > float(tau)) else 0
        assert got_gen[b] == want_flag, b
    assert got_gen[5] == 0 and got_gen[6] == 1
    assert np.array_equal(maxr.cpu().numpy(), r.max(axis=1))
    # rejected arguments
    with pytest.raises(B.SpecsError) as e:
        B.specs_select_and_switch(ctx, t(lt), t(ld), t(r), -1.0, 0.5, t(u), gen, idx)
    assert e.value.code == 4
    B.specs_ctx_destroy(ctx)
