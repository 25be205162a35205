"""Each contraction kernel on its own against the oracle's definition, on identical operands
(bf16 inputs are exactly representable on both sides, so only accumulation order differs).
Shapes span several tiles with ragged tails, plus the 7B-class benchmark shapes."""
import numpy as np
import pytest
import torch

import oracle
import workload as W
from workload.configs import ModelDesc, HostWeights

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    from paper_2506_15733_amd import binding as B
    ws = torch.zeros(3 << 30, dtype=torch.uint8, device=DEV)
    c = B.specs_ctx_create(0, torch.cuda.current_stream().cuda_stream, ws)
    yield c
    B.specs_ctx_destroy(c)


def draw(name, shape, std=1.0, dtype="bf16"):
    a = W.rng.normal_tensor(7, name, shape, std, dtype)
    t = torch.from_numpy(a).to(DEV)
    return a, (t.to(torch.bfloat16) if dtype == "bf16" else t)


def close(got, want, rel):
    scale = np.sqrt((want ** 2).mean()) + 1e-30
    err = np.abs(got - want).max() / scale
    assert err < rel, err
    return err


LINEAR_SHAPES = [(45, 100, 64), (256, 256, 64), (300, 1152, 128), (130, 257, 192), (300, 1152, 256), (130, 257, 320),
                 (77, 2100, 448), (2048, 4608, 3584),
                 (1024, 1536, 8960), (256, 1024, 2816), (2048, 3584, 18944),
                 # tile counts that are no multiple of the CU count, with ragged edges
                 (2000, 4500, 3584), (1000, 3000, 1024), (4100, 1500, 2048), (2048, 1536, 8960), (4096, 8960, 1536),
                 # a few rows (one position of every candidate during generation): the weight-streaming kernel
                 (16, 4608, 3584), (16, 3584, 18944), (5, 301, 128), (32, 2050, 1280), (17, 1536, 8960), (1, 64, 256)]


@pytest.mark.parametrize("M,N,K", LINEAR_SHAPES)
def test_linear_bf16(ctx, M, N, K):
    from paper_2506_15733_amd import binding as B
    a, ta = draw(f"a{M}.{K}", (M, K))
    w, tw = draw(f"w{N}.{K}", (N, K), 0.02)
    c0, _ = draw(f"c{M}.{N}", (M, N), 1.0, "f32")
    out = torch.from_numpy(c0).to(DEV)
    B.specs_op_linear(ctx, ta, tw, out, accumulate=False)
    torch.cuda.synchronize()
    want = oracle.linear(a, w)
    close(out.cpu().numpy().astype(np.float64), want, 2e-5)
    out = torch.from_numpy(c0).to(DEV)
    B.specs_op_linear(ctx, ta, tw, out, accumulate=True)
    torch.cuda.synchronize()
    close(out.cpu().numpy().astype(np.float64), want + c0, 2e-5)


def test_linear_f32(ctx):
    from paper_2506_15733_amd import binding as B
    a, ta = draw("fa", (70, 100), 1.0, "f32")
    w, tw = draw("fw", (130, 100), 0.05, "f32")
    out = torch.zeros((70, 130), dtype=torch.float32, device=DEV)
    B.specs_op_linear(ctx, ta, tw, out)
    torch.cuda.synchronize()
    close(out.cpu().numpy().astype(np.float64), oracle.linear(a, w), 2e-6)


@pytest.mark.parametrize("M,F,K", [(45, 96, 64), (300, 160, 128), (300, 1120, 256), (256, 2816, 1024), (2048, 18944, 3584),
                                   (16, 18944, 3584), (7, 96, 128), (32, 8960, 1536), (19, 160, 384)])
def test_gate_up_bf16(ctx, M, F, K):
    from paper_2506_15733_amd import binding as B
    from paper_2506_15733_amd.synthetic import pack_gate_up
    a, ta = draw(f"ga{M}.{K}", (M, K))
    wg, tg = draw(f"wg{F}.{K}", (F, K), 0.02)
    wu, tu = draw(f"wu{F}.{K}", (F, K), 0.02)
    act = torch.zeros((M, F), dtype=torch.bfloat16, device=DEV)
    B.specs_op_gate_up(ctx, ta, pack_gate_up(tg, tu), act)
    torch.cuda.synchronize()
    got = act.float().cpu().numpy().astype(np.float64)
    exact = oracle.silu(oracle.linear(a, wg)) * oracle.linear(a, wu)
    want = oracle.round_bf16(exact)
    # identical except where float accumulation order moves a value across a bf16 rounding boundary:
    # never more than one bf16 step (plus the float accumulation error itself for values near zero)
    rms = np.sqrt((exact ** 2).mean())
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 1e-4 * rms)
    assert (got != want).mean() < 5e-3
    assert np.all(np.abs(got - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-4 * rms)


@pytest.mark.parametrize("M,V,K", [(45, 301, 64), (100, 1000, 128), (300, 5000, 256), (256, 32768, 1024), (512, 152064, 3584),
                                   (300, 151936, 896)])
def test_lmhead_logprob_bf16(ctx, M, V, K):
    from paper_2506_15733_amd import binding as B
    a, ta = draw(f"la{M}.{K}", (M, K))
    w, tw = draw(f"lw{V}.{K}", (V, K), 0.02)
    tok = W.rng.zipf_tokens(3, f"t{M}.{V}", M, V)
    tok[0], tok[-1] = V - 1, 0
    out = torch.zeros(M, dtype=torch.float32, device=DEV)
    B.specs_op_lmhead_logprob(ctx, ta, tw, torch.from_numpy(tok).to(DEV), out)
    torch.cuda.synchronize()
    want = oracle.token_logprob(a, w, tok)
    assert np.abs(out.cpu().numpy() - want).max() < 2e-5 * max(1.0, np.abs(want).max())


def test_lmhead_logprob_f32(ctx):
    from paper_2506_15733_amd import binding as B
    a, ta = draw("lfa", (37, 72), 1.0, "f32")
    w, tw = draw("lfw", (515, 72), 0.3, "f32")
    tok = W.rng.uniform_tokens(3, "lft", 37, 515)
    out = torch.zeros(37, dtype=torch.float32, device=DEV)
    B.specs_op_lmhead_logprob(ctx, ta, tw, torch.from_numpy(tok).to(DEV), out)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - oracle.token_logprob(a, w, tok)).max() < 5e-6


def attention_case(ctx, desc, Bn, n, L, lens, page_tokens, sample_rows=None):
    """Attention of layer 0 on random q/k/v and a random paged prefix, against oracle.attention row by row."""
    from paper_2506_15733_amd import binding as B
    tdt = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
    Hq, Hkv, hd = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    M = Bn * n * L
    need = [(l + page_tokens - 1) // page_tokens for l in lens]
    perm = W.rng.permutation(5, "pg", sum(need))
    table = np.full((Bn, max(need)), -1, np.int32)
    o = 0
    for b in range(Bn):
        table[b, :need[b]] = perm[o:o + need[b]]
        o += need[b]
    num_pages = sum(need)
    q, tq = draw("aq", (M, Hq, hd), 1.0, desc.dtype)
    kb, tkb = draw("akb", (M, Hkv, hd), 1.0, desc.dtype)
    vb, tvb = draw("avb", (M, Hkv, hd), 1.0, desc.dtype)
    pool, tpool = draw("apool", (1, 2, num_pages, Hkv, page_tokens, hd), 1.0, desc.dtype)
    # device layout: key page-heads [token][dim], value page-heads transposed [dim][token]
    tpool = torch.stack([tpool[:, 0].reshape(1, num_pages, Hkv, -1),
                         tpool[:, 1].transpose(-1, -2).reshape(1, num_pages, Hkv, -1)], dim=1).contiguous()
    cdesc = B.make_desc(1, desc.d_model, Hq, Hkv, hd, desc.ffn, desc.vocab, desc.dtype, "prm")
    dummy = torch.zeros(max(desc.d_model, 64), dtype=tdt, device=DEV)
    ones = torch.ones(desc.d_model, dtype=torch.float32, device=DEV)
    layer = dict(wqkv=dummy, wo=dummy, wgu=dummy, wd=dummy, g_attn=ones, g_ffn=ones)
    model = B.specs_model_create(ctx, cdesc, dummy, dummy, ones, [layer])
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    h_last = torch.zeros((Bn, desc.d_model), dtype=torch.float32, device=DEV)
    ttable = torch.from_numpy(table).to(DEV)
    prefix = B.specs_prefix_create(ctx, model, lens, lens_dev, page_tokens, tpool, num_pages, ttable, h_last)
    out = torch.zeros((M, Hq * hd), dtype=tdt, device=DEV)
    B.specs_op_attention(ctx, model, prefix, 0, tq, tkb, tvb, n, L, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    B.specs_prefix_destroy(prefix)
    B.specs_model_destroy(model)
    worst = 0.0
    cands = [(b, i) for b in range(Bn) for i in range(n)]
    if sample_rows is not None:
        cands = [cands[j] for j in sample_rows]
    for b, i in cands:
        P = lens[b]
        pk = np.stack([pool[0, 0, table[b, j // page_tokens], :, j % page_tokens, :] for j in range(P)])
        pv = np.stack([pool[0, 1, table[b, j // page_tokens], :, j % page_tokens, :] for j in range(P)])
        r0 = (b * n + i) * L
        k = np.concatenate([pk, kb[r0:r0 + L]]).astype(np.float64)
        v = np.concatenate([pv, vb[r0:r0 + L]]).astype(np.float64)
        mask = np.concatenate([np.ones((L, P), bool), np.tril(np.ones((L, L), bool))], 1)
        want = oracle.operand(oracle.attention(q[r0:r0 + L].astype(np.float64), k, v, mask, desc.dtype), desc.dtype)
        worst = max(worst, np.abs(got[r0:r0 + L] - want).max())
    return worst


def test_attention_f32_ragged(ctx):
    d = ModelDesc("target", 1, 96, 6, 2, 16, 160, 301, "f32", "lm")
    assert attention_case(ctx, d, 3, 3, 5, [38, 8, 20], 4) < 2e-6


@pytest.mark.parametrize("Hq,Hkv,hd,Bn,n,L,lens,pt", [
    (6, 2, 16, 3, 3, 5, [38, 8, 20], 4),             # SIMT path: head_dim 16
    (16, 8, 64, 1, 8, 32, [512], 16),                # config-2 shape
    (12, 2, 128, 2, 3, 64, [333, 1000], 16),         # ragged prefix lengths, group of 6
    (28, 4, 128, 1, 16, 128, [4096], 16),            # config-4 shape (sampled candidates)
    (14, 2, 64, 1, 2, 70, [100], 16),                # block length not a multiple of any tile
    (12, 2, 128, 2, 3, 64, [1, 17], 16),             # prefixes shorter than a key tile: one and two pages
    (8, 8, 64, 3, 2, 16, [64, 65, 127], 16),         # prefix ends on, just after and just before a tile boundary
    (8, 8, 64, 20, 4, 32, [5, 300, 64, 64, 17, 200, 129, 1, 333, 64, 250, 90, 31, 400, 128, 77, 300, 12, 160, 222], 16),
                                                     # 20 ragged beams with equal lengths among them: the two-phase
                                                     # kernel deals beams to the XCDs by decreasing length
    (8, 2, 128, 17, 5, 64, [700 - 37 * b for b in range(17)], 16),   # the same with groups of 4 and a beam count that
                                                                     # leaves XCD slots empty
])
def test_attention_bf16(ctx, Hq, Hkv, hd, Bn, n, L, lens, pt):
    d = ModelDesc("target", 1, Hq * hd, Hq, Hkv, hd, 64, 64, "bf16", "lm")
    sample = None if Bn * n <= 8 else [0, 7, Bn * n - 1] if Bn < 16 else list(range(0, Bn * n, 3)) + [Bn * n - 1]
    err = attention_case(ctx, d, Bn, n, L, lens, pt, sample)
    # outputs are averages of unit normals rounded to bf16: one bf16 ulp of the largest plausible value, which is
    # below 2 when hundreds of keys are averaged and below 4 when a row sees only two or three keys
    assert err < 2.0 ** -7 or (min(lens) < 64 and err <= 2.0 ** -6), err

@pytest.mark.parametrize("dtype,Hq,Hkv,hd,d_model,Bn,n,L,lens", [
    ("bf16", 28, 4, 128, 3584, 1, 4, 128, [4096]),        # 7B layer: rotary embedding inside the GEMM epilogue, head_dim 128
    ("bf16", 6, 2, 64, 384, 3, 2, 70, [100, 17, 333]),    # head_dim 64, block length off every tile: zeroed padding of vT
    ("bf16", 12, 2, 128, 1536, 2, 8, 2, [50, 2000]),      # 32 rows: the few-row path (projection, then the rotary kernel)
    ("f32", 6, 2, 16, 96, 3, 3, 5, [38, 8, 20]),          # float: plain kernels
])
def test_qkv_projection_with_rotary_embedding(ctx, dtype, Hq, Hkv, hd, d_model, Bn, n, L, lens):
    """q, k, v of one layer on given operands against the definition: y = A W^T in float64, q and k heads rotated
    by oracle.rope at absolute position lens[b] + t, everything rounded once to the operand type; block keys per row,
    block values transposed per candidate with zeroed padding. A bf16 output is the rounding of a float-accumulated
    value: within half a unit in the last place plus the accumulation error of the exact one, and equal to the
    oracle's rounding for all but the values that sit on a rounding boundary."""
    from paper_2506_15733_amd import binding as B
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    M = Bn * n * L
    width = (Hq + 2 * Hkv) * hd
    A, tA = draw("qa", (M, d_model), 1.0, dtype)
    Wm, tW = draw("qw", (width, d_model), 0.02, dtype)
    page_tokens = 16 if dtype == "bf16" else 4
    need = [(l + page_tokens - 1) // page_tokens for l in lens]
    table = np.zeros((Bn, max(need)), np.int32)
    cdesc = B.make_desc(1, d_model, Hq, Hkv, hd, 64, 64, dtype, "prm")
    dummy = torch.zeros(max(d_model, 64), dtype=tdt, device=DEV)
    ones = torch.ones(d_model, dtype=torch.float32, device=DEV)
    layer = dict(wqkv=dummy, wo=dummy, wgu=dummy, wd=dummy, g_attn=ones, g_ffn=ones)
    model = B.specs_model_create(ctx, cdesc, dummy, dummy, ones, [layer])
    pool = torch.zeros((1, 2, 1, Hkv, page_tokens * hd), dtype=tdt, device=DEV)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    h_last = torch.zeros((Bn, d_model), dtype=torch.float32, device=DEV)
    prefix = B.specs_prefix_create(ctx, model, lens, lens_dev, page_tokens, pool, 1, torch.from_numpy(table).to(DEV), h_last)
    Lp = (L + 15) // 16 * 16
    q = torch.full((M, Hq, hd), 7.0, dtype=tdt, device=DEV)
    kb = torch.full((M, Hkv, hd), 7.0, dtype=tdt, device=DEV)
    vT = torch.full((Bn * n, Hkv, hd, Lp), 7.0, dtype=tdt, device=DEV)
    B.specs_op_qkv_rope(ctx, model, prefix, tA, tW, n, L, q, kb, vT)
    torch.cuda.synchronize()
    assert B.specs_ctx_status(ctx) == 0
    B.specs_prefix_destroy(prefix)
    B.specs_model_destroy(model)
    y = A.astype(np.float64) @ Wm.astype(np.float64).T
    pos = np.concatenate([lens[b] + np.tile(np.arange(L), n) for b in range(Bn)])
    wq = oracle.rope(y[:, :Hq * hd].reshape(M, Hq, hd), pos, 10000.0)
    wk = oracle.rope(y[:, Hq * hd:(Hq + Hkv) * hd].reshape(M, Hkv, hd), pos, 10000.0)
    wv = y[:, (Hq + Hkv) * hd:].reshape(Bn * n, L, Hkv, hd).transpose(0, 2, 3, 1)          # [cand][Hkv][hd][L]
    gq, gk = q.float().cpu().numpy().astype(np.float64), kb.float().cpu().numpy().astype(np.float64)
    gv = vT.float().cpu().numpy().astype(np.float64)
    assert np.all(gv[..., L:] == 0.0)                                 # padding zeroed
    for got, want in ((gq, wq), (gk, wk), (gv[..., :L], wv)):
        if dtype == "f32":
            assert np.abs(got - want).max() < 2e-5 * max(1.0, np.abs(want).max())
        else:
            # half a unit in the last place of the stored value (its rounding) plus the float accumulation error of
            # the product, 2e-5 of the operands' scale as in the GEMM tests (a rotated pair may cancel to a value far
            # smaller than its two terms)
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.maximum(np.abs(want), np.abs(got)), 2.0 ** -30))) - 7)
            delta = 2e-5 * np.sqrt((y ** 2).mean())
            assert np.all(np.abs(got - want) <= 0.5 * ulp + delta), float((np.abs(got - want) - 0.5 * ulp).max())
            assert np.mean(got == oracle.operand(want, "bf16")) > 0.99   # and nearly all values round identically
