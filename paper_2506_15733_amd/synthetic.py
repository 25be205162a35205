"""Device-side set-up of a synthetic scoring step: weights, KV pools, contexts, inputs.

Plumbing for tests, smoke() and bench.py: it draws inputs with the `workload` generators,
places them in device memory with torch and calls the C ABI through the binding. No arithmetic
of the method happens here.
"""
import numpy as np
import torch

import workload as W
from workload.configs import device_tensor, weight_shapes
from . import binding as B


def pack_gate_up(wg, wu):
    """[F,d],[F,d] -> [2F,d] with gate/up rows interleaved in groups of 32 (layout of specs_layer_weights.wgu)."""
    F, d = wg.shape
    g = B.GATE_UP_GROUP
    return torch.stack([wg.view(F // g, g, d), wu.view(F // g, g, d)], dim=1).reshape(2 * F, d).contiguous()


class DeviceModel:
    """Weights of one model in device memory + its ABI handles (context with own workspace, model)."""

    def __init__(self, desc, device, stream, max_rows, max_blocks, seed=0):
        self.desc, self.device = desc, device
        top, per_layer = weight_shapes(desc)
        gen = lambda name, shape: device_tensor(desc, seed, name, shape, device)
        self.embed = gen("embed", top["embed"])
        self.head = gen("head", top["head"])
        self.g_final = torch.ones(desc.d_model, dtype=torch.float32, device=device)
        self.layers = []
        for l in range(desc.n_layers):
            wg, wu = gen(f"L{l}/wg", per_layer["wg"]), gen(f"L{l}/wu", per_layer["wu"])
            self.layers.append(dict(wqkv=gen(f"L{l}/wqkv", per_layer["wqkv"]), wo=gen(f"L{l}/wo", per_layer["wo"]),
                                    wgu=pack_gate_up(wg, wu), wd=gen(f"L{l}/wd", per_layer["wd"]),
                                    g_attn=self.g_final, g_ffn=self.g_final))
            del wg, wu
        self.cdesc = B.make_desc(desc.n_layers, desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.ffn,
                                 desc.vocab, desc.dtype, desc.head, desc.rope_base, desc.rms_eps)
        nbytes = B.specs_workspace_bytes(self.cdesc, max_rows, max_blocks)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        # the block may still be written by queued work of the allocating stream: order the context's stream after it
        stream.wait_stream(torch.cuda.current_stream())
        self.workspace.record_stream(stream)
        self.ctx = B.specs_ctx_create(torch.device(device).index or 0, stream.cuda_stream, self.workspace)
        self.model = B.specs_model_create(self.ctx, self.cdesc, self.embed, self.head, self.g_final, self.layers)

    def close(self):
        B.specs_model_destroy(self.model)
        B.specs_ctx_destroy(self.ctx)


class DevicePrefix:
    """Paged KV pool, page table, lengths and h_last of B beams for one model."""

    def __init__(self, dm: DeviceModel, lens, page_table, num_pages, page_tokens):
        d, dev = dm.desc, dm.device
        tdt = torch.bfloat16 if d.dtype == "bf16" else torch.float32
        # [layer][K|V][page][kv head][page_tokens*head_dim]; K page-heads are [token][dim], V page-heads [dim][token]
        self.kv_pool = torch.zeros((d.n_layers, 2, num_pages, d.n_kv_heads, page_tokens * d.head_dim), dtype=tdt, device=dev)
        self.page_table = torch.from_numpy(np.ascontiguousarray(page_table)).to(dev)
        self.lens_host = [int(x) for x in lens]
        self.lens_dev = torch.tensor(self.lens_host, dtype=torch.int32, device=dev)
        self.h_last = torch.zeros((len(lens), d.d_model), dtype=torch.float32, device=dev)
        self.handle = B.specs_prefix_create(dm.ctx, dm.model, self.lens_host, self.lens_dev, page_tokens, self.kv_pool,
                                            num_pages, self.page_table, self.h_last)

    def close(self):
        B.specs_prefix_destroy(self.handle)


class ScoringStep:
    """One step of the hot path on a synthetic workload: score the n blocks of every beam under target,
    draft and PRM, then SubSample per (beam, beta)."""

    ROLES = ("target", "draft", "prm")

    def __init__(self, wl: W.Workload, device="cuda:0", extra_tokens=0, prefill_rows=2048, concurrent=True):
        """concurrent: each role gets its own context on its own stream (default priority), so that the three
        independent passes overlap where one of them leaves CUs idle (the paper runs target and PRM scoring
        concurrently and pays for the slower of the two); SubSample joins them on the caller's stream."""
        self.wl, self.device = wl, device
        torch.cuda.set_device(device)
        self.stream = torch.cuda.current_stream()
        self.concurrent = concurrent
        self.role_streams = {r: (torch.cuda.Stream(device=device) if concurrent else self.stream) for r in self.ROLES}
        lens = wl.prefix_lens()
        rows = max(wl.B * wl.n * wl.L, min(int(lens.max()), prefill_rows))
        table, num_pages = wl.page_table(extra_tokens)
        self.models, self.prefixes = {}, {}
        for role, desc in wl.models().items():
            self.models[role] = DeviceModel(desc, device, self.role_streams[role], rows, wl.B * wl.n, wl.seed)
            self.prefixes[role] = DevicePrefix(self.models[role], lens, table, num_pages, wl.page_tokens)
        self.cand = torch.from_numpy(wl.candidates()).to(device)
        self.prefix_tokens = torch.from_numpy(np.concatenate(wl.prefix_tokens()).astype(np.int32)).to(device)
        self.u = torch.from_numpy(wl.uniforms()).to(device)
        f = lambda *s: torch.zeros(s, dtype=torch.float32, device=device)
        self.out = {r: f(wl.B, wl.n) for r in self.ROLES}
        self.tok = {r: f(wl.B, wl.n, wl.L) for r in ("target", "draft")}
        self.idx = torch.zeros((wl.B, len(wl.betas)), dtype=torch.int32, device=device)
        self.max_reward = f(wl.B)
        # SubSample runs on the caller's stream after the three passes have joined it
        self.sel_ws = torch.zeros(4096, dtype=torch.uint8, device=device)
        self.sel_ctx = B.specs_ctx_create(torch.device(device).index or 0, self.stream.cuda_stream, self.sel_ws)

    def _fork(self):
        if self.concurrent:
            for r in self.ROLES:
                self.role_streams[r].wait_stream(self.stream)

    def _join(self):
        if self.concurrent:
            for r in self.ROLES:
                self.stream.wait_stream(self.role_streams[r])

    def prefill(self):
        self._fork()
        for r in self.ROLES:
            B.specs_prefill(self.models[r].ctx, self.models[r].model, self.prefixes[r].handle, self.prefix_tokens)
        self._join()

    def score(self, role, cand=None, out=None, tok=None):
        dm = self.models[role]
        B.specs_score_blocks(dm.ctx, dm.model, self.prefixes[role].handle, self.cand if cand is None else cand,
                             self.out[role] if out is None else out,
                             (self.tok.get(role) if tok is None else tok))

    def enqueue_step(self):
        self._fork()
        for r in self.ROLES:
            self.score(r)
        self._join()
        B.specs_subsample(self.sel_ctx, self.out["target"], self.out["draft"], self.out["prm"],
                          self.wl.betas, self.u, self.idx, None, self.max_reward)

    def status(self):
        st = {r: B.specs_ctx_status(self.models[r].ctx) for r in self.ROLES}
        st["subsample"] = B.specs_ctx_status(self.sel_ctx)
        return st

    def score_and_select(self):
        self.enqueue_step()
        torch.cuda.synchronize()
        st = self.status()
        assert all(v == 0 for v in st.values()), st
        res = {r: self.out[r].cpu().numpy() for r in self.ROLES}
        res["tok_target"] = self.tok["target"].cpu().numpy()
        res["tok_draft"] = self.tok["draft"].cpu().numpy()
        res["idx"] = self.idx.cpu().numpy()
        res["max_reward"] = self.max_reward.cpu().numpy()
        return res

    def close(self):
        B.specs_ctx_destroy(self.sel_ctx)
        for r in self.ROLES:
            self.prefixes[r].close()
            self.models[r].close()


def run_specs_loop(step: ScoringStep, blocks, tau, beta_index=0, start_with_target=True, fast_path=True):
    """Alg. 1 with a synthetic generator: for each iteration h, blocks[h] is the [B, n, L] candidate set the
    generator proposed (token ids; generation itself is outside this path). Everything the method decides happens
    behind the C ABI: specs_select_and_switch applies Eq. 1 with the beam's current generator as pi_gen, draws
    SubSample's index and performs Step III's switch on the device-resident generator flags; specs_commit_block_dev
    appends the chosen block (Step II) from the device-resident index. This function only moves inputs and
    chooses which passes to enqueue from a host copy of the flags.
    fast_path: in an iteration where EVERY beam's generator is the target, no log-likelihood enters the score, so
    only the PRM scores the n candidates; target and draft then run over the one chosen block per beam (n = 1),
    which is all their caches need.
    Returns the chosen indices [H, B], the generator flags [H, B] (True = draft generated that iteration) and,
    per iteration, whether the PRM-only path ran."""
    wl, dev = step.wl, step.device
    gen = torch.full((wl.B,), 0 if start_with_target else 1, dtype=torch.uint8, device=dev)
    chosen_all, gen_all, fast_all = [], [], []
    u_all = W.rng.uniform_f64(wl.u_seed, "loop/u", len(blocks) * wl.B).reshape(len(blocks), wl.B)
    beta = wl.betas[beta_index]
    idx = torch.zeros((wl.B,), dtype=torch.int32, device=dev)
    zeros = torch.zeros((wl.B, wl.n), dtype=torch.float32, device=dev)
    zero_idx = torch.zeros((wl.B,), dtype=torch.int32, device=dev)
    out1 = {r: torch.zeros((wl.B, 1), dtype=torch.float32, device=dev) for r in ("target", "draft")}
    tok1 = {r: torch.zeros((wl.B, 1, wl.L), dtype=torch.float32, device=dev) for r in ("target", "draft")}
    beams = torch.arange(wl.B, device=dev)
    for h, cand in enumerate(blocks):
        step.cand = torch.from_numpy(np.ascontiguousarray(cand.astype(np.int32))).to(dev)
        flags = gen.cpu().numpy().astype(bool)              # host copy: which passes to enqueue
        fast = fast_path and not flags.any()
        u = torch.from_numpy(u_all[h].copy()).to(dev)
        step._fork()
        for r in (("prm",) if fast else step.ROLES):
            step.score(r)
        step._join()
        lt, ld = (zeros, zeros) if fast else (step.out["target"], step.out["draft"])
        B.specs_select_and_switch(step.sel_ctx, lt, ld, step.out["prm"], beta, tau, u, gen, idx, None, step.max_reward)
        gen_all.append(flags.copy())
        fast_all.append(fast)
        if fast:                                          # gathered on the caller's stream, before the fork
            picked = step.cand[beams, idx.long()][:, None, :].contiguous()             # [B, 1, L]
        step._fork()
        if fast:
            for r in ("target", "draft"):
                step.score(r, cand=picked, out=out1[r], tok=tok1[r])
                B.specs_commit_block_dev(step.models[r].ctx, step.models[r].model, step.prefixes[r].handle, zero_idx)
            B.specs_commit_block_dev(step.models["prm"].ctx, step.models["prm"].model, step.prefixes["prm"].handle, idx)
        else:
            for r in step.ROLES:
                B.specs_commit_block_dev(step.models[r].ctx, step.models[r].model, step.prefixes[r].handle, idx)
        step._join()
        chosen_all.append(idx.cpu().numpy().copy())
    torch.cuda.synchronize()
    return np.array(chosen_all), np.array(gen_all), np.array(fast_all)


def run_specs_generation_loop(step: ScoringStep, H, tau, beta_index=0, start_with_target=True):
    """Alg. 1 end to end on the GPU for H iterations: Step I, the current generator of every beam (the target until
    Step III switches the beam to the draft model, for good, once max_i r(Y_i|tr) > tau) draws n blocks of L tokens
    with specs_generate_blocks; Steps II-III, scores, specs_select_and_switch and specs_commit_block_dev as in
    run_specs_loop. What has to run depends on who generated (read from a host copy of the device-resident flags):
      all beams by the target: log pi_gen = log pi_target cancels in Eq. 1, only the PRM scores the candidates; the
        target commits what it generated, the draft model runs over the one chosen block to keep its cache current;
      all beams by the draft: its block log-likelihoods came out of the generation pass, so only target and PRM score;
      mixed: both models generate for every beam, each beam keeps its generator's blocks, and all three models score.
    Uniforms: stream "gen/u" [H, B, n, L] for the tokens, "loop/u" [H, B] for SubSample (seed wl.u_seed).
    Returns (tokens [H, B, n, L], chosen [H, B], generator flags [H, B])."""
    wl, dev = step.wl, step.device
    Bn, n, L = wl.B, wl.n, wl.L
    gen = torch.full((Bn,), 0 if start_with_target else 1, dtype=torch.uint8, device=dev)
    u_gen = W.rng.uniform_f64(wl.u_seed, "gen/u", H * Bn * n * L).reshape(H, Bn, n, L)
    u_sel = W.rng.uniform_f64(wl.u_seed, "loop/u", H * Bn).reshape(H, Bn)
    beta = wl.betas[beta_index]
    limit = min(m.vocab for m in wl.models().values() if m.head == "lm")
    f = lambda *s: torch.zeros(s, dtype=torch.float32, device=dev)
    gen_cand = {r: torch.zeros((Bn, n, L), dtype=torch.int32, device=dev) for r in ("target", "draft")}
    gen_logp = {r: f(Bn, n) for r in ("target", "draft")}
    out1 = {r: f(Bn, 1) for r in ("target", "draft")}
    tok1 = {r: f(Bn, 1, L) for r in ("target", "draft")}
    zeros, idx = f(Bn, n), torch.zeros((Bn,), dtype=torch.int32, device=dev)
    zero_idx = torch.zeros((Bn,), dtype=torch.int32, device=dev)
    beams = torch.arange(Bn, device=dev)
    tokens_all, chosen_all, gen_all = [], [], []

    def generate(role, ud):
        dm = step.models[role]
        B.specs_generate_blocks(dm.ctx, dm.model, step.prefixes[role].handle, ud, gen_cand[role], gen_logp[role], None,
                                limit)

    def commit(role, which):
        dm = step.models[role]
        B.specs_commit_block_dev(dm.ctx, dm.model, step.prefixes[role].handle, which)

    for h in range(H):
        ud = torch.from_numpy(u_gen[h]).to(dev)
        us = torch.from_numpy(u_sel[h].copy()).to(dev)
        flags = gen.cpu().numpy().astype(bool)              # host copy: which passes to enqueue
        gens = sorted({"draft" if d else "target" for d in flags})
        step._fork()
        for r in gens:
            generate(r, ud)
        step._join()
        if len(gens) == 1:
            step.cand = gen_cand[gens[0]]
        else:
            step.cand = torch.where(gen.bool()[:, None, None], gen_cand["draft"], gen_cand["target"]).contiguous()
        step._fork()
        if gens == ["target"]:
            step.score("prm")
        elif gens == ["draft"]:
            step.score("target")
            step.score("prm")
        else:
            for r in step.ROLES:
                step.score(r)
        step._join()
        if gens == ["target"]:
            lt, ld = zeros, zeros                       # not read: every flag is 0
        elif gens == ["draft"]:
            lt, ld = step.out["target"], gen_logp["draft"]
        else:
            lt, ld = step.out["target"], step.out["draft"]
        B.specs_select_and_switch(step.sel_ctx, lt, ld, step.out["prm"], beta, tau, us, gen, idx, None, step.max_reward)
        tokens_all.append(step.cand.cpu().numpy().copy())
        gen_all.append(flags.copy())
        if gens == ["target"]:                            # gathered on the caller's stream, before the fork
            picked = step.cand[beams, idx.long()][:, None, :].contiguous()
        step._fork()
        if len(gens) == 1:
            other = "draft" if gens[0] == "target" else "target"
            commit(gens[0], idx)                        # its workspace holds the blocks it generated
            commit("prm", idx)
            if gens == ["draft"]:
                commit("target", idx)                   # the target scored all n candidates
            else:                                       # the draft saw none of them: run it over the chosen block
                step.score(other, cand=picked, out=out1[other], tok=tok1[other])
                commit(other, zero_idx)
        else:
            for r in step.ROLES:
                commit(r, idx)
        step._join()
        chosen_all.append(idx.cpu().numpy().copy())
    torch.cuda.synchronize()
    return np.array(tokens_all), np.array(chosen_all), np.array(gen_all)
