"""Benchmark of the SPECS scoring + SubSample step on one MI355X.

A step = score the n candidate blocks of every beam under target, draft and PRM (three
specs_score_blocks calls) + one specs_subsample, inputs resident in HBM. Prints ONE JSON line:
candidate tokens scored per second, the roofline of the dominant kernel (timed live with
events on the launch stream) and the CPU oracle timed on a bounded sample of the same workload.

usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4_7b] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM-side bytes per launch of the dominant kernel come from the committed rocprofv3 --pmc summary of that kernel
# (FETCH_SIZE and WRITE_SIZE runs, each scaled by what the counter reads for a device copy of known size). The
# summary carries one machine-readable line per workload, "traffic_bytes_per_launch <workload> <bytes>"; a workload
# without such a line reports null.
TRAFFIC_PROFILE = os.path.join("profiles", "gemm_gate_up_c4_7b_pmc.md")


def measured_traffic(workload):
    try:
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
            for ln in f:
                w = ln.split()
                if len(w) == 3 and w[0] == "traffic_bytes_per_launch" and w[1] == workload:
                    return float(w[2])
    except OSError:
        pass
    return None

def role_flops(d, M, P_total_rows_ctx, n, L, B):
    """Algorithmic FLOPs of one scoring pass (GEMMs + attention), for reporting."""
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    per_layer = 2.0 * M * d.d_model * (qd + 2 * kvd) + 2.0 * M * qd * d.d_model + 2.0 * M * d.d_model * 2 * d.ffn \
        + 2.0 * M * d.ffn * d.d_model
    attn = 4.0 * d.n_q_heads * d.head_dim * (P_total_rows_ctx + B * n * L * (L + 1) / 2.0)
    if d.head == "lm":
        return d.n_layers * (per_layer + attn) + 2.0 * M * d.d_model * d.vocab
    # PRM: the reward reads the last token of every block only, so the last layer needs its keys/values for all M
    # rows but its attention output, O projection and feed-forward for B*n rows
    C = B * n
    last = 2.0 * M * d.d_model * (qd + 2 * kvd) + (per_layer - 2.0 * M * d.d_model * (qd + 2 * kvd)) * C / M + attn / L
    return (d.n_layers - 1) * (per_layer + attn) + last + 2.0 * C * d.d_model


def cpu_baseline(wl, budget_layers=2, n_sub=2):
    """The oracle, untuned, on a bounded sample: n_sub candidates of beam 0 through `budget_layers`
    layers of each role (prefix keys/values random-filled, as only time is measured) plus the head;
    scaled linearly to all layers and all candidates."""
    import dataclasses
    import numpy as np
    import oracle
    from workload.configs import HostWeights
    P = int(wl.prefix_lens()[0])
    cand = wl.candidates()[0:1, :n_sub]
    rng = np.random.default_rng(0)
    total = 0.0
    for role, desc in wl.models().items():
        sub = dataclasses.replace(desc, n_layers=min(budget_layers, desc.n_layers))
        hw = HostWeights(sub, wl.seed)
        cached = {l: hw.layer(l) for l in range(sub.n_layers)}
        head = hw.head()
        hw.layer = lambda l, c=cached: c[l]
        hw.head = lambda h=head: h
        kv = [rng.standard_normal((P, desc.n_kv_heads, desc.head_dim)) for _ in range(sub.n_layers)]
        cache = oracle.PrefixCache(P, kv, kv, rng.standard_normal(desc.d_model))
        t0 = time.perf_counter()
        oracle.forward_sequences(sub, hw, [cand[0]], prefixes=[cache])
        t_layers = time.perf_counter() - t0
        t0 = time.perf_counter()
        if desc.head == "lm":
            oracle.token_logprob(rng.standard_normal((n_sub * wl.L, desc.d_model)), head, cand[0].reshape(-1))
        t_head = time.perf_counter() - t0
        total += (t_layers * desc.n_layers / sub.n_layers + t_head) * (wl.n / n_sub)
    total *= wl.B
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    return {"value": wl.B * wl.n * wl.L / total, "unit": "candidate tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"beam 0, {n_sub} of {wl.n} candidates, {budget_layers} layers per role + head, "
                      f"float64 numpy; scaled linearly to all layers, candidates and beams"}


def kernel_bench(args):
    """Loop one contraction kernel of the pass at the workload's target-model shape (for profiling and tuning)."""
    import torch
    import workload as W
    from workload.configs import device_tensor
    from paper_2506_15733_amd import binding as B, synthetic
    wl = W.get_config(args.workload)
    d = wl.target
    dev = "cuda:0"
    M = args.rows if args.rows else wl.B * wl.n * wl.L     # --rows 16: one position of every candidate (generation)
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    ws = torch.zeros(3 << 30, dtype=torch.uint8, device=dev)
    ctx = B.specs_ctx_create(0, torch.cuda.current_stream().cuda_stream, ws)
    bf = lambda *s: (torch.randn(s, device=dev) * 0.5).to(torch.bfloat16)
    wt = lambda n, k: device_tensor(d, 0, f"bench/{n}.{k}", (n, k), dev)
    k = args.kernel
    if k == "gate_up":
        A, Wm, out = bf(M, d.d_model), wt(2 * d.ffn, d.d_model), torch.empty((M, d.ffn), dtype=torch.bfloat16, device=dev)
        fn, flops = (lambda: B.specs_op_gate_up(ctx, A, Wm, out)), 2.0 * M * d.d_model * 2 * d.ffn
    elif k in ("qkv", "o", "down"):
        N, K = {"qkv": (qd + 2 * kvd, d.d_model), "o": (d.d_model, qd), "down": (d.d_model, d.ffn)}[k]
        A, Wm, out = bf(M, K), wt(N, K), torch.zeros((M, N), dtype=torch.float32, device=dev)
        fn, flops = (lambda: B.specs_op_linear(ctx, A, Wm, out, accumulate=(k != "qkv"))), 2.0 * M * N * K
    elif k == "lmhead":
        A, Wm = bf(M, d.d_model), wt(d.vocab, d.d_model)
        tok = torch.randint(0, d.vocab, (M,), dtype=torch.int32, device=dev)
        out = torch.empty(M, dtype=torch.float32, device=dev)
        fn, flops = (lambda: B.specs_op_lmhead_logprob(ctx, A, Wm, tok, out)), 2.0 * M * d.d_model * d.vocab
    elif k == "attn":
        step_prefix_len = wl.prefix_lens()
        table, num_pages = wl.page_table()
        cdesc = B.make_desc(1, d.d_model, d.n_q_heads, d.n_kv_heads, d.head_dim, d.ffn, d.vocab, d.dtype, "prm")
        dummy = torch.zeros(max(d.d_model, 64), dtype=torch.bfloat16, device=dev)
        ones = torch.ones(d.d_model, dtype=torch.float32, device=dev)
        model = B.specs_model_create(ctx, cdesc, dummy, dummy, ones,
                                     [dict(wqkv=dummy, wo=dummy, wgu=dummy, wd=dummy, g_attn=ones, g_ffn=ones)])
        pool = bf(1, 2, num_pages, d.n_kv_heads, wl.page_tokens * d.head_dim)
        lens = [int(x) for x in step_prefix_len]
        lens_dev = torch.tensor(lens, dtype=torch.int32, device=dev)
        h_last = torch.zeros((wl.B, d.d_model), dtype=torch.float32, device=dev)
        ttab = torch.from_numpy(table).to(dev)
        prefix = B.specs_prefix_create(ctx, model, lens, lens_dev, wl.page_tokens, pool, num_pages, ttab, h_last)
        q, kb, vb = bf(M, qd), bf(M, kvd), bf(M, kvd)
        out = torch.empty((M, qd), dtype=torch.bfloat16, device=dev)
        fn = lambda: B.specs_op_attention(ctx, model, prefix, 0, q, kb, vb, wl.n, wl.L, out)
        flops = 4.0 * qd * (sum(l * wl.n * wl.L for l in lens) + wl.B * wl.n * wl.L * (wl.L + 1) / 2.0)
    elif k == "copy":
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per launch
        dst = torch.empty_like(src)
        fn, flops = (lambda: dst.copy_(src)), 0.0
    else:
        raise SystemExit(f"unknown kernel {k}")
    for _ in range(3):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.reps
    line = {"kernel": k, "workload": wl.name, "rows": M, "ms": ms, "tflops": flops / ms / 1e9,
            "frac_mfma_peak": flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS}
    if k in ("gate_up", "qkv", "o", "down", "lmhead"):
        line["weight_GBps"] = Wm.numel() * Wm.element_size() / ms / 1e6       # the binding figure for a few rows
    print(json.dumps(line))


def model_bytes(d):
    """bf16 bytes a decoding step must stream: every layer's matrices and the vocabulary head (embedding rows are
    gathered, not streamed)."""
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    per_layer = d.d_model * (qd + 2 * kvd) + qd * d.d_model + 3 * d.d_model * d.ffn
    es = 2 if d.dtype == "bf16" else 4
    return es * (d.n_layers * per_layer + d.vocab * d.d_model)


def generate_bench(args):
    """Block generation by one model: n blocks of L tokens per beam, token by token. The step streams the whole
    model once per token position, so the binding roof is HBM bandwidth."""
    import numpy as np
    import torch
    import workload as W
    from paper_2506_15733_amd import synthetic, binding as B
    wl = W.get_config(args.workload)
    role = args.generate
    step = synthetic.ScoringStep(wl, device="cuda:0", concurrent=False)
    step.prefill()
    dm, pf = step.models[role], step.prefixes[role]
    u = torch.from_numpy(W.rng.uniform_f64(wl.u_seed, "bench/gen", wl.B * wl.n * wl.L).reshape(wl.B, wl.n, wl.L)).cuda()
    cand = torch.zeros((wl.B, wl.n, wl.L), dtype=torch.int32, device="cuda:0")
    logp = torch.zeros((wl.B, wl.n), dtype=torch.float32, device="cuda:0")
    limit = min(m.vocab for m in wl.models().values() if m.head == "lm")
    run = lambda: B.specs_generate_blocks(dm.ctx, dm.model, pf.handle, u, cand, logp, None, limit)
    run()
    torch.cuda.synchronize()
    assert B.specs_ctx_status(dm.ctx) == 0
    t0 = time.perf_counter()
    for _ in range(args.reps):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.reps
    B.specs_ctx_profile(dm.ctx, True)
    run()
    prof = B.specs_ctx_profile_read(dm.ctx)
    B.specs_ctx_profile(dm.ctx, False)
    d = wl.models()[role]
    streamed = model_bytes(d) * wl.L
    line = {"metric": "generated candidate tokens/sec (n blocks x L) on 1 MI355X", "value": wl.B * wl.n * wl.L / dt,
            "unit": "tokens/s", "ms_per_block_set": dt * 1e3, "ms_per_position": dt * 1e3 / wl.L,
            "config": {"workload": wl.name, "generator": role, "B": wl.B, "n": wl.n, "L": wl.L},
            "roofline": {"bound": "hbm", "achieved": streamed / dt / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": streamed / dt / 1e9 / 8000.0, "bytes_per_position": model_bytes(d)},
            "kernel_ms_per_position": {k: ms / wl.L for k, (ms, n) in prof.items()},
            "kernel_launches_per_position": {k: n / wl.L for k, (ms, n) in prof.items()}}
    print(json.dumps(line))


def loop_bench(args):
    """Whole iterations of Alg. 1 with the draft model as the generator (after the switch of Step III) and with the
    target as the generator (before it): generation, scoring by the models still needed, SubSample, commit."""
    import torch
    import workload as W
    from paper_2506_15733_amd import synthetic
    wl = W.get_config(args.workload)
    H = args.specs_loop
    out = {"metric": "Alg. 1 iterations (generate n blocks, score, SubSample, commit) on 1 MI355X",
           "config": {"workload": wl.name, "B": wl.B, "n": wl.n, "L": wl.L, "iterations": H}}
    step = synthetic.ScoringStep(wl, device="cuda:0", extra_tokens=2 * (H + 1) * wl.L)
    step.prefill()
    torch.cuda.synchronize()
    for name, start_with_target, tau in (("draft_generates", False, 2.0), ("target_generates", True, 2.0)):
        synthetic.run_specs_generation_loop(step, 1, tau, start_with_target=start_with_target)     # warm-up iteration
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        synthetic.run_specs_generation_loop(step, H, tau, start_with_target=start_with_target)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / H
        out[name] = {"ms_per_iteration": dt * 1e3, "accepted_tokens_per_s": wl.B * wl.L / dt,
                     "candidate_tokens_per_s": wl.B * wl.n * wl.L / dt}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kernel", default=None, help="gate_up|qkv|o|down|lmhead|attn|copy: time that kernel alone")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--rows", type=int, default=0, help="with --kernel: activation rows (default: the workload's B*n*L)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4_7b")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--serial", action="store_true", help="one stream for the three passes instead of one each")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (three passes + SubSample) in a HIP graph and time its replays (measured: "
                         "no faster than eager launches, the small configurations are bound by the device-side "
                         "dispatch of ~500 dependent kernels, not by the host)")
    ap.add_argument("--generate", default=None, help="draft|target: time block generation (Alg. 1 Step I) by that model")
    ap.add_argument("--specs-loop", type=int, default=0, metavar="H",
                    help="time H full iterations of Alg. 1 (generate, score, SubSample, commit) per generator")
    args = ap.parse_args()
    if args.kernel:
        return kernel_bench(args)
    if args.generate:
        return generate_bench(args)
    if args.specs_loop:
        return loop_bench(args)
    if args.gpus != 1:
        print("bench.py measures the one-GPU share of the path; --gpus must be 1 (nothing here uses a second GPU)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import workload as W
    from paper_2506_15733_amd import synthetic, binding as B
    wl = W.get_config(args.workload)
    t_setup = time.time()
    main_stream = torch.cuda.Stream(device="cuda:0") if args.graph else torch.cuda.current_stream()
    with torch.cuda.stream(main_stream):          # a graph cannot be captured on the default stream
        step = synthetic.ScoringStep(wl, device="cuda:0", concurrent=not args.serial)
        step.prefill()
        torch.cuda.synchronize()
        print(f"# setup + prefill {time.time() - t_setup:.1f}s", file=sys.stderr, flush=True)
        run = step.enqueue_step
        if args.graph:
            step.enqueue_step()                   # eager once: every kernel configured before the capture
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=main_stream):
                step.enqueue_step()
            run = graph.replay
        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
    assert all(v == 0 for v in step.status().values())

    # per-role time with events on the launch stream
    role_ms = {}
    for r in step.ROLES:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(step.role_streams[r]):
            e0.record()
            for _ in range(3):
                step.score(r)
            e1.record()
        torch.cuda.synchronize()
        role_ms[r] = e0.elapsed_time(e1) / 3

    # Per-kernel durations inside the real pass: events on the launch stream around every launch of the
    # target-model scoring call (recorded in extra passes after the timed region, not inside it).
    d = wl.target
    M = wl.B * wl.n * wl.L
    dm = step.models["target"]
    B.specs_ctx_profile(dm.ctx, True)
    for _ in range(3):
        step.score("target")
    prof = B.specs_ctx_profile_read(dm.ctx)
    B.specs_ctx_profile(dm.ctx, False)
    kernel_us = {k: (1e3 * ms / n if n else 0.0) for k, (ms, n) in prof.items()}
    # dominant kernel: the fused gate/up SwiGLU GEMM of the target/PRM model
    k_ms = kernel_us["gate_up"] / 1e3
    flops = 2.0 * M * d.d_model * 2 * d.ffn
    achieved = flops / (k_ms * 1e-3) / 1e12
    traffic = measured_traffic(args.workload)

    lens = wl.prefix_lens()
    ctx_rows = float(sum(int(l) * wl.n * wl.L for l in lens))
    # fraction of the bf16 MFMA peak of every contraction of the target pass, from the same live per-launch times
    qd, kvd = d.n_q_heads * d.head_dim, d.n_kv_heads * d.head_dim
    kflops = {"qkv": 2.0 * M * d.d_model * (qd + 2 * kvd), "oproj": 2.0 * M * qd * d.d_model,
              "gate_up": 2.0 * M * d.d_model * 2 * d.ffn, "down": 2.0 * M * d.ffn * d.d_model,
              "lmhead": 2.0 * M * d.d_model * d.vocab,
              "attention": 4.0 * qd * (ctx_rows + wl.B * wl.n * wl.L * (wl.L + 1) / 2.0)}
    kfrac = {k: (v / (kernel_us[k] * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS if kernel_us.get(k) else None)
             for k, v in kflops.items()}
    total_flops = sum(role_flops(m, M, ctx_rows, wl.n, wl.L, wl.B) for m in wl.models().values())
    line = {
        "metric": "candidate tokens scored/sec (n blocks x L) on 1 MI355X",
        "value": M / dt, "unit": "candidate tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if d.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "n": wl.n, "L": wl.L, "prefix_tokens": int(lens.sum()),
                   "roles": "target+draft+prm+subsample", "streams": 1 if args.serial else 3,
                   "launch": "graph replay" if args.graph else "eager"},
        "step_tflops": total_flops / dt / 1e12, "step_frac_of_mfma_peak": total_flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "role_ms_alone": role_ms, "target_kernel_us_per_launch": kernel_us, "target_kernel_frac_of_mfma_peak": kfrac,
        "roofline": {"kernel": "gemm_mfma_kernel<256, SWIGLU> (gate/up projection + SiLU*mul)", "bound": "mfma",
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_source": TRAFFIC_PROFILE if traffic is not None else None,
                     "ms_per_launch": k_ms,
                     "shape": [M, 2 * d.ffn, d.d_model]},
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
