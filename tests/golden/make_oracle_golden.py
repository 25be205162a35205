"""Writes tests/golden/oracle_<config>.json: the CPU oracle's outputs on a seeded benchmark configuration.

Calls only `oracle` (and the input generators in `workload`); nothing here touches the HIP path.
The large configurations take minutes (c3) to an hour (c4) of float64 BLAS time, which is why
their expected values are stored instead of being recomputed inside the GPU test run.

With --floor it also evaluates every role under oracle.float_accumulation_jitter (a relative error of 2e-7 in every
value that gets rounded to bf16) and stores how far that moves the outputs: what a float-accumulating evaluation of the
same rounding contract can be expected to differ from the float64 oracle by.

With --noise it also evaluates every role WITHOUT operand rounding (same bf16-valued weights, all
arithmetic float64) and stores how far that moves the outputs: the sensitivity of the result to the
bf16 rounding of matrix operands, i.e. the floor under which no two bf16 evaluations can be expected to
agree. The GPU parity test scales its tolerance by it.

--layers K evaluates every role with its first K layers only, at full widths, and writes
oracle_<config>_L<K>.json: the depth series that separates an error that grows with depth (rounding
decisions that decorrelate) from one that is there at depth 1 (a mistake).

--append adds the given beams to the beams a stored file already holds (configuration 5: each beam
costs up to an hour), keeping what is stored.

--generate T (with --layers K) stores block generation instead of scoring: T positions of all n candidates of beam 0
drawn by oracle.generate_blocks from every language model of the configuration (first K layers, full widths, the
configuration's prefix), with the uniforms of stream "gen/u"; a model whose vocabulary exceeds the token vocabulary
draws from the first token_vocab ids. Written to oracle_gen_<config>_L<K>.json.

usage: python tests/golden/make_oracle_golden.py c3_1p5b [--beams 0,1] [--noise] [--layers 2] [--append]
"""
import dataclasses
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workload as W  # noqa: E402
from workload.configs import HostWeights  # noqa: E402


def append_beams(args, wl, beams, old, path):
    """Scores `beams` and appends them, beam by beam, to the lists of a stored file (written after every beam and role)."""
    pt_all, cand_all = wl.prefix_tokens(), wl.candidates()
    partial = path[:-5] + ".partial.json"
    done = json.load(open(partial)) if os.path.exists(partial) else {}
    for b in beams:
        for role in args.roles.split(","):
            key = f"{b}/{role}"
            if key in done:
                continue
            desc = wl.models()[role]
            t0 = time.time()
            hw = HostWeights(desc, wl.seed)
            res = oracle.score_cached(desc, hw, oracle.prefill(desc, hw, [pt_all[b]]), cand_all[[b]])
            done[key] = np.asarray(res).tolist() if desc.head == "prm" else [res[0].tolist(), res[1].tolist()]
            print("beam", b, role, round(time.time() - t0, 1), "s", flush=True)
            json.dump(done, open(partial, "w"))
    for b in beams:
        old["beams"].append(b)
        for role in args.roles.split(","):
            r = done[f"{b}/{role}"]
            if wl.models()[role].head == "prm":
                old[role] += r
            else:
                old[role] += r[0]
                old["tok_" + role] += r[1]
    old["note_appended"] = ("noise_* and seconds_* fields were measured on the first two beams stored; "
                            "later beams were appended without a sensitivity run")
    json.dump(old, open(path, "w"))
    os.remove(partial)
    print("appended", beams, "to", path)


def generation(args, wl, tag):
    """Alg. 1 step I by the oracle: T positions for the n candidates of beam 0, per language model."""
    T = args.generate
    u = W.rng.uniform_f64(wl.u_seed, "gen/u", wl.n * T).reshape(wl.n, T)
    out = {"config": args.config, "layers": args.layers, "positions": T, "u_stream": "gen/u",
           "note": "float64 oracle, oracle.generate_blocks on beam 0; bounds = interval of uniforms mapped to each id"}
    path = os.path.join(ROOT, "tests", "golden", f"oracle_gen_{tag}.json")
    for role, desc in wl.models().items():
        if desc.head != "lm":
            continue
        t0 = time.time()
        hw = HostWeights(desc, wl.seed)
        cache = oracle.prefill(desc, hw, [wl.prefix_tokens()[0]])[0]
        limit = wl.token_vocab if desc.vocab > wl.token_vocab else None
        p_max = np.zeros((wl.n, T))
        tokens, tok, blk, _, bounds = oracle.generate_blocks(desc, hw, cache, wl.n, T, u, vocab_limit=limit, p_max=p_max)
        out[role] = {"vocab_limit": limit or 0, "tokens": tokens.tolist(), "tok": tok.tolist(), "block": blk.tolist(),
                     "bounds": bounds.tolist(), "p_max": p_max.tolist()}
        print(role, round(time.time() - t0, 1), "s", flush=True)
        json.dump(out, open(path, "w"))
    print("wrote", path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("config")
    ap.add_argument("--beams", default=None, help="comma-separated beam indices (default: all)")
    ap.add_argument("--roles", default="target,draft,prm")
    ap.add_argument("--noise", action="store_true")
    ap.add_argument("--floor", action="store_true",
                    help="also evaluate with oracle.float_accumulation_jitter and store the distance (fp32_floor_*)")
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--append", action="store_true")
    ap.add_argument("--generate", type=int, default=0, help="store T generated positions instead of scores")
    args = ap.parse_args()
    wl = W.get_config(args.config)
    tag = args.config
    if args.layers:
        wl = W.configs.scaled(wl, **{r: dataclasses.replace(m, n_layers=min(args.layers, m.n_layers))
                                     for r, m in wl.models().items()})
        tag = f"{args.config}_L{args.layers}"
    if args.generate:
        return generation(args, wl, tag)
    beams = list(range(wl.B)) if args.beams is None else [int(b) for b in args.beams.split(",")]
    pt_all, cand_all = wl.prefix_tokens(), wl.candidates()
    pt, cand = [pt_all[b] for b in beams], cand_all[beams]
    out = {"config": args.config, "beams": beams, "seed": wl.seed,
           "note": "float64 oracle, cached mode (proved equal to full recompute in tests/test_oracle_scoring.py)"}
    if args.layers:
        out["layers"] = args.layers
    path = os.path.join(ROOT, "tests", "golden", f"oracle_{tag}.json")
    old = json.load(open(path)) if os.path.exists(path) else None
    if args.append:
        assert old is not None and not args.noise and not set(beams) & set(old["beams"])
        return append_beams(args, wl, beams, old, path)
    if old is not None and old.get("beams") == beams:
        out.update({k: v for k, v in old.items() if k not in out})
    for role in args.roles.split(","):
        desc = wl.models()[role]
        t0 = time.time()
        hw = HostWeights(desc, wl.seed)
        caches = oracle.prefill(desc, hw, pt)
        t1 = time.time()
        res = oracle.score_cached(desc, hw, caches, cand)
        t2 = time.time()
        if desc.head == "prm":
            out[role] = np.asarray(res).tolist()
        else:
            out[role] = res[0].tolist()
            out["tok_" + role] = res[1].tolist()
        out[f"seconds_{role}"] = {"prefill": round(t1 - t0, 1), "score": round(t2 - t1, 1)}
        if args.noise:
            exact = dataclasses.replace(desc, dtype="f32")      # no rounding points; weights stay bf16-valued
            res_x = oracle.score_cached(exact, hw, oracle.prefill(exact, hw, pt), cand)
            if desc.head == "prm":
                out[f"noise_{role}"] = {"max": float(np.abs(np.asarray(res_x) - np.asarray(res)).max())}
            else:
                dt, db = res_x[1] - res[1], res_x[0] - res[0]
                out[f"noise_{role}"] = {"tok_rms": float(np.sqrt((dt ** 2).mean())), "tok_max": float(np.abs(dt).max()),
                                        "block_rms": float(np.sqrt((db ** 2).mean())),
                                        "block_max": float(np.abs(db).max())}
            print(role, "noise", out[f"noise_{role}"], flush=True)
        if args.floor:
            # the same rounding contract with float-sized errors in the values that get rounded: how close a
            # float-accumulating evaluation can come to the float64 one (see oracle/rounding.py)
            with oracle.float_accumulation_jitter(2.0e-7, seed=1):
                res_j = oracle.score_cached(desc, hw, oracle.prefill(desc, hw, pt), cand)
            if desc.head == "prm":
                out[f"fp32_floor_{role}"] = {"max": float(np.abs(np.asarray(res_j) - np.asarray(res)).max())}
            else:
                dt, db = res_j[1] - res[1], res_j[0] - res[0]
                out[f"fp32_floor_{role}"] = {"tok_rms": float(np.sqrt((dt ** 2).mean())), "tok_max": float(np.abs(dt).max()),
                                             "block_rms": float(np.sqrt((db ** 2).mean())),
                                             "block_max": float(np.abs(db).max())}
            print(role, "fp32 floor", out[f"fp32_floor_{role}"], flush=True)
        print(role, out[f"seconds_{role}"], flush=True)
        json.dump(out, open(path, "w"))
    print("wrote", path)


if __name__ == "__main__":
    main()
