#!/usr/bin/env python3
"""Benchmark of the EAGLE speculative step on one MI355X.

A "step" is one pass of the whole hot path -- draft-tree expansion with the Autoregression Head, one
tree-masked target forward, acceptance, KV/feature compaction -- for one batch of sequences.  The workload is
the LLaMA2-7B-shaped bf16 configuration (bs=1, 512-token prompt, 26-node depth-5 tree, greedy, draft logits
biased toward the target's greedy continuation so that the mean accepted length is ~3.5).  Inputs are seeded
and synthetic (random-init weights N(0, 0.02), uniform-random prompt); they stand in for the chat benchmarks
the paper measures on.

Prints ONE JSON line: decode tokens/s (`value`), ms per step, the verify-phase time, a per-kernel table of the
verify phase (every launch timed by start/stop events attached to the dispatch, on the library's stream), the
roofline of the dominant kernel of that table, a bare streaming-read ceiling measured in the same process, and
the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402


HINT_BIAS = 1.0e4   # far above any head logit (a random-init head feeds its own growing features back)


def solve_alpha(tau: float, D: int) -> float:
    lo, hi = 0.0, 0.999999
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if sum(mid ** i for i in range(D + 1)) < tau:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def bench_head_loss(args, shape, torch, synth, pkg) -> int:
    """Forward + gradient of the head's training loss on R rows (only the LM head of the shape is loaded).  A step is
    one call: 2R rows through the LM head, the row-wise loss, R rows through its transpose.  Bound: the bf16 MFMA
    rate (6 R V d algorithmic flop; the kernels multiply two bf16 planes per activation, i.e. twice that)."""
    R, K, W = args.head_loss_rows, args.steps, args.warmup
    par, rk = synth.TREES["T8"]
    eng = pkg.Eagle(shape.twin(1), par, rk, max_batch=1, max_seq=128, head_loss_rows=R)
    spec = [t for t in synth.tensor_specs(shape) if t[0] == "lm_head"][0]
    eng.load_named("lm_head", synth.gen_tensor(shape, args.seed, spec, synth.device_fmt(shape)))
    g = torch.Generator(device="cpu").manual_seed(args.seed)
    f = torch.randn(R, shape.d_model, generator=g).cuda()
    fhat = (f.cpu() + 0.6 * torch.randn(R, shape.d_model, generator=g)).cuda()
    grad = torch.empty_like(f)
    for _ in range(W):
        eng.head_loss_device(f, fhat, grad)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        loss = eng.head_loss_device(f, fhat, grad)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flop = 6.0 * R * shape.vocab * shape.d_model
    out = {"metric": "head training loss (forward + gradient), rows/s", "value": R * K / dt, "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{shape.name} LM head ({shape.vocab} x {shape.d_model}), {R} rows of N(0,1) features, prediction = label + 0.6 N(0,1), w_cls 0.1"},
           "loss": {"L": loss[0], "L_reg": loss[1], "L_cls": loss[2]},
           "roofline": {"bound": "mfma", "achieved": flop / (dt / K) / 1e12, "peak": 2500.0, "unit": "TFLOP/s", "frac": flop / (dt / K) / 2.5e15,
                        "traffic": None, "note": "algorithmic flop 6 R V d over the whole call (its GEMMs, the row-wise loss kernel and the partial-sum pass)"},
           "cpu_baseline": None}
    print(json.dumps(out))
    eng.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=73)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--shape", default="llama2-7b")
    ap.add_argument("--layers", type=int, default=0, help="override the number of target layers (0 = the shape's own)")
    ap.add_argument("--prompt", type=int, default=512)
    ap.add_argument("--tau", type=float, default=3.5)
    ap.add_argument("--tree", default="T26")
    ap.add_argument("--alpha", type=float, default=None, help="per-position hit probability of the knob (default: solved from --tau for this tree depth)")
    ap.add_argument("--seed", type=int, default=2)
    ap.add_argument("--kv-dtype", default="fp32", choices=["fp32", "bf16"], help="storage type of the KV cache (the default, fp32, is what the parity tests of the bf16 configurations use)")
    ap.add_argument("--batch", type=int, default=1, help="sequences decoded together (each with its own prompt and knob)")
    ap.add_argument("--temperature", type=float, default=0.0, help="> 0: stochastic tree acceptance, no knob (natural acceptance)")
    ap.add_argument("--weight-bits", type=int, default=16, choices=[16, 4], help="4: the library quantises the weight matrices to 4 bits as it loads them (the paper's int4 case study); algorithmic bytes are then counted at 0.5 B per weight plus the group scales")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=3)
    ap.add_argument("--cpu-prompt", type=int, default=48)
    ap.add_argument("--head-loss-rows", type=int, default=0, help="> 0: time the head's training loss instead (Sec. 3.2: Smooth L1 + w_cls x cross entropy over the "
                    "LM head, forward and gradient) on this many rows of synthetic features; prints its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no cross-GPU exchange); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import synth
    import paper_2401_15077_amd as pkg

    shape = synth.SHAPES[args.shape]
    if args.layers:
        shape = shape.twin(args.layers)
    if args.head_loss_rows > 0:
        return bench_head_loss(args, shape, torch, synth, pkg)
    par, rk = synth.TREES[args.tree]
    K, W = args.steps, args.warmup
    M = len(par)
    depth = [0] * M
    for v in range(1, M):
        depth[v] = depth[int(par[v])] + 1
    D = max(depth)
    n_future = (K + W + 2) * (D + 1) + 8
    max_seq = args.prompt + n_future + M + 16 + 64
    B = args.batch
    stochastic = args.temperature > 0.0
    t0 = time.time()
    eng = pkg.Eagle(shape, par, rk, max_batch=B, max_seq=max_seq, temperature=args.temperature, seed=args.seed, kv_dtype=args.kv_dtype,
                    weight_bits=args.weight_bits)
    eng.load_weights(synth.iter_weights(shape, args.seed, synth.device_fmt(shape)))
    t_load = time.time() - t0
    prompts = [synth.prompt(args.seed + 1000 * b, args.prompt, shape.vocab) for b in range(B)]
    prompt = prompts[0]

    # the target's own continuation (vanilla decoding with the same kernels), outside the timed region: the knob's
    # hints when greedy, and the vanilla tokens/s in any case
    futures = [list(prompts[b]) + [eng.prefill(b, prompts[b])] for b in range(B)]
    torch.cuda.synchronize()
    tv0 = time.time()
    for _ in range(n_future):
        tk = eng.vanilla_step()
        for b in range(B):
            futures[b].append(int(tk[b]))
    torch.cuda.synchronize()
    vanilla_tok_s = n_future * B / (time.time() - tv0)
    if not stochastic and B > 1:
        # With several sequences the verify rows take another kernel path than vanilla decoding, so the two can part
        # at an arg-max near-tie.  The knob must hint at what THIS path will emit: an untimed speculative run without
        # hints emits exactly that (the output of greedy speculation is decided by the verify logits alone).
        eng.reset()
        for b in range(B):
            futures[b] = list(prompts[b]) + [eng.prefill(b, prompts[b])]
        need = args.prompt + 1 + n_future
        while min(len(f) for f in futures) < need and max(len(f) for f in futures) < need + 48:
            toks, lens, _ = eng.step()
            for b in range(B):
                futures[b] += [int(t) for t in toks[b][:lens[b]]]
    future = futures[0]
    alpha = args.alpha if args.alpha is not None else solve_alpha(args.tau, D)
    hint_seed = 20240126

    hist = np.zeros(D + 2, np.int64)                  # accepted draft tokens per sequence and step (timed run)
    prefill_ms = [0.0]

    def run(mode: int, steps: int):
        eng.reset()
        torch.cuda.synchronize()
        tp = time.perf_counter()
        for b in range(B):
            eng.prefill(b, prompts[b])
        torch.cuda.synchronize()
        prefill_ms[0] = (time.perf_counter() - tp) * 1e3
        for b in range(B):
            if not stochastic:
                eng.set_hint(b, futures[b], alpha, HINT_BIAS, hint_seed + b)
        eng.set_profiling(0)
        for _ in range(W):
            eng.step()
        eng.set_profiling(mode)
        eng.get_profile(reset=True)
        torch.cuda.synchronize()
        t = time.perf_counter()
        emitted = 0
        for _ in range(steps):
            _, lens, _ = eng.step()
            emitted += int(lens.sum())
            if mode == 0:
                for b in range(B):
                    hist[int(lens[b]) - 1] += 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        prof = eng.get_profile(reset=True)
        eng.set_profiling(0)
        return dt, emitted, prof

    # A tree node's key sits at another cache slot than the same token's key in vanilla decoding, so the two runs agree
    # only up to rounding and can part at an arg-max near-tie; the knob must hint at what the speculative run itself
    # emits.  Untimed rehearsal: if the hinted run leaves the hinted continuation, continue it without hints, take ITS
    # tokens as the continuation and rehearse again (runs are deterministic: the timed run then repeats the rehearsal).
    repairs = 0
    while not stochastic and repairs < 3:
        run(0, K)
        emitted_toks = [list(eng.get_buffer(pkg.BUF_TOKENS, b)) for b in range(B)]
        if all(t == futures[b][:len(t)] for b, t in enumerate(emitted_toks)):
            break
        repairs += 1
        need = args.prompt + 1 + n_future
        for b in range(B):
            eng.set_hint(b, futures[b], 0.0, 0.0, hint_seed + b)      # knob off for the continuation
        guard = 0
        while min(len(t) for t in emitted_toks) < need and guard < 2 * n_future:
            toks, lens, _ = eng.step()
            for b in range(B):
                emitted_toks[b] += [int(t) for t in toks[b][:lens[b]]]
            guard += 1
        for b in range(B):
            futures[b] = emitted_toks[b]
    hist[:] = 0
    dt, emitted, _ = run(0, K)                       # the timed region: exactly K steps
    prefill_ms_timed = prefill_ms[0]
    # acceptance rate by depth: of the steps whose accepted path reached depth n, the share that also accepted a token
    # at depth n + 1 -- a token drafted from an input holding n predicted features.  With `--tree chain5` this is the
    # paper's n-alpha (Metrics paragraph of the experiments section, defined on chain drafts); on tree drafts it is the
    # per-depth acceptance of the best of the node's children.
    reached = np.cumsum(hist[::-1])[::-1]             # reached[n] = steps with at least n accepted draft tokens
    accept_by_depth = [float(reached[n + 1] / reached[n]) if reached[n] > 0 else None for n in range(D)]
    stale = False
    if not stochastic:
        for b in range(B):
            toks = eng.get_buffer(pkg.BUF_TOKENS, b)
            stale = stale or not np.array_equal(toks, np.asarray(futures[b][:len(toks)], np.int32))
    _, _, prof1 = run(1, K)                          # same K steps with phase events
    eng.get_kernel_stats(0); eng.get_kernel_stats(1)
    _, _, prof2 = run(2, min(K, 16))                 # start/stop events on every GEMM and attention launch
    kstats = {"draft": eng.get_kernel_stats(0), "verify": eng.get_kernel_stats(1)}

    verify_ms = prof1["verify_ms"] / max(1, prof1["steps"])
    draft_ms = prof1["draft_ms"] / max(1, prof1["steps"])
    accept_ms = prof1["accept_ms"] / max(1, prof1["steps"])
    verify_bytes = (prof1["verify_weight_bytes"] + prof1["verify_kv_bytes"]) / max(1, prof1["steps"])
    n_timed_steps = max(1, prof2["steps"])

    def table(rows):
        out_rows = []
        for r in rows:
            us = r["ms"] * 1e3 / max(1, r["launches"])
            bpl = r["bytes"] / max(1, r["launches"])
            out_rows.append({"name": r["name"], "kernel": r["kernel"], "launches_per_step": r["launches"] / n_timed_steps,
                             "avg_launch_us": us, "bytes_per_launch": bpl, "us_per_step": r["ms"] * 1e3 / n_timed_steps,
                             "gb_per_s": bpl / (us * 1e-6) / 1e9 if us > 0 else None,
                             "frac_of_8TBs": bpl / (us * 1e-6) / 8e12 if us > 0 else None})
        return out_rows

    verify_table, draft_table = table(kstats["verify"]), table(kstats["draft"])
    # the dominant kernel: the kernel TEMPLATE with the largest summed time in the verify phase (one template serves
    # several matrices: its launches are pooled -- bytes over time)
    pools = {}
    for r in verify_table:
        if r["name"] == "attention":
            continue
        p = pools.setdefault(r["kernel"], {"kernel": r["kernel"], "names": [], "us": 0.0, "bytes": 0.0, "launches": 0.0})
        p["names"].append(r["name"]); p["us"] += r["us_per_step"]; p["bytes"] += r["bytes_per_launch"] * r["launches_per_step"]
        p["launches"] += r["launches_per_step"]
    dominant = max(pools.values(), key=lambda p: p["us"]) if pools else None
    if dominant:
        dominant["name"] = "+".join(dominant["names"])
        dominant["launches_per_step"] = dominant["launches"]
        dominant["avg_launch_us"] = dominant["us"] / dominant["launches"]
        dominant["bytes_per_launch"] = dominant["bytes"] / dominant["launches"]
        dominant["gb_per_s"] = dominant["bytes"] / (dominant["us"] * 1e-6) / 1e9
        dominant["frac_of_8TBs"] = dominant["gb_per_s"] / 8000.0
    # HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE counters (each scaled by what
    # the counter reads for a copy of known size): taken from the committed summary under profiles/, which names the
    # commit it was measured on; only quoted for the workload it was measured on
    default_workload = (args.shape == "llama2-7b" and not args.layers and args.tree == "T26" and args.prompt == 512
                        and B == 1 and not stochastic and args.kv_dtype == "fp32" and args.weight_bits == 16)
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_llama2-7b_bs1_T26.txt")
    if default_workload and dominant and os.path.exists(tpath):
        for ln in open(tpath):
            f = ln.split()
            if len(f) >= 4 and f[0] == "TRAFFIC" and f[1] == dominant["kernel"].replace(" ", "_"):
                traffic, traffic_src = float(f[2]), f"profiles/hbm_traffic_llama2-7b_bs1_T26.txt (measured at commit {f[3]})"
    stream_gbs = pkg.probe_stream_read(2 << 30, 5)   # beyond the 256 MB memory-side cache
    out = {
        "metric": "decode tokens/s + verify-step ms, LLaMA2-7B shape bs=1; % HBM roofline",
        "value": emitted / dt, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}{' int4 weights' if args.weight_bits == 4 else ''} bs={B} prompt={args.prompt} tree={args.tree}({M} nodes, depth {D}) "
                               + (f"temperature {args.temperature} (Alg. 1), no knob" if stochastic else f"greedy knob alpha={alpha:.4f}"),
                   "global_batch": B, "seq_len": args.prompt,
                   "n_layers": shape.n_layers},
        "tau": emitted / K / B, "verify_ms": verify_ms, "draft_ms": draft_ms, "accept_ms": accept_ms,
        "verify_hbm_frac": verify_bytes / (verify_ms * 1e-3) / 8e12 if verify_ms > 0 else None,
        "verify_bytes": verify_bytes, "vanilla_tokens_per_s": vanilla_tok_s, "hint_stale": bool(stale), "hint_repairs": repairs,
        "load_s": t_load, "prefill_ms": prefill_ms_timed, "prefill_tokens_per_s": B * args.prompt / (prefill_ms_timed * 1e-3),
        "accept_rate_by_depth": accept_by_depth,
        "stream_ceiling_gbs": stream_gbs,
        "verify_kernels": verify_table, "draft_kernels": draft_table,
        "roofline": {"bound": "hbm",
                     "kernel": f"{dominant['kernel']} ({dominant['name']}: the kernel template with the largest summed time in the verify phase; its launches pooled)",
                     "achieved": dominant["gb_per_s"], "peak": 8000.0, "unit": "GB/s", "frac": dominant["frac_of_8TBs"],
                     "traffic": traffic, "traffic_source": traffic_src,
                     "launches_per_step": dominant["launches_per_step"], "avg_launch_us": dominant["avg_launch_us"],
                     "bytes_per_launch": dominant["bytes_per_launch"],
                     "all_gemm_launches_gb_per_s": prof2["gemm_weight_bytes"] / (prof2["gemm_ms"] * 1e-3) / 1e9 if prof2["gemm_ms"] > 0 else None},
    }
    eng.close()
    del eng
    torch.cuda.empty_cache()

    if not args.no_cpu_baseline and B == 1 and not stochastic and args.weight_bits == 16:
        from oracle.eagle_oracle import Oracle
        cp = args.cpu_prompt
        Wo = synth.make_weights(shape, args.seed, synth.oracle_fmt(shape))
        orc = Oracle(shape, Wo, par, rk, max_seq=cp + (args.cpu_steps + 1) * (D + 1) + M + 8, dtype=np.float32)
        cprompt = prompt[:cp]
        # the knob needs the target's greedy continuation of THIS prompt: the oracle's own vanilla run (untimed)
        n_fut = (args.cpu_steps + 1) * (D + 1)
        van = Oracle(shape, Wo, par, rk, max_seq=cp + n_fut + 8, dtype=np.float32)
        cfuture = list(cprompt) + van.generate_vanilla(cprompt, n_fut)
        del van
        orc.set_hint(cfuture, alpha, HINT_BIAS, hint_seed)
        orc.prefill(cprompt)
        tc = time.perf_counter()
        cpu0 = time.process_time()
        em = 0
        for _ in range(args.cpu_steps):
            em += orc.spec_step()["length"]
        dtc = time.perf_counter() - tc
        # threads the oracle actually kept busy: CPU time of the process over wall time of the timed steps
        cores = max(1, round((time.process_time() - cpu0) / dtc))
        out["cpu_baseline"] = {"value": em / dtc, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{args.cpu_steps} speculative steps of the same {shape.name} model after a "
                                         f"{cp}-token prompt, fp32 numpy oracle, same knob (tau={em / args.cpu_steps:.2f}); "
                                         f"{dtc / args.cpu_steps * 1e3:.0f} ms per step",
                               "ms_per_step": dtc / args.cpu_steps * 1e3}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
