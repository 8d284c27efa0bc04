#!/usr/bin/env python3
"""Benchmark of the router-gated decode step on one MI355X.

A step = one call of first_decode_step (embed -> kept layers -> final norm -> LM head ->
argmax) for the batch, free-running on the device (each step feeds its own greedy token).
Workload: the 8B-class bf16 decoder, batch 1, prompt 1024, with a seeded skip mask (first and
last layers kept) fed through first_set_mask; prefill + route runs once per mask before the
timed region, so weights, KV and tokens are resident in HBM when timing starts.

Prints ONE JSON line: decode tokens/s (headline skip fraction), a sweep over the skip
fractions, the HBM roofline of the dominant kernel (the persistent whole-step kernel) measured
with events on the library's stream, and the CPU oracle timed on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def step_bytes(desc, n_kept, ctx_len, logits=True):
    """Algorithmic HBM bytes of one batch-1 decode step: kept-layer weights once, LM head,
    embedding row, KV read of all previous positions plus append, fp32 logits write."""
    e = desc.bytes_per_elem
    kvb = 2 * desc.n_kv_heads * desc.head_dim * e
    w = n_kept * (desc.layer_params * e + 2 * desc.d_model * 4)
    head = desc.vocab * desc.d_model * e + desc.d_model * 4
    kv = n_kept * kvb * (ctx_len + 1) + n_kept * kvb
    return w + head + desc.d_model * e + kv + (desc.vocab * 4 if logits else 0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="cfg3_8b",
                    choices=["cfg3_8b", "cfg3_3b", "cfg2_1b", "cfg1_tiny", "cfg4_8b_b16", "cfg5_8b_16k"])
    ap.add_argument("--prompt", type=int, default=0, help="override the prompt length of a batch workload")
    ap.add_argument("--skips", default="", help="comma-separated numbers of skipped layers to sweep instead of the workload's own")
    ap.add_argument("--headline-skip", type=float, default=0.25)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--per-op", action="store_true", help="one kernel per fused op instead of the persistent kernel")
    ap.add_argument("--sample", action="store_true",
                    help="also time the headline mask with the paper's decoding rule (temperature 0.8, top-k 10) instead of greedy")
    ap.add_argument("--no-tpot-grid", action="store_true",
                    help="skip the sweep over the paper's skip fractions (random and fixed-interval masks, 8B and 3B-class shapes)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the two batch workloads (cfg4_8b_b16, cfg5_8b_16k) that the default run appends")
    ap.add_argument("--train-forward", action="store_true",
                    help="also time the training-side pieces: soft-skip forward + loss terms over the prompt, LoRA merge of the gate matrices")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import paper_2410_12513_amd as P
    from synth import CONFIGS, WORKLOADS, make_interval_mask, make_prompt, make_router, make_skip_mask, make_weights

    wl = WORKLOADS[args.workload]
    desc = CONFIGS[wl["model"]]
    if wl["batch"] > 1:
        return bench_batch(args, wl, desc, args.workload)
    seed = wl["seed"]
    n_prompt, L = wl["prompt"], desc.n_layers
    K, W = args.steps, args.warmup
    skips = sorted(set(int(x) for x in args.skips.split(","))) if args.skips else sorted(set(wl["skip"]))
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    t0 = time.time()
    weights = make_weights(desc, seed, device="cuda")
    router = make_router(desc, seed, device="cuda")
    prompt = make_prompt(desc.vocab, n_prompt, seed).cuda()
    torch.cuda.synchronize()
    t_gen = time.time() - t0

    ctx = P.FirstContext(desc, weights, router, max_batch=1, max_seq_len=n_prompt + 2 * (W + K) + 160, stream=stream)
    if args.no_graph:
        ctx.set_option(1, 0)
    ctx.set_option(3, 0 if args.per_op else 1)       # persistent kernel or error: never a silent fallback
    logits = torch.zeros(1, desc.vocab, device="cuda")
    tok = torch.zeros(1, dtype=torch.int32, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    sweep, prefill_ms = [], None
    for k in skips:
        mask = [0] * L if k >= L else make_skip_mask(L, k, seed).tolist()      # k = L: every layer skipped
        ev0.record(stream)
        ctx.prefill_route(prompt, [n_prompt], token=tok)          # synchronises
        ev1.record(stream)
        ev1.synchronize()
        prefill_ms = ev0.elapsed_time(ev1)
        ctx.set_mask(0, mask)
        assert len(ctx.get_kept(0)) == L - k
        for _ in range(W):
            ctx.decode_step(tok, logits, tok)
        ctx.sync()
        ev0.record(stream)
        for _ in range(K):
            ctx.decode_step(tok, logits, tok)
        ev1.record(stream)
        ev1.synchronize()
        ms = ev0.elapsed_time(ev1) / K
        mid_ctx = n_prompt + W + K // 2
        by = step_bytes(desc, L - k, mid_ctx)
        sweep.append({"skip_fraction": k / L, "kept_layers": L - k, "tokens_per_s": 1000.0 / ms,
                      "ms_per_step": ms, "step_bytes": by,
                      "hbm_frac": by / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9),
                      "per_step_ms": per_step_distribution(ctx, stream, tok, logits, min(K, 128))})
    head = min(sweep, key=lambda r: abs(r["skip_fraction"] - args.headline_skip))

    sampled = None
    if args.sample:
        # same mask, the paper's decoding rule instead of greedy, the sampled token feeds the next step: once as part of
        # the step (first_decode_step_sampled: inside the persistent kernel), once as first_sample_top_k on the logits
        # of a greedy step, and greedy under the same conditions.  Launched directly, not through a captured graph: the
        # address of each step's uniform number is an argument of the launch.
        k = L - head["kept_layers"]
        gen = torch.Generator(device="cpu").manual_seed(seed)
        uni = torch.rand(W + K, generator=gen).cuda()
        scratch = torch.zeros(1, dtype=torch.int32, device="cuda")
        times = {}
        ctx.set_option(1, 0)                               # USE_GRAPH off
        for mode in ("greedy", "in_step", "separate"):
            ctx.prefill_route(prompt, [n_prompt], token=tok)
            ctx.set_mask(0, [0] * L if k >= L else make_skip_mask(L, k, seed).tolist())
            for i in range(W + K):
                if i == W:
                    ctx.sync()
                    ev0.record(stream)
                if mode == "in_step":
                    ctx.decode_step_sampled(tok, uni[i:i + 1], 0.8, 10, None, tok)
                elif mode == "separate":
                    ctx.decode_step(tok, logits, scratch)
                    ctx.sample_top_k(logits, uni[i:i + 1], 0.8, 10, tok)
                else:
                    ctx.decode_step(tok, None, tok)
            ev1.record(stream)
            ev1.synchronize()
            times[mode] = ev0.elapsed_time(ev1) / K
        ctx.set_option(1, 0 if args.no_graph else 1)
        ms = times["in_step"]
        sampled = {"temperature": 0.8, "top_k": 10, "kept_layers": head["kept_layers"], "ms_per_step": ms,
                   "tokens_per_s": 1000.0 / ms, "greedy_ms_per_step": times["greedy"],
                   "ms_per_step_separate_sampling_kernels": times["separate"], "launch": "direct (no graph)"}

    train = None
    if args.train_forward:
        # soft-skip forward with all three loss terms over the workload's prompt (every layer runs on every
        # position, plus the LM head on every position), then a rank-8 merge into each layer's gate matrix
        targets = torch.roll(prompt, -1).to(torch.int32)
        targets[-1] = -1
        terms = torch.zeros(1, 4, device="cuda")
        ctx.soft_forward(prompt, [n_prompt], targets, 0.01, 0.05, terms)          # allocates its workspace
        ev0.record(stream)
        ctx.soft_forward(prompt, [n_prompt], targets, 0.01, 0.05, terms)
        ev1.record(stream)
        ev1.synchronize()
        sf_ms = ev0.elapsed_time(ev1)
        flops = 2.0 * n_prompt * (L * desc.layer_params + desc.vocab * desc.d_model)
        gen = torch.Generator(device="cpu").manual_seed(seed)
        A = (torch.randn(8, desc.d_model, generator=gen) * 0.01).cuda()
        Bz = torch.zeros(desc.d_ffn, 8, device="cuda")                             # B = 0: the weights stay what they are
        with torch.cuda.stream(stream):
            P.lora_merge(weights["layers"][0]["w_gate"], A, Bz, 4.0, stream=stream)
            ev0.record(stream)
            for i in range(L):
                P.lora_merge(weights["layers"][i]["w_gate"], A, Bz, 4.0, stream=stream)
            ev1.record(stream)
        ev1.synchronize()
        lm_us = ev0.elapsed_time(ev1) * 1e3 / L
        lm_bytes = 2.0 * desc.d_ffn * desc.d_model * desc.bytes_per_elem
        train = {"soft_forward": {"tokens": n_prompt, "ms": sf_ms, "tokens_per_s": n_prompt / (sf_ms * 1e-3),
                                  "tflops": flops / (sf_ms * 1e-3) / 1e12, "terms": [float(x) for x in terms[0].cpu()]},
                 "lora_merge": {"matrix": [desc.d_ffn, desc.d_model], "rank": 8, "us": lm_us, "bytes": lm_bytes,
                                "GB/s": lm_bytes / (lm_us * 1e-6) / 1e9, "hbm_frac": lm_bytes / (lm_us * 1e-6) / (HBM_PEAK_GBS * 1e9)}}

    # Dominant kernel.  With the persistent path the whole step is ONE kernel (k_step), so its
    # launch duration is the step time measured above with events on the library's stream;
    # with the per-op path it is the gate/up mat-vec, timed below over all layers' weights.
    persistent = head["ms_per_step"] is not None and not args.per_op
    reps = max(64, K)
    for i in range(8):
        ctx.op_gateup(i % L)
    ctx.sync()
    ev0.record(stream)
    for i in range(reps):
        ctx.op_gateup(i % L)                                      # rotate: no launch finds its weights cached
    ev1.record(stream)
    ev1.synchronize()
    gu_ms = ev0.elapsed_time(ev1) / reps
    gu_bytes = 2 * desc.d_ffn * desc.d_model * desc.bytes_per_elem       # both matrices, once
    per_op = {"kernel": "k_gateup (RMSNorm + gate/up mat-vec + SiLU*up of one layer, per-op path)",
              "bytes_per_launch": gu_bytes, "avg_launch_us": gu_ms * 1e3, "GB/s": gu_bytes / (gu_ms * 1e-3) / 1e9}
    # HBM bytes per launch from the committed counter runs (profiles/): valid for the headline mask only
    traffic, traffic_detail = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic_detail = json.load(open(tpath)).get("k_step" if persistent else "k_gateup")
            # the counter runs describe the kernel as it was then: they count only while its source is unchanged
            if traffic_detail and traffic_detail.get("kept_layers") == head["kept_layers"] and \
               traffic_detail.get("kernel_source_sha256") == kernel_source_hash():
                traffic = traffic_detail["bytes_per_launch"]
        except Exception:
            traffic, traffic_detail = None, None
    if persistent:
        achieved = head["step_bytes"] / (head["ms_per_step"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_step (whole decode step of the kept layers + LM head as one persistent kernel)",
                    "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": traffic, "traffic_detail": traffic_detail, "bytes_per_launch": head["step_bytes"],
                    "avg_launch_us": head["ms_per_step"] * 1e3, "launches_timed": K, "per_op_gateup": per_op}
    else:
        roofline = {"bound": "hbm", "kernel": per_op["kernel"], "achieved": per_op["GB/s"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": per_op["GB/s"] / HBM_PEAK_GBS, "traffic": traffic,
                    "bytes_per_launch": gu_bytes, "avg_launch_us": gu_ms * 1e3, "launches_timed": reps}

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    grid = None
    if not args.no_tpot_grid and not args.per_op and args.workload == "cfg3_8b":
        grid = tpot_grid(P, args, stream, (desc, weights, router, ctx))

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(desc, weights, router, head, seed, n_prompt)

    out = {
        "metric": "decode tokens/sec at skip fraction s, batch 1 (8B-class); % of HBM roofline",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if desc.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {wl['model']} Llama-style decoder, batch 1, prompt {n_prompt}, "
                               f"greedy decode, seeded skip mask (first/last kept)",
                   "skip_fraction": head["skip_fraction"], "kept_layers": head["kept_layers"],
                   "kv_page_tokens": 16, "graph": not args.no_graph,
                   "decode_path": "per-op kernels" if args.per_op else "persistent kernel"},
        "hbm_roofline_frac_step": head["hbm_frac"],
        "sweep": sweep,
        "tpot_grid": grid,
        "sampled_decode": sampled,
        "train_forward": train,
        "prefill": {"tokens": n_prompt, "ms": prefill_ms,
                    "tflops": (2.0 * n_prompt * L * desc.layer_params + 2.0 * desc.vocab * desc.d_model)
                              / (prefill_ms * 1e-3) / 1e12},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "setup_s": {"generate_weights": t_gen},
    }
    ctx.close()
    if args.workload == "cfg3_8b" and not args.per_op and not args.no_other_workloads:
        # the two batch workloads, 64 timed steps each, so that one default run carries every configuration
        del ctx, weights, router
        torch.cuda.empty_cache()
        other = []
        for name in ("cfg4_8b_b16", "cfg5_8b_16k"):
            r = bench_batch(args, WORKLOADS[name], CONFIGS[WORKLOADS[name]["model"]], name, steps=64, emit=False)
            other.append({"workload": r["config"]["workload"], "tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
                          "steps": r["steps"], "step_bytes": r["roofline"]["bytes_per_launch"], "hbm_frac": r["roofline"]["frac"],
                          "mean_kept_layers": r["config"]["mean_kept_layers"], "prefill": r["prefill"]})
        out["other_workloads"] = other
    print(json.dumps(out))


def kernel_source_hash():
    """sha256 of the sources of the decode kernels (what profiles/traffic.json was measured on)."""
    import hashlib
    h = hashlib.sha256()
    for f in ("step_kernel.h", "decode_kernels.h", "common.h"):
        with open(os.path.join(ROOT, "paper_2410_12513_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def per_step_distribution(ctx, stream, tok, logits, n):
    """Median and 10th / 90th percentile of n further decode steps, one event pair per step on the library's stream
    (outside the timed region above: the events sit between the launches)."""
    import torch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    evs[0].record(stream)
    for i in range(n):
        ctx.decode_step(tok, logits, tok)
        evs[i + 1].record(stream)
    evs[n].synchronize()
    t = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n))
    return {"n": n, "median": t[n // 2], "p10": t[n // 10], "p90": t[(9 * n) // 10]}


def tpot_grid(P, args, stream, have):
    """Time per output token against the fraction of layers skipped, on the paper's own grid (10 / 15 / 20 / 25 / 35 %:
    Section 5.2) for the two model geometries it used, with random-skip and fixed-interval masks (the two mask rules
    of its baselines, Section 5.1) fed through first_set_mask.  Shapes and masks only: no trained routers, no datasets.
    `have` = (desc, weights, router, ctx) of the model the caller already built, reused for its workload."""
    import torch
    from synth import CONFIGS, WORKLOADS, make_interval_mask, make_prompt, make_router, make_skip_mask, make_weights
    rows = []
    K, W = 64, 8
    for workload in ("cfg3_8b", "cfg3_3b"):
        wl = WORKLOADS[workload]
        desc = CONFIGS[wl["model"]]
        seed, n_prompt, L = wl["seed"], wl["prompt"], desc.n_layers
        if have is not None and have[0] is desc:
            weights, router, ctx, own = have[1], have[2], have[3], False
        else:
            weights = make_weights(desc, seed, device="cuda")
            router = make_router(desc, seed, device="cuda")
            ctx = P.FirstContext(desc, weights, router, max_batch=1, max_seq_len=n_prompt + 2 * (W + K) + 16, stream=stream)
            ctx.set_option(3, 0 if args.per_op else 1)
            own = True
        prompt = make_prompt(desc.vocab, n_prompt, seed).cuda()
        logits = torch.zeros(1, desc.vocab, device="cuda")
        tok = torch.zeros(1, dtype=torch.int32, device="cuda")
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        base = None
        for frac in (0.0, 0.10, 0.15, 0.20, 0.25, 0.35):
            k = int(round(frac * L))
            for rule in (("none",) if k == 0 else ("random", "interval")):
                mask = (make_interval_mask(L, k) if rule == "interval" else make_skip_mask(L, k, seed)).tolist()
                ctx.prefill_route(prompt, [n_prompt], token=tok)
                ctx.set_mask(0, mask)
                for _ in range(W):
                    ctx.decode_step(tok, logits, tok)
                ctx.sync()
                ev0.record(stream)
                for _ in range(K):
                    ctx.decode_step(tok, logits, tok)
                ev1.record(stream)
                ev1.synchronize()
                ms = ev0.elapsed_time(ev1) / K
                base = ms if k == 0 else base
                by = step_bytes(desc, L - k, n_prompt + W + K // 2)
                rows.append({"model": wl["model"], "layers": L, "skipped": k, "skip_fraction": k / L, "mask_rule": rule,
                             "tpot_ms": ms, "tokens_per_s": 1000.0 / ms, "tpot_vs_no_skip": ms / base,
                             "hbm_frac": by / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9)})
        if own:
            ctx.close()
            del weights, router, ctx
            torch.cuda.empty_cache()
    return rows


def batch_step_bytes(desc, masks, ctx_lens):
    """Algorithmic HBM bytes of one decode step of a batch: the weights of every layer that at
    least one sequence keeps, once; LM head once; per sequence its embedding row, the KV of its
    kept layers (read + append) and its logits."""
    e = desc.bytes_per_elem
    kvb = 2 * desc.n_kv_heads * desc.head_dim * e
    L = desc.n_layers
    used = sum(1 for i in range(L) if any(m[i] for m in masks))
    by = used * (desc.layer_params * e + 2 * desc.d_model * 4) + desc.vocab * desc.d_model * e + desc.d_model * 4
    for m, n in zip(masks, ctx_lens):
        by += desc.d_model * e + sum(m) * kvb * (n + 2) + desc.vocab * 4
    return by, used


def bench_batch(args, wl, desc, name, steps=None, emit=True):
    """Decode of a batch with one skip mask per sequence (the batch-16 mixed-mask and the batch-4
    long-context workloads): aggregate tokens/s over all sequences.  Prints its JSON line (emit) or returns it."""
    import numpy as np
    import torch
    import paper_2410_12513_amd as P
    from synth import make_prompt, make_router, make_skip_mask, make_weights

    seed, B, L = wl["seed"], wl["batch"], desc.n_layers
    K, W = min(steps or args.steps, wl["decode"]), args.warmup
    rng = np.random.Generator(np.random.PCG64(seed))
    if isinstance(wl["prompt"], tuple):
        lens = [int(x) for x in rng.integers(wl["prompt"][0], wl["prompt"][1] + 1, size=B)]
    else:
        lens = [int(args.prompt or wl["prompt"])] * B
    if isinstance(wl["skip"], str):                                  # "U[0,0.5]": one skip fraction per sequence
        skips = [min(L - 2, int(round(float(f) * L))) for f in rng.uniform(0.0, 0.5, size=B)]
    else:
        skips = [int(wl["skip"][0])] * B
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    weights = make_weights(desc, seed, device="cuda")
    router = make_router(desc, seed, device="cuda")
    ctx = P.FirstContext(desc, weights, router, max_batch=B, max_seq_len=max(lens) + W + K + 16, stream=stream)
    ctx.set_option(6, 0 if args.per_op else 1)                      # shared pass over the weights, or error
    prompts = [make_prompt(desc.vocab, n, seed * 100 + b).cuda() for b, n in enumerate(lens)]
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    logits = torch.zeros(B, desc.vocab, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    ctx.prefill_route(torch.cat(prompts).to(torch.int32), lens, token=tok)
    ev1.record(stream)
    ev1.synchronize()
    prefill_ms = ev0.elapsed_time(ev1)
    # per-sequence draws for the mixed-mask workload; one common set of skipped layers otherwise
    mixed = isinstance(wl["skip"], str)
    masks = [make_skip_mask(L, k, seed * 100 + (b if mixed else 0)).tolist() for b, k in enumerate(skips)]
    for b, m in enumerate(masks):
        ctx.set_mask(b, m)
    for _ in range(W):
        ctx.decode_step(tok, logits, tok)
    ctx.sync()
    ev0.record(stream)
    for _ in range(K):
        ctx.decode_step(tok, logits, tok)
    ev1.record(stream)
    ev1.synchronize()
    ms = ev0.elapsed_time(ev1) / K
    by, used = batch_step_bytes(desc, masks, [n + W + K // 2 for n in lens])
    achieved = by / (ms * 1e-3) / 1e9
    out = {
        "metric": "decode tokens/sec, batch with per-sequence skip masks (8B-class); % of HBM roofline",
        "value": B * 1000.0 / ms, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if desc.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{name}: {wl['model']} Llama-style decoder, batch {B}, prompts {min(lens)}..{max(lens)} "
                               f"tokens, skipped layers per sequence {min(skips)}..{max(skips)} of {L}",
                   "layers_kept_by_some_sequence": used, "mean_kept_layers": sum(sum(m) for m in masks) / B,
                   "kv_page_tokens": 16, "decode_path": "one pass per sequence" if args.per_op else "shared pass per layer"},
        "prefill": {"tokens": sum(lens), "ms": prefill_ms},
        "roofline": {"bound": "hbm", "kernel": "whole decode step (batched mat-vec, attention and LM-head kernels)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_launch": by, "avg_launch_us": ms * 1e3, "launches_timed": K},
        "cpu_baseline": None,
    }
    ctx.close()
    del ctx, weights, router, logits, prompts
    torch.cuda.empty_cache()
    if not emit:
        return out
    print(json.dumps(out))


def cpu_baseline(desc, weights, router, head, seed, n_ctx):
    """The CPU oracle, as it stands, on this box's host cores, in its fp32 mode ("full precision"), on a bounded
    sample of the same workload: decode steps of the same model and mask at the workload's context length.  The
    oracle's own prompt pass over n_ctx tokens would take minutes on the 8B shape, so its state is set up by a
    16-token prompt pass and the KV cache of every layer is then filled to n_ctx positions with seeded synthetic
    keys / values (decode cost depends on the cache's length, not on its contents)."""
    import torch
    from oracle import first_oracle as O
    from synth import make_prompt, make_skip_mask
    from synth.generators import to_device
    t0 = time.time()
    w_cpu = to_device(weights, "cpu")
    r_cpu = router.cpu()
    t_copy = time.time() - t0
    L = desc.n_layers
    mask = make_skip_mask(L, L - head["kept_layers"], seed)
    cdt = torch.float32
    st = O.prefill_route(desc, w_cpu, r_cpu, make_prompt(desc.vocab, 16, seed), cdt=cdt)
    st.set_mask(mask)
    g = torch.Generator().manual_seed(seed)
    kv_dt = st.K[0].dtype
    for i in range(L):
        st.K[i] = (torch.randn(n_ctx, desc.n_kv_heads, desc.head_dim, generator=g) * 0.5).to(kv_dt)
        st.V[i] = (torch.randn(n_ctx, desc.n_kv_heads, desc.head_dim, generator=g) * 0.5).to(kv_dt)
    st.pos = n_ctx
    tok, n, t_dec = st.token, 0, 0.0
    while n < 2 or (t_dec < 12.0 and n < 64):
        t1 = time.time()
        _, tok = O.decode_step(desc, w_cpu, st, tok, cdt=cdt)
        t_dec += time.time() - t1
        n += 1
    return {"value": n / t_dec, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{n} decode steps of the same model and mask at context {n_ctx} (the oracle in its fp32 mode; its "
                      f"state from a 16-token prompt pass, the cache of every layer then filled to {n_ctx} positions with "
                      f"seeded synthetic keys / values); weights copied device->host in {t_copy:.1f} s"}


if __name__ == "__main__":
    main()
