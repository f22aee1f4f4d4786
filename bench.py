#!/usr/bin/env python3
"""Benchmark of the rollout decode step on one MI355X.

One step = the whole hot path over one batch: allocator (+1 token per row, one commit),
K/V append, paged GQA decode attention (work dealing, split-K partial, merge) and
temperature / top-p sampling with log-prob recording.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2|c3|c4|c5]

Without --config the line's own fields are those of c5 (the largest configuration that fits one
GPU), and `per_config` holds the same fields for c3, c2 and c4 (its 200-step refill loop), every
configuration with its roofline, its CPU-oracle baseline and the parity of all its rows.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published peak


def profiled_traffic(workload: str, algorithmic_bytes: float):
    """HBM bytes per launch of the attention kernel from the rocprofv3 --pmc summary under
    profiles/ (lines `traffic_bytes_per_launch[<workload>]` and `algorithmic_bytes_in_that_run[...]`),
    scaled from the profiled run's algorithmic bytes to this run's.  None if no summary covers
    the workload."""
    key = re.escape(workload)
    pat_t = re.compile(r"traffic_bytes_per_launch\[" + key + r"\]:\s*([0-9.eE+]+)")
    pat_a = re.compile(r"algorithmic_bytes_in_that_run\[" + key + r"\]:\s*([0-9.eE+]+)")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")) +
                       glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        text = open(path).read()
        mt, ma = pat_t.search(text), pat_a.search(text)
        if mt and ma:
            return float(mt.group(1)) * algorithmic_bytes / float(ma.group(1))
    return None


def profiled_valu_per_logit(workload: str):
    """Vector instructions per logit of the sampling kernel from the rocprofv3 --pmc summary under
    profiles/ (`sample_rows_<workload>_valu_counters.txt`); None if there is none."""
    path = os.path.join(ROOT, "profiles", f"sample_rows_{workload}_valu_counters.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"=\s*([0-9.]+) per logit", open(path).read())
    return float(m.group(1)) if m else None


def equal_rows_bench(args, torch, rb, wl, DecodeBatch):
    """The plain attention launch (roll_decode_attn) on the config's batch with every row at the same
    length: the mean of the config's lengths rounded to the number of steps that gives every
    workgroup whole rows.  (The ragged batch is what the default run measures; a second batch in one
    process lands elsewhere in memory and times ~10 us slower, so it is not repeated here.)"""
    cfg = wl.CONFIGS[args.config]
    ragged = wl.draw_lengths(cfg.lengths, cfg.batch, args.seed, cfg.max_len).astype(np.int64)
    steps = max(1, int(round(ragged.mean() / 32.0)))
    out = {}
    for name, lengths in (("equal_rows", np.full(cfg.batch, 32 * steps, np.int64)),):
        batch = DecodeBatch(cfg, args.seed, lengths, headroom_tokens=8)
        torch.cuda.synchronize()
        desc, n = batch.desc, max(args.steps, 5)
        evs = [(rb.ProfEvent(), rb.ProfEvent()) for _ in range(n)]
        for _ in range(max(args.warmup, 1)):
            rb.roll_decode_attn(batch.q, batch.k_pages, batch.v_pages, batch.page_table, batch.seq_lens, batch.out,
                                desc, batch._ws)
        torch.cuda.synchronize()
        for a, b in evs:
            rb.roll_prof_attn_events(a, b)
            rb.roll_decode_attn(batch.q, batch.k_pages, batch.v_pages, batch.page_table, batch.seq_lens, batch.out,
                                desc, batch._ws)
        torch.cuda.synchronize()
        rb.roll_prof_attn_events(None, None)
        ms = float(np.mean([a.elapsed_ms(b) for a, b in evs]))
        kv_bytes = cfg.kv_bytes_per_token * batch.total_tokens()
        out[name] = {"sum_seq_lens": int(batch.total_tokens()), "avg_launch_ms": ms,
                     "GBps": kv_bytes / (ms * 1e-3) / 1e9, "frac_of_peak": kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        batch.close()
        del batch
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "KV-read GB/s of the plain attention launch on equal rows",
                      "unit": "GB/s", "n_gpus": 1, "steps": max(args.steps, 5), "warmup": max(args.warmup, 1),
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: B={cfg.batch} Hq={cfg.num_q_heads} Hkv={cfg.num_kv_heads} "
                                             f"D={cfg.head_dim} P={cfg.page_size}, rows of {32 * steps} tokens"},
                      "roofline": {"bound": "hbm", "kernel": "attn_stream", "achieved": out["equal_rows"]["GBps"],
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": out["equal_rows"]["frac_of_peak"],
                                   "traffic": None},
                      **out}))


def policy_loss_bench(args, torch, rb, wl):
    """Tokens/s of roll_policy_loss on ragged batches of responses with lognormal lengths, one launch pair
    per objective; HBM roofline on the bytes a token moves (its 3-4 fp32 inputs and 3 fp32 outputs).
    Two batches: a rollout-sized one (512 responses, ~50 MB: it stays in the last-level cache between
    launches) and one of 4096 responses (~400 MB, more than the 256 MB cache holds), which is the
    headline."""
    out = {}
    for label, n_resp in (("512_responses", 512), ("4096_responses", 4096)):
        b = {k: v.cuda() for k, v in wl.make_policy_batch(n_resp, args.seed).items()}
        T, n = b["logp_old"].numel(), b["offsets"].numel() - 1
        value, grad, w = (torch.empty(T, device="cuda") for _ in range(3))
        seq_mean, batch_mean = torch.empty(n, device="cuda"), torch.empty(1, device="cuda")
        res = {}
        for kind in ["ppo", "decoupled_ppo", "tis", "cispo", "topr"]:
            prox = b["logp_prox"] if kind == "decoupled_ppo" else None
            call = lambda: rb.roll_policy_loss(kind, b["logp_theta"], b["logp_old"], prox, b["signal"], b["offsets"],
                                               value, grad, w, seq_mean, batch_mean)
            for _ in range(args.warmup):
                call()
            e0, e1 = rb.ProfEvent(), rb.ProfEvent()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                call()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_ms(e1) / args.steps
            nbytes = T * (4 * (3 + (1 if prox is not None else 0)) + 12)
            res[kind] = {"ms": ms, "tokens_per_s": T / (ms * 1e-3), "GBps": nbytes / (ms * 1e-3) / 1e9,
                         "bytes": nbytes}
        out[label] = {"tokens": T, "longest_response": int((b["offsets"][1:] - b["offsets"][:-1]).max().item()),
                      "per_objective": res}
        del b, value, grad, w
        torch.cuda.empty_cache()
    big = out["4096_responses"]
    best = big["per_objective"]["ppo"]
    return ({"metric": "policy-loss tokens/s (value, derivative, IS weight, ragged means)",
                      "value": best["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": best["ms"], "higher_is_better": True,
                      "dtype": "f64 arithmetic on f32 data", "data": "synthetic",
                      "config": {"workload": f"4096 ragged responses, {big['tokens']} tokens, lognormal(2048) lengths, "
                                             f"longest {big['longest_response']}: {best['bytes'] / 1e6:.0f} MB per launch pair, "
                                             "more than the 256 MB last-level cache"},
                      "roofline": {"bound": "hbm", "kernel": "policy_loss_tokens", "achieved": best["GBps"],
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": best["GBps"] / HBM_PEAK_GBS,
                                   "traffic": None},
                      "batches": out})


def attn_timeline_bench(args, torch, rb, wl):
    """Where the attention launch spends its time, wave by wave: needs the library built with
    `python -m paper_2510_11345_amd.build --timeline`, whose kernel stamps the 100 MHz clock at five
    places per wave.  Runs the configuration's decode loop and reports, over the timed launches
    that took the single fused launch: the launch's span, how long a wave takes to its first
    finished step, the steady step time, when the waves run out of work (by XCD too) and how many
    microseconds the average wave idles at the end.  Steps are synchronised one by one, so the
    step rate of this run means nothing."""
    from paper_2510_11345_amd.harness import DecodeBatch, RefillLoop
    cfg = wl.CONFIGS[args.config]
    K, W = args.steps, args.warmup
    loop = None
    if cfg.name == "c4":
        plan = wl.draw_refill_plan(cfg.batch, cfg.batch + 4 * (K + W) + 64, args.seed)
        loop = RefillLoop(cfg, plan, args.seed, max_len=cfg.max_len + K + W + 2)
        batch, step_fn = loop.batch, loop.step
    else:
        lengths = wl.draw_lengths(cfg.lengths, cfg.batch, args.seed, cfg.max_len).astype(np.int64)
        batch = DecodeBatch(cfg, args.seed, lengths - 1, headroom_tokens=K + W + 2)
        step_fn = batch.step
    logits = wl.make_logits(cfg, args.seed, "cuda")
    for i in range(W):
        step_fn(logits, i)
    torch.cuda.synchronize()
    buf = torch.zeros((1024, 8), dtype=torch.int64, device="cuda")
    rb.roll_prof_attn_timeline(buf)
    per_launch = []
    for i in range(K):
        buf.zero_()
        fused_before = rb.roll_kv_fused_steps(batch.pool)
        step_fn(logits, W + i)
        torch.cuda.synchronize()
        if rb.roll_kv_fused_steps(batch.pool) == fused_before:
            continue                      # a refill tick: two launches, not the one profiled here
        t = buf.cpu().numpy().astype(np.float64)
        t = t[t[:, 0] > 0]
        ticks = 0.01                      # microseconds per tick of the 100 MHz clock
        t0 = t[:, 0].min()
        entry, prefix, first, last, exit_ = ((t[:, k] - t0) * ticks for k in range(5))
        steps, xcd = t[:, 5], t[:, 6].astype(int)
        span = exit_.max()
        work = steps > 1
        step_us = float(np.median((last[work] - first[work]) / (steps[work] - 1)))
        kv_bytes = cfg.kv_bytes_per_token * batch.total_tokens()
        per_launch.append({
            "span_us": float(span), "GBps_over_span": kv_bytes / span / 1e3,
            "entry_skew_us": float(entry.max()), "prefix_build_us": float(np.median(prefix - entry)),
            "first_step_done_us": float(np.median(first[steps > 0])),
            "step_us": step_us,
            "last_step_p10_p50_p90_max_us": [float(np.percentile(last, q)) for q in (10, 50, 90)] + [float(last.max())],
            "exit_p10_p50_p90_max_us": [float(np.percentile(exit_, q)) for q in (10, 50, 90)] + [float(exit_.max())],
            "mean_idle_at_end_us": float((span - exit_).mean()),
            "mean_start_over_one_step_us": float(np.mean(first[steps > 0] - step_us)),
            "after_last_step_us": float(np.median(exit_ - last)),
            "last_step_mean_by_xcd_us": [float(last[xcd == x].mean()) if (xcd == x).any() else None for x in range(8)],
            "steps_per_wave_min_max": [int(steps.min()), int(steps.max())], "waves": int(len(t)),
        })
    rb.roll_prof_attn_timeline(None)
    keys = [k for k in per_launch[0] if not isinstance(per_launch[0][k], list)]
    mean = {k: float(np.mean([p[k] for p in per_launch])) for k in keys}
    for k in per_launch[0]:
        if isinstance(per_launch[0][k], list) and k != "steps_per_wave_min_max":
            mean[k] = [float(np.mean([p[k][i] for p in per_launch])) for i in range(len(per_launch[0][k]))]
    print(json.dumps({"metric": "per-wave timeline of the attention launch (attn_stream, fused decode step)",
                      "unit": "us", "n_gpus": 1, "steps": K, "warmup": W, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: B={cfg.batch} Hq={cfg.num_q_heads} Hkv={cfg.num_kv_heads} "
                                             f"D={cfg.head_dim} P={cfg.page_size} lengths={cfg.lengths}",
                                 "sum_seq_lens": int(batch.total_tokens())},
                      "launches_profiled": len(per_launch), "mean_over_launches": mean,
                      "first_launch": per_launch[0]}), flush=True)
    batch.close()


MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak


def prefill_bench(args, torch, rb, wl):
    """Tokens/s of roll_prefill_attn on prompts with the 7B-class head shape of c2 / c4.  Two
    workloads: the refill queue's prompt lengths (128..1024, 64 prompts in one call) and long
    prompts (8 x 8192, prefilled in chunks of 2048); the long prompts once more with 32 query
    heads on 8 KV heads (4 per KV head: a workgroup's seven computing waves span two or three spans of query tokens).  Matrix-core
    roofline on the algorithmic flops of causal attention: 4 D Hq per (query, visible key) pair."""
    import numpy as np
    cfg = wl.CONFIGS["c2"]
    D, P = cfg.head_dim, cfg.page_size
    rng = np.random.default_rng([args.seed, 0x505245])
    res = {}
    for name, lens, chunk, heads in [
            ("refill_prompts_64x128..1024", rng.integers(128, 1025, size=64), None, (cfg.num_q_heads, cfg.num_kv_heads)),
            ("long_prompts_8x8192_chunks_of_2048", np.full(8, 8192), 2048, (cfg.num_q_heads, cfg.num_kv_heads)),
            ("long_prompts_8x8192_chunks_of_2048_Hq32_Hkv8", np.full(8, 8192), 2048, (32, 8))]:
        Hq, Hkv = heads
        n_slots, cap = len(lens), int(lens.max())
        max_pages = (cap + P - 1) // P
        num_pages = n_slots * max_pages + 8
        page_table = torch.empty((n_slots, max_pages), dtype=torch.int32, device="cuda")
        seq_lens = torch.zeros((n_slots,), dtype=torch.int32, device="cuda")
        pool = rb.KvPool(num_pages, P, n_slots, max_pages, page_table, seq_lens)
        for s_, n in enumerate(lens):
            rb.roll_kv_alloc(pool, s_, int(n))
        rb.roll_kv_commit(pool)
        k_pages, v_pages = rb.new_kv_pools(num_pages, Hkv, D, P, fill=0)
        # calls: one per chunk round; every call holds one chunk per prompt that still has tokens
        calls = []
        step = int(lens.max()) if chunk is None else chunk
        for start in range(0, int(lens.max()), step):
            ch = [(s_, start, int(min(step, n - start))) for s_, n in enumerate(lens) if n > start]
            T = sum(c[2] for c in ch)
            off = np.concatenate([[0], np.cumsum([c[2] for c in ch])]).astype(np.int32)
            calls.append(dict(
                q=wl.randn_bf16((T, Hq, D), args.seed, 40 + start, "cuda"),
                k=wl.randn_bf16((T, Hkv, D), args.seed, 41 + start, "cuda"),
                v=wl.randn_bf16((T, Hkv, D), args.seed, 42 + start, "cuda"),
                slot=torch.tensor([c[0] for c in ch], dtype=torch.int32, device="cuda"),
                start=torch.tensor([c[1] for c in ch], dtype=torch.int32, device="cuda"),
                off=torch.from_numpy(off).cuda(),
                out=torch.empty((T, Hq, D), dtype=torch.bfloat16, device="cuda"),
                pairs=sum(n * st + n * (n + 1) // 2 for _, st, n in ch), T=T))
        kernel_events = []   # one pair per attention launch of the timed steps

        def run(timed=False):
            for c in calls:
                if timed:
                    kernel_events.append((rb.ProfEvent(), rb.ProfEvent()))
                    rb.roll_prof_prefill_events(*kernel_events[-1])
                rb.roll_prefill_attn(c["q"], c["k"], c["v"], c["slot"], c["start"], c["off"], k_pages, v_pages,
                                     page_table, c["out"], P)
        for _ in range(args.warmup):
            run()
        e0, e1 = rb.ProfEvent(), rb.ProfEvent()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            run(timed=True)
        e1.record()
        torch.cuda.synchronize()
        rb.roll_prof_prefill_events(None, None)
        ms = e0.elapsed_ms(e1) / args.steps
        launch_ms = [a.elapsed_ms(b) for a, b in kernel_events]
        attn_ms = sum(launch_ms) / args.steps     # the attention launches of one pass over the prompts
        tokens, pairs = sum(c["T"] for c in calls), sum(c["pairs"] for c in calls)
        flops = 4.0 * D * Hq * pairs
        res[name] = {"Hq": Hq, "Hkv": Hkv, "ms": ms, "tokens": tokens, "launch_pairs": len(calls), "tokens_per_s": tokens / (ms * 1e-3),
                     "TFLOPs_of_the_call": flops / (ms * 1e-3) / 1e12,
                     "attn_launch_ms": spread(launch_ms), "attn_ms_per_pass": attn_ms,
                     "TFLOPs": flops / (attn_ms * 1e-3) / 1e12}
        pool.close()
    head = res["long_prompts_8x8192_chunks_of_2048"]
    Hq, Hkv = cfg.num_q_heads, cfg.num_kv_heads
    return ({"metric": "prefill tokens/s (one attention layer, K/V written into pages)",
                      "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": head["ms"], "higher_is_better": True,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"8 prompts x 8192 tokens in chunks of 2048, Hq={Hq} Hkv={Hkv} D={D} P={P}"},
                      "roofline": {"bound": "mfma", "kernel": "prefill_attn", "achieved": head["TFLOPs"],
                                   "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": head["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                                   "launch_ms": head["attn_launch_ms"],
                                   "note": "algorithmic flops of a pass / the attention launches' own time (events "
                                           "around the kernel); with the K/V writer and the gaps between launches: "
                                           f"{head['TFLOPs_of_the_call']:.0f} TFLOP/s"},
                      "per_workload": res})


def prefill_groups_bench(args, torch, rb, wl):
    """roll_prefill_attn across numbers of query heads per KV head (4 KV heads, head_dim 128, 16-token
    pages, bf16 result, 8 prompts in one call): TFLOP/s with the units per workgroup as the launch
    chooses them, and with one span and all its heads per workgroup (up to 8 heads per KV head)."""
    D, P, Hkv, n_slots = 128, 16, 4, 8
    out = {}
    for n in (4096, 512):
        max_pages = n // P
        num_pages = n_slots * max_pages + 8
        page_table = torch.empty((n_slots, max_pages), dtype=torch.int32, device="cuda")
        seq_lens = torch.zeros((n_slots,), dtype=torch.int32, device="cuda")
        pool = rb.KvPool(num_pages, P, n_slots, max_pages, page_table, seq_lens)
        for s_ in range(n_slots):
            rb.roll_kv_alloc(pool, s_, n)
        rb.roll_kv_commit(pool)
        k_pages, v_pages = rb.new_kv_pools(num_pages, Hkv, D, P, fill=0)
        T = n_slots * n
        k = wl.randn_bf16((T, Hkv, D), args.seed, 41, "cuda")
        v = wl.randn_bf16((T, Hkv, D), args.seed, 42, "cuda")
        slot = torch.arange(n_slots, dtype=torch.int32, device="cuda")
        start = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        off = torch.arange(n_slots + 1, dtype=torch.int32, device="cuda") * n
        pairs = n_slots * n * (n + 1) // 2
        rows = {}
        for G in (7, 1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16):      # (the first one warms the clocks and is measured again)
            Hq = G * Hkv
            q = wl.randn_bf16((T, Hq, D), args.seed, 40, "cuda")
            res = torch.empty((T, Hq, D), dtype=torch.bfloat16, device="cuda")
            row = {}
            for label, units in (("one_span_per_workgroup", G if G <= 8 else None), ("chosen_by_the_launch", 0)):
                if units is None:
                    continue
                rb.roll_prof_prefill_units(units)
                for _ in range(args.warmup):
                    rb.roll_prefill_attn(q, k, v, slot, start, off, k_pages, v_pages, page_table, res, P)
                e0, e1 = rb.ProfEvent(), rb.ProfEvent()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(args.steps):
                    rb.roll_prefill_attn(q, k, v, slot, start, off, k_pages, v_pages, page_table, res, P)
                e1.record()
                torch.cuda.synchronize()
                rb.roll_prof_prefill_units(0)
                ms = e0.elapsed_ms(e1) / args.steps
                row[label] = {"ms": ms, "TFLOPs": 4.0 * D * Hq * pairs / (ms * 1e-3) / 1e12}
            rows[f"G={G}"] = row
            del q, res
        out[f"8x{n}"] = rows
        pool.close()
    print(json.dumps({"metric": "prefill TFLOP/s by query heads per KV head (K/V writer included)", "unit": "TFLOP/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"8 prompts in one call, Hkv={Hkv} D={D} P={P}, Hq = G x Hkv"},
                      "per_workload": out}), flush=True)


def prefill_timeline_bench(args, torch, rb, wl):
    """A prefill workgroup's life: needs the library built with
    `python -m paper_2510_11345_amd.build --timeline`, whose kernel stamps the 100 MHz clock per
    workgroup at entry, with its block found, before and after its step loop and after its stores,
    with the compute unit it ran on.  For three prompt shapes (7B-class heads, bf16 result) the
    last call of a pass is profiled: what a block costs beyond its steps (before the loop, after
    it, and the time between the end of one workgroup and the first instruction of the next on
    the same compute unit), the step time inside the loop, and how the launch's span divides."""
    cfg = wl.CONFIGS["c2"]
    Hq, Hkv, D, P = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size
    out = {}
    for n_slots, n, chunk in ((8, 8192, 2048), (8, 4096, 4096), (8, 2048, 2048)):
        max_pages = n // P
        num_pages = n_slots * max_pages + 8
        page_table = torch.empty((n_slots, max_pages), dtype=torch.int32, device="cuda")
        seq_lens = torch.zeros((n_slots,), dtype=torch.int32, device="cuda")
        pool = rb.KvPool(num_pages, P, n_slots, max_pages, page_table, seq_lens)
        for s_ in range(n_slots):
            rb.roll_kv_alloc(pool, s_, n)
        rb.roll_kv_commit(pool)
        k_pages, v_pages = rb.new_kv_pools(num_pages, Hkv, D, P, fill=0)
        T = n_slots * chunk
        q = wl.randn_bf16((T, Hq, D), args.seed, 40, "cuda")
        k = wl.randn_bf16((T, Hkv, D), args.seed, 41, "cuda")
        v = wl.randn_bf16((T, Hkv, D), args.seed, 42, "cuda")
        slot = torch.arange(n_slots, dtype=torch.int32, device="cuda")
        starts = [torch.full((n_slots,), s0, dtype=torch.int32, device="cuda") for s0 in range(0, n, chunk)]
        off = torch.arange(n_slots + 1, dtype=torch.int32, device="cuda") * chunk
        res = torch.empty((T, Hq, D), dtype=torch.bfloat16, device="cuda")

        def call(st):
            rb.roll_prefill_attn(q, k, v, slot, st, off, k_pages, v_pages, page_table, res, P)
        for _ in range(args.warmup):
            for st in starts:
                call(st)
        torch.cuda.synchronize()
        n_wg = (T // 32 + n_slots) * Hkv
        buf = torch.zeros((n_wg, 8), dtype=torch.int64, device="cuda")
        rb.roll_prof_prefill_timeline(buf)
        rb.roll_prof_prefill_units(Hq // Hkv)     # a span with all its heads per workgroup (what a launch of this size gets anyway)
        call(starts[-1])
        torch.cuda.synchronize()
        rb.roll_prof_prefill_units(0)
        rb.roll_prof_prefill_timeline(None)
        t = buf.cpu().numpy()
        t = t[t[:, 7] == 1]
        ts = (t[:, :5] - t[:, 0].min()) * 0.01                     # microseconds
        steps = t[:, 6].astype(np.float64)
        hw, xcc = t[:, 5] & 0xFFFFFFFF, t[:, 5] >> 32
        cu = xcc * 4096 + ((hw >> 13) & 7) * 512 + ((hw >> 12) & 1) * 256 + ((hw >> 8) & 15)   # XCC, SE, SH, CU
        units = np.unique(cu)
        loop = ts[:, 3] - ts[:, 2]
        gaps, in_wg, idle_end = [], [], []
        for c in units:
            m = np.flatnonzero(cu == c)
            o = m[np.argsort(ts[m, 0])]
            gaps.extend((ts[o[1:], 0] - ts[o[:-1], 4]).tolist())
            in_wg.append(float((ts[o, 4] - ts[o, 0]).sum()))
            idle_end.append(float(ts[:, 4].max() - ts[o[-1], 4]))
        span = float(ts[:, 4].max())
        pairs = n_slots * (chunk * (n - chunk) + chunk * (chunk + 1) // 2)
        pct = lambda a: [float(np.percentile(a, p_)) for p_ in (10, 50, 90)]
        out[f"{n_slots}x{n}_last_chunk_of_{chunk}"] = {
            "workgroups": int(len(t)), "compute_units": int(len(units)), "steps_min_max": [int(steps.min()), int(steps.max())],
            "span_us": span, "TFLOPs_over_span": 4.0 * D * Hq * pairs / span / 1e6,
            "entry_to_block_found_us_p10_p50_p90": pct(ts[:, 1] - ts[:, 0]),
            "entry_to_loop_us_p10_p50_p90": pct(ts[:, 2] - ts[:, 0]),
            "loop_end_to_stores_done_us_p10_p50_p90": pct(ts[:, 4] - ts[:, 3]),
            "between_workgroups_on_a_unit_us_p10_p50_p90": pct(gaps) if gaps else None,
            "between_workgroups_min_us": float(np.min(gaps)) if gaps else None,
            "loop_us_per_step_mean": float(loop.sum() / steps.sum()),
            # a step is 32 queries x 32 keys per query head of the group; all units in their loops at once
            "TFLOPs_inside_the_loops": 4.0 * D * (Hq // Hkv) * 32 * 32 * steps.sum() / loop.sum() * len(units) / 1e6,
            "share_of_span_in_workgroups": float(np.mean(in_wg) / span),
            "share_of_span_in_loops": float(loop.sum() / len(units) / span),
            "idle_at_the_end_us_mean_max": [float(np.mean(idle_end)), float(np.max(idle_end))],
        }
        pool.close()
    print(json.dumps({"metric": "per-workgroup timeline of the prefill attention launch (prefill_attn)", "unit": "us",
                      "n_gpus": 1, "steps": 1, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"prompts of 7B-class heads, Hq={Hq} Hkv={Hkv} D={D} P={P}, bf16 result"},
                      "per_workload": out}), flush=True)


def spread(xs):
    """mean, median, 10th and 90th percentile of a list of milliseconds."""
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "p10": float(np.percentile(a, 10)),
            "p90": float(np.percentile(a, 90)), "n": int(a.size)}


def ceiling_probe(torch, rb, batch, n=12):
    """GB/s of a plain streaming read of the batch's paged KV bytes through its page table
    (roll_prof_kv_read_probe): what this machine's memory system gives to the access pattern of the
    step, with no arithmetic and nothing written.  Median of n launches."""
    sink = torch.empty(2048 * 256, dtype=torch.int32, device="cuda")
    per_page = 0
    for _ in range(3):
        per_page = rb.roll_prof_kv_read_probe(batch.k_pages, batch.v_pages, batch.page_table, batch.seq_lens,
                                              batch.desc, sink)
    evs = [(rb.ProfEvent(), rb.ProfEvent()) for _ in range(n)]
    torch.cuda.synchronize()
    for a, b in evs:
        a.record()
        rb.roll_prof_kv_read_probe(batch.k_pages, batch.v_pages, batch.page_table, batch.seq_lens, batch.desc, sink)
        b.record()
    torch.cuda.synchronize()
    P = batch.cfg.page_size
    pages = int(((batch.lengths + P - 1) // P).sum())
    ms = float(np.median([a.elapsed_ms(b) for a, b in evs]))
    return {"GBps": per_page * pages / (ms * 1e-3) / 1e9, "bytes": per_page * pages, "median_launch_ms": ms}


def run_config(name, K, W, args, torch, rb, wl):
    """W warm-up steps, then K timed steps of the whole path on config `name`; the attention launch
    timed by HIP events on its stream; the sampling launch alone; the bandwidth ceiling; the CPU
    oracle on every row with the parity of the last step.  Returns the fields of one result."""
    from paper_2510_11345_amd.harness import DecodeBatch
    cfg = wl.CONFIGS[name]
    extra = {}
    pool_kw = dict(side_by_side=False, run_pages=1) if args.dense_pools else {}
    loop = None
    if cfg.name == "c4":
        # continuous refill: slots finish by pre-drawn length and are refilled from the prompt queue
        from paper_2510_11345_amd.harness import RefillLoop
        plan = wl.draw_refill_plan(cfg.batch, cfg.batch + 4 * (K + W) + 64, args.seed)
        loop = RefillLoop(cfg, plan, args.seed, max_len=cfg.max_len + K + W + 2, **pool_kw)
        batch = loop.batch
        step_fn = loop.step
    else:
        lengths = wl.draw_lengths(cfg.lengths, cfg.batch, args.seed, cfg.max_len).astype(np.int64)
        # seq_lens count the token being decoded: start one short, every step appends one token
        batch = DecodeBatch(cfg, args.seed, lengths - 1, headroom_tokens=K + W + 2, profile_events=False, **pool_kw)
        step_fn = batch.step
    logits = wl.make_logits(cfg, args.seed, "cuda")
    torch.cuda.synchronize()

    step_index = 0
    for _ in range(W):
        step_fn(logits, step_index)
        step_index += 1
    torch.cuda.synchronize()
    batch.ev_spare = [(rb.ProfEvent(), rb.ProfEvent()) for _ in range(K)]
    batch.profile_events = True
    refills_before = loop.refills if loop else 0
    t0 = time.perf_counter()
    for _ in range(K):
        step_fn(logits, step_index)
        step_index += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    batch.profile_events = False
    if loop:
        extra = {"refills_in_timed_steps": loop.refills - refills_before,
                 "free_pages_at_end": rb.roll_kv_free_pages(batch.pool),
                 "note": "refill (release, alloc, chunked prefill of the new prompts into pages) is inside the timed steps"}

    ms_per_step = (t1 - t0) * 1e3 / K
    beta = cfg.kv_bytes_per_token
    kern_ms = [a.elapsed_ms(b) for a, b, _ in batch.ev_pairs]
    kv_bytes = [beta * tot for _, _, tot in batch.ev_pairs]
    # one step on the GPU's clock: from the start of an attention launch to the start of the next
    step_gpu_ms = [batch.ev_pairs[i][0].elapsed_ms(batch.ev_pairs[i + 1][0]) for i in range(len(batch.ev_pairs) - 1)]
    avg_kern_ms = float(np.mean(kern_ms))
    avg_kv_bytes = float(np.mean(kv_bytes))
    achieved = avg_kv_bytes / (avg_kern_ms * 1e-3) / 1e9
    workload = (f"{cfg.name}: B={cfg.batch} Hq={cfg.num_q_heads} Hkv={cfg.num_kv_heads} D={cfg.head_dim} "
                f"P={cfg.page_size} lengths={cfg.lengths} V={cfg.vocab} T={cfg.temperature} top_p={cfg.top_p}")
    ceiling = ceiling_probe(torch, rb, batch)

    result = {
        "value": cfg.batch / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "config": {"workload": workload, "seed": args.seed, "sum_seq_lens": int(batch.total_tokens()),
                   "kv_pools": ("two dense allocations, single pages" if args.dense_pools else
                                f"one allocation, K and V of a page side by side, pages in runs of {batch.run_pages}"),
                   **extra},
        "kv_read_GBps": achieved,
        "kv_read_frac_of_peak": achieved / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "attn_stream", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": profiled_traffic(cfg.name, avg_kv_bytes),
                     "algorithmic_bytes_per_launch": avg_kv_bytes, "avg_launch_ms": avg_kern_ms,
                     "launch_ms": spread(kern_ms),
                     "ceiling_GBps": ceiling["GBps"], "frac_of_ceiling": achieved / ceiling["GBps"],
                     "ceiling": "median of 12 launches of roll_prof_kv_read_probe: a plain streaming read of the "
                                "same pages through the same page table, no arithmetic, nothing written"},
    }
    if step_gpu_ms:
        result["step_ms_on_gpu_clock"] = spread(step_gpu_ms)

    # The sampling launch alone (after the timed region): its bound is the vector ALU, not HBM, so
    # it is reported as logits per second and vector instructions per logit.
    n_s = 20
    s0, s1 = rb.ProfEvent(), rb.ProfEvent()
    sdesc = rb.sample_desc(logits)
    s0.record()
    for i in range(n_s):
        rb.roll_sample_logprob(logits, cfg.temperature, cfg.top_p, args.seed, step_index + i, batch.tokens,
                               batch.logprob, sdesc, None)
    s1.record()
    torch.cuda.synchronize()
    samp_ms = s0.elapsed_ms(s1) / n_s
    result["sampling"] = {"kernel": "sample_rows", "bound": "alu", "avg_launch_ms": samp_ms,
                          "Gelem_per_s": cfg.batch * cfg.vocab / (samp_ms * 1e-3) / 1e9,
                          "vector_instructions_per_logit": profiled_valu_per_logit(cfg.name),
                          "peak_lane_ops_per_s": 256 * 4 * 16 * 2.4e9,
                          "compulsory_bytes": cfg.batch * cfg.vocab * (2 if cfg.logits_dtype == "bf16" else 4)}
    # share of a step's wall time in which the step's own kernels run (the attention launch timed in
    # place, the sampling launch as timed alone; c4: plus the prefill launches of the refill ticks)
    prefill_ms = sum(a.elapsed_ms(b) for a, b in loop.prefill_events) / K if loop else 0.0
    result["gpu_busy_frac"] = (avg_kern_ms + samp_ms + prefill_ms) / ms_per_step
    if loop:
        result["config"]["prefill_ms_per_step"] = prefill_ms
    n_layers = 64 if cfg.name == "c5" else 28
    result["extrapolation"] = {
        "what": "tokens/s if every step ran n_layers such attention launches and one sampling launch "
                "(the attention and sampling times measured above; nothing else of a model counted)",
        "n_layers": n_layers,
        "tokens_per_s": cfg.batch / ((n_layers * avg_kern_ms + samp_ms) * 1e-3)}
    # the step that parity is checked on must be the last one the batch ran
    rb.roll_sample_logprob(logits, cfg.temperature, cfg.top_p, args.seed, step_index - 1, batch.tokens,
                           batch.logprob, sdesc, None)
    torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        import oracle
        n = cfg.batch if args.oracle_rows <= 0 else min(args.oracle_rows, cfg.batch)
        rows = [int(r) for r in np.linspace(0, cfg.batch - 1, n).round().astype(int)]
        rows = sorted(set(rows))
        q, k, v, table, lens = batch.gather_rows(rows)
        last_step = step_index - 1
        gpu_out = batch.out[torch.tensor(rows, device="cuda")].double().cpu().numpy()
        gpu_tok = batch.tokens.cpu().numpy()[rows]
        gpu_lp = batch.logprob.double().cpu().numpy()[rows]
        lg_host = wl.logits_numpy(logits[torch.tensor(rows, device="cuda")])
        c0 = time.perf_counter()
        ref_out, threads = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads,
                                              cfg.head_dim, cfg.page_size, return_threads=True)
        c1 = time.perf_counter()
        ref = oracle.sample_logprob(lg_host, cfg.temperature, cfg.top_p, args.seed, last_step, row_ids=rows)
        c2 = time.perf_counter()
        differ = gpu_tok != ref["tokens"]
        x = logits[torch.tensor(rows, device="cuda")].float().cpu().numpy()
        # rows whose tokens differ and one of the two lies between the cuts for top_p -+ 1e-5
        in_band = sum(any(ref["x_cut_plus"][i] <= x[i, t] < ref["x_cut_minus"][i]
                          for t in (gpu_tok[i], ref["tokens"][i]) if 0 <= t < cfg.vocab)
                      for i in np.flatnonzero(differ))
        near_tie = int((differ & (ref["gap"] < 1e-5)).sum())
        result["cpu_baseline"] = {
            "value": len(rows) / (c2 - c0), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{len(rows)} of {cfg.batch} rows" + (" (all)" if len(rows) == cfg.batch else " (evenly spaced)") +
                      f", {int(lens.sum())} KV tokens: attention {c1 - c0:.2f} s + sampling {c2 - c1:.2f} s",
        }
        result["parity_on_sample"] = {
            "rows_compared": len(rows),
            "attn_max_abs_err_bf16_out": float(np.abs(gpu_out - ref_out).max()),
            "logprob_max_abs_err": float(np.abs(gpu_lp - ref["logprob"])[~differ].max()) if not differ.all() else None,
            "token_mismatches": int(differ.sum()),
            "token_mismatches_at_near_ties_below_1e-5": near_tie,
            "token_mismatches_in_top_p_boundary_band": int(in_band),
            "near_ties_below_1e-5": int((ref["gap"] < 1e-5).sum()),
        }
    batch.close()
    del batch, loop, logits
    torch.cuda.empty_cache()
    return result


C4_STEPS = 200  # the refill workload is defined over 200 decode steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None, choices=["c2", "c3", "c4", "c5"],
                    help="one configuration only.  Default: the headline is c5, the largest single-GPU "
                         "configuration, and c2, c3 and c4 (the 200-step refill loop) follow under per_config")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--oracle-rows", type=int, default=0, help="rows timed on the CPU oracle (0 = the whole batch)")
    ap.add_argument("--policy-loss", action="store_true",
                    help="measure roll_policy_loss (the consumer of logprob_out) instead of the decode step")
    ap.add_argument("--prefill", action="store_true",
                    help="measure roll_prefill_attn (chunked prefill into pages) instead of the decode step")
    ap.add_argument("--equal-rows", action="store_true",
                    help="measure the plain attention launch on a batch of equal rows of the config's mean "
                         "length (no row is cut, little is written): what the kernel reads when nothing is ragged")
    ap.add_argument("--dense-pools", action="store_true",
                    help="K and V in two dense allocations and pages handed out one by one, instead of one "
                         "allocation with the K and V block of a page side by side and pages in runs of 32 / P")
    ap.add_argument("--prefill-groups", action="store_true",
                    help="prefill attention across numbers of query heads per KV head, units per workgroup chosen "
                         "by the launch against one span per workgroup")
    ap.add_argument("--prefill-timeline", action="store_true",
                    help="per-workgroup timestamps of the prefill attention launch on three prompt shapes; needs "
                         "the library built with `python -m paper_2510_11345_amd.build --timeline`")
    ap.add_argument("--attn-timeline", action="store_true",
                    help="per-wave timestamps of the attention launch on --config (default c4): needs the "
                         "library built with `python -m paper_2510_11345_amd.build --timeline`")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU: rollout decode is data-parallel over sequences with "
              "no exchange between GPUs, so --gpus N > 1 is not implemented; run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_11345_amd import binding as rb
    from paper_2510_11345_amd import workloads as wl
    from paper_2510_11345_amd.harness import DecodeBatch
    if args.attn_timeline or args.prefill_timeline:
        from paper_2510_11345_amd import build as hip_build
        if not os.path.exists(hip_build.TIMELINE_LIB):
            print("bench.py --attn-timeline / --prefill-timeline: build the instrumented library first: "
                  "python -m paper_2510_11345_amd.build --timeline", file=sys.stderr)
            sys.exit(1)
        rb.LIB_PATH = hip_build.TIMELINE_LIB

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    rb.lib()  # fail loudly if the HIP library is missing
    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_calibration": "one device copy", "bytes_read": src.numel() * 4,
                          "bytes_written": dst.numel() * 4}))
        return
    if args.prefill_timeline:
        prefill_timeline_bench(args, torch, rb, wl)
        return
    if args.prefill_groups:
        prefill_groups_bench(args, torch, rb, wl)
        return
    if args.attn_timeline:
        args.config = args.config or "c4"
        attn_timeline_bench(args, torch, rb, wl)
        return
    if args.equal_rows:
        args.config = args.config or "c2"
        equal_rows_bench(args, torch, rb, wl, DecodeBatch)
        return
    if args.policy_loss:
        print(json.dumps(policy_loss_bench(args, torch, rb, wl)), flush=True)
        return
    if args.prefill:
        print(json.dumps(prefill_bench(args, torch, rb, wl)), flush=True)
        return

    K, W = args.steps, args.warmup
    head_name = args.config or "c5"
    say = lambda m: print(m, file=sys.stderr, flush=True)
    say(f"bench: {head_name}, {K} steps")
    head = run_config(head_name, K, W, args, torch, rb, wl)
    result = {
        "metric": "decode tokens/s (one attention layer + sampling per step)",
        "value": head.pop("value"),
        "unit": head.pop("unit"),
        "n_gpus": 1,
        "steps": head.pop("steps"),
        "warmup": head.pop("warmup"),
        "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        **head,
    }
    if args.config is None:
        # the other single-GPU configurations, each a whole run of its own (same fields)
        result["per_config"] = {}
        for name in ("c3", "c2", "c4"):
            k = C4_STEPS if name == "c4" else K
            say(f"bench: {name}, {k} steps")
            result["per_config"][name] = run_config(name, k, W, args, torch, rb, wl)
        # the kernels beside the decode step (prefill of refilled prompts, the consumer of the recorded
        # log-probs), a short run of each with its own roofline block; a failure here is reported in
        # place of the figures and does not take the decode figures with it
        result["other_kernels"] = {}
        for name, fn, k, w in (("prefill_attn", prefill_bench, 10, 3), ("policy_loss", policy_loss_bench, 20, 3)):
            say(f"bench: {name}, {k} steps")
            sub = argparse.Namespace(**{**vars(args), "steps": k, "warmup": w})
            try:
                r = fn(sub, torch, rb, wl)
                result["other_kernels"][name] = {key: r[key] for key in ("metric", "value", "unit", "steps", "warmup",
                                                                         "ms_per_step", "dtype", "config", "roofline")}
            except Exception as e:   # noqa: BLE001
                result["other_kernels"][name] = {"error": f"{type(e).__name__}: {e}"}
            torch.cuda.empty_cache()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
