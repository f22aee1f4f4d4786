"""Seeded random shapes and parameters for every GPU entry point against the oracle (needs an
MI355X).  The fixed-case files pick their edge cases by hand; this one draws many small ones.
ROLL_FUZZ_SEED=<n> draws another sweep and ROLL_FUZZ_ROUNDS=<k> makes it k times as long (give pytest
a longer --timeout with it); without them the sweep is the same on every run."""
import dataclasses
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from paper_2510_11345_amd.harness import DecodeBatch
from gpu_helpers import compare_sampling, oracle_attn, run_attn, say

pytestmark = pytest.mark.gpu

SEED = 1000 * int(os.environ.get("ROLL_FUZZ_SEED", "0"))
ROUNDS = max(1, int(os.environ.get("ROLL_FUZZ_ROUNDS", "1")))

HEADS = [(1, 1), (4, 1), (7, 1), (8, 2), (12, 4), (16, 16), (28, 4), (32, 2), (64, 8), (6, 3), (12, 6), (20, 5)]


def _draw_lengths(rng, B, cap):
    kind = rng.integers(0, 4)
    if kind == 0:
        L = rng.integers(0, min(cap, 80) + 1, size=B)              # short rows, some empty
    elif kind == 1:
        L = np.minimum(cap, (rng.pareto(1.2, size=B) * 40 + 1).astype(np.int64))   # long tail
    elif kind == 2:
        L = rng.choice([1, 15, 16, 17, 31, 32, 33, 63, 64, 65, cap], size=B)        # boundaries
    else:
        L = rng.integers(1, cap + 1, size=B)
    return np.minimum(L, cap).astype(np.int32)


def test_decode_attention_random_cases():
    rng = np.random.default_rng(101 + SEED)
    worst32 = worst16 = 0.0
    for case in range(24 * ROUNDS):
        Hq, Hkv = HEADS[rng.integers(0, len(HEADS))]
        D = int(rng.choice([64, 128]))
        P = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 40))
        cap = int(rng.choice([100, 700, 3000]))
        lengths = _draw_lengths(rng, B, cap)
        if lengths.max() == 0:
            lengths[0] = 1
        cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                                  page_size=P)
        inp = wl.make_attn_inputs(cfg, 1000 + case, "cpu", lengths=np.maximum(lengths, 1))
        inp["seq_lens"] = lengths                      # rows drawn empty keep their one page
        scale = 0.0 if rng.random() < 0.7 else float(rng.uniform(0.02, 0.3))
        out_dtype = torch.float32 if rng.random() < 0.5 else torch.bfloat16
        layout = ["dense", "side_by_side", "padded"][case % 3]
        got = run_attn(inp, cfg, out_dtype=out_dtype, softmax_scale=scale, layout=layout)
        want = oracle_attn(inp, cfg, scale=None if scale == 0.0 else scale)
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all()
        if out_dtype == torch.float32:
            worst32 = max(worst32, err)
            assert err <= 1e-4, (case, Hq, Hkv, D, P, B, cap, err)
        else:
            worst16 = max(worst16, err)
            assert err <= 2e-2, (case, Hq, Hkv, D, P, B, cap, err)
    say(f"  decode attention, {24 * ROUNDS} random cases: worst abs err {worst32:.2e} (fp32 out), {worst16:.2e} (bf16 out)")


def test_fused_steps_random_cases():
    rng = np.random.default_rng(202 + SEED)
    for case in range(8 * ROUNDS):
        Hq, Hkv = HEADS[rng.integers(0, len(HEADS))]
        D = int(rng.choice([64, 128]))
        P = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 30))
        start = np.maximum(_draw_lengths(rng, B, 400), 1) - 1       # zero = the slot starts its sequence
        cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                                  page_size=P, vocab=512)
        # pools side by side with runs of pages (the default), side by side with single pages, or
        # two dense allocations with runs of four
        kind = case % 3
        b = DecodeBatch(cfg, 300 + case, start, headroom_tokens=8, out_dtype=torch.float32,
                        side_by_side=kind != 2, run_pages=[None, 1, 4][kind])
        logits = wl.make_logits(cfg, 300 + case, "cuda")
        for step in range(5):
            b.k_new.copy_(wl.randn_bf16(tuple(b.k_new.shape), 300 + case, 50 + step, "cuda"))
            b.v_new.copy_(wl.randn_bf16(tuple(b.v_new.shape), 300 + case, 60 + step, "cuda"))
            b.step(logits, step)
            torch.cuda.synchronize()
            q, k, v, table, lens = b.gather_rows(list(range(B)))
            want = oracle.decode_attn(q, k, v, table, lens, Hq, Hkv, D, P)
            err = float(np.abs(b.out.double().cpu().numpy() - want).max())
            assert err <= 1e-4, (case, step, Hq, Hkv, D, P, B, err)
            assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32))
        assert rb.roll_kv_fused_steps(b.pool) >= 4
        b.close()


def test_prefill_random_cases():
    rng = np.random.default_rng(303 + SEED)
    worst = 0.0
    for case in range(12 * ROUNDS):
        Hq, Hkv = (HEADS + [(24, 1), (40, 2), (9, 1)])[rng.integers(0, len(HEADS) + 3)]   # prefill takes any group size
        D = int(rng.choice([64, 128]))
        P = int(rng.choice([16, 32, 64]))
        n_slots = int(rng.integers(1, 7))
        chunks, need = [], np.zeros(n_slots, np.int64)
        for slot in range(n_slots):
            pos = int(rng.integers(0, 60)) if rng.random() < 0.5 else 0
            for _ in range(int(rng.integers(0, 3))):                 # up to two chunks of a slot, in order
                n = int(rng.choice([0, 1, 7, 8, 9, 16, 31, 32, 33, 50, 120, 257, 400]))
                chunks.append((slot, pos, n))
                pos += n
            need[slot] = pos
        if not chunks or sum(c[2] for c in chunks) == 0:
            chunks.append((0, int(need[0]), 5))
            need[0] += 5
        order = rng.permutation(len(chunks))
        chunks = [chunks[i] for i in order]                           # call order is free
        cap = int(max(need.max(), 1))
        max_pages = (cap + P - 1) // P
        num_pages = n_slots * max_pages + 4
        page_table = torch.empty((n_slots, max_pages), dtype=torch.int32, device="cuda")
        seq_lens = torch.zeros((n_slots,), dtype=torch.int32, device="cuda")
        pool = rb.KvPool(num_pages, P, n_slots, max_pages, page_table, seq_lens)
        for slot in range(n_slots):
            if need[slot]:
                rb.roll_kv_alloc(pool, slot, int(need[slot]))
        rb.roll_kv_commit(pool)
        k_pages = wl.randn_bf16((num_pages, Hkv, D // 8, P, 8), 400 + case, 2, "cuda")
        v_pages = wl.randn_bf16((num_pages, Hkv, P // 8, D, 8), 400 + case, 3, "cuda")
        T = sum(c[2] for c in chunks)
        q = wl.randn_bf16((T, Hq, D), 400 + case, 11, "cuda")
        k_new = wl.randn_bf16((T, Hkv, D), 400 + case, 12, "cuda")
        v_new = wl.randn_bf16((T, Hkv, D), 400 + case, 13, "cuda")
        cs = np.array([c[0] for c in chunks], np.int32)
        st = np.array([c[1] for c in chunks], np.int32)
        off = np.concatenate([[0], np.cumsum([c[2] for c in chunks])]).astype(np.int32)
        kp_host, vp_host = wl.bits(k_pages).reshape(-1).copy(), wl.bits(v_pages).reshape(-1).copy()
        out_dtype = torch.float32 if rng.random() < 0.5 else torch.bfloat16
        out = torch.full((T, Hq, D), float("nan"), dtype=out_dtype, device="cuda")
        # units (span of query tokens x query head) per workgroup: fixed at 1 .. 8, or chosen by the launch
        rb.roll_prof_prefill_units(int(rng.integers(0, 9)))
        rb.roll_prefill_attn(q, k_new, v_new, torch.from_numpy(cs).cuda(), torch.from_numpy(st).cuda(),
                             torch.from_numpy(off).cuda(), k_pages, v_pages, page_table, out, P)
        rb.roll_prof_prefill_units(0)
        torch.cuda.synchronize()
        table = np.full((n_slots, max_pages), -1, np.int32)
        for slot in range(n_slots):
            pr = rb.roll_kv_slot_pages(pool, slot)
            table[slot, :len(pr)] = pr
        want = oracle.prefill_attn(wl.bits(q), wl.bits(k_new), wl.bits(v_new), cs, st, off, kp_host, vp_host, table,
                                   Hq, Hkv, D, P)
        got = out.double().cpu().numpy()
        assert not np.isnan(got).any()
        err = float(np.abs(got - want).max())
        worst = max(worst, err if out_dtype == torch.float32 else 0.0)
        assert err <= (1e-4 if out_dtype == torch.float32 else 2e-2), (case, Hq, Hkv, D, P, chunks, err)
        assert np.array_equal(wl.bits(k_pages).reshape(-1), kp_host), case
        assert np.array_equal(wl.bits(v_pages).reshape(-1), vp_host), case
        pool.close()
    say(f"  prefill, {12 * ROUNDS} random cases: worst abs err {worst:.2e} (fp32 out)")


def test_sampling_random_cases():
    rng = np.random.default_rng(404 + SEED)
    for case in range(16 * ROUNDS):
        B = int(rng.integers(1, 12))
        V = int(rng.choice([3, 17, 256, 1000, 4099, 32003]))
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        kind = str(rng.choice(["normal1", "normal2", "zipf"]))
        cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=B, vocab=V, logits_dtype=dtype, logits=kind)
        stride = V + int(rng.choice([0, 8, 16])) * (1 if rng.random() < 0.5 else 0)
        stride = (stride + 7) // 8 * 8                                # rows stay 16-byte aligned
        full = torch.zeros((B, stride), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
        full[:, :V] = wl.make_logits(cfg, 500 + case, "cuda")
        logits = full[:, :V]
        if rng.random() < 0.3:                                        # masked entries
            mask = torch.from_numpy(rng.random((B, V)) < 0.3).cuda()
            mask[:, 0] = False
            logits.masked_fill_(mask, float("-inf"))
        T = float(rng.choice([0.3, 0.7, 1.0, 1.5]))
        top_p = float(rng.choice([1.0, 0.99, 0.9, 0.5, 0.05]))
        seed = int(rng.integers(0, 2**63 - 1))
        step = int(rng.integers(0, 2**40))
        rows = None if rng.random() < 0.5 else [int(x) for x in rng.integers(0, 2**31 - 1, size=B)]
        compare_sampling(logits, T, top_p, seed, step, row_ids=rows)
