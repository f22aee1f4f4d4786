"""Queue-scheduled continuous refill through the C ABI (needs an MI355X): slots finish by
pre-drawn target length, are released and refilled from a prompt queue, and every step's
sampling (and a subset of steps' attention) is checked against the oracle."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from paper_2510_11345_amd.harness import DecodeBatch, RefillLoop
from gpu_helpers import say

pytestmark = pytest.mark.gpu


def test_refill_loop_reduced():
    # config 4 at reduced size: 24 slots, 7B-class heads, 48 steps, short targets so that
    # about one slot finishes per step
    cfg = dataclasses.replace(wl.CONFIGS["c4"], batch=24, vocab=8192)
    steps = 48
    plan = wl.draw_refill_plan(cfg.batch, cfg.batch + 200, seed=3, prompt_range=(5, 90),
                               target_median=30.0, target_clip=(2, 400))
    loop = RefillLoop(cfg, plan, seed=3, max_len=90 + 400 + steps + 2, out_dtype=torch.float32)
    b = loop.batch
    total_pages = b.num_pages
    attn_checked = prefill_checked = 0
    for step in range(steps):
        logits = wl.make_logits(cfg, 3, "cuda", salt=100 + step)
        refilled = loop.step(logits, step)
        torch.cuda.synchronize()
        # allocator invariants after every tick
        assert b.pages_held() + rb.roll_kv_free_pages(b.pool) == total_pages
        assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32))
        # sampling parity every step (row id = slot, step = decode step)
        ref = oracle.sample_logprob(wl.logits_numpy(logits), cfg.temperature, cfg.top_p, 3, step)
        tok, lp = b.tokens.cpu().numpy(), b.logprob.double().cpu().numpy()
        bad = [r for r in range(cfg.batch) if tok[r] != ref["tokens"][r] and ref["gap"][r] >= 1e-5]
        assert not bad, (step, bad)
        same = tok == ref["tokens"]
        assert np.abs(lp - ref["logprob"])[same].max() <= 1e-3
        # the prefill of the refilled prompts: its output for the last prompt token is a decode
        # step over the prompt (the pages are read back after the step; the token appended by
        # the step lies beyond the prompt's length)
        if refilled:
            qp, outp, meta = loop.last_prefill
            assert [m[0] for m in meta] == refilled
            _, kq, vq, tq, _ = b.gather_rows(refilled)
            last = [m[2] + m[1] - 1 for m in meta]
            want_p = oracle.decode_attn(wl.bits(qp[last]), kq, vq, tq, np.array([m[1] for m in meta], np.int32),
                                        cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size)
            err_p = np.abs(outp[last].double().cpu().numpy() - want_p).max()
            assert err_p <= 1e-4, (step, err_p)
            prefill_checked += len(refilled)
        # attention parity on the first and last step, every 8th, and right after a refill
        if step in (0, steps - 1) or step % 8 == 0 or refilled:
            rows = list(range(cfg.batch))
            q, k, v, table, lens = b.gather_rows(rows)
            want = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads,
                                      cfg.head_dim, cfg.page_size)
            err = np.abs(b.out.double().cpu().numpy() - want).max()
            assert err <= 1e-4, (step, err)
            attn_checked += 1
    say(f"  refill loop: {steps} steps, {loop.refills} refills, attention checked on {attn_checked} steps, "
        f"free pages at the end {rb.roll_kv_free_pages(b.pool)}, prefills checked {prefill_checked}")
    assert loop.refills >= 10
    loop.close()


def test_abort_mid_sequence_then_refill():
    # ABORT = release of a live slot; its pages go back and the next prompt reuses them
    cfg = dataclasses.replace(wl.CONFIGS["c4"], batch=4, vocab=4096)
    plan = wl.draw_refill_plan(4, 12, seed=5, prompt_range=(20, 40), target_median=1000.0,
                               target_clip=(900, 1000))
    loop = RefillLoop(cfg, plan, seed=5, max_len=1100, out_dtype=torch.float32)
    b = loop.batch
    logits = wl.make_logits(cfg, 5, "cuda")
    loop.step(logits, 0)
    free_before = rb.roll_kv_free_pages(b.pool)
    pages = rb.roll_kv_slot_pages(b.pool, 2)
    loop.generated[2] = 10**9            # force slot 2 to be reclaimed at the next tick
    refilled = loop.step(logits, 1)
    assert refilled == [2]
    new_pages = rb.roll_kv_slot_pages(b.pool, 2)
    assert set(new_pages) <= set(pages) or len(new_pages) <= len(pages)
    assert rb.roll_kv_free_pages(b.pool) >= free_before
    torch.cuda.synchronize()
    q, k, v, table, lens = b.gather_rows([0, 1, 2, 3])
    want = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                              cfg.page_size)
    assert np.abs(b.out.double().cpu().numpy() - want).max() <= 1e-4
    loop.close()


def test_random_release_refill_schedule():
    # slots come and go at random (releases without refill leave empty slots in the batch, prompts of
    # awkward lengths, several events per tick): the device tables must follow the host state at
    # every step, whichever route (one launch or two) the step takes
    rng = np.random.default_rng(17)
    cfg = dataclasses.replace(wl.CONFIGS["c4"], batch=12, vocab=2048)
    P, B, steps = cfg.page_size, cfg.batch, 90
    start = rng.integers(1, 70, size=B)
    b = DecodeBatch(cfg, 17, start, max_len=400, out_dtype=torch.float32, num_pages=B * 26)
    logits = wl.make_logits(cfg, 17, "cuda")
    live = np.ones(B, dtype=bool)
    bank_q = wl.randn_bf16((256, cfg.num_q_heads, cfg.head_dim), 17, 70, "cuda")
    bank_k = wl.randn_bf16((256, cfg.num_kv_heads, cfg.head_dim), 17, 71, "cuda")
    bank_v = wl.randn_bf16((256, cfg.num_kv_heads, cfg.head_dim), 17, 72, "cuda")
    checked = 0
    for step in range(steps):
        changed = False
        for slot in np.flatnonzero(live):
            if rng.random() < 0.06 or b.lengths[slot] > 300:
                rb.roll_kv_release(b.pool, int(slot))
                b.lengths[slot] = 0
                live[slot] = False
                changed = True
        chunks = []
        for slot in np.flatnonzero(~live):
            if rng.random() < 0.3:
                n = int(rng.choice([1, P - 1, P, P + 1, 2 * P, 37, 95]))
                rb.roll_kv_alloc(b.pool, int(slot), n)
                b.lengths[slot] = n
                live[slot] = True
                chunks.append((int(slot), n))
                changed = True
        if chunks:
            rb.roll_kv_commit(b.pool)
            T = sum(n for _, n in chunks)
            off = np.concatenate([[0], np.cumsum([n for _, n in chunks])]).astype(np.int32)
            out = torch.empty((T, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
            rb.roll_prefill_attn(bank_q[:T], bank_k[:T], bank_v[:T],
                                 torch.tensor([s for s, _ in chunks], dtype=torch.int32, device="cuda"),
                                 torch.zeros(len(chunks), dtype=torch.int32, device="cuda"),
                                 torch.from_numpy(off).cuda(), b.k_pages, b.v_pages, b.page_table, out, P)
        elif changed and rng.random() < 0.5:
            rb.roll_kv_commit(b.pool)       # sometimes the release is published before the step
        # one decode step over the live slots only
        slots = np.flatnonzero(live).astype(np.int32)
        if len(slots):
            rb.roll_kv_alloc_batch(b.pool, slots, np.ones(len(slots), dtype=np.int32))
            b.lengths[slots] += 1
        rb.roll_decode_step_attn(b.pool, b.k_new, b.v_new, b.q, b.k_pages, b.v_pages, b.out, b.desc, b._ws)
        torch.cuda.synchronize()
        assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32)), step
        table = b.page_table.cpu().numpy()
        for slot in range(B):
            pages = rb.roll_kv_slot_pages(b.pool, slot)
            assert list(table[slot, :len(pages)]) == pages, (step, slot)
        assert b.pages_held() + rb.roll_kv_free_pages(b.pool) == b.num_pages
        if step % 6 == 0 or step == steps - 1 or chunks:
            q, k, v, tb, lens = b.gather_rows(list(range(B)))
            want = oracle.decode_attn(q, k, v, tb, lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, P)
            err = np.abs(b.out.double().cpu().numpy() - want).max()
            assert err <= 1e-4, (step, err)
            checked += 1
    fused = rb.roll_kv_fused_steps(b.pool)
    say(f"  random schedule: {steps} steps, {fused} in one launch, attention checked on {checked}")
    assert 10 <= fused < steps
    b.close()
