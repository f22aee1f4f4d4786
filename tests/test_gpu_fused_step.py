"""The single-launch decode step (allocator commit + K/V append + attention) through the C ABI
(needs an MI355X): against the oracle, against the two-launch route bit for bit, and on the
cases where it has to take the two-launch route."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from paper_2510_11345_amd.harness import DecodeBatch
from gpu_helpers import say

pytestmark = pytest.mark.gpu


def _fresh_kv(batch: DecodeBatch, seed: int, step: int):
    cfg = batch.cfg
    shape = (cfg.batch, cfg.num_kv_heads, cfg.head_dim)
    batch.k_new.copy_(wl.randn_bf16(shape, seed, 500 + 2 * step, "cuda"))
    batch.v_new.copy_(wl.randn_bf16(shape, seed, 501 + 2 * step, "cuda"))
    batch.q.copy_(wl.randn_bf16((cfg.batch, cfg.num_q_heads, cfg.head_dim), seed, 900 + step, "cuda"))


def _oracle_err(batch: DecodeBatch) -> float:
    cfg = batch.cfg
    rows = list(range(cfg.batch))
    q, k, v, table, lens = batch.gather_rows(rows)
    want = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                              cfg.page_size)
    return float(np.abs(batch.out.double().cpu().numpy() - want).max())


def _lengths(B: int, P: int, seed: int) -> np.ndarray:
    """Lengths AFTER the first step: page starts, page ends, multiples of the 32-token step and
    of it plus one, a row of one token, rows long enough to be cut across waves."""
    rng = np.random.default_rng([seed, 0x465553])
    special = [1, 2, P, P + 1, 2 * P, 31, 32, 33, 64, 65, 4 * P + 1, 96, 97, 1024, 1025, 3000, 2048 + 1]
    L = rng.integers(1, 700, size=B)
    L[:min(B, len(special))] = special[:B]
    return L.astype(np.int64)


@pytest.mark.parametrize("D,P,Hq,Hkv", [(128, 16, 28, 4), (128, 32, 64, 8), (64, 64, 8, 2), (64, 16, 16, 16)])
def test_fused_step_matches_oracle_and_two_launches(D, P, Hq, Hkv):
    B, steps, seed = 40, 6, 11
    cfg = dataclasses.replace(wl.CONFIGS["c2"], batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                              page_size=P, vocab=2048)
    first = _lengths(B, P, seed)
    logits = wl.make_logits(cfg, seed, "cuda")
    runs = {}
    for fused in (True, False):
        b = DecodeBatch(cfg, seed, first - 1, headroom_tokens=steps + 2, out_dtype=torch.float32, fused=fused)
        outs = []
        for step in range(steps):
            _fresh_kv(b, seed, step)
            b.step(logits, step)
            torch.cuda.synchronize()
            if fused:
                err = _oracle_err(b)
                assert err <= 1e-4, (step, err)
                assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32))
            outs.append(b.out.clone())
        runs[fused] = (b, outs)
    bf, outs_f = runs[True]
    bu, outs_u = runs[False]
    # rows of length 0 before the first step start a sequence there: that step takes the
    # two-launch route, every later one the single launch
    expect = steps - (1 if (first == 1).any() else 0)
    assert rb.roll_kv_fused_steps(bf.pool) == expect, rb.roll_kv_fused_steps(bf.pool)
    assert rb.roll_kv_fused_steps(bu.pool) == 0
    for step in range(steps):
        assert torch.equal(outs_f[step], outs_u[step]), step
    assert torch.equal(bf.seq_lens, bu.seq_lens)
    # same allocation order, so the same physical pages: pools and tables must be identical
    for slot in range(B):
        assert rb.roll_kv_slot_pages(bf.pool, slot) == rb.roll_kv_slot_pages(bu.pool, slot)
        n = len(rb.roll_kv_slot_pages(bf.pool, slot))
        assert torch.equal(bf.page_table[slot, :n], bu.page_table[slot, :n])
    assert torch.equal(bf.k_pages.view(torch.int16), bu.k_pages.view(torch.int16))
    assert torch.equal(bf.v_pages.view(torch.int16), bu.v_pages.view(torch.int16))
    say(f"  fused step D={D} P={P} Hq={Hq} Hkv={Hkv}: {steps} steps bit-identical to two launches, "
        f"{expect} in one launch")
    bf.close()
    bu.close()


def test_fused_step_bf16_out_and_empty_slots():
    B, seed = 24, 5
    cfg = dataclasses.replace(wl.CONFIGS["c2"], batch=B, vocab=2048)
    L = _lengths(B, cfg.page_size, seed)
    b = DecodeBatch(cfg, seed, L, headroom_tokens=8, out_dtype=torch.bfloat16)
    # empty three slots; they must stay empty and give zeros
    for slot in (3, 9, 23):
        rb.roll_kv_release(b.pool, slot)
        b.lengths[slot] = 0
    rb.roll_kv_commit(b.pool)
    live = np.array([s for s in range(B) if s not in (3, 9, 23)], dtype=np.int32)
    logits = wl.make_logits(cfg, seed, "cuda")
    for step in range(3):
        _fresh_kv(b, seed, step)
        rb.roll_kv_alloc_batch(b.pool, live, np.ones(len(live), dtype=np.int32))
        b.lengths[live] += 1
        rb.roll_decode_step_attn(b.pool, b.k_new, b.v_new, b.q, b.k_pages, b.v_pages, b.out, b.desc, b._ws)
        torch.cuda.synchronize()
        assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32))
        assert _oracle_err(b) <= 2e-2
        assert float(b.out[[3, 9, 23]].abs().max()) == 0.0
    assert rb.roll_kv_fused_steps(b.pool) == 3
    b.close()


def test_fused_step_falls_back_when_not_a_plain_step():
    B, seed = 160, 7
    cfg = dataclasses.replace(wl.CONFIGS["c2"], batch=B, vocab=2048)
    P = cfg.page_size
    # every slot at a page end: the next step opens B = 160 > 128 pages at once
    b = DecodeBatch(cfg, seed, np.full(B, 3 * P), headroom_tokens=3 * P, out_dtype=torch.float32)
    logits = wl.make_logits(cfg, seed, "cuda")
    _fresh_kv(b, seed, 0)
    b.step(logits, 0)
    torch.cuda.synchronize()
    assert rb.roll_kv_fused_steps(b.pool) == 0
    assert _oracle_err(b) <= 1e-4
    # the next one is a plain step again
    _fresh_kv(b, seed, 1)
    b.step(logits, 1)
    torch.cuda.synchronize()
    assert rb.roll_kv_fused_steps(b.pool) == 1
    assert _oracle_err(b) <= 1e-4
    # a refill (release + new prompt) that was not committed: two launches, same results
    rb.roll_kv_release(b.pool, 5)
    rb.roll_kv_alloc(b.pool, 5, 40)
    b.lengths[5] = 40
    _fresh_kv(b, seed, 2)
    b.step(logits, 2)
    torch.cuda.synchronize()
    assert rb.roll_kv_fused_steps(b.pool) == 1
    assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32))
    # slot 5's first 40 positions were never written by the prompt writer; they hold whatever
    # the pages held, which the oracle reads too (it sees the same pools)
    assert _oracle_err(b) <= 1e-4
    _fresh_kv(b, seed, 3)
    b.step(logits, 3)
    torch.cuda.synchronize()
    assert rb.roll_kv_fused_steps(b.pool) == 2
    assert _oracle_err(b) <= 1e-4
    b.close()


def test_fused_step_rejects_a_desc_that_is_not_the_pools():
    cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=4)
    b = DecodeBatch(cfg, 0, np.array([5, 6, 7, 8]), headroom_tokens=4, out_dtype=torch.float32)
    desc = rb.attn_desc(b.q[:3], b.k_pages, b.page_table[:3], cfg.page_size, torch.float32)
    with pytest.raises(rb.RollError):
        rb.roll_decode_step_attn(b.pool, b.k_new, b.v_new, b.q, b.k_pages, b.v_pages, b.out, desc, b._ws)
    b.close()
