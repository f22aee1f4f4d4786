"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (needs an MI355X): one decode step of c2, c3 and c5 through the harness with EVERY row's
attention output, token and log-prob compared with the oracle, and config 4 (256 slots, 200 steps
of continuous refill) with sampling parity at every step and attention parity on a schedule."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from paper_2510_11345_amd.harness import DecodeBatch, RefillLoop
from gpu_helpers import say

pytestmark = pytest.mark.gpu


def check_sampling(tok, lp, ref, logits_rows, vocab, where=""):
    """The bar on tokens and log-probs for the rows of `ref`: identical tokens unless the oracle's
    top-two gap is below 1e-5 or a token lies in the top-p boundary band; log-probs within 1e-3
    wherever the tokens agree.  Returns (near-tie mismatches, boundary-band mismatches)."""
    same = tok == ref["tokens"]
    assert ((tok >= 0) & (tok < vocab)).all(), where
    if same.any():
        assert np.abs(lp - ref["logprob"])[same].max() <= 1e-3, where
    ties = band = 0
    for i in np.flatnonzero(~same):
        x = logits_rows(int(i))
        in_band = lambda t: ref["x_cut_plus"][i] <= x[t] < ref["x_cut_minus"][i]
        if ref["gap"][i] < 1e-5:
            ties += 1
        else:
            assert in_band(tok[i]) or in_band(ref["tokens"][i]), (where, int(i), int(tok[i]), int(ref["tokens"][i]))
            band += 1
    return ties, band


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["c2", "c3", "c5"])
def test_full_size_step_matches_oracle_on_every_row(name, capsys):
    cfg = wl.CONFIGS[name]
    lengths = wl.draw_lengths(cfg.lengths, cfg.batch, 0, cfg.max_len).astype(np.int64)
    with capsys.disabled():
        say(f"\n  full-size case {name}: B={cfg.batch} sum L={int(lengths.sum())} max L={int(lengths.max())}")
    batch = DecodeBatch(cfg, 0, lengths - 1, headroom_tokens=4)
    logits = wl.make_logits(cfg, 0, "cuda")
    batch.step(logits, 0)
    torch.cuda.synchronize()
    assert np.array_equal(batch.lengths, lengths)
    rb.roll_decode_attn_workspace_check(batch._ws)
    got = batch.out.double().cpu().numpy()
    assert np.isfinite(got).all()
    # attention, every row, in slices so that the host copy of the pages stays small
    worst = 0.0
    for first in range(0, cfg.batch, 32):
        rows = list(range(first, min(first + 32, cfg.batch)))
        q, k, v, table, lens = batch.gather_rows(rows)
        want = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                  cfg.page_size)
        err = float(np.abs(got[rows] - want).max())
        worst = max(worst, err)
        assert err <= 2e-2, (name, first, err)
        with capsys.disabled():
            say(f"    attention rows {first}..{rows[-1]}: max abs err {err:.3e} (bf16 out)")
    # sampling, every row
    ref = oracle.sample_logprob(wl.logits_numpy(logits), cfg.temperature, cfg.top_p, 0, 0)
    tok = batch.tokens.cpu().numpy()
    lp = batch.logprob.double().cpu().numpy()
    ties, band = check_sampling(tok, lp, ref, lambda i: logits[i].float().cpu().numpy(), cfg.vocab, name)
    with capsys.disabled():
        say(f"    {name}: attention on all {cfg.batch} rows max abs err {worst:.3e}; sampling on all rows: "
            f"near-tie mismatches {ties}, boundary-band mismatches {band}")
    batch.close()


@pytest.mark.timeout(900)
def test_config4_full_size_refill_loop(capsys):
    # 256 slots, 200 decode steps, finish by pre-drawn target length, release + refill from the prompt
    # queue with chunked prefill; fresh logits every step.  Every step: sampling parity on all rows,
    # allocator conservation, device lengths.  Attention parity on all rows at steps 0, 199 and
    # every 20th; right after a refill on the refilled rows and 15 rows spread over the batch.
    cfg = wl.CONFIGS["c4"]
    steps, seed = 200, 0
    plan = wl.draw_refill_plan(cfg.batch, cfg.batch + 4 * steps + 64, seed)
    loop = RefillLoop(cfg, plan, seed, max_len=cfg.max_len + steps + 2)
    b = loop.batch
    total_pages = b.num_pages
    spread = [int(r) for r in np.linspace(0, cfg.batch - 1, 15).round()]
    checked_all = checked_some = ties = band = 0
    worst = 0.0
    for step in range(steps):
        logits = wl.make_logits(cfg, seed, "cuda", salt=1000 + step)
        refilled = loop.step(logits, step)
        torch.cuda.synchronize()
        assert b.pages_held() + rb.roll_kv_free_pages(b.pool) == total_pages, step
        assert np.array_equal(b.seq_lens.cpu().numpy(), b.lengths.astype(np.int32)), step
        ref = oracle.sample_logprob(wl.logits_numpy(logits), cfg.temperature, cfg.top_p, seed, step)
        t, bd = check_sampling(b.tokens.cpu().numpy(), b.logprob.double().cpu().numpy(), ref,
                               lambda i: logits[i].float().cpu().numpy(), cfg.vocab, f"step {step}")
        ties, band = ties + t, band + bd
        everything = step in (0, steps - 1) or step % 20 == 0
        rows = list(range(cfg.batch)) if everything else (sorted(set(refilled + spread)) if refilled else [])
        for first in range(0, len(rows), 64):
            part = rows[first:first + 64]
            q, k, v, table, lens = b.gather_rows(part)
            want = oracle.decode_attn(q, k, v, table, lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                      cfg.page_size)
            err = float(np.abs(b.out[torch.tensor(part, device="cuda")].double().cpu().numpy() - want).max())
            worst = max(worst, err)
            assert err <= 2e-2, (step, first, err)
        checked_all += everything
        checked_some += bool(rows) and not everything
        if step % 10 == 0 or step == steps - 1:
            with capsys.disabled():
                say(f"    c4 step {step}: refills so far {loop.refills}, sum L {b.total_tokens()}, "
                    f"attention max abs err so far {worst:.3e}")
    rb.roll_decode_attn_workspace_check(b._ws)
    with capsys.disabled():
        say(f"  c4 full size: {steps} steps, {loop.refills} refills, attention checked on all rows at {checked_all} "
            f"steps and on the refilled + 15 spread rows at {checked_some}, near-tie mismatches {ties}, "
            f"boundary-band mismatches {band}, {rb.roll_kv_fused_steps(b.pool)} steps in one launch")
    assert loop.refills >= 20 and checked_some >= 10
    loop.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (32, 8)])
def test_prefill_full_size_sampled_tokens(capsys, Hq, Hkv):
    """bench.py --prefill's long-prompt workloads in their launch configuration (8 prompts x 8192
    tokens in chunks of 2048, 16-token pages, side-by-side pools, bf16 result: blocks of up to 256
    steps in the pipelined loop; 7B-class heads, and 32 heads on 8, whose workgroups of seven
    computing waves reach over two or three spans of query tokens in a launch of this size).  The oracle cannot afford all 65536 tokens; it
    computes sampled ones one by one, as decode steps over the slot's first pos + 1 tokens read
    from the pools the library wrote: the first tokens, both sides of every chunk, span and step
    boundary, the last token, of three slots."""
    D, P = 128, 16
    n_slots, n, chunk = 8, 8192, 2048
    max_pages = n // P
    num_pages = n_slots * max_pages + 8
    page_table = torch.empty((n_slots, max_pages), dtype=torch.int32, device="cuda")
    seq_lens = torch.zeros((n_slots,), dtype=torch.int32, device="cuda")
    pool = rb.KvPool(num_pages, P, n_slots, max_pages, page_table, seq_lens)
    for s in range(n_slots):
        rb.roll_kv_alloc(pool, s, n)
    rb.roll_kv_commit(pool)
    k_pages, v_pages = rb.new_kv_pools(num_pages, Hkv, D, P, fill=0)
    T = n_slots * chunk
    slot = torch.arange(n_slots, dtype=torch.int32, device="cuda")
    off = torch.arange(n_slots + 1, dtype=torch.int32, device="cuda") * chunk
    qs, outs = [], []
    for ci, start in enumerate(range(0, n, chunk)):
        q = wl.randn_bf16((T, Hq, D), 3, 40 + ci, "cuda")
        k = wl.randn_bf16((T, Hkv, D), 3, 50 + ci, "cuda")
        v = wl.randn_bf16((T, Hkv, D), 3, 60 + ci, "cuda")
        out = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        rb.roll_prefill_attn(q, k, v, slot, torch.full((n_slots,), start, dtype=torch.int32, device="cuda"), off,
                             k_pages, v_pages, page_table, out, P)
        qs.append(q)
        outs.append(out)
        del k, v
    torch.cuda.synchronize()
    with capsys.disabled():
        say("  prefill full size: 4 calls of 8 x 2048 tokens done, comparing sampled tokens with the oracle")
    positions = [0, 1, 15, 16, 31, 32, 33, 63, 64, 2047, 2048, 2049, 2079, 2080, 2111, 2112, 4095, 4096, 5555, 6143,
                 6144, 8190, 8191]
    samples = [(s, p) for s in (0, 3, 7) for p in positions]
    table = np.full((n_slots, max_pages), -1, np.int32)
    for s in range(n_slots):
        pr = rb.roll_kv_slot_pages(pool, s)
        table[s, :len(pr)] = pr
    kb, vb = wl.bits(k_pages).reshape(-1), wl.bits(v_pages).reshape(-1)
    q_rows = np.stack([wl.bits(qs[p // chunk][s * chunk + p % chunk]) for s, p in samples])
    got = np.stack([outs[p // chunk][s * chunk + p % chunk].double().cpu().numpy() for s, p in samples])
    want = oracle.decode_attn(np.ascontiguousarray(q_rows), kb, vb, np.ascontiguousarray(table[[s for s, _ in samples]]),
                              np.array([p + 1 for _, p in samples], np.int32), Hq, Hkv, D, P)
    assert not np.isnan(got).any()
    err = np.abs(got - want).max(axis=(1, 2))
    with capsys.disabled():
        say(f"  prefill full size: {len(samples)} sampled tokens, max abs err {err.max():.2e} (bf16 result)")
    assert err.max() <= 2e-2, [(samples[i], float(err[i])) for i in np.flatnonzero(err > 2e-2)]
    pool.close()
