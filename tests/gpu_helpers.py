"""Shared plumbing of the GPU parity tests: upload seeded inputs, call the C ABI through the
binding, fetch results.  No arithmetic of the decode step lives here."""
import numpy as np
import torch

from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl


def say(msg):
    print(msg, flush=True)


def side_by_side(k_pages, v_pages, extra_heads=0):
    """The two pools copied into ONE allocation with the K and the V block of a page next to each
    other (plus extra_heads unused head blocks per page, filled with NaN): strided views of it."""
    N, Hkv, d8, P, _ = k_pages.shape
    D = d8 * 8
    blk = Hkv * P * D
    both = torch.full((N, 2 * blk + extra_heads * P * D), float("nan"), dtype=torch.bfloat16, device=k_pages.device)
    both[:, :blk] = k_pages.reshape(N, blk)
    both[:, blk:2 * blk] = v_pages.reshape(N, blk)
    return both[:, :blk].view(N, Hkv, d8, P, 8), both[:, blk:2 * blk].view(N, Hkv, P // 8, D, 8)


def run_attn(inp, cfg, out_dtype=torch.float32, softmax_scale=0.0, seq_lens=None, layout="dense"):
    """inp: dict from workloads.make_attn_inputs (cpu or cuda tensors). Returns out on host (float64).
    layout: "dense" (two allocations), "side_by_side" (one, K and V of a page adjacent), or
    "padded" (the same with three unused head blocks per page)."""
    dev = "cuda"
    q = inp["q"].to(dev)
    k_pages = inp["k_pages"].to(dev)
    v_pages = inp["v_pages"].to(dev)
    if layout != "dense":
        k_pages, v_pages = side_by_side(k_pages, v_pages, 3 if layout == "padded" else 0)
    table = torch.from_numpy(np.ascontiguousarray(inp["page_table"])).to(dev)
    lens = torch.from_numpy(np.ascontiguousarray(inp["seq_lens"] if seq_lens is None else seq_lens)).to(dev)
    B, Hq, D = q.shape
    out = torch.full((B, Hq, D), float("nan"), dtype=out_dtype, device=dev)
    desc = rb.attn_desc(q, k_pages, table, cfg.page_size, out_dtype, softmax_scale)
    ws = rb.new_attn_workspace(desc, dev)
    rb.roll_decode_attn(q, k_pages, v_pages, table, lens, out, desc, ws)
    torch.cuda.synchronize()
    return out.double().cpu().numpy()


def oracle_attn(inp, cfg, rows=None, scale=None, seq_lens=None):
    import oracle
    return oracle.decode_attn(wl.bits(inp["q"]), wl.bits(inp["k_pages"]).reshape(-1),
                              wl.bits(inp["v_pages"]).reshape(-1), inp["page_table"],
                              inp["seq_lens"] if seq_lens is None else seq_lens,
                              cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size,
                              scale=scale, rows=rows)


def run_sample(logits, T, top_p, seed, step, row_ids=None, want_raw=False):
    dev = "cuda"
    lg = logits if logits.is_cuda else logits.to(dev)
    B = lg.shape[0]
    tokens = torch.full((B,), -7, dtype=torch.int32, device=dev)
    lp = torch.full((B,), float("nan"), dtype=torch.float32, device=dev)
    rid = None if row_ids is None else torch.tensor(row_ids, dtype=torch.int32, device=dev)
    raw = torch.full((B,), float("nan"), dtype=torch.float32, device=dev) if want_raw else None
    desc = rb.sample_desc(lg, rid, raw)
    ws = torch.empty(rb.roll_sample_logprob_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    rb.roll_sample_logprob(lg, T, top_p, seed, step, tokens, lp, desc, ws)
    torch.cuda.synchronize()
    if want_raw:
        return tokens.cpu().numpy(), lp.double().cpu().numpy(), raw.double().cpu().numpy()
    return tokens.cpu().numpy(), lp.double().cpu().numpy()


def compare_sampling(logits, T, top_p, seed, step, row_ids=None, lp_tol=1e-3):
    """Runs both sides; returns (n_mismatch_excused_tie, n_mismatch_excused_band). Asserts the bar:
    token ids identical unless the oracle's top-two gap is below 1e-5 or a token lies in the
    top-p boundary band; log-probs within lp_tol wherever the tokens agree."""
    import oracle
    tok, lp, raw = run_sample(logits, T, top_p, seed, step, row_ids, want_raw=True)
    tok2, lp2 = run_sample(logits, T, top_p, seed, step, row_ids)        # without the raw output
    assert np.array_equal(tok, tok2) and np.array_equal(lp, lp2)
    ref = oracle.sample_logprob(wl.logits_numpy(logits), T, top_p, seed, step, row_ids=row_ids)
    x = wl.logits_numpy(logits)
    if x.dtype == np.uint16:
        x = (x.astype(np.uint32) << 16).view(np.float32)
    ties = band = 0
    for r in range(len(tok)):
        if tok[r] == ref["tokens"][r]:
            assert abs(lp[r] - ref["logprob"][r]) <= lp_tol, (r, lp[r], ref["logprob"][r])
            assert abs(raw[r] - ref["raw_logprob"][r]) <= lp_tol, (r, raw[r], ref["raw_logprob"][r])
            continue
        in_band = lambda t: ref["x_cut_plus"][r] <= x[r, t] < ref["x_cut_minus"][r]
        if ref["gap"][r] < 1e-5:
            ties += 1
        elif 0 <= tok[r] < x.shape[1] and (in_band(tok[r]) or in_band(ref["tokens"][r])):
            band += 1
        else:
            raise AssertionError(f"row {r}: token {tok[r]} != oracle {ref['tokens'][r]} "
                                 f"(gap {ref['gap'][r]:.3e})")
    say(f"    sampling parity: {len(tok)} rows, near-tie mismatches {ties}, boundary-band mismatches {band}")
    return ties, band
