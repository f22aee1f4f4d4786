"""roll_decode_attn_static, the entry point that allocates nothing (needs an MI355X): its results
against roll_decode_attn's on the same inputs, on two calls in a row, the second on a smaller
batch (the static scratch keeps the first call's contents), and against the oracle."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from gpu_helpers import oracle_attn, say

pytestmark = pytest.mark.gpu


def _both(cfg, lengths, seed, out_dtype):
    """(static entry's out, workspace entry's out) on the same device inputs, as host float64."""
    lens = np.asarray(lengths, np.int32)
    inp = wl.make_attn_inputs(cfg, seed, "cpu", lengths=np.maximum(lens, 1))
    dev = "cuda"
    q, k, v = inp["q"].to(dev), inp["k_pages"].to(dev), inp["v_pages"].to(dev)
    table = torch.from_numpy(np.ascontiguousarray(inp["page_table"])).to(dev)
    sl = torch.from_numpy(lens).to(dev)
    B, Hq, D = q.shape
    desc = rb.attn_desc(q, k, table, cfg.page_size, out_dtype)
    out_static = torch.full((B, Hq, D), float("nan"), dtype=out_dtype, device=dev)
    out_ws = torch.full((B, Hq, D), float("nan"), dtype=out_dtype, device=dev)
    ws = rb.new_attn_workspace(desc, dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    say(f"  no-alloc case B={B} Hq={Hq} Hkv={cfg.num_kv_heads} D={D} P={cfg.page_size} sumL={int(lens.sum())} "
        f"maxL={int(lens.max())} out={out_dtype}")
    rb.roll_decode_attn_static(q, k, v, table, sl, out_static, desc)
    assert torch.cuda.memory_allocated() == before      # nothing came from torch's allocator either
    rb.roll_decode_attn(q, k, v, table, sl, out_ws, desc, ws)
    torch.cuda.synchronize()
    rb.roll_decode_attn_workspace_check(ws)
    return inp, lens, out_static, out_ws


def test_static_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    cfg = wl.CONFIGS["c2"]
    rng = np.random.default_rng(23)
    # first call: long-tailed rows, many of them cut across workgroups (pieces go through the scratch,
    # rows of more than 16 pieces take the second merge level)
    big = np.concatenate([rng.integers(1, 3000, size=90), [40000, 0, 17000, 1, 33]]).astype(np.int32)
    # second call: a smaller batch, other lengths, other output type
    small = np.concatenate([rng.integers(1, 900, size=21), [9000, 0, 31]]).astype(np.int32)
    for lens, seed, dt, tol in [(big, 3, torch.float32, 1e-4), (small, 4, torch.bfloat16, 2e-2)]:
        c = dataclasses.replace(cfg, batch=len(lens))
        inp, lens, got_static, got_ws = _both(c, lens, seed, dt)
        # same kernel, same dealing: the two entry points agree bit for bit
        assert torch.equal(got_static.view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                           got_ws.view(torch.int16 if dt == torch.bfloat16 else torch.int32))
        ref = oracle_attn(inp, c, seq_lens=lens)
        err = np.abs(got_static.double().cpu().numpy() - ref).max()
        say(f"    static entry against the oracle: max abs err {err:.3e}")
        assert err <= tol
        assert not got_static[torch.from_numpy(lens == 0).cuda()].any()


def test_static_entry_point_refuses_a_shape_beyond_its_scratch():
    # 16 KV heads with a group of 16 heads of 128: the pieces of such a launch do not fit 48 MiB
    q = torch.zeros((2, 256, 128), dtype=torch.bfloat16, device="cuda")
    k, v = rb.new_kv_pools(4, 16, 128, 16, fill=0)
    table = torch.zeros((2, 2), dtype=torch.int32, device="cuda")
    sl = torch.ones((2,), dtype=torch.int32, device="cuda")
    out = torch.full((2, 256, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    desc = rb.attn_desc(q, k, table, 16)
    with pytest.raises(rb.RollError) as e:
        rb.roll_decode_attn_static(q, k, v, table, sl, out, desc)
    assert e.value.status == -6 and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())           # nothing was launched
