"""GPU parity of roll_decode_attn against the fp64 oracle, element by element (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2510_11345_amd import workloads as wl
import oracle
from gpu_helpers import oracle_attn, run_attn, say

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4   # fp32 output, absolute
TOL_BF16 = 2e-2  # bf16 output, absolute

EDGE_LENGTHS = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 511, 512, 513, 1023, 1024,
                1025, 1537, 2048, 2049]


def check(cfg, lengths, seed, bf16_too=True, scale=0.0, layout="dense"):
    say(f"  attn case {cfg.name} B={len(lengths)} Hq={cfg.num_q_heads} Hkv={cfg.num_kv_heads} "
        f"D={cfg.head_dim} P={cfg.page_size} seed={seed} maxL={max(lengths)}")
    inp = wl.make_attn_inputs(cfg, seed, "cpu", lengths=np.asarray(lengths, np.int32))
    ref = oracle_attn(inp, cfg, scale=scale if scale else None)
    got = run_attn(inp, cfg, torch.float32, softmax_scale=scale, layout=layout)
    err = np.abs(got - ref).max()
    say(f"    fp32 out ({layout} pools): max abs err {err:.3e}")
    assert np.isfinite(got).all() and err <= TOL_F32
    if bf16_too:
        got16 = run_attn(inp, cfg, torch.bfloat16, softmax_scale=scale, layout=layout)
        err16 = np.abs(got16 - ref).max()
        say(f"    bf16 out: max abs err {err16:.3e}")
        assert np.isfinite(got16).all() and err16 <= TOL_BF16
    return inp, ref


def test_config1_exact_shape():
    cfg = wl.CONFIGS["c1"]
    check(cfg, wl.draw_lengths(cfg.lengths, cfg.batch, 0), seed=0)


def test_7b_shape_edge_lengths():
    cfg = wl.CONFIGS["c2"]
    check(cfg, EDGE_LENGTHS, seed=1)


@pytest.mark.parametrize("lengths", [[40000], [3, 30000, 5], [1] * 40, [33] * 300, [20000, 20000, 1, 0, 7]])
def test_rows_cut_across_many_waves_and_tiny_batches(lengths):
    # one row longer than all the others together is spread over hundreds of waves; a batch of
    # one-token rows leaves most waves idle; both ends of the work dealing
    cfg = wl.CONFIGS["c2"]
    lens = np.asarray(lengths, np.int32)
    inp = wl.make_attn_inputs(cfg, 11, "cpu", lengths=np.maximum(lens, 1))
    ref = oracle_attn(inp, cfg, seq_lens=lens)
    got = run_attn(inp, cfg, torch.float32, seq_lens=lens)
    err = np.abs(got - ref).max()
    say(f"  attn cut-rows case {lengths[:5]}... max abs err {err:.3e}")
    assert np.isfinite(got).all() and err <= TOL_F32


@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (16, 2), (24, 8), (12, 6)])
def test_short_rows_clustered_beside_long_ones(Hq, Hkv):
    # Ranges are equal in cost, a row costing about a step beyond its steps: a range of one-step
    # rows holds fewer steps than one inside a long row, and range ends fall at every place of a
    # row (its first step, its last, the gap between two rows, empty rows between).
    rng = np.random.default_rng(Hq * 100 + Hkv)
    short = rng.integers(0, 70, size=700)
    short[rng.integers(0, 700, size=60)] = 0
    lens = np.concatenate([short[:350], rng.integers(1500, 6000, size=12), short[350:], [9000, 1, 0, 33, 32, 31]]).astype(np.int32)
    cfg = dataclasses.replace(wl.CONFIGS["c2"], batch=len(lens), num_q_heads=Hq, num_kv_heads=Hkv)
    inp = wl.make_attn_inputs(cfg, 17, "cpu", lengths=np.maximum(lens, 1))
    ref = oracle_attn(inp, cfg, seq_lens=lens)
    got = run_attn(inp, cfg, torch.float32, seq_lens=lens)
    err = np.abs(got - ref).max()
    say(f"  attn clustered short rows Hq={Hq} Hkv={Hkv} B={len(lens)} sumL={int(lens.sum())}: max abs err {err:.3e}")
    assert np.isfinite(got).all() and err <= TOL_F32
    assert not got[lens == 0].any()


@pytest.mark.parametrize("layout", ["dense", "side_by_side"])
def test_7b_shape_lognormal_lengths(layout):
    cfg = wl.CONFIGS["c2"]
    L = np.minimum(wl.draw_lengths(cfg.lengths, 24, 2), 6000)
    check(cfg, L, seed=2, layout=layout)


@pytest.mark.parametrize("layout", ["dense", "side_by_side", "padded"])
def test_32b_shape_page32(layout):
    cfg = wl.CONFIGS["c5"]
    L = [64, 65, 95, 96, 97, 1000, 2047, 2048, 3000, 31, 1, 33]
    check(cfg, L, seed=3, layout=layout)


@pytest.mark.parametrize("Hq,Hkv,D,P", [(4, 4, 64, 64), (16, 1, 64, 16), (16, 1, 128, 64), (6, 2, 128, 32),
                                        (6, 3, 128, 16), (12, 6, 64, 16), (20, 5, 128, 32), (24, 12, 64, 16)])
@pytest.mark.parametrize("layout", ["dense", "side_by_side"])
def test_other_head_and_page_shapes(Hq, Hkv, D, P, layout):
    # KV head counts of every kind for the dealing of heads to a workgroup's four waves: fewer than
    # four (1, 2: the range is cut again; 3: a wave stays idle), more than four and not a multiple
    # of four (5, 6: the waves get unequal numbers of heads), multiples of four (4, 12)
    cfg = dataclasses.replace(wl.CONFIGS["c1"], name=f"h{Hq}_{Hkv}_d{D}_p{P}", num_q_heads=Hq,
                              num_kv_heads=Hkv, head_dim=D, page_size=P)
    check(cfg, [1, 7, 63, 64, 65, 200, 513, 700, 129], seed=4, layout=layout)


def test_custom_softmax_scale():
    cfg = wl.CONFIGS["c1"]
    check(cfg, [5, 100, 513, 40], seed=5, scale=0.31, bf16_too=False)


def test_zero_length_rows_give_zeros():
    cfg = wl.CONFIGS["c2"]
    L = np.array([0, 37, 0, 600, 0], np.int32)
    full = np.array([16, 37, 16, 600, 16], np.int32)     # pages exist, lengths say empty
    inp = wl.make_attn_inputs(cfg, 6, "cpu", lengths=full)
    ref = oracle_attn(inp, cfg, seq_lens=L)
    got = run_attn(inp, cfg, torch.float32, seq_lens=L)
    assert not got[[0, 2, 4]].any()
    assert np.abs(got - ref).max() <= TOL_F32
    got = run_attn(inp, cfg, torch.bfloat16, seq_lens=np.zeros(5, np.int32))
    assert not got.any()


def test_garbage_past_the_length_is_never_used():
    # NaN bit patterns in every slot past a row's length (rest of the last page and spare
    # pages) and -1 in unused page-table entries must not reach the output
    cfg = wl.CONFIGS["c2"]
    L = np.array([1, 17, 250, 513, 1030], np.int32)
    inp = wl.make_attn_inputs(cfg, 7, "cpu", lengths=L)
    ref = oracle_attn(inp, cfg)
    P = cfg.page_size
    k = inp["k_pages"].view(torch.int16)
    v = inp["v_pages"].view(torch.int16)
    used = np.zeros((inp["num_pages"], P), bool)
    for b, l in enumerate(L):
        for j in range(l):
            used[inp["page_table"][b, j // P], j % P] = True
    nan = np.int16(0x7FC0)
    for page in range(inp["num_pages"]):
        for t in range(P):
            if not used[page, t]:
                k[page, :, :, oracle.k_slot(t, P), :] = nan   # [N, Hkv, D/8, P (permuted), 8]
                v[page, :, t // 8, :, t % 8] = nan  # [N, Hkv, P/8, D, 8]
    got = run_attn(inp, cfg, torch.float32)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= TOL_F32


def test_seq_lens_beyond_the_table_are_clamped():
    cfg = wl.CONFIGS["c1"]
    L = np.array([40, 64], np.int32)
    inp = wl.make_attn_inputs(cfg, 8, "cpu", lengths=L)        # table has 4 pages per row
    ref = oracle_attn(inp, cfg, seq_lens=np.array([40, 64], np.int32))
    got = run_attn(inp, cfg, torch.float32, seq_lens=np.array([40, 100000], np.int32))
    assert np.abs(got - ref).max() <= TOL_F32


def test_repeat_calls_are_bit_identical():
    cfg = wl.CONFIGS["c2"]
    inp = wl.make_attn_inputs(cfg, 9, "cpu", lengths=np.array([700, 33, 1500], np.int32))
    a = run_attn(inp, cfg, torch.float32)
    b = run_attn(inp, cfg, torch.float32)
    assert np.array_equal(a, b)


def test_maximum_batch_of_short_and_empty_rows():
    # 8192 rows (the limit of the row prefix in LDS), most of a few tokens, many empty, some longer
    B = 8192
    rng = np.random.default_rng(B)
    lengths = rng.integers(0, 40, size=B).astype(np.int32)
    lengths[::97] = 300
    cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=B, num_q_heads=4, num_kv_heads=2, head_dim=64, page_size=16)
    inp = wl.make_attn_inputs(cfg, 31, "cpu", lengths=np.maximum(lengths, 1))
    inp["seq_lens"] = lengths
    got = run_attn(inp, cfg, out_dtype=torch.float32)
    want = oracle_attn(inp, cfg)
    assert np.abs(got - want).max() <= 1e-4
    assert not got[lengths == 0].any()


def test_unprepared_workspace_is_refused_by_the_kernel_and_found_by_the_check():
    # A workspace that roll_decode_attn_workspace_init never saw holds arbitrary arrival counters,
    # with which cut rows would merge too early or never.  The kernel refuses it: nothing is
    # written, and the diagnostic call says why.
    from paper_2510_11345_amd import binding as rb
    cfg = wl.CONFIGS["c2"]
    lens = np.asarray([5000, 3, 700, 0, 64], np.int32)
    inp = wl.make_attn_inputs(cfg, 5, "cuda", lengths=np.maximum(lens, 1))
    q, k, v = inp["q"], inp["k_pages"], inp["v_pages"]
    table = torch.from_numpy(inp["page_table"]).cuda()
    sl = torch.from_numpy(lens).cuda()
    out = torch.full(q.shape, 3.0, dtype=torch.float32, device="cuda")
    desc = rb.attn_desc(q, k, table, cfg.page_size, torch.float32)
    ws = torch.full((rb.roll_decode_attn_workspace_bytes(desc),), 0xA5, dtype=torch.uint8, device="cuda")
    rb.roll_decode_attn(q, k, v, table, sl, out, desc, ws)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
    with pytest.raises(rb.RollError) as e:
        rb.roll_decode_attn_workspace_check(ws)
    assert e.value.status == -6 and "never prepared" in str(e.value)
    # a tag without a clean header (here: a counter left over) is found too
    rb.roll_decode_attn_workspace_init(ws)
    rb.roll_decode_attn_workspace_check(ws)
    ws[4096:4100] = 1
    with pytest.raises(rb.RollError) as e:
        rb.roll_decode_attn_workspace_check(ws)
    assert "not zero" in str(e.value)
    # prepared: the same call now computes, and leaves the header clean
    rb.roll_decode_attn_workspace_init(ws)
    rb.roll_decode_attn(q, k, v, table, sl, out, desc, ws)
    torch.cuda.synchronize()
    rb.roll_decode_attn_workspace_check(ws)
    ref = oracle.decode_attn(wl.bits(q), wl.bits(k).reshape(-1), wl.bits(v).reshape(-1), inp["page_table"], lens,
                             cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size)
    assert np.abs(out.double().cpu().numpy() - ref).max() <= TOL_F32
