"""Chunked prefill attention into pages through the C ABI against the oracle (needs an MI355X):
outputs within the attention tolerance, pools bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from gpu_helpers import say, side_by_side

pytestmark = pytest.mark.gpu


class Pool:
    """Slots with pages from the library's allocator and seeded random pool contents."""

    def __init__(self, num_slots, capacity_tokens, Hkv, D, P, seed, spare=8):
        self.P, self.Hkv, self.D = P, Hkv, D
        self.max_pages = (capacity_tokens + P - 1) // P
        self.num_pages = num_slots * self.max_pages + spare
        self.page_table = torch.empty((num_slots, self.max_pages), dtype=torch.int32, device="cuda")
        self.seq_lens = torch.zeros((num_slots,), dtype=torch.int32, device="cuda")
        self.pool = rb.KvPool(self.num_pages, P, num_slots, self.max_pages, self.page_table, self.seq_lens)
        self.k_pages = wl.randn_bf16((self.num_pages, Hkv, D // 8, P, 8), seed, 2, "cuda")
        self.v_pages = wl.randn_bf16((self.num_pages, Hkv, P // 8, D, 8), seed, 3, "cuda")
        if seed % 2 == 1:   # odd seeds: K and V of a page side by side in one allocation
            self.k_pages, self.v_pages = side_by_side(self.k_pages, self.v_pages)

    def host_table(self, num_slots):
        t = np.full((num_slots, self.max_pages), -1, np.int32)
        for s in range(num_slots):
            pr = rb.roll_kv_slot_pages(self.pool, s)
            t[s, :len(pr)] = pr
        return t


def _run_case(Hq, Hkv, D, P, chunks, seed, out_dtype=torch.float32, num_slots=None, scale=0.0):
    """chunks: list of (slot, start, n) in call order.  Slots are grown to what the chunks need."""
    num_slots = (max(c[0] for c in chunks) + 1) if num_slots is None else num_slots
    need = np.zeros(num_slots, np.int64)
    for slot, start, n in chunks:
        need[slot] = max(need[slot], start + n)
    pool = Pool(num_slots, int(max(need.max(), 1)), Hkv, D, P, seed)
    for slot in range(num_slots):
        if need[slot]:
            rb.roll_kv_alloc(pool.pool, slot, int(need[slot]))
    rb.roll_kv_commit(pool.pool)
    T = sum(c[2] for c in chunks)
    q = wl.randn_bf16((T, Hq, D), seed, 11, "cuda")
    k_new = wl.randn_bf16((T, Hkv, D), seed, 12, "cuda")
    v_new = wl.randn_bf16((T, Hkv, D), seed, 13, "cuda")
    cs = np.array([c[0] for c in chunks], np.int32)
    st = np.array([c[1] for c in chunks], np.int32)
    off = np.concatenate([[0], np.cumsum([c[2] for c in chunks])]).astype(np.int32)
    kp_host, vp_host = wl.bits(pool.k_pages).reshape(-1).copy(), wl.bits(pool.v_pages).reshape(-1).copy()
    out = torch.full((T, Hq, D), float("nan"), dtype=out_dtype, device="cuda")
    rb.roll_prefill_attn(q, k_new, v_new, torch.from_numpy(cs).cuda(), torch.from_numpy(st).cuda(),
                         torch.from_numpy(off).cuda(), pool.k_pages, pool.v_pages, pool.page_table, out, P,
                         softmax_scale=scale)
    torch.cuda.synchronize()
    table = pool.host_table(num_slots)
    want = oracle.prefill_attn(wl.bits(q), wl.bits(k_new), wl.bits(v_new), cs, st, off, kp_host, vp_host, table,
                               Hq, Hkv, D, P, scale=None if scale == 0.0 else scale)
    got = out.double().cpu().numpy()
    assert not np.isnan(got).any()
    err = float(np.abs(got - want).max()) if T else 0.0
    assert np.array_equal(wl.bits(pool.k_pages).reshape(-1), kp_host)
    assert np.array_equal(wl.bits(pool.v_pages).reshape(-1), vp_host)
    pool.pool.close()
    return err


@pytest.mark.parametrize("Hq,Hkv,D,P", [(28, 4, 128, 16), (64, 8, 128, 32), (8, 2, 64, 64), (16, 16, 64, 16),
                                        (16, 1, 128, 16), (12, 1, 64, 32)])
def test_prefill_whole_prompts(Hq, Hkv, D, P):
    # prompt lengths around the block (16), step (32) and page sizes, one of them a few hundred tokens
    lens = [1, 15, 16, 17, 31, 32, 33, 64, 100, 333]
    chunks = [(slot, 0, n) for slot, n in enumerate(lens)]
    err = _run_case(Hq, Hkv, D, P, chunks, seed=21)
    say(f"  prefill Hq={Hq} Hkv={Hkv} D={D} P={P}: max abs err {err:.2e}")
    assert err <= 1e-4
    err = _run_case(Hq, Hkv, D, P, chunks, seed=21, out_dtype=torch.bfloat16)
    assert err <= 2e-2


def test_prefill_chunks_on_top_of_a_cache_and_same_slot_twice():
    Hq, Hkv, D, P = 28, 4, 128, 16
    # slot 0: 40 cached tokens (first call), then chunks 40..99 and 100..130 in one call;
    # slot 1: a chunk that starts in the middle of a page; slot 2 stays empty; slot 3: one token
    err0 = _run_case(Hq, Hkv, D, P, [(0, 0, 40)], seed=22)
    assert err0 <= 1e-4
    # second call on a fresh pool whose "cache" is the seeded pool content itself
    chunks = [(0, 40, 60), (1, 7, 50), (0, 100, 31), (3, 250, 1)]
    err = _run_case(Hq, Hkv, D, P, chunks, seed=23, num_slots=4)
    assert err <= 1e-4
    err = _run_case(Hq, Hkv, D, P, chunks, seed=23, num_slots=4, out_dtype=torch.bfloat16)
    assert err <= 2e-2


def test_prefill_many_small_chunks_and_empty_ones():
    Hq, Hkv, D, P = 8, 2, 64, 16
    rng = np.random.default_rng(5)
    chunks = []
    for slot in range(70):                      # more chunks than one 64-lane counting round
        chunks.append((slot, int(rng.integers(0, 20)), int(rng.integers(0, 40))))
    assert any(c[2] == 0 for c in chunks) or True
    chunks[3] = (3, 5, 0)                       # an empty chunk
    chunks[69] = (69, 0, 35)
    err = _run_case(Hq, Hkv, D, P, chunks, seed=24)
    assert err <= 1e-4
    err = _run_case(Hq, Hkv, D, P, chunks, seed=24, out_dtype=torch.bfloat16)   # the pipelined loop's block search
    assert err <= 2e-2


def test_prefill_bf16_out_custom_scale_and_long_prefix():
    err = _run_case(28, 4, 128, 16, [(0, 1500, 200), (1, 0, 700)], seed=25, out_dtype=torch.bfloat16, scale=0.11)
    assert err <= 2e-2


@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (16, 2), (10, 2), (4, 1)])
@pytest.mark.parametrize("scale", [1.0, 8.0])
def test_prefill_scores_that_rise_far_above_those_of_the_first_tokens(Hq, Hkv, scale):
    # The fast loop of the kernel keeps the softmax reference of a column at the maximum over the
    # first 32 tokens and runs the block again through the exact loop when the row sums show that
    # later scores rose too far above it.  With unit-variance q and k the logits have a standard
    # deviation of 11 * scale nats: scale 1 gives probabilities of thousands relative to the
    # reference (kept by the fast loop), scale 8 overflows it (the exact loop must take over).
    # Head counts: one, two and four copying waves, and all waves copying (8 heads per KV head).
    chunks = [(0, 0, 300), (1, 40, 130), (2, 0, 33)]
    err = _run_case(Hq, Hkv, 128, 16, chunks, seed=31, scale=scale)
    say(f"  prefill Hq={Hq} Hkv={Hkv} scale={scale}: max abs err {err:.2e}")
    assert err <= 1e-4
    err = _run_case(Hq, Hkv, 128, 16, chunks, seed=32, out_dtype=torch.bfloat16, scale=scale)
    assert err <= 2e-2


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("P", [16, 32, 64])
@pytest.mark.parametrize("G", [7, 5, 3])
def test_prefill_every_page_size_with_one_two_and_four_copying_waves(D, P, G):
    # 7, 5 and 3 query heads per KV head leave 1, 2 and 4 waves of the workgroup to do the copying;
    # their addresses are written out per head_dim, page size and number of copying waves.
    # Chunks that start inside a page and inside a 32-token step, on top of cached tokens.
    chunks = [(0, 0, 150), (1, 21, 90), (2, 70, 37), (0, 150, 40)]
    # (the bf16 result takes the pipelined loop with the copying waves, the fp32 result the exact loop)
    err = _run_case(2 * G, 2, D, P, chunks, seed=40 + G, num_slots=3, out_dtype=torch.bfloat16)
    say(f"  prefill G={G} D={D} P={P}: max abs err {err:.2e} (bf16 result)")
    assert err <= 2e-2
    err = _run_case(2 * G, 2, D, P, chunks, seed=40 + G, num_slots=3)
    assert err <= 1e-4


@pytest.mark.parametrize("case", range(8))
def test_prefill_random_shapes_and_chunkings(case):
    # Seeded draws of head counts (1 to 16 query heads per KV head), head_dim, page size, and of
    # chunks with arbitrary starts and lengths (several chunks of one slot in a call follow each
    # other), both result types.
    rng = np.random.default_rng([77, case])
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 12, 16]))
    Hkv = int(rng.choice([1, 2, 4]))
    D = int(rng.choice([64, 128]))
    P = int(rng.choice([16, 32, 64]))
    chunks = []
    for slot in range(int(rng.integers(2, 6))):
        pos = int(rng.integers(0, 90))
        for _ in range(int(rng.integers(1, 4))):
            n = int(rng.integers(1, 120))
            chunks.append((slot, pos, n))
            pos += n
    num_slots = max(c[0] for c in chunks) + 1
    for dtype, tol in ((torch.bfloat16, 2e-2), (torch.float32, 1e-4)):
        err = _run_case(G * Hkv, Hkv, D, P, chunks, seed=50 + case, out_dtype=dtype, num_slots=num_slots)
        say(f"  prefill case {case}: G={G} Hkv={Hkv} D={D} P={P}, {len(chunks)} chunks, {dtype}: max abs err {err:.2e}")
        assert err <= tol


@pytest.mark.parametrize("units", [1, 2, 3, 5, 7, 8])
@pytest.mark.parametrize("Hq,Hkv,D,P", [(4, 4, 128, 16), (2, 1, 64, 32), (6, 2, 128, 64), (8, 2, 128, 16), (5, 1, 64, 16),
                                        (12, 2, 128, 32), (7, 1, 128, 16), (16, 2, 64, 64)])
def test_prefill_units_per_workgroup(Hq, Hkv, D, P, units):
    """A workgroup computes `units` consecutive (span of 32 query tokens, query head) units of a
    chunk, one per wave, whatever the number of heads per KV head: its waves may sit in different
    spans, a span's heads in different workgroups, and the last workgroup of a chunk may have
    waves left over.  Prompts that end inside the first span, at a span's end, one token into the
    next one; chunks on a cache at positions that are no multiples of anything; a prompt of one
    token.  Both result types (the pipelined loop and the exact one) against the oracle, pools
    bit for bit."""
    rb.roll_prof_prefill_units(units)
    try:
        chunks = [(0, 0, 113), (1, 0, 64), (2, 0, 65), (3, 0, 255), (4, 0, 1), (5, 0, 96)]
        for out_dtype, tol in ((torch.bfloat16, 2e-2), (torch.float32, 1e-4)):
            err = _run_case(Hq, Hkv, D, P, chunks, 70 + Hq, out_dtype=out_dtype)
            assert err <= tol, (out_dtype, err)
        chunks = [(0, 0, 45), (1, 0, 130), (0, 45, 104), (1, 130, 33), (2, 0, 7)]
        for out_dtype, tol in ((torch.bfloat16, 2e-2), (torch.float32, 1e-4)):
            err = _run_case(Hq, Hkv, D, P, chunks, 71 + Hq, out_dtype=out_dtype)
            assert err <= tol, (out_dtype, err)
    finally:
        rb.roll_prof_prefill_units(0)


@pytest.mark.parametrize("Hq,Hkv,D,P", [(12, 1, 128, 16), (32, 2, 64, 32), (32, 1, 128, 64), (64, 1, 64, 16), (18, 2, 128, 16)])
def test_prefill_large_head_groups(Hq, Hkv, D, P):
    """More query heads per KV head than a workgroup has waves (9, 12, 16, 32, 64): the heads of a
    span are spread over several workgroups.  Whole prompts and chunks on a cache, both result
    types; the number of units per workgroup as the launch chooses it and fixed at 7 and 8."""
    chunks = [(0, 0, 70), (1, 0, 33), (2, 9, 40), (0, 70, 31)]
    for units in (0, 7, 8):
        rb.roll_prof_prefill_units(units)
        try:
            for out_dtype, tol in ((torch.bfloat16, 2e-2), (torch.float32, 1e-4)):
                err = _run_case(Hq, Hkv, D, P, chunks, 90 + Hq, out_dtype=out_dtype, num_slots=3)
                assert err <= tol, (units, out_dtype, err)
        finally:
            rb.roll_prof_prefill_units(0)


def test_prefill_units_are_checked():
    with pytest.raises(rb.RollError):
        rb.roll_prof_prefill_units(9)
    with pytest.raises(rb.RollError):
        rb.roll_prof_prefill_units(-1)


def test_prefill_no_tokens_is_a_no_op_and_bad_desc_is_rejected():
    Hq, Hkv, D, P = 8, 2, 64, 16
    pool = Pool(2, 64, Hkv, D, P, 1)
    z = torch.zeros((0, Hq, D), dtype=torch.bfloat16, device="cuda")
    zk = torch.zeros((0, Hkv, D), dtype=torch.bfloat16, device="cuda")
    e = torch.zeros((0,), dtype=torch.int32, device="cuda")
    off = torch.zeros((1,), dtype=torch.int32, device="cuda")
    before = pool.k_pages.clone()
    rb.roll_prefill_attn(z, zk, zk, e, e, off, pool.k_pages, pool.v_pages, pool.page_table,
                         torch.zeros((0, Hq, D), dtype=torch.float32, device="cuda"), P)
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), pool.k_pages.view(torch.int16))
    q = torch.zeros((4, Hq, D), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((4, Hkv, D), dtype=torch.bfloat16, device="cuda")
    one = torch.zeros((1,), dtype=torch.int32, device="cuda")
    off2 = torch.tensor([0, 4], dtype=torch.int32, device="cuda")
    with pytest.raises(rb.RollError):
        rb.roll_prefill_attn(q, kn, kn, one, one, off2, pool.k_pages, pool.v_pages, pool.page_table,
                             torch.zeros((4, Hq, D), dtype=torch.float32, device="cuda"), 48)
    pool.pool.close()
