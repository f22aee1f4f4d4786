"""GPU checks of the allocator's device tables and the paged token writer (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from gpu_helpers import say

pytestmark = pytest.mark.gpu


def make_pool(num_pages, P, slots, max_pages):
    table = torch.zeros((slots, max_pages), dtype=torch.int32, device="cuda")
    lens = torch.full((slots,), 123, dtype=torch.int32, device="cuda")
    return rb.KvPool(num_pages, P, slots, max_pages, table, lens), table, lens


def test_commit_publishes_tables():
    pool, table, lens = make_pool(64, 16, 4, 8)
    rb.roll_kv_alloc(pool, 0, 40)
    rb.roll_kv_alloc(pool, 2, 1)
    rb.roll_kv_commit(pool)
    torch.cuda.synchronize()
    t, l = table.cpu().numpy(), lens.cpu().numpy()
    assert list(l) == [40, 0, 1, 0]
    assert list(t[0, :3]) == rb.roll_kv_slot_pages(pool, 0) and (t[0, 3:] == -1).all()
    assert t[2, 0] == rb.roll_kv_slot_pages(pool, 2)[0] and (t[1] == -1).all()
    # release + refill between two commits: the device sees only the final state
    rb.roll_kv_release(pool, 0)
    rb.roll_kv_alloc(pool, 1, 20)
    rb.roll_kv_alloc(pool, 0, 17)
    rb.roll_kv_commit(pool)
    rb.roll_kv_commit(pool)   # an empty commit is fine
    torch.cuda.synchronize()
    t, l = table.cpu().numpy(), lens.cpu().numpy()
    assert list(l) == [17, 20, 1, 0]
    for s in range(3):
        pages = rb.roll_kv_slot_pages(pool, s)
        assert list(t[s, :len(pages)]) == pages
    pool.close()


def test_many_deltas_span_several_staging_blocks():
    slots, max_pages, P = 64, 600, 16
    pool, table, lens = make_pool(slots * max_pages, P, slots, max_pages)
    rng = np.random.default_rng(0)
    L = rng.integers(1, max_pages * P, size=slots)
    for s in range(slots):
        rb.roll_kv_alloc(pool, s, int(L[s]))       # ~19k page deltas > one 8192-pair block
    rb.roll_kv_commit(pool)
    torch.cuda.synchronize()
    t = table.cpu().numpy()
    assert np.array_equal(lens.cpu().numpy(), L.astype(np.int32))
    for s in range(slots):
        pages = rb.roll_kv_slot_pages(pool, s)
        assert list(t[s, :len(pages)]) == pages
    pool.close()


def zero_pools(num_pages, Hkv, D, P, side_by_side):
    if side_by_side:
        return rb.new_kv_pools(num_pages, Hkv, D, P, fill=0)
    return (torch.zeros((num_pages, Hkv, D // 8, P, 8), dtype=torch.bfloat16, device="cuda"),
            torch.zeros((num_pages, Hkv, P // 8, D, 8), dtype=torch.bfloat16, device="cuda"))


@pytest.mark.parametrize("side_by_side", [False, True])
@pytest.mark.parametrize("Hkv,D,P", [(4, 128, 16), (8, 128, 32), (2, 64, 64)])
def test_append_tokens_writes_the_documented_layouts(Hkv, D, P, side_by_side):
    say(f"  append case Hkv={Hkv} D={D} P={P} side_by_side={side_by_side}")
    slots, max_pages = 3, 6
    num_pages = slots * max_pages
    pool, table, lens = make_pool(num_pages, P, slots, max_pages)
    L = [P * 2 + 3, 1, P * 5]
    for s, l in enumerate(L):
        rb.roll_kv_alloc(pool, s, l)
    rb.roll_kv_commit(pool)
    slot_ids = np.concatenate([np.full(l, s) for s, l in enumerate(L)]).astype(np.int32)
    pos = np.concatenate([np.arange(l) for l in L]).astype(np.int32)
    n = len(pos)
    k_new = wl.randn_bf16((n, Hkv, D), 1, 50)
    v_new = wl.randn_bf16((n, Hkv, D), 1, 51)
    k_pages, v_pages = zero_pools(num_pages, Hkv, D, P, side_by_side)
    rb.roll_kv_append_tokens(k_new.cuda(), v_new.cuda(), torch.from_numpy(slot_ids).cuda(),
                             torch.from_numpy(pos).cuda(), None, k_pages, v_pages, table, P)
    torch.cuda.synchronize()
    # expected pools: the oracle's own writer, token by token
    ek = np.zeros(num_pages * Hkv * D * P, np.uint16)
    ev = np.zeros_like(ek)
    kb, vb = wl.bits(k_new), wl.bits(v_new)
    for i in range(n):
        page = rb.roll_kv_slot_pages(pool, int(slot_ids[i]))[pos[i] // P]
        oracle.kv_store(ek, ev, page, int(pos[i] % P), kb[i], vb[i], Hkv, D, P)
    assert np.array_equal(wl.bits(k_pages).reshape(-1), ek)
    assert np.array_equal(wl.bits(v_pages).reshape(-1), ev)
    pool.close()


@pytest.mark.parametrize("side_by_side", [False, True])
@pytest.mark.parametrize("Hkv,D,P", [(4, 128, 16), (8, 128, 32)])
def test_commit_append_publishes_and_writes_in_one_launch(Hkv, D, P, side_by_side):
    say(f"  commit_append case Hkv={Hkv} D={D} P={P} side_by_side={side_by_side}")
    slots, max_pages = 6, 5
    num_pages = slots * max_pages
    pool, table, lens = make_pool(num_pages, P, slots, max_pages)
    k_pages, v_pages = zero_pools(num_pages, Hkv, D, P, side_by_side)
    ek = np.zeros(num_pages * Hkv * D * P, np.uint16)
    ev = np.zeros_like(ek)
    L = [P - 1, 0, 2 * P, 5, 0, 3 * P + 7]           # slots 1 and 4 stay empty
    for s, l in enumerate(L):
        if l:
            rb.roll_kv_alloc(pool, s, l)
    live = np.array([s for s, l in enumerate(L) if l], np.int32)
    for step in range(3):                            # crosses a page boundary for slots 0 and 2
        rb.roll_kv_alloc_batch(pool, live, np.ones(len(live), np.int32))
        k_new = wl.randn_bf16((slots, Hkv, D), 2, 60 + step)
        v_new = wl.randn_bf16((slots, Hkv, D), 2, 70 + step)
        rb.roll_kv_commit_append(pool, k_new.cuda(), v_new.cuda(), k_pages, v_pages)
        kb, vb = wl.bits(k_new), wl.bits(v_new)
        for s in live:
            pos = rb.roll_kv_seq_len(pool, int(s)) - 1
            page = rb.roll_kv_slot_pages(pool, int(s))[pos // P]
            oracle.kv_store(ek, ev, page, pos % P, kb[s], vb[s], Hkv, D, P)
    torch.cuda.synchronize()
    assert np.array_equal(wl.bits(k_pages).reshape(-1), ek)
    assert np.array_equal(wl.bits(v_pages).reshape(-1), ev)
    t, l = table.cpu().numpy(), lens.cpu().numpy()
    assert list(l) == [x + 3 if x else 0 for x in L]
    for s in range(slots):
        pages = rb.roll_kv_slot_pages(pool, s)
        assert list(t[s, :len(pages)]) == pages
    pool.close()
