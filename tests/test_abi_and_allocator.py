"""CPU-only checks: the C-ABI library loads and exports what the header declares, argument
validation rejects bad input before anything touches a GPU, and the host allocator logic
(host-only pool) keeps its invariants."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_11345_amd import binding as rb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "roll_decode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(roll_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = rb.lib()
    syms = declared_symbols()
    assert len(syms) >= 18
    for s in syms:
        assert hasattr(L, s), f"{s} declared in roll_decode.h but not exported"
    assert sorted(rb.EXPORTS) == syms  # the binding covers the same set
    assert rb.roll_version()


def host_pool(num_pages=64, P=16, slots=4, max_pages=8):
    return rb.KvPool(num_pages, P, slots, max_pages)


def owned(pool, slots):
    return [rb.roll_kv_slot_pages(pool, s) for s in range(slots)]


def check_conservation(pool, slots, num_pages):
    pages = [p for lst in owned(pool, slots) for p in lst]
    assert len(pages) == len(set(pages)), "a page is owned twice"
    assert all(0 <= p < num_pages for p in pages)
    assert rb.roll_kv_free_pages(pool) + len(pages) == num_pages


def test_alloc_grows_by_pages_and_conserves():
    pool = host_pool()
    rb.roll_kv_alloc(pool, 0, 1)
    assert rb.roll_kv_seq_len(pool, 0) == 1 and rb.roll_kv_slot_pages(pool, 0) == [0]
    rb.roll_kv_alloc(pool, 0, 15)          # fills the page, no new one
    assert rb.roll_kv_slot_pages(pool, 0) == [0]
    rb.roll_kv_alloc(pool, 0, 1)           # crosses the boundary
    assert rb.roll_kv_slot_pages(pool, 0) == [0, 1] and rb.roll_kv_seq_len(pool, 0) == 17
    rb.roll_kv_alloc(pool, 2, 40)
    assert rb.roll_kv_slot_pages(pool, 2) == [2, 3, 4]
    check_conservation(pool, 4, 64)


def test_release_returns_everything_and_refill_reuses():
    pool = host_pool()
    rb.roll_kv_alloc(pool, 1, 100)
    before = rb.roll_kv_slot_pages(pool, 1)
    assert rb.roll_kv_free_pages(pool) == 64 - 7
    rb.roll_kv_release(pool, 1)            # finish or ABORT
    assert rb.roll_kv_free_pages(pool) == 64 and rb.roll_kv_seq_len(pool, 1) == 0
    rb.roll_kv_alloc(pool, 3, 100)         # the refill gets the same pages back
    assert rb.roll_kv_slot_pages(pool, 3) == before
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_release(pool, 1)        # double release
    assert e.value.status == -3


def test_errors_leave_state_unchanged():
    pool = host_pool(num_pages=10, max_pages=8)
    rb.roll_kv_alloc(pool, 0, 5 * 16)
    snap = (owned(pool, 4), rb.roll_kv_free_pages(pool))
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_alloc(pool, 1, 6 * 16)  # needs 6, 5 free
    assert e.value.status == -2
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_alloc(pool, 0, 4 * 16)  # would need 9 > max_pages_per_seq
    assert e.value.status == -5
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_alloc(pool, 4, 1)
    assert e.value.status == -4
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_alloc(pool, 0, 0)
    assert e.value.status == -1
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_commit(pool)            # host-only pool
    assert e.value.status == -1
    assert (owned(pool, 4), rb.roll_kv_free_pages(pool)) == snap
    assert "host-only" in rb.lib().roll_last_error().decode()


def test_random_alloc_release_keeps_invariants():
    rng = np.random.default_rng(0)
    slots, num_pages = 16, 300
    pool = host_pool(num_pages=num_pages, slots=slots, max_pages=40)
    lens = [0] * slots
    for _ in range(3000):
        s = int(rng.integers(slots))
        if lens[s] and rng.random() < 0.15:
            rb.roll_kv_release(pool, s); lens[s] = 0
        else:
            n = int(rng.integers(1, 50))
            try:
                rb.roll_kv_alloc(pool, s, n); lens[s] += n
            except rb.RollError as e:
                assert e.status in (-2, -5)
        assert rb.roll_kv_seq_len(pool, s) == lens[s]
    check_conservation(pool, slots, num_pages)
    for s in range(slots):
        assert len(rb.roll_kv_slot_pages(pool, s)) == (lens[s] + 15) // 16


def test_bad_pool_config_is_rejected():
    for args in [(0, 16, 4, 8), (64, 8, 4, 8), (64, 16, 0, 8), (64, 16, 4, 0)]:
        with pytest.raises(rb.RollError):
            rb.KvPool(*args)


def test_attention_and_sampling_reject_bad_descriptors_on_the_host():
    L = rb.lib()
    good = rb.AttnDesc(4, 8, 2, 64, 16, 8, 32, rb.ROLL_BF16, 0.0, 0)
    assert L.roll_decode_attn_workspace_bytes(C.byref(good)) > 0
    for field, val in [("head_dim", 96), ("num_kv_heads", 3), ("page_size", 8), ("batch", 8193),
                       ("batch", 0), ("out_dtype", 7), ("num_q_heads", 64)]:
        d = rb.AttnDesc(4, 8, 2, 64, 16, 8, 32, rb.ROLL_BF16, 0.0, 0)
        if field == "num_q_heads":
            d.num_kv_heads = 2  # group of 32 > 16
        setattr(d, field, val)
        assert L.roll_decode_attn_workspace_bytes(C.byref(d)) == 0
        assert L.roll_decode_attn(16, 16, 16, 16, 16, 16, C.byref(d), 256, 1 << 30, None) == -1
    # NULL / misaligned pointers and a short workspace never reach a kernel launch
    assert L.roll_decode_attn(None, 16, 16, 16, 16, 16, C.byref(good), 256, 1 << 30, None) == -1
    assert L.roll_decode_attn(8, 16, 16, 16, 16, 16, C.byref(good), 256, 1 << 30, None) == -1
    assert L.roll_decode_attn(16, 16, 16, 16, 16, 16, C.byref(good), 256, 8, None) == -6
    assert L.roll_decode_attn(16, 16, 16, 16, 16, 16, C.byref(good), None, 1 << 30, None) == -6
    sd = rb.SampleDesc(2, 4096, 4096, rb.ROLL_F32, 0, None, None)
    assert L.roll_sample_logprob_workspace_bytes(C.byref(sd)) > 0
    for T, p in [(0.0, 1.0), (-1.0, 1.0), (1.0, 0.0), (1.0, 1.5), (float("nan"), 1.0), (1.0, float("nan"))]:
        assert L.roll_sample_logprob(16, T, p, 0, 0, 16, 16, C.byref(sd), None, 0, None) == -1
    bad = rb.SampleDesc(2, 4096, 4095, rb.ROLL_F32, 0, None, None)
    assert L.roll_sample_logprob(16, 1.0, 1.0, 0, 0, 16, 16, C.byref(bad), None, 0, None) == -1
    bad = rb.SampleDesc(2, 4097, 4097, rb.ROLL_BF16, 0, None, None)  # rows would not be 16-byte aligned
    assert L.roll_sample_logprob(16, 1.0, 1.0, 0, 0, 16, 16, C.byref(bad), None, 0, None) == -1
    assert L.roll_sample_logprob(None, 1.0, 1.0, 0, 0, 16, 16, C.byref(sd), None, 0, None) == -1


def test_alloc_batch_is_all_or_nothing():
    pool = host_pool(num_pages=10, slots=4, max_pages=8)
    rb.roll_kv_alloc_batch(pool, np.array([0, 2], np.int32), np.array([20, 1], np.int32))
    assert rb.roll_kv_seq_len(pool, 0) == 20 and rb.roll_kv_seq_len(pool, 2) == 1
    snap = (owned(pool, 4), rb.roll_kv_free_pages(pool))
    for slots, n, status in [([0, 0], [1, 1], -1),          # repeated slot
                             ([1, 3], [5 * 16, 4 * 16], -2),  # 9 pages needed, 7 free
                             ([1, 0], [1, 8 * 16], -5),       # slot 0 would exceed max_pages
                             ([1, 7], [1, 1], -4),
                             ([1, 3], [1, 0], -1)]:
        with pytest.raises(rb.RollError) as e:
            rb.roll_kv_alloc_batch(pool, np.array(slots, np.int32), np.array(n, np.int32))
        assert e.value.status == status
        assert (owned(pool, 4), rb.roll_kv_free_pages(pool)) == snap
    rb.roll_kv_alloc_batch(pool, np.array([], np.int32), np.array([], np.int32))
    check_conservation(pool, 4, 10)


@pytest.mark.parametrize("R", [2, 4, 8])
def test_runs_of_pages_are_aligned_adjacent_and_conserved(R):
    # pages handed out in aligned runs of R: logical pages R j .. R j + R - 1 of a slot are the
    # physical pages R k .. R k + R - 1 of one run, however the pool has been churned
    rng = np.random.default_rng(R)
    slots, num_pages, max_pages = 12, 40 * R + 3, 24     # the 3 pages past the last whole run are never used
    pool = rb.KvPool(num_pages, 16, slots, max_pages, run_pages=R)
    usable = num_pages // R * R
    assert rb.roll_kv_free_pages(pool) == usable
    lens = [0] * slots
    for it in range(4000):
        s = int(rng.integers(slots))
        if lens[s] and rng.random() < 0.2:
            rb.roll_kv_release(pool, s); lens[s] = 0
        else:
            n = int(rng.integers(1, 60))
            free_before, pages_before = rb.roll_kv_free_pages(pool), rb.roll_kv_slot_pages(pool, s)
            try:
                rb.roll_kv_alloc(pool, s, n); lens[s] += n
            except rb.RollError as e:
                assert e.status in (-2, -5)
                assert rb.roll_kv_free_pages(pool) == free_before and rb.roll_kv_slot_pages(pool, s) == pages_before
        if it % 50 == 0 or it == 3999:
            held, seen = 0, set()
            for t in range(slots):
                pages = rb.roll_kv_slot_pages(pool, t)
                assert len(pages) == (lens[t] + 15) // 16
                for j, p in enumerate(pages):
                    assert 0 <= p < usable and p not in seen
                    seen.add(p)
                    if j % R == 0:
                        assert p % R == 0                    # a run starts at a multiple of R
                    else:
                        assert p == pages[j - 1] + 1          # and continues page by page
                held += (len(pages) + R - 1) // R * R
            assert held + rb.roll_kv_free_pages(pool) == usable
    # release + re-alloc hands the same pages back in the same order
    s = max(range(slots), key=lambda t: lens[t])
    before = rb.roll_kv_slot_pages(pool, s)
    rb.roll_kv_release(pool, s)
    rb.roll_kv_alloc(pool, s, lens[s])
    assert rb.roll_kv_slot_pages(pool, s) == before


def test_runs_batch_alloc_is_all_or_nothing_and_bad_run_lengths_are_rejected():
    pool = rb.KvPool(8, 16, 4, 8, run_pages=2)           # 4 runs of 2 pages
    rb.roll_kv_alloc_batch(pool, np.array([0, 1, 2], np.int32), np.array([1, 17, 33], np.int32))   # 1 + 1 + 2 runs
    assert rb.roll_kv_free_pages(pool) == 0
    snap = [rb.roll_kv_slot_pages(pool, s) for s in range(4)]
    with pytest.raises(rb.RollError) as e:
        rb.roll_kv_alloc_batch(pool, np.array([0, 3], np.int32), np.array([15, 1], np.int32))  # slot 0 fits its run, slot 3 needs one
    assert e.value.status == -2
    assert [rb.roll_kv_slot_pages(pool, s) for s in range(4)] == snap and rb.roll_kv_seq_len(pool, 0) == 1
    rb.roll_kv_alloc(pool, 0, 31)                        # the second page of slot 0's run: no new run needed
    assert rb.roll_kv_slot_pages(pool, 0) == [snap[0][0], snap[0][0] + 1]
    for R in (3, 5, 16, -1):
        with pytest.raises(rb.RollError):
            rb.KvPool(64, 16, 4, 8, run_pages=R)


def test_page_stride_must_be_whole_head_blocks_that_hold_all_heads():
    L = rb.lib()
    base = dict(batch=4, Hq=8, Hkv=2, D=64, P=16)
    block = base["P"] * base["D"]

    def desc(stride):
        return rb.AttnDesc(base["batch"], base["Hq"], base["Hkv"], base["D"], base["P"], 8, 32, rb.ROLL_BF16, 0.0,
                           stride)
    for ok in (0, 2 * block, 4 * block, 7 * block):      # dense; exactly the heads; K and V side by side; padded
        assert L.roll_decode_attn_workspace_bytes(C.byref(desc(ok))) > 0
    for bad in (block, 2 * block + 8, -2 * block, 2 * block - 1):
        assert L.roll_decode_attn_workspace_bytes(C.byref(desc(bad))) == 0
        assert L.roll_decode_attn(16, 16, 16, 16, 16, 16, C.byref(desc(bad)), 256, 1 << 30, None) == -1


def test_step_count_of_a_batch_must_fit_32_bits():
    # the kernel keeps the rows' step counts as 32-bit prefix sums: a desc that could exceed them is
    # refused on the host
    L = rb.lib()
    ok = rb.AttnDesc(8192, 8, 2, 64, 64, (1 << 24) // 64 // 4, 32, rb.ROLL_BF16, 0.0, 0)
    assert L.roll_decode_attn_workspace_bytes(C.byref(ok)) > 0
    big = rb.AttnDesc(8192, 8, 2, 64, 64, (1 << 24) // 64, 32, rb.ROLL_BF16, 0.0, 0)
    assert L.roll_decode_attn_workspace_bytes(C.byref(big)) == 0
    assert L.roll_decode_attn(16, 16, 16, 16, 16, 16, C.byref(big), 256, 1 << 30, None) == -5


def test_static_entry_point_and_workspace_check_reject_bad_arguments_on_the_host():
    L = rb.lib()
    good = rb.AttnDesc(4, 8, 2, 64, 16, 8, 32, rb.ROLL_BF16, 0.0, 0)
    bad = rb.AttnDesc(4, 8, 2, 96, 16, 8, 32, rb.ROLL_BF16, 0.0, 0)
    assert L.roll_decode_attn_static(16, 16, 16, 16, 16, 16, C.byref(bad), None) == -1
    assert L.roll_decode_attn_static(None, 16, 16, 16, 16, 16, C.byref(good), None) == -1
    assert L.roll_decode_attn_static(8, 16, 16, 16, 16, 16, C.byref(good), None) == -1
    assert L.roll_decode_attn_workspace_check(None, 1 << 30, None) == -6
    assert L.roll_decode_attn_workspace_check(128, 1 << 30, None) == -6
    assert L.roll_decode_attn_workspace_check(256, 8, None) == -6
    assert L.roll_decode_attn_workspace_init(256, 8, None) == -6
    assert L.roll_prof_attn_events(16, None) == -1
    assert L.roll_prof_attn_events(None, None) == 0
    assert L.roll_prof_prefill_events(None, 16) == -1
    assert L.roll_prof_prefill_events(None, None) == 0
    # the product library has no timestamps in its kernels and says so
    assert L.roll_prof_attn_timeline(None, 0) == -1
    assert L.roll_prof_prefill_timeline(None, 0) == -1
    assert L.roll_prof_prefill_units(9) == -1 and L.roll_prof_prefill_units(-1) == -1
    assert L.roll_prof_prefill_units(8) == 0 and L.roll_prof_prefill_units(0) == 0
    # the decode step checks its pointers and workspace before it touches the allocator's pending changes
    pool = host_pool()
    rb.roll_kv_alloc(pool, 0, 3)
    assert L.roll_decode_step_attn(pool._h, 16, 16, None, 16, 16, 16, C.byref(good), 256, 1 << 30, None) == -1
    assert L.roll_decode_step_attn(pool._h, 16, 16, 16, 16, 16, 16, C.byref(good), 256, 8, None) == -6
    assert rb.roll_kv_seq_len(pool, 0) == 3
