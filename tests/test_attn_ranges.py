"""Host arithmetic of the attention kernel's work dealing (roll_decode_attn_ranges): no GPU needed.

The kernel and this call share the arithmetic, so what is pinned here is what the kernel does:
ranges of equal cost on a line where a row with tokens takes 2 units (starting it) and each of
its 32-token steps 2 more (ROLL Flash, arXiv 2510.11345, Section 1: long-tailed lengths)."""
import numpy as np
import pytest

from paper_2510_11345_amd import binding as rb

STEP, STEP_COST, ROW_COST = 32, 2, 2


def desc(B, Hq=28, Hkv=4, D=128, P=16, max_pages=2048):
    return rb.AttnDesc(B, Hq, Hkv, D, P, max_pages, 1 << 20, rb.ROLL_BF16, 0.0, 0)


def by_definition(lens, num_ranges):
    """The cost line unit by unit: which range owns which step."""
    units = []        # step id of every unit, -1 for a unit that starts a row
    step = 0
    for L in lens:
        n = (int(L) + STEP - 1) // STEP
        if n == 0:
            continue
        units += [-1] * ROW_COST
        for _ in range(n):
            units += [step] * STEP_COST
            step += 1
    T = len(units)
    first_unit = {}
    for x, s in enumerate(units):
        if s >= 0 and s not in first_unit:
            first_unit[s] = x
    starts = [c * T // num_ranges for c in range(num_ranges)]
    first = []
    for c in range(num_ranges):
        owned = [s for s, x in first_unit.items() if x >= starts[c]]
        first.append(min(owned) if owned else step)
    return np.array(first + [step], dtype=np.int64)


@pytest.mark.parametrize("seed", range(12))
def test_small_batches_against_the_definition_unit_by_unit(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 30))
    kind = seed % 4
    if kind == 0:
        lens = rng.integers(0, 300, B)
    elif kind == 1:
        lens = rng.integers(0, 3, B) * rng.integers(0, 70, B)
    elif kind == 2:
        lens = np.clip(np.rint(np.exp(rng.normal(5.5, 1.5, B))), 0, 20000).astype(np.int64)
    else:
        lens = rng.integers(1, 34, B)
    for groups in (1, 2, 3, 7, 64, 256):
        got = rb.roll_decode_attn_ranges(desc(B), lens, groups)
        steps = int(((lens + STEP - 1) // STEP).sum())
        want_nc = max(1, min((steps + 3) // 4, groups))
        assert len(got) == want_nc + 1
        assert np.array_equal(got, by_definition(lens, want_nc)), (lens, groups)


def test_ranges_partition_the_steps_and_are_equal_in_cost():
    rng = np.random.default_rng(100)
    lens = np.clip(np.rint(np.exp(rng.normal(np.log(2048), 1.0, 256))), 16, 16384).astype(np.int64)
    first = rb.roll_decode_attn_ranges(desc(256), lens, 256)
    n = (lens + STEP - 1) // STEP
    pre = np.concatenate([[0], np.cumsum(n)])
    assert first[0] == 0 and first[-1] == pre[-1] and np.all(np.diff(first) > 0) and len(first) == 257
    T = STEP_COST * pre[-1] + ROW_COST * (n > 0).sum()
    for c in range(256):
        rows_started = np.count_nonzero((pre[:-1] >= first[c]) & (pre[:-1] < first[c + 1]) & (n > 0))
        cost = STEP_COST * (first[c + 1] - first[c]) + ROW_COST * rows_started
        assert abs(cost - T / 256) <= STEP_COST + ROW_COST + 1, (c, cost, T / 256)


def test_equal_rows_one_range_each_and_no_row_is_cut():
    first = rb.roll_decode_attn_ranges(desc(256), np.full(256, 3456), 256)
    assert np.array_equal(first, np.arange(257) * 108)


def test_a_range_of_short_rows_gets_fewer_steps_than_one_inside_a_long_row():
    lens = np.concatenate([np.full(2000, 20), np.full(8, 64000)])   # one-step rows, then long rows
    first = rb.roll_decode_attn_ranges(desc(len(lens), max_pages=4096), lens, 64)
    size = np.diff(first)
    short, long_ = size[0], size[-1]
    assert first[-1] == 2000 + 8 * 2000
    # a one-step row costs 2 + 2, a step inside a long row 2
    assert abs(long_ / short - 2.0) < 0.1, (short, long_)


@pytest.mark.parametrize("Hkv,cut", [(1, 4), (2, 2), (4, 1), (8, 1), (3, 1)])
def test_few_kv_heads_cut_the_workgroups_range_again(Hkv, cut):
    lens = np.full(64, 4096)
    first = rb.roll_decode_attn_ranges(desc(64, Hq=Hkv * 4, Hkv=Hkv), lens, 256)
    assert len(first) - 1 == 256 * cut


def test_lengths_are_clamped_like_the_kernel_clamps_them():
    d = desc(4, max_pages=8)            # 8 pages of 16 tokens: at most 128 tokens = 4 steps per row
    first = rb.roll_decode_attn_ranges(d, np.array([-5, 1 << 30, 0, 33]), 256)
    assert first[-1] == 0 + 4 + 0 + 2


def test_empty_batch_and_errors():
    first = rb.roll_decode_attn_ranges(desc(5), np.zeros(5), 256)
    assert np.array_equal(first, [0, 0])
    with pytest.raises(rb.RollError):
        rb.roll_decode_attn_ranges(desc(5), np.ones(5), 0)
    with pytest.raises(ValueError):
        rb.roll_decode_attn_ranges(desc(5), np.ones(4), 8)
