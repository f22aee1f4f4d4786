"""GPU parity of roll_sample_logprob against the fp64 oracle (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from gpu_helpers import compare_sampling, run_sample, say

pytestmark = pytest.mark.gpu


def test_config1_exact():
    cfg = wl.CONFIGS["c1"]
    say("  sample case c1: fp32 N(0,1) V=4096 B=8 T=1 p=1 seed 0")
    lg = wl.make_logits(cfg, 0)
    for step in range(4):
        compare_sampling(lg, 1.0, 1.0, seed=0, step=step)


@pytest.mark.parametrize("name,T,p", [("c2", 1.0, 1.0), ("c3", 0.7, 0.95), ("c5", 1.0, 0.99)])
def test_full_vocab_reduced_batch(name, T, p):
    cfg = wl.CONFIGS[name]
    say(f"  sample case {name}: {cfg.logits_dtype} {cfg.logits} V={cfg.vocab} B=12 T={T} p={p}")
    lg = wl.make_logits(cfg, 1, batch=12)
    compare_sampling(lg, T, p, seed=42, step=3)


@pytest.mark.parametrize("dtype,V,stride", [("bf16", 1001, 1008), ("f32", 4099, 4100), ("bf16", 5, 8),
                                            ("f32", 3, 4), ("bf16", 8200, 8200), ("f32", 70001, 70004)])
@pytest.mark.parametrize("T,p", [(1.0, 1.0), (0.8, 0.9)])
def test_odd_vocab_sizes_and_strides(dtype, V, stride, T, p):
    say(f"  sample case odd: {dtype} V={V} stride={stride} T={T} p={p}")
    cfg = dataclasses.replace(wl.CONFIGS["c2"], vocab=stride, logits_dtype=dtype)
    lg = wl.make_logits(cfg, 2, batch=5).cuda()[:, :V]   # a strided view: rows dense, stride > V
    assert lg.stride(0) == stride and lg.is_cuda
    compare_sampling(lg, T, p, seed=7, step=11)


def test_row_ids_and_step_define_the_draw():
    cfg = dataclasses.replace(wl.CONFIGS["c2"], vocab=4096)
    lg = wl.make_logits(cfg, 3, batch=6)
    t0, l0 = run_sample(lg, 1.0, 1.0, 5, 9)
    perm = [4, 2, 0, 5, 1, 3]
    t1, l1 = run_sample(lg[perm].contiguous(), 1.0, 1.0, 5, 9, row_ids=perm)
    assert np.array_equal(t1, t0[perm]) and np.array_equal(l1, l0[perm])
    t2, _ = run_sample(lg, 1.0, 1.0, 5, 10)
    t3, _ = run_sample(lg, 1.0, 1.0, 6, 9)
    assert not np.array_equal(t2, t0) and not np.array_equal(t3, t0)
    compare_sampling(lg[perm].contiguous(), 1.0, 1.0, 5, 9, row_ids=perm)
    compare_sampling(lg, 1.3, 0.7, (1 << 40) + 17, (1 << 33) + 5)   # 64-bit seed and step


def test_masked_and_dominant_entries():
    cfg = dataclasses.replace(wl.CONFIGS["c2"], vocab=2048)
    lg = wl.make_logits(cfg, 4, batch=4).float()
    lg[0, 100:] = float("-inf")           # only the first 100 entries can be drawn
    lg[1, 777] = 60.0                     # one entry holds all the mass
    lg[2, :] = 0.5                        # uniform
    lg = lg.to(torch.bfloat16)
    for T, p in [(1.0, 1.0), (1.0, 0.9), (0.5, 0.3)]:
        tok, lp = run_sample(lg, T, p, 1, 2)
        assert tok[0] < 100 and tok[1] == 777 and abs(lp[1]) < 1e-6
        assert abs(lp[2] + np.log(2048)) < 1e-3
        compare_sampling(lg, T, p, 1, 2)


def test_tiny_top_p_keeps_the_top_class():
    cfg = dataclasses.replace(wl.CONFIGS["c2"], vocab=4096)
    lg = wl.make_logits(cfg, 5, batch=8)
    tok, lp = run_sample(lg, 1.0, 1e-6, 3, 0)
    x = lg.float().numpy()
    for r in range(8):
        assert x[r, tok[r]] == x[r].max()
    compare_sampling(lg, 1.0, 1e-6, 3, 0)


def test_many_steps_small_vocab_all_tokens_match():
    # the sampler as a whole: every draw of a long run equals the oracle's draw
    cfg = dataclasses.replace(wl.CONFIGS["c1"], vocab=16)
    lg = (wl.make_logits(cfg, 6, batch=64) * 1.5).contiguous()
    ties = 0
    for step in range(40):
        t, _ = compare_sampling(lg, 0.9, 0.95, seed=99, step=step)
        ties += t
    assert ties <= 2


def test_policy_version_tag_is_recorded_beside_the_logprob():
    # a trajectory that is generated under version 3, aborted, and resumed under version 5
    # carries both tags token by token; tokens and log-probs do not depend on the tag output
    cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=6, vocab=5000)
    logits = wl.make_logits(cfg, 9, "cuda")
    steps, B = 4, cfg.batch
    tags = torch.full((steps, B), -1, dtype=torch.int32, device="cuda")
    toks = torch.zeros((steps, B), dtype=torch.int32, device="cuda")
    lps = torch.zeros((steps, B), dtype=torch.float32, device="cuda")
    for step in range(steps):
        version = 3 if step < 2 else 5
        desc = rb.sample_desc(logits, policy_version=version, policy_version_out=tags[step])
        rb.roll_sample_logprob(logits, 1.0, 1.0, 9, step, toks[step], lps[step], desc, None)
    torch.cuda.synchronize()
    assert tags.cpu().tolist() == [[3] * B, [3] * B, [5] * B, [5] * B]
    for step in range(steps):
        t, lp = run_sample(logits, 1.0, 1.0, 9, step)
        assert np.array_equal(t, toks[step].cpu().numpy())
        assert np.array_equal(lp, lps[step].double().cpu().numpy())


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_top_p_cut_at_every_depth_of_the_row(dtype):
    # Rows built so that the cut value falls (0) within the same binade as the max, (1) a few
    # binades below it, (2) at tiny positive values, (3) at negative values, (4) in a row whose
    # max is zero with both signed zeros present, (5) in a row of one repeated value, (6) in a
    # sorted row (descending, then (7) ascending), (8) in a row with a single finite entry.
    g = torch.Generator().manual_seed(77)
    V = 6000
    rows = []
    base = torch.randn((V,), generator=g)
    rows.append(8.0 + 0.5 * base)                                   # 0: everything in [4, 16)
    rows.append(torch.where(torch.arange(V) < 40, 6.0 + base, 0.05 * base.abs() + 0.02))   # 1
    rows.append(torch.where(torch.arange(V) < 3, 1.0 + 0 * base, 1e-4 * (1 + base.abs())))  # 2
    rows.append(base * 3.0 - 4.0)                                    # 3: mostly negative
    z = -base.abs() * 2.0
    z[::7] = 0.0
    z[3::7] = -0.0
    rows.append(z)                                                   # 4
    rows.append(torch.full((V,), -1.25))                             # 5
    rows.append(torch.sort(base * 2.0, descending=True).values)      # 6
    rows.append(torch.sort(base * 2.0).values)                       # 7
    one = torch.full((V,), float("-inf"))
    one[4321] = -3.0
    rows.append(one)                                                 # 8
    lg = torch.stack(rows).to(dtype).contiguous()
    for T, p in [(1.0, 0.9), (0.6, 0.5), (1.7, 0.999), (1.0, 0.02)]:
        for step in range(3):
            compare_sampling(lg, T, p, seed=1234, step=step)


def test_fp32_top_p_with_crowded_cut_bucket():
    # fp32 rows whose cut value shares its upper 16 key bits with few, 8192, 8193 and all of the
    # row's entries (equal values and distinct ones): the lower key bits are resolved over those
    # entries alone when they fit on chip and over the whole row otherwise, with one result.
    g = torch.Generator().manual_seed(91)
    V = 20000
    fine = 2.0 + torch.randint(0, 1 << 16, (V,), generator=g).float() * 2.0 ** -22   # one bucket: [2, 2 + 2^-6)
    rows = []
    for crowd in (300, 8192, 8193, V):
        r = -3.0 + 0.5 * torch.randn((V,), generator=g)
        idx = torch.randperm(V, generator=g)[:crowd]
        r[idx] = fine[idx]
        rows.append(r)
    rows.append(torch.full((V,), 0.75))
    eq = -3.0 + 0.5 * torch.randn((V,), generator=g)
    eq[torch.randperm(V, generator=g)[:9000]] = 2.0
    rows.append(eq)
    lg = torch.stack(rows).contiguous()
    assert lg.dtype == torch.float32
    for T, p in [(1.0, 0.9), (0.5, 0.4), (1.0, 0.999), (2.0, 0.05)]:
        for step in range(2):
            compare_sampling(lg, T, p, seed=4321, step=step)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_row_without_a_finite_entry_gives_no_token(dtype):
    # row 1 is masked entirely: token -1 and NaN log-probs, as the oracle says; its neighbours are
    # untouched by it, with and without top-p
    cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=3, vocab=3001)
    lg = wl.make_logits(cfg, 12).to(dtype)
    full = torch.zeros((3, 3008), dtype=dtype, device="cuda")    # rows dense, stride a multiple of 8
    full[:, :3001] = lg.cuda()
    full[1, :] = float("-inf")
    lg = full[:, :3001]
    import oracle
    for T, p in [(1.0, 1.0), (0.8, 0.9)]:
        tok, lp, raw = run_sample(lg, T, p, 5, 1, want_raw=True)
        ref = oracle.sample_logprob(wl.logits_numpy(lg), T, p, 5, 1)
        assert tok[1] == -1 and ref["tokens"][1] == -1
        assert np.isnan(lp[1]) and np.isnan(raw[1])
        for r in (0, 2):
            assert tok[r] == ref["tokens"][r] and abs(lp[r] - ref["logprob"][r]) <= 1e-3


@pytest.mark.parametrize("T", [0.01, 0.05, 10.0, 100.0])
def test_extreme_temperatures_and_tiny_vocabularies(T):
    # T = 0.01 multiplies the logits by 100 (nearly greedy, exponents hundreds of binary orders
    # apart), T = 100 flattens them; vocabularies of one and two entries have nothing to sweep
    for dtype in ("bf16", "f32"):
        for V in (1, 2, 9, 4097):
            cfg = dataclasses.replace(wl.CONFIGS["c1"], batch=6, vocab=V, logits_dtype=dtype, logits="normal2")
            stride = (V + 7) // 8 * 8
            full = torch.zeros((6, stride), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                               device="cuda")
            full[:, :V] = wl.make_logits(cfg, 77 + V, "cuda")
            for p in (1.0, 0.5, 0.999):
                compare_sampling(full[:, :V], T, p, 9, 3)


def test_bf16_top_p_rows_that_overflow_the_value_counters():
    # bf16 rows with top-p count the entries of every value in 16-bit counters; a row with 65536
    # or more equal entries overflows one, is noticed and takes the histogram route, with the same
    # result.  Rows: one repeated value; 70 000 equal entries among Gaussian ones (as the row max,
    # as a low value); 40 000 entries of +0 and 40 000 of -0 (one value, two bit patterns); exactly
    # 65 535 and 65 536 equal entries; a row masked but for 300 entries (-inf is not counted).
    g = torch.Generator().manual_seed(5)
    V = 152064
    base = torch.randn((V,), generator=g) * 2.0
    perm = torch.randperm(V, generator=g)
    rows = [torch.full((V,), 0.375)]
    for value in (9.5, -3.0):
        r = base.clone()
        r[perm[:70000]] = value
        rows.append(r)
    z = -base.abs() - 0.5
    z[perm[:40000]] = 0.0
    z[perm[40000:80000]] = -0.0
    rows.append(z)
    for n in (65535, 65536):
        r = base.clone()
        r[perm[:n]] = 1.25
        rows.append(r)
    masked = torch.full((V,), float("-inf"))
    masked[perm[:300]] = base[perm[:300]]
    rows.append(masked)
    lg = torch.stack(rows).to(torch.bfloat16).contiguous()
    for T, p in [(1.0, 0.9), (0.7, 0.95), (1.3, 0.3)]:
        compare_sampling(lg, T, p, seed=77, step=2)
