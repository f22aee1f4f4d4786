"""Pins for the oracle's temperature / top-p Gumbel-max sampler and its log-probs (CPU only)."""
import itertools

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import oracle
from oracle_helpers import from_bf16_bits, to_bf16_bits


def test_logprob_is_library_log_softmax_at_T1_p1():
    # the paper's enforced setting (temperature 1, top_p 1): the recorded value must be the
    # plain log-softmax of the raw logits at the sampled token
    rng = np.random.default_rng(0)
    x = (rng.standard_normal((6, 997)) * 2).astype(np.float32)
    r = oracle.sample_logprob(x, 1.0, 1.0, seed=3, step=5)
    ref = scipy.special.log_softmax(x.astype(np.float64), axis=1)
    ref_t = torch.log_softmax(torch.from_numpy(x).double(), dim=1).numpy()
    for b in range(6):
        assert abs(r["logprob"][b] - ref[b, r["tokens"][b]]) < 1e-12
        assert abs(r["logprob"][b] - ref_t[b, r["tokens"][b]]) < 1e-12
    assert (r["kept"] == 997).all() and np.isneginf(r["x_cut"]).all()


def test_logprob_bf16_logits_and_temperature():
    rng = np.random.default_rng(1)
    xb = to_bf16_bits(rng.standard_normal((4, 513)) * 2)
    x = from_bf16_bits(xb)
    T = 0.7
    r = oracle.sample_logprob(xb, T, 1.0, seed=1, step=0)
    Tf = float(np.float32(T))
    ref = scipy.special.log_softmax(x / Tf, axis=1)
    for b in range(4):
        assert abs(r["logprob"][b] - ref[b, r["tokens"][b]]) < 1e-12


def test_raw_logprob_is_library_log_softmax_whatever_the_sampling_setting():
    rng = np.random.default_rng(11)
    xb = to_bf16_bits(rng.standard_normal((5, 700)) * 2)
    ref = scipy.special.log_softmax(from_bf16_bits(xb), axis=1)
    for T, p in [(1.0, 1.0), (0.7, 0.95), (1.4, 0.5)]:
        r = oracle.sample_logprob(xb, T, p, seed=2, step=1)
        for b in range(5):
            assert abs(r["raw_logprob"][b] - ref[b, r["tokens"][b]]) < 1e-12
        if T == 1.0 and p == 1.0:
            np.testing.assert_allclose(r["raw_logprob"], r["logprob"], atol=1e-12)
        else:
            assert not np.allclose(r["raw_logprob"], r["logprob"])


def test_uniform_logits_give_minus_log_V():
    x = np.full((2, 300), 1.25, dtype=np.float32)
    r = oracle.sample_logprob(x, 1.0, 1.0, seed=0, step=0)
    np.testing.assert_allclose(r["logprob"], -np.log(300), atol=1e-13)
    # top-p < 1 on uniform logits: every value ties with the cut, so everything is kept
    r = oracle.sample_logprob(x, 1.0, 0.5, seed=0, step=0)
    assert (r["kept"] == 300).all()
    np.testing.assert_allclose(r["logprob"], -np.log(300), atol=1e-13)


def test_shift_and_scale_invariance():
    rng = np.random.default_rng(2)
    x = rng.integers(-40, 40, size=(3, 200)).astype(np.float32) / 8  # exact under +c and *2
    a = oracle.sample_logprob(x, 1.0, 0.9, seed=5, step=2)
    b = oracle.sample_logprob(x + 4.0, 1.0, 0.9, seed=5, step=2)
    c = oracle.sample_logprob(x * 2, 2.0, 0.9, seed=5, step=2)
    for o in (b, c):
        assert np.array_equal(a["tokens"], o["tokens"])
        np.testing.assert_allclose(a["logprob"], o["logprob"], atol=1e-12)
        assert np.array_equal(a["kept"], o["kept"])


def test_kept_logprobs_logsumexp_to_zero():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(400) * 2).astype(np.float32)
    for T, p in [(1.0, 1.0), (0.7, 0.95), (1.3, 0.5)]:
        pert, kept = oracle.row_detail(x, T, p, seed=0, step=0)
        r = oracle.sample_logprob(x[None], T, p, seed=0, step=0)
        tok = r["tokens"][0]
        lse_kept = r["logprob"][0] * -1 + x[tok].astype(np.float64) / float(np.float32(T))
        z = x.astype(np.float64) / float(np.float32(T))
        assert abs(scipy.special.logsumexp(z[kept] - lse_kept)) < 1e-12
        assert kept[tok]


def brute_force_kept(x, T, p):
    """Enumerate every subset: the answer is the smallest value-closed upper set
    (contains everything >= its minimum) whose softmax mass is >= p."""
    V = len(x)
    prob = scipy.special.softmax(np.asarray(x, np.float64) / T)
    best = None
    for r in range(1, V + 1):
        for sub in itertools.combinations(range(V), r):
            s = set(sub)
            lo = min(x[i] for i in s)
            if any(x[i] >= lo and i not in s for i in range(V)):
                continue  # not an upper set closed under ties
            if prob[list(s)].sum() >= p:
                if best is None or len(s) < len(best):
                    best = s
        if best is not None:
            break
    return best


@pytest.mark.parametrize("seed", range(6))
def test_top_p_set_matches_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    V = 8
    x = rng.integers(-6, 7, size=V).astype(np.float32) / 2  # coarse grid -> exact ties occur
    for p in (0.3, 0.6, 0.9, 0.999):
        for T in (1.0, 0.5):
            _, kept = oracle.row_detail(x, T, p, seed=0, step=0)
            assert set(np.flatnonzero(kept)) == brute_force_kept(x, T, p)


def test_top_p_properties():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(3000) * 2).astype(np.float32)
    z = x.astype(np.float64)
    prob = scipy.special.softmax(z)
    prev = None
    for p in (0.1, 0.5, 0.9, 0.95, 0.99, 0.9999):
        pf = float(np.float32(p))
        cut = oracle.top_p_cut(z, 1.0, pf)
        kept = z >= cut
        assert prob[kept].sum() >= pf - 1e-15
        assert prob[z > cut].sum() < pf          # dropping the lowest kept class falls short
        if prev is not None:
            assert not (prev & ~kept).any()      # monotone in p
        prev = kept
    assert np.isneginf(oracle.top_p_cut(z, 1.0, 1.0))
    # a dominant token with p >= top_p is the whole kept set and its log-prob is exactly 0
    x2 = x.copy(); x2[17] = 40.0
    r = oracle.sample_logprob(x2[None], 1.0, 0.9, seed=0, step=0)
    assert r["kept"][0] == 1 and r["tokens"][0] == 17 and r["logprob"][0] == 0.0


def test_top_p_one_equals_untruncated_sampling():
    rng = np.random.default_rng(5)
    xb = to_bf16_bits(rng.standard_normal((5, 2000)) * 2)
    a = oracle.sample_logprob(xb, 1.0, 1.0, seed=9, step=4)
    pert = np.stack([oracle.row_detail(xb[b], 1.0, 1.0, 9, 4, b)[0] for b in range(5)])
    assert np.array_equal(a["tokens"], pert.argmax(1))
    # a top_p so close to 1 that nothing is cut gives the same tokens and log-probs
    c = oracle.sample_logprob(xb, 1.0, 1.0 - 1e-7, seed=9, step=4)
    assert (c["kept"] >= 1999).all()


def test_argmax_ties_take_lowest_index_and_gap():
    x = np.zeros((1, 64), np.float32)
    pert, kept = oracle.row_detail(x[0], 1.0, 1.0, seed=2, step=0)
    r = oracle.sample_logprob(x, 1.0, 1.0, seed=2, step=0)
    order = np.sort(pert)[::-1]
    assert r["tokens"][0] == int(np.argmax(pert))
    assert abs(r["gap"][0] - (order[0] - order[1])) < 1e-15


def test_gumbel_formula_and_determinism():
    x = np.linspace(-1, 1, 16).astype(np.float32)
    pert, _ = oracle.row_detail(x, 0.5, 1.0, seed=77, step=3, row_id=2)
    for i in range(16):
        u = oracle.uniform(77, 3, 2, i)
        assert abs(pert[i] - (float(x[i]) / 0.5 - np.log(-np.log(u)))) < 1e-15
    # the draw depends on (seed, step, row id) only, not on batch composition
    X = np.stack([x, x[::-1].copy(), x])
    a = oracle.sample_logprob(X, 0.5, 1.0, seed=77, step=3)
    b = oracle.sample_logprob(X[[2, 0]], 0.5, 1.0, seed=77, step=3, row_ids=[2, 0])
    assert a["tokens"][2] == b["tokens"][0] and a["tokens"][0] == b["tokens"][1]
    c = oracle.sample_logprob(X, 0.5, 1.0, seed=77, step=4)
    assert not np.array_equal(pert, oracle.row_detail(x, 0.5, 1.0, 77, 4, 2)[0])
    assert a["logprob"].shape == c["logprob"].shape


@pytest.mark.parametrize("T,p,V", [(1.0, 1.0, 6), (0.7, 0.8, 12), (1.5, 0.95, 16)])
def test_sampled_frequencies_match_distribution(T, p, V):
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(V) * 1.5).astype(np.float32)
    n = 200000
    counts = oracle.sample_counts(x, T, p, seed=123, step0=0, n_draws=n)
    _, kept = oracle.row_detail(x, T, p, 123, 0)
    z = x.astype(np.float64) / float(np.float32(T))
    prob = np.where(kept, np.exp(z - z.max()), 0.0)
    prob /= prob.sum()
    assert counts[~kept].sum() == 0
    chi2 = ((counts[kept] - n * prob[kept]) ** 2 / (n * prob[kept])).sum()
    dof = kept.sum() - 1
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, dof)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("T,top_p", [(1.0, 1.0), (0.7, 0.95), (1.0, 0.5)])
def test_row_with_every_token_masked_draws_nothing(dtype, T, top_p):
    # -inf entries are masked tokens; a row in which every entry is masked defines no distribution:
    # token -1, log-probs NaN (nothing for the importance weight of Appendix A.1 to divide by),
    # nothing kept.  The neighbouring rows are untouched by it.
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((3, 41)) * 2).astype(np.float32)
    x[1, :] = -np.inf
    x[2, 5:] = -np.inf          # a row with SOME masked entries is an ordinary row
    xin = to_bf16_bits(x) if dtype == "bf16" else x
    r = oracle.sample_logprob(xin, T, top_p, seed=9, step=4)
    assert r["tokens"][1] == -1
    assert np.isnan(r["logprob"][1]) and np.isnan(r["raw_logprob"][1])
    assert r["kept"][1] == 0 and np.isposinf(r["gap"][1])
    assert np.isnan(r["x_cut"][1]) and np.isnan(r["x_cut_minus"][1]) and np.isnan(r["x_cut_plus"][1])
    # the other rows: same result as when sampled alone under their own row ids
    for b in (0, 2):
        alone = oracle.sample_logprob(xin[b:b + 1], T, top_p, seed=9, step=4, row_ids=[b])
        assert alone["tokens"][0] == r["tokens"][b] and alone["logprob"][0] == r["logprob"][b]
        assert 0 <= r["tokens"][b] < 41 and np.isfinite(r["logprob"][b])
    # masked entries can never be drawn; under a cut they are not in the kept set either (at
    # top_p = 1 the cut is -inf and the count is the whole row, masked entries carrying no mass)
    assert r["tokens"][2] < 5 and (1 <= r["kept"][2] <= 5 if top_p < 1 else r["kept"][2] == 41)
    # the helpers agree: no cut, nothing kept, nothing counted
    row = xin[1]
    assert np.isnan(oracle.top_p_cut(np.full(41, -np.inf), T, top_p))
    _, kept = oracle.row_detail(row, T, top_p, seed=9, step=4, row_id=1)
    assert not kept.any()
    assert oracle.sample_counts(row, T, top_p, seed=9, step0=0, n_draws=50).sum() == 0


def test_single_finite_entry_among_masked_ones_is_drawn_with_logprob_zero():
    # the smallest distribution there is: one unmasked token has probability 1 whatever T and top_p
    x = np.full((1, 33), -np.inf, dtype=np.float32)
    x[0, 17] = -3.5
    for T, p in [(1.0, 1.0), (0.7, 0.95), (2.0, 1e-6)]:
        r = oracle.sample_logprob(x, T, p, seed=1, step=2)
        assert r["tokens"][0] == 17 and r["logprob"][0] == 0.0 and r["raw_logprob"][0] == 0.0
        assert np.isposinf(r["gap"][0]) and r["kept"][0] == (1 if p < 1 else 33)
