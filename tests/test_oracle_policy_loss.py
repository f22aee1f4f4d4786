"""Pins for the oracle's off-policy objectives (Section 3.2 of the paper): closed forms, the
reductions between the objectives that the paper's own description implies, a numerical
derivative, and hand-computed values."""
import numpy as np
import pytest

import oracle


def rand_batch(rng, n_seq=5, max_len=40):
    lens = rng.integers(0, max_len, size=n_seq)
    lens[0] = 0                                     # an empty response
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(off[-1])
    lo = -np.abs(rng.standard_normal(T)).astype(np.float32) * 2
    lt = (lo + rng.standard_normal(T).astype(np.float32) * 0.6).astype(np.float32)
    lp = (lo + rng.standard_normal(T).astype(np.float32) * 0.3).astype(np.float32)
    R = rng.standard_normal(T).astype(np.float32)
    return lt, lo, lp, R, off


def test_hand_computed_values():
    # r = e^{0.5} = 1.6487; eps 0.2; c = 1.5; R = 2 and R = -2; log pi_theta = -1
    lt, lo = np.float32([-1.0, -1.0]), np.float32([-1.5, -1.5])
    R, off = np.float32([2.0, -2.0]), np.int64([0, 2])
    r = np.exp(0.5)
    ppo = oracle.policy_loss("ppo", lt, lo, None, R, off, 0.2, 0.2)
    assert np.allclose(ppo["value"], [2 * 1.2, -2 * r])       # positive signal clipped, negative not
    assert np.allclose(ppo["grad"], [0.0, -2 * r])
    tis = oracle.policy_loss("tis", lt, lo, None, R, off, c=1.5)
    assert np.allclose(tis["value"], [1.5 * 2 * -1, 1.5 * -2 * -1]) and np.allclose(tis["grad"], [3.0, -3.0])
    assert np.allclose(tis["is_weight"], [1.5, 1.5])
    topr = oracle.policy_loss("topr", lt, lo, None, R, off, c=1.5)
    assert np.allclose(topr["value"], [1.0 * 2 * -1, 1.5 * -2 * -1])   # T+ untouched, T- truncated
    cispo = oracle.policy_loss("cispo", lt, lo, None, R, off, 0.1, 0.3)
    assert np.allclose(cispo["grad"], [1.3 * 2, 1.3 * -2])
    assert np.isclose(ppo["seq_mean"][0], (2.4 - 2 * r) / 2) and np.isclose(ppo["batch_mean"], ppo["seq_mean"][0])


def test_reductions_between_objectives():
    rng = np.random.default_rng(0)
    lt, lo, lp, R, off = rand_batch(rng)
    # a proximal policy equal to the behaviour policy turns Decoupled PPO into PPO
    a = oracle.policy_loss("ppo", lt, lo, None, R, off, 0.2, 0.3)
    b = oracle.policy_loss("decoupled_ppo", lt, lo, lo, R, off, 0.2, 0.3)
    assert np.allclose(a["value"], b["value"], atol=1e-14) and np.allclose(a["grad"], b["grad"], atol=1e-14)
    # CISPO with the interval [0, c] is Truncated IS
    t = oracle.policy_loss("tis", lt, lo, None, R, off, c=3.0)
    ci = oracle.policy_loss("cispo", lt, lo, None, R, off, 1.0, 2.0)
    assert np.allclose(t["value"], ci["value"], atol=1e-14) and np.allclose(t["grad"], ci["grad"], atol=1e-14)
    # TOPR is Truncated IS on negative signals and plain R log pi on positive ones
    tp = oracle.policy_loss("topr", lt, lo, None, R, off, c=3.0)
    neg = R <= 0
    assert np.allclose(tp["value"][neg], t["value"][neg])
    assert np.allclose(tp["value"][~neg], (R * lt).astype(np.float64)[~neg])
    # with a huge clip range PPO is the unclipped surrogate R r, whose derivative in log pi is R r
    wide = oracle.policy_loss("ppo", lt, lo, None, R, off, 1.0, 1e9)
    ratio = np.exp(lt.astype(np.float64) - lo.astype(np.float64))
    assert np.allclose(wide["value"], R * ratio) and np.allclose(wide["grad"], R * ratio)
    # on-policy data (pi_theta = pi_old): every IS weight is 1
    on = oracle.policy_loss("tis", lo, lo, None, R, off, c=5.0)
    assert np.allclose(on["is_weight"], 1.0) and np.allclose(on["grad"], R)


@pytest.mark.parametrize("kind", ["ppo", "decoupled_ppo"])
def test_derivative_matches_finite_difference(kind):
    rng = np.random.default_rng(1)
    lt, lo, lp, R, off = rand_batch(rng, n_seq=6, max_len=60)
    base = oracle.policy_loss(kind, lt, lo, lp, R, off, 0.2, 0.2)
    h = 1e-3
    up = oracle.policy_loss(kind, (lt + np.float32(h)).astype(np.float32), lo, lp, R, off, 0.2, 0.2)
    dn = oracle.policy_loss(kind, (lt - np.float32(h)).astype(np.float32), lo, lp, R, off, 0.2, 0.2)
    step = (lt + np.float32(h)).astype(np.float64) - (lt - np.float32(h)).astype(np.float64)
    fd = (up["value"] - dn["value"]) / step
    # away from the kinks of min / clip the analytic derivative equals the numerical one
    ref = lp if kind == "decoupled_ppo" else lo
    rr = np.exp(lt.astype(np.float64) - ref.astype(np.float64))
    smooth = (np.abs(rr - 0.8) > 0.02) & (np.abs(rr - 1.2) > 0.02) & (np.abs(up["grad"] - dn["grad"]) < 1e-2 * (1 + np.abs(base["grad"])))
    assert smooth.sum() > 20
    assert np.allclose(fd[smooth], base["grad"][smooth], rtol=2e-3, atol=2e-3)


def test_sg_objectives_have_constant_coefficient():
    # for TIS / CISPO / TOPR the value is coefficient * R * log pi and the derivative is coefficient * R
    rng = np.random.default_rng(2)
    lt, lo, lp, R, off = rand_batch(rng)
    for kind in ("tis", "cispo", "topr"):
        r = oracle.policy_loss(kind, lt, lo, None, R, off, 0.2, 0.3, 2.0)
        nz = np.abs(lt) > 1e-3
        assert np.allclose(r["value"][nz] / lt.astype(np.float64)[nz], r["grad"][nz], rtol=1e-12)


def test_ragged_means():
    rng = np.random.default_rng(3)
    lt, lo, lp, R, off = rand_batch(rng, n_seq=7)
    r = oracle.policy_loss("ppo", lt, lo, None, R, off)
    means = [r["value"][off[s]:off[s + 1]].mean() if off[s + 1] > off[s] else 0.0 for s in range(7)]
    assert np.allclose(r["seq_mean"], means)
    live = [m for s, m in enumerate(means) if off[s + 1] > off[s]]
    assert np.isclose(r["batch_mean"], np.mean(live))
