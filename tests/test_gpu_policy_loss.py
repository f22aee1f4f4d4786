"""GPU parity of roll_policy_loss against the fp64 oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_11345_amd import binding as rb
from paper_2510_11345_amd import workloads as wl
from gpu_helpers import say

pytestmark = pytest.mark.gpu

KINDS = ["ppo", "decoupled_ppo", "tis", "cispo", "topr"]


def run_gpu(kind, b, eps_lo, eps_hi, c, outputs=True):
    d = {k: v.cuda() for k, v in b.items()}
    T, n = d["logp_old"].numel(), d["offsets"].numel() - 1
    mk = lambda m: torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
    value, grad, w = (mk(T), mk(T), mk(T)) if outputs else (None, None, None)
    seq_mean, batch_mean = mk(n), mk(1)
    rb.roll_policy_loss(kind, d["logp_theta"], d["logp_old"], d["logp_prox"] if kind == "decoupled_ppo" else None,
                        d["signal"], d["offsets"], value, grad, w, seq_mean, batch_mean, eps_lo, eps_hi, c)
    torch.cuda.synchronize()
    f = lambda t: None if t is None else t.double().cpu().numpy()
    return f(value), f(grad), f(w), f(seq_mean), float(batch_mean.item())


@pytest.mark.parametrize("kind", KINDS)
def test_policy_loss_matches_oracle(kind):
    b = wl.make_policy_batch(96, seed=1, max_len=3000)
    eps_lo, eps_hi, c = 0.2, 0.28, 5.0
    say(f"  policy loss {kind}: {b['offsets'].numel() - 1} responses, {b['logp_old'].numel()} tokens")
    ref = oracle.policy_loss(kind, b["logp_theta"].numpy(), b["logp_old"].numpy(),
                             b["logp_prox"].numpy() if kind == "decoupled_ppo" else None,
                             b["signal"].numpy(), b["offsets"].numpy(), np.float32(eps_lo), np.float32(eps_hi),
                             np.float32(c))
    value, grad, w, seq_mean, batch_mean = run_gpu(kind, b, eps_lo, eps_hi, c)
    # outputs are fp32 roundings of the same fp64 arithmetic
    tol = lambda x: 1e-6 * (1 + np.abs(x))
    assert (np.abs(value - ref["value"]) <= tol(ref["value"])).all()
    assert (np.abs(grad - ref["grad"]) <= tol(ref["grad"])).all()
    assert (np.abs(w - ref["is_weight"]) <= tol(ref["is_weight"])).all()
    assert (np.abs(seq_mean - ref["seq_mean"]) <= tol(ref["seq_mean"])).all()
    assert abs(batch_mean - ref["batch_mean"]) <= 1e-6 * (1 + abs(ref["batch_mean"]))
    # the per-token outputs are optional
    _, _, _, seq_mean2, batch_mean2 = run_gpu(kind, b, eps_lo, eps_hi, c, outputs=False)
    assert np.array_equal(seq_mean, seq_mean2) and batch_mean == batch_mean2


def test_on_policy_weights_are_one_and_empty_batch_edges():
    b = wl.make_policy_batch(8, seed=2, max_len=200)
    b["logp_theta"] = b["logp_old"].clone()
    value, grad, w, seq_mean, _ = run_gpu("tis", b, 0.2, 0.2, 5.0)
    assert np.array_equal(w, np.ones_like(w))
    assert np.allclose(grad, b["signal"].numpy())
    # a batch whose responses are all empty
    e = dict(logp_old=torch.zeros(1), logp_theta=torch.zeros(1), logp_prox=torch.zeros(1), signal=torch.zeros(1),
             offsets=torch.zeros(4, dtype=torch.int64))
    _, _, _, seq_mean, batch_mean = run_gpu("ppo", e, 0.2, 0.2, 5.0, outputs=False)
    assert not seq_mean.any() and batch_mean == 0.0


def test_bad_arguments():
    b = {k: v.cuda() for k, v in wl.make_policy_batch(4, seed=3, max_len=50).items()}
    n = b["offsets"].numel() - 1
    sm, bm = torch.zeros(n, device="cuda"), torch.zeros(1, device="cuda")
    with pytest.raises(rb.RollError):   # Decoupled PPO without the proximal policy
        rb.roll_policy_loss("decoupled_ppo", b["logp_theta"], b["logp_old"], None, b["signal"], b["offsets"],
                            None, None, None, sm, bm)
    with pytest.raises(rb.RollError):
        rb.roll_policy_loss("tis", b["logp_theta"], b["logp_old"], None, b["signal"], b["offsets"],
                            None, None, None, sm, bm, c=0.0)


@pytest.mark.parametrize("shape", ["one_long", "many_tiny", "mixed", "fewer_tokens_than_waves", "many_responses"])
def test_token_shares_and_partial_sums_at_every_kind_of_boundary(shape):
    # The batch's tokens are dealt to the waves in equal shares whatever the responses' lengths: one
    # response spread over every wave, thousands of one- and two-token responses (dozens per
    # share), responses that begin or end exactly at share boundaries with empty ones between,
    # fewer tokens than waves (most shares empty), and more responses than the on-chip offset
    # table holds.
    rng = np.random.default_rng(["one_long", "many_tiny", "mixed", "fewer_tokens_than_waves", "many_responses"].index(shape))
    if shape == "one_long":
        lens = np.array([0, 300000, 0, 5])
    elif shape == "many_tiny":
        lens = rng.integers(0, 3, size=6000)
    elif shape == "mixed":
        lens = np.concatenate([[4096 * 7, 0, 0, 4096, 1, 4095, 0], rng.integers(0, 9000, size=40), [0]])
    elif shape == "fewer_tokens_than_waves":
        lens = np.array([3, 0, 700, 1, 0, 0, 2])
    else:
        lens = rng.integers(0, 40, size=9000)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(offsets[-1])
    g = torch.Generator().manual_seed(T)
    lo = -(torch.randn(T, generator=g).abs() * 1.5 + 0.01)
    b = dict(logp_old=lo, logp_theta=lo + torch.randn(T, generator=g) * 0.3, logp_prox=lo + torch.randn(T, generator=g) * 0.1,
             signal=torch.randn(T, generator=g), offsets=torch.from_numpy(offsets))
    say(f"  policy loss shares {shape}: {len(lens)} responses, {T} tokens")
    for kind in ("ppo", "decoupled_ppo", "topr"):
        ref = oracle.policy_loss(kind, b["logp_theta"].numpy(), b["logp_old"].numpy(),
                                 b["logp_prox"].numpy() if kind == "decoupled_ppo" else None,
                                 b["signal"].numpy(), offsets, np.float32(0.2), np.float32(0.28), np.float32(5.0))
        value, grad, w, seq_mean, batch_mean = run_gpu(kind, b, 0.2, 0.28, 5.0)
        tol = lambda x: 1e-6 * (1 + np.abs(x))
        assert (np.abs(value - ref["value"]) <= tol(ref["value"])).all()
        assert (np.abs(grad - ref["grad"]) <= tol(ref["grad"])).all()
        assert (np.abs(w - ref["is_weight"]) <= tol(ref["is_weight"])).all()
        assert (np.abs(seq_mean - ref["seq_mean"]) <= tol(ref["seq_mean"])).all()
        assert abs(batch_mean - ref["batch_mean"]) <= 1e-6 * (1 + abs(ref["batch_mean"]))
        again = run_gpu(kind, b, 0.2, 0.28, 5.0)
        assert np.array_equal(seq_mean, again[3]) and batch_mean == again[4]     # reproducible
