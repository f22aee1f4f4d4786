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
