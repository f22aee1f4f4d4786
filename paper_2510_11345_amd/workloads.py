"""Seeded synthetic inputs with the shapes of the paper's rollout workloads.

This module holds no arithmetic of the decode step: it only draws lengths,
Gaussian tensors and page assignments.  Both the CPU oracle and the GPU
library are fed from here so that they see identical bits.

What the synthetic inputs stand in for (ROLL Flash, arXiv 2510.11345): the
paper rolls out Qwen3-class GQA models on math / agentic prompts with a 32k
sequence limit (Section 3.3, Appendix A); response lengths are long-tailed
with the longest above 20x the median (Section 1).  Neither the weights nor
the prompt sets are available here, so Q/K/V are N(0,1) in bf16, lengths are
drawn from long-tailed laws and logits are Gaussian (optionally with a
Zipf-shaped bias) over a Qwen-sized vocabulary.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class DecodeConfig:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    vocab: int
    logits_dtype: str  # "bf16" | "f32"
    temperature: float
    top_p: float
    lengths: str  # name of the length law, see draw_lengths
    logits: str  # "normal1" | "normal2" | "zipf"
    max_len: int

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def kv_bytes_per_token(self) -> int:
        """K and V, bf16, all KV heads of one layer."""
        return 2 * self.num_kv_heads * self.head_dim * 2


CONFIGS = {
    # small correctness case
    "c1": DecodeConfig("c1", 8, 8, 2, 64, 16, 4096, "f32", 1.0, 1.0, "uniform_1_512", "normal1", 512),
    # 7B-class GQA shape, lognormal lengths
    "c2": DecodeConfig("c2", 256, 28, 4, 128, 16, 152064, "bf16", 1.0, 1.0, "lognormal_2048", "normal2", 16384),
    # long-tail rollout batch
    "c3": DecodeConfig("c3", 512, 28, 4, 128, 16, 152064, "bf16", 0.7, 0.95, "longtail_32768", "normal2", 32768),
    # continuous refill uses c2's shape; lengths come from the refill scheduler
    "c4": DecodeConfig("c4", 256, 28, 4, 128, 16, 152064, "bf16", 1.0, 1.0, "refill", "normal2", 17408),
    # 32B-class GQA shape
    "c5": DecodeConfig("c5", 128, 64, 8, 128, 32, 151936, "bf16", 1.0, 0.99, "lognormal_8192", "zipf", 65536),
}


def scaled(cfg: DecodeConfig, **kw) -> DecodeConfig:
    """A copy of cfg with some fields replaced (reduced sizes for CPU-speed tests)."""
    return dataclasses.replace(cfg, **kw)


def draw_lengths(law: str, batch: int, seed: int, max_len: Optional[int] = None) -> np.ndarray:
    """KV length per row (counts the token being decoded), int32 [batch]."""
    rng = np.random.default_rng([seed, 0x4C454E])
    if law == "uniform_1_512":
        L = rng.integers(1, 513, size=batch)
    elif law == "lognormal_2048":
        L = np.clip(np.rint(np.exp(rng.normal(math.log(2048.0), 1.0, size=batch))), 16, 16384)
    elif law == "lognormal_8192":
        L = np.clip(np.rint(np.exp(rng.normal(math.log(8192.0), 1.0, size=batch))), 64, 65536)
    elif law == "longtail_32768":
        L = rng.integers(256, 4097, size=batch)
        n_long = int(round(0.05 * batch))
        idx = rng.permutation(batch)[:n_long]
        L[idx] = 32768
    else:
        raise ValueError(law)
    L = L.astype(np.int64)
    if max_len is not None:
        L = np.minimum(L, max_len)
    return L.astype(np.int32)


def _gen(seed: int, salt: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + salt) & 0x7FFFFFFFFFFFFFFF)
    return g


def randn_bf16(shape, seed: int, salt: int, device="cpu", std: float = 1.0) -> torch.Tensor:
    """N(0, std^2) rounded to nearest-even bf16, generated in slabs to bound memory."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    g = _gen(seed, salt, device)
    slab = 1 << 26
    for s in range(0, flat.numel(), slab):
        n = min(slab, flat.numel() - s)
        x = torch.randn(n, generator=g, device=device, dtype=torch.float32)
        if std != 1.0:
            x *= std
        flat[s:s + n] = x.to(torch.bfloat16)
    return out


def bits(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16 tensor (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def assign_pages(lengths: np.ndarray, page_size: int, seed: int, spare_pages: int = 3,
                 shuffle: bool = True):
    """Give every row ceil(L/P) distinct physical pages.

    Returns (page_table int32 [B, max_pages] filled with -1 past the row's
    pages, num_pages).  With shuffle the physical ids are a seeded random
    permutation, which is what a pool looks like after many refills.
    """
    n_pages = (lengths.astype(np.int64) + page_size - 1) // page_size
    total = int(n_pages.sum())
    num_pages = total + spare_pages
    ids = np.arange(num_pages, dtype=np.int32)
    if shuffle:
        ids = np.random.default_rng([seed, 0x504147]).permutation(num_pages).astype(np.int32)
    max_pages = max(1, int(n_pages.max()) if len(n_pages) else 1)
    table = np.full((len(lengths), max_pages), -1, dtype=np.int32)
    pos = 0
    for b, n in enumerate(n_pages):
        table[b, :n] = ids[pos:pos + n]
        pos += int(n)
    return table, num_pages


def make_attn_inputs(cfg: DecodeConfig, seed: int, device="cpu", lengths=None,
                     shuffle_pages: bool = True):
    """Q and the two paged pools filled with i.i.d. N(0,1) bf16.

    The pools are filled in physical order (the values are i.i.d., so the
    page layout does not enter); each consumer applies its own index formula.
    Returns dict(q, k_pages, v_pages [torch bf16], page_table, seq_lens
    [numpy int32], num_pages).
    """
    if lengths is None:
        lengths = draw_lengths(cfg.lengths, cfg.batch, seed, cfg.max_len)
    lengths = np.asarray(lengths, dtype=np.int32)
    table, num_pages = assign_pages(lengths, cfg.page_size, seed, shuffle=shuffle_pages)
    B, Hq, Hkv, D, P = len(lengths), cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.page_size
    q = randn_bf16((B, Hq, D), seed, 1, device)
    k_pages = randn_bf16((num_pages, Hkv, D // 8, P, 8), seed, 2, device)
    v_pages = randn_bf16((num_pages, Hkv, P // 8, D, 8), seed, 3, device)
    return dict(q=q, k_pages=k_pages, v_pages=v_pages, page_table=table, seq_lens=lengths,
                num_pages=num_pages)


def make_logits(cfg: DecodeConfig, seed: int, device="cpu", batch: Optional[int] = None,
                salt: int = 4) -> torch.Tensor:
    """Logits [B, V] in cfg.logits_dtype.

    normal1: N(0,1); normal2: N(0, std 2); zipf: -1.1 ln(rank_i) + N(0,1) with
    rank a seeded permutation of 1..V shared by the rows.
    """
    B = cfg.batch if batch is None else batch
    V = cfg.vocab
    g = _gen(seed, salt, device)
    x = torch.randn((B, V), generator=g, device=device, dtype=torch.float32)
    if cfg.logits == "normal2":
        x *= 2.0
    elif cfg.logits == "zipf":
        rank = np.random.default_rng([seed, 0x5A4950]).permutation(V).astype(np.float64) + 1.0
        bias = torch.from_numpy((-1.1 * np.log(rank)).astype(np.float32)).to(device)
        x += bias
    elif cfg.logits != "normal1":
        raise ValueError(cfg.logits)
    if cfg.logits_dtype == "bf16":
        return x.to(torch.bfloat16)
    return x


def logits_numpy(t: torch.Tensor) -> np.ndarray:
    """Host array the oracle reads: uint16 bits for bf16, float32 otherwise."""
    if t.dtype == torch.bfloat16:
        return bits(t)
    return t.detach().cpu().contiguous().numpy()


# --------------------------------------------------------------------------
# Continuous refill (queue scheduling: a freed slot is given the next prompt)
# --------------------------------------------------------------------------

@dataclasses.dataclass
class RefillPlan:
    """Pre-drawn prompt queue: prompt length and target response length per request."""
    prompt_len: np.ndarray
    target_len: np.ndarray
    start_generated: np.ndarray  # tokens already generated by the initial occupants


def draw_refill_plan(num_slots: int, num_requests: int, seed: int, prompt_range=(128, 1024),
                     target_median: float = 1500.0, target_clip=(16, 16384)) -> RefillPlan:
    """Prompt queue of the continuous-refill workload: request i has a prompt of prompt_len[i]
    tokens and finishes after target_len[i] generated tokens.  The first num_slots requests
    occupy the slots at step 0 and have already generated start_generated[i] < target_len[i]
    tokens, so that finishes are spread over the run instead of bunched at its start."""
    rng = np.random.default_rng([seed, 0x52454649])
    prompt = rng.integers(prompt_range[0], prompt_range[1] + 1, size=num_requests).astype(np.int32)
    target = np.clip(np.rint(np.exp(rng.normal(math.log(target_median), 1.0, size=num_requests))),
                     target_clip[0], target_clip[1]).astype(np.int32)
    start = np.zeros(num_requests, dtype=np.int32)
    start[:num_slots] = (rng.random(num_slots) * target[:num_slots]).astype(np.int32)
    return RefillPlan(prompt, target, start)


# --------------------------------------------------------------------------
# A rollout batch as the trainer sees it: ragged responses with recorded log-probs
# --------------------------------------------------------------------------

def make_policy_batch(num_seqs: int, seed: int, length_law: str = "lognormal_2048", max_len: int = 16384,
                      group: int = 8, drift: float = 0.3, device="cpu"):
    """Ragged responses (lengths from a long-tailed law, a few empty), per-token log-probs of the
    rollout policy (negative, a few nats), of the current and proximal policies (the rollout's plus
    Gaussian drift, i.e. stale by a few policy versions), and a per-response learning signal
    normalised within groups of `group` responses (GRPO-style advantage), broadcast to tokens.
    Returns dict of torch tensors: logp_old, logp_theta, logp_prox, signal [T] fp32; offsets int64."""
    rng = np.random.default_rng([seed, 0x504F4C])
    lens = draw_lengths(length_law, num_seqs, seed, max_len).astype(np.int64)
    lens[rng.integers(0, num_seqs, size=max(1, num_seqs // 64))] = 0
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(offsets[-1])
    g = _gen(seed, 77, "cpu")
    lo = -(torch.randn(T, generator=g).abs() * 1.5 + 0.01)
    lt = lo + torch.randn(T, generator=g) * drift
    lp = lo + torch.randn(T, generator=g) * (0.5 * drift)
    reward = rng.random(num_seqs) < 0.4                      # verifiable reward: right or wrong
    adv = np.zeros(num_seqs, np.float32)
    for s0 in range(0, num_seqs, group):
        r = reward[s0:s0 + group].astype(np.float32)
        adv[s0:s0 + group] = (r - r.mean()) / (r.std() + 1e-6)
    signal = torch.from_numpy(np.repeat(adv, lens))
    out = dict(logp_old=lo.float(), logp_theta=lt.float(), logp_prox=lp.float(), signal=signal.float(),
               offsets=torch.from_numpy(offsets))
    return {k: v.to(device) for k, v in out.items()}
