"""Helpers for oracle tests: bf16 packing and logical-to-paged KV placement (CPU only)."""
import numpy as np
import torch

import oracle


def to_bf16_bits(x):
    """float array -> uint16 bf16 bit patterns (round to nearest even, via torch)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def from_bf16_bits(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def k_slot_bits(t, P):
    """Third, bit-level statement of the K token permutation: inside blocks of min(P, 32)
    tokens, bit 2 of the in-block index moves to the top and the bits above it shift down."""
    nbits = 4 if P == 16 else 5
    u, blk = t & ((1 << nbits) - 1), t >> nbits
    low, b2, high = u & 3, (u >> 2) & 1, u >> 3
    return (blk << nbits) | (b2 << (nbits - 1)) | (high << 2) | low


def build_paged(K, V, lens, P, rng=None, spare=2):
    """K, V: float arrays [B, Lmax, Hkv, D] (logical).  Returns bf16-bit pools in the
    oracle's page layouts with a (optionally shuffled) page table, plus the rounded
    logical values as float64."""
    B, Lmax, Hkv, D = K.shape
    Kb, Vb = to_bf16_bits(K), to_bf16_bits(V)
    n_pages = [(int(l) + P - 1) // P for l in lens]
    total = sum(n_pages) + spare
    ids = np.arange(total, dtype=np.int32) if rng is None else rng.permutation(total).astype(np.int32)
    max_pages = max(1, max(n_pages))
    table = np.full((B, max_pages), -1, dtype=np.int32)
    k_pages = np.zeros(total * Hkv * D * P, dtype=np.uint16)
    v_pages = np.zeros(total * Hkv * D * P, dtype=np.uint16)
    pos = 0
    for b in range(B):
        table[b, :n_pages[b]] = ids[pos:pos + n_pages[b]]
        pos += n_pages[b]
        for j in range(int(lens[b])):
            oracle.kv_store(k_pages, v_pages, int(table[b, j // P]), j % P, Kb[b, j], Vb[b, j], Hkv, D, P)
    return k_pages, v_pages, table, from_bf16_bits(Kb), from_bf16_bits(Vb)
