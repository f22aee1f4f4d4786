"""Pins of the oracle's chunked prefill against things other than itself: dense causal attention
written out with numpy, invariance to how the prompt is cut into chunks, the decode definition
for the last token, causality, and the page layout."""
import numpy as np
import pytest

import oracle
from oracle_helpers import to_bf16_bits as bf16_bits, from_bf16_bits as bf16_value


def _setup(seed, n_slots, lens, Hq, Hkv, D, P, extra_pages=2):
    rng = np.random.default_rng(seed)
    pages_per = [(L + P - 1) // P for L in lens]
    num_pages = sum(pages_per) + extra_pages
    ids = rng.permutation(num_pages).astype(np.int32)
    max_pages = max(pages_per)
    table = np.full((n_slots, max_pages), -1, np.int32)
    pos = 0
    for s, n in enumerate(pages_per):
        table[s, :n] = ids[pos:pos + n]
        pos += n
    k_pages = bf16_bits(rng.normal(size=num_pages * Hkv * D * P).astype(np.float32))
    v_pages = bf16_bits(rng.normal(size=num_pages * Hkv * D * P).astype(np.float32))
    return rng, table, k_pages, v_pages


def _tokens(rng, T, Hq, Hkv, D):
    q = bf16_bits(rng.normal(size=(T, Hq, D)).astype(np.float32))
    k = bf16_bits(rng.normal(size=(T, Hkv, D)).astype(np.float32))
    v = bf16_bits(rng.normal(size=(T, Hkv, D)).astype(np.float32))
    return q, k, v


def _dense_causal(q, k, v, Hq, Hkv, n_before=0, scale=None):
    """q [n, Hq, D], k / v [n_before + n, Hkv, D] as float64: textbook masked softmax attention."""
    n, _, D = q.shape
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    G = Hq // Hkv
    out = np.zeros((n, Hq, D))
    for h in range(Hq):
        S = q[:, h, :] @ k[:, h // G, :].T * scale            # [n, n_before + n]
        mask = np.arange(k.shape[0])[None, :] > (n_before + np.arange(n))[:, None]
        S = np.where(mask, -np.inf, S)
        S = S - S.max(axis=1, keepdims=True)
        W = np.exp(S)
        W /= W.sum(axis=1, keepdims=True)
        out[:, h, :] = W @ v[:, h // G, :]
    return out


@pytest.mark.parametrize("Hq,Hkv,D,P", [(4, 2, 64, 16), (7, 1, 128, 32), (2, 2, 64, 64)])
def test_prefill_equals_dense_causal_attention(Hq, Hkv, D, P):
    n = 45
    rng, table, kp, vp = _setup(1, 1, [n], Hq, Hkv, D, P)
    q, k, v = _tokens(rng, n, Hq, Hkv, D)
    out = oracle.prefill_attn(q, k, v, [0], [0], [0, n], kp, vp, table, Hq, Hkv, D, P)
    want = _dense_causal(bf16_value(q), bf16_value(k), bf16_value(v), Hq, Hkv)
    assert np.abs(out - want).max() < 1e-12


def test_prefill_on_top_of_cached_tokens_and_custom_scale():
    Hq, Hkv, D, P = 6, 2, 64, 16
    n0, n1 = 21, 30
    rng, table, kp, vp = _setup(2, 1, [n0 + n1], Hq, Hkv, D, P)
    q0, k0, v0 = _tokens(rng, n0, Hq, Hkv, D)
    q1, k1, v1 = _tokens(rng, n1, Hq, Hkv, D)
    oracle.prefill_attn(q0, k0, v0, [0], [0], [0, n0], kp, vp, table, Hq, Hkv, D, P)
    out = oracle.prefill_attn(q1, k1, v1, [0], [n0], [0, n1], kp, vp, table, Hq, Hkv, D, P, scale=0.3)
    kk = np.concatenate([bf16_value(k0), bf16_value(k1)])
    vv = np.concatenate([bf16_value(v0), bf16_value(v1)])
    want = _dense_causal(bf16_value(q1), kk, vv, Hq, Hkv, n_before=n0, scale=0.3)
    assert np.abs(out - want).max() < 1e-12


def test_prefill_does_not_depend_on_the_chunking():
    Hq, Hkv, D, P = 4, 2, 64, 16
    lens = [50, 37]
    rng, table, kp, vp = _setup(3, 2, lens, Hq, Hkv, D, P)
    q, k, v = _tokens(rng, sum(lens), Hq, Hkv, D)
    kp1, vp1 = kp.copy(), vp.copy()
    whole = oracle.prefill_attn(q, k, v, [0, 1], [0, 0], [0, 50, 87], kp1, vp1, table, Hq, Hkv, D, P)
    # the same prompts cut as slot 0: 20 + 30, slot 1: 37, in one call (chunks of one slot in order)
    kp2, vp2 = kp.copy(), vp.copy()
    order = np.r_[0:20, 50:87, 20:50]
    cut = oracle.prefill_attn(q[order], k[order], v[order], [0, 1, 0], [0, 0, 20], [0, 20, 57, 87],
                              kp2, vp2, table, Hq, Hkv, D, P)
    back = np.empty_like(cut)
    back[order] = cut
    assert np.abs(back - whole).max() < 1e-12
    assert np.array_equal(kp1, kp2) and np.array_equal(vp1, vp2)
    # and in two calls
    kp3, vp3 = kp.copy(), vp.copy()
    a = oracle.prefill_attn(q[:20], k[:20], v[:20], [0], [0], [0, 20], kp3, vp3, table, Hq, Hkv, D, P)
    b = oracle.prefill_attn(q[20:50], k[20:50], v[20:50], [0], [20], [0, 30], kp3, vp3, table, Hq, Hkv, D, P)
    assert np.abs(np.concatenate([a, b]) - whole[:50]).max() < 1e-12


def test_last_prefill_token_is_a_decode_step_and_pages_hold_the_tokens():
    Hq, Hkv, D, P = 8, 2, 64, 16
    n = 40
    rng, table, kp, vp = _setup(4, 1, [n], Hq, Hkv, D, P)
    q, k, v = _tokens(rng, n, Hq, Hkv, D)
    out = oracle.prefill_attn(q, k, v, [0], [0], [0, n], kp, vp, table, Hq, Hkv, D, P)
    dec = oracle.decode_attn(np.ascontiguousarray(q[n - 1:n]), kp, vp, table, np.array([n], np.int32), Hq, Hkv, D, P)
    assert np.abs(dec[0] - out[n - 1]).max() < 1e-12
    for t in (0, 7, 15, 16, 39):
        for h in range(Hkv):
            for d in (0, 5, 63):
                page = int(table[0, t // P])
                assert kp[oracle.k_index(page, h, t % P, d, Hkv, D, P)] == k[t, h, d]
                assert vp[oracle.v_index(page, h, t % P, d, Hkv, D, P)] == v[t, h, d]


def test_prefill_is_causal():
    Hq, Hkv, D, P = 4, 1, 64, 32
    n = 33
    rng, table, kp, vp = _setup(5, 1, [n], Hq, Hkv, D, P)
    q, k, v = _tokens(rng, n, Hq, Hkv, D)
    a = oracle.prefill_attn(q, k, v, [0], [0], [0, n], kp.copy(), vp.copy(), table, Hq, Hkv, D, P)
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[20:] = bf16_bits(rng.normal(size=k2[20:].shape).astype(np.float32))
    v2[20:] = bf16_bits(rng.normal(size=v2[20:].shape).astype(np.float32))
    q2[20:] = bf16_bits(rng.normal(size=q2[20:].shape).astype(np.float32))
    b = oracle.prefill_attn(q2, k2, v2, [0], [0], [0, n], kp.copy(), vp.copy(), table, Hq, Hkv, D, P)
    assert np.array_equal(a[:20], b[:20])
    assert np.abs(a[20:] - b[20:]).max() > 1e-3
    # the first token sees only itself: its output is its own V row
    G = Hq // Hkv
    for h in range(Hq):
        assert np.abs(a[0, h] - bf16_value(v[0, h // G])).max() < 1e-15
