"""Pins for the oracle's paged GQA decode attention (CPU only).

Each test fixes the oracle to something other than itself: exact special
cases, closed forms, invariants, and a dense library computation.
"""
import numpy as np
import pytest
import scipy.special

import oracle
from oracle_helpers import build_paged, from_bf16_bits, k_slot_bits, to_bf16_bits


def rand_case(rng, B=3, Hq=8, Hkv=2, D=64, P=16, Lmax=70, lens=None):
    lens = rng.integers(1, Lmax + 1, size=B) if lens is None else np.asarray(lens)
    Lm = int(max(lens))
    K = rng.standard_normal((B, Lm, Hkv, D))
    V = rng.standard_normal((B, Lm, Hkv, D))
    Q = rng.standard_normal((B, Hq, D))
    return Q, K, V, lens.astype(np.int32)


def run(Q, K, V, lens, P, rng=None, scale=None):
    B, Hq, D = Q.shape
    Hkv = K.shape[2]
    kp, vp, table, Kr, Vr = build_paged(K, V, lens, P, rng)
    qb = to_bf16_bits(Q)
    out = oracle.decode_attn(qb, kp, vp, table, lens, Hq, Hkv, D, P, scale=scale)
    return out, from_bf16_bits(qb), Kr, Vr, (qb, kp, vp, table)


@pytest.mark.parametrize("P", [16, 32, 64])
def test_layout_index_formulas(P):
    # K: [page][h][d/8][kpos(t)][d%8]; V: [page][h][t/8][d][t%8] -- check against numpy reshapes
    Hkv, D, N = 2, 64, 3
    k = np.arange(N * Hkv * D * P).reshape(N, Hkv, D // 8, P, 8)
    v = np.arange(N * Hkv * D * P).reshape(N, Hkv, P // 8, D, 8)
    slots = [oracle.k_slot(t, P) for t in range(P)]
    assert sorted(slots) == list(range(P))                       # a permutation of the page
    assert slots == [k_slot_bits(t, P) for t in range(P)]
    # the first four of every eight tokens fill the first half of each block, in order
    W = min(P, 32)
    first_half = [t for t in range(W) if t % 8 < 4]
    assert [slots[t] for t in first_half] == list(range(W // 2))
    assert [slots[t] for t in range(W) if t % 8 >= 4] == list(range(W // 2, W))
    if P == 64:
        assert slots[32:] == [32 + s for s in slots[:32]]
    for (pg, h, t, d) in [(0, 0, 0, 0), (2, 1, P - 1, 63), (1, 0, 9, 17), (1, 1, 7, 8), (0, 1, 12, 5)]:
        assert oracle.k_index(pg, h, t, d, Hkv, D, P) == k[pg, h, d // 8, slots[t], d % 8]
        assert oracle.v_index(pg, h, t, d, Hkv, D, P) == v[pg, h, t // 8, d, t % 8]


def test_single_key_returns_its_value():
    rng = np.random.default_rng(0)
    Q, K, V, lens = rand_case(rng, lens=[1, 1, 1])
    out, _, _, Vr, _ = run(Q, K, V, lens, 16, rng)
    G = Q.shape[1] // K.shape[2]
    for b in range(3):
        for h in range(Q.shape[1]):
            assert np.array_equal(out[b, h], Vr[b, 0, h // G])  # exact bf16 value


def test_identical_keys_give_mean_of_values():
    rng = np.random.default_rng(1)
    Q, K, V, lens = rand_case(rng, lens=[37, 5, 64])
    K[:] = K[:, :1]  # every position of a row holds the same key
    out, _, _, Vr, _ = run(Q, K, V, lens, 16, rng)
    G = Q.shape[1] // K.shape[2]
    for b in range(3):
        for h in range(Q.shape[1]):
            np.testing.assert_allclose(out[b, h], Vr[b, :lens[b], h // G].mean(0), atol=1e-14)


def test_zero_query_gives_mean_of_values():
    rng = np.random.default_rng(2)
    Q, K, V, lens = rand_case(rng)
    Q[:] = 0
    out, _, _, Vr, _ = run(Q, K, V, lens, 16, rng)
    G = Q.shape[1] // K.shape[2]
    for b in range(len(lens)):
        np.testing.assert_allclose(out[b, 3], Vr[b, :lens[b], 3 // G].mean(0), atol=1e-14)


def test_dominant_key_selects_its_value():
    rng = np.random.default_rng(3)
    B, Hq, Hkv, D = 1, 2, 1, 64
    L, hot = 40, 23
    Q = np.zeros((B, Hq, D)); Q[..., 0] = 16.0
    K = rng.standard_normal((B, L, Hkv, D)); K[..., 0] = 0.0
    K[0, hot, 0, 0] = 32.0  # score 16*32/8 = 64 above all the others (which are 0)
    V = rng.standard_normal((B, L, Hkv, D))
    out, _, _, Vr, _ = run(Q, K, V, np.array([L], np.int32), 16)
    np.testing.assert_allclose(out[0, 0], Vr[0, hot, 0], atol=1e-15)


def test_two_keys_closed_form():
    # two keys: p_0 = sigmoid(s_0 - s_1)
    rng = np.random.default_rng(4)
    Q, K, V, lens = rand_case(rng, B=1, Hq=2, Hkv=1, D=64, lens=[2])
    out, Qr, Kr, Vr, _ = run(Q, K, V, lens, 16)
    for h in range(2):
        s = Kr[0, :2, 0] @ Qr[0, h] / 8.0
        p0 = 1.0 / (1.0 + np.exp(-(s[0] - s[1])))
        np.testing.assert_allclose(out[0, h], p0 * Vr[0, 0, 0] + (1 - p0) * Vr[0, 1, 0], atol=1e-14)


def test_output_in_convex_hull():
    rng = np.random.default_rng(5)
    Q, K, V, lens = rand_case(rng, B=4, Lmax=100)
    out, _, _, Vr, _ = run(Q, K, V, lens, 16, rng)
    G = Q.shape[1] // K.shape[2]
    for b in range(4):
        for h in range(Q.shape[1]):
            v = Vr[b, :lens[b], h // G]
            assert np.all(out[b, h] <= v.max(0) + 1e-12) and np.all(out[b, h] >= v.min(0) - 1e-12)


@pytest.mark.parametrize("P,D,Hq,Hkv", [(16, 64, 8, 2), (32, 128, 8, 1), (16, 128, 14, 2)])
def test_matches_dense_library_softmax(P, D, Hq, Hkv):
    rng = np.random.default_rng(6)
    Q, K, V, lens = rand_case(rng, B=3, Hq=Hq, Hkv=Hkv, D=D, P=P, Lmax=90)
    out, Qr, Kr, Vr, _ = run(Q, K, V, lens, P, rng)
    G = Hq // Hkv
    for b in range(3):
        L = lens[b]
        for h in range(Hq):
            s = Kr[b, :L, h // G] @ Qr[b, h] / np.sqrt(D)
            p = scipy.special.softmax(s)
            np.testing.assert_allclose(out[b, h], p @ Vr[b, :L, h // G], rtol=0, atol=2e-14)


def test_custom_scale():
    rng = np.random.default_rng(7)
    Q, K, V, lens = rand_case(rng, B=1, Hq=2, Hkv=1, lens=[33])
    out, Qr, Kr, Vr, _ = run(Q, K, V, lens, 16, scale=0.3)
    p = scipy.special.softmax(Kr[0, :33, 0] @ Qr[0, 1] * 0.3)
    np.testing.assert_allclose(out[0, 1], p @ Vr[0, :33, 0], atol=2e-14)


def test_page_permutation_invariance():
    rng = np.random.default_rng(8)
    Q, K, V, lens = rand_case(rng, B=3, Lmax=120)
    a, *_ = run(Q, K, V, lens, 16, None)
    b, *_ = run(Q, K, V, lens, 16, np.random.default_rng(99))
    assert np.array_equal(a, b)  # same logical cache, different physical pages: identical bits


def test_gqa_heads_of_a_group_share_kv():
    rng = np.random.default_rng(9)
    Q, K, V, lens = rand_case(rng, B=2, Hq=8, Hkv=2)
    Q[:, 1:4] = Q[:, :1]      # heads 0..3 form KV group 0
    Q[:, 4] = Q[:, 0]         # head 4 uses KV head 1: must differ
    out, *_ = run(Q, K, V, lens, 16, rng)
    for h in (1, 2, 3):
        assert np.array_equal(out[:, h], out[:, 0])
    assert not np.allclose(out[:, 4], out[:, 0])


def test_split_and_lse_merge_equals_whole():
    # the split-K identity the GPU path relies on, checked on the oracle's own pieces
    rng = np.random.default_rng(10)
    Q, K, V, lens = rand_case(rng, B=1, Hq=4, Hkv=2, lens=[77])
    out, _, _, _, (qb, kp, vp, table) = run(Q, K, V, lens, 16, rng)
    for h in range(4):
        for a in (1, 16, 40, 76):
            m1, l1, acc1 = oracle.attn_range(qb, kp, vp, table, 0, h, 0, a, 4, 2, 64, 16)
            m2, l2, acc2 = oracle.attn_range(qb, kp, vp, table, 0, h, a, 77, 4, 2, 64, 16)
            M = max(m1, m2)
            l = l1 * np.exp(m1 - M) + l2 * np.exp(m2 - M)
            merged = (acc1 * np.exp(m1 - M) + acc2 * np.exp(m2 - M)) / l
            np.testing.assert_allclose(merged, out[0, h], atol=1e-12)
    m0, l0, acc0 = oracle.attn_range(qb, kp, vp, table, 0, 0, 5, 5, 4, 2, 64, 16)
    assert m0 == -np.inf and l0 == 0 and not acc0.any()


def test_zero_length_row_gives_zeros_and_rows_subset():
    rng = np.random.default_rng(11)
    Q, K, V, lens = rand_case(rng, B=3, lens=[9, 1, 30])
    lens2 = lens.copy(); lens2[1] = 0
    kp, vp, table, _, _ = build_paged(K, V, lens, 16, rng)
    qb = to_bf16_bits(Q)
    full = oracle.decode_attn(qb, kp, vp, table, lens2, 8, 2, 64, 16)
    assert not full[1].any()
    sub = oracle.decode_attn(qb, kp, vp, table, lens2, 8, 2, 64, 16, rows=[2])
    assert np.array_equal(sub[2], full[2]) and not sub[0].any()
