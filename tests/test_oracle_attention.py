"""Pins of the oracle's block-sparse attention: Eq. (1), the candidate-set form of Sec. 5.1 and Lemma 1."""
import numpy as np
import pytest
from scipy.special import logsumexp

import oracle
from workloads import f32_to_bf16_bits, bf16_bits_to_f32


def dense_attention(Q, K, V, scale, mask=None, bias=None):
    """Textbook softmax attention in float64 (Eq. 1), optional boolean mask [n_q, n_k] and logit bias [n_k]."""
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * scale
    if bias is not None:
        S = S + bias[None, :]
    if mask is not None:
        S = np.where(mask, S, -np.inf)
    lse = logsumexp(S, axis=1)
    P = np.exp(S - lse[:, None])
    return P @ V.astype(np.float64), lse


def rand_qkv(rng, H, n_q, C, d):
    return (rng.standard_normal((H, n_q, d)).astype(np.float32),
            rng.standard_normal((H, C, d)).astype(np.float32),
            rng.standard_normal((H, C, d)).astype(np.float32))


def test_full_selection_is_dense_attention():
    rng = np.random.default_rng(0)
    H, n_q, C, d, BQ, BK = 2, 70, 200, 64, 32, 64          # ragged query and key tails
    Q, K, V = rand_qkv(rng, H, n_q, C, d)
    length = np.array([200, 137], np.int32)
    sel, nsel = oracle.full_selection(H, n_q, BQ, length, BK)
    O, lse = oracle.sparse_attn_fwd(Q, K, V, None, length, sel, nsel, BQ, BK, d ** -0.5)
    for h in range(H):
        L = length[h]
        Od, lsed = dense_attention(Q[h], K[h, :L], V[h, :L], d ** -0.5)
        assert np.abs(O[h] - Od).max() < 1e-5       # the invariant's bound; fp64 agrees far tighter
        assert np.abs(O[h] - Od).max() < 1e-12
        assert np.abs(lse[h] - lsed).max() < 1e-12


def test_selection_equals_masked_dense():
    rng = np.random.default_rng(1)
    H, n_q, C, d, BQ, BK, n_sel = 3, 100, 300, 32, 32, 16, 5
    Q, K, V = rand_qkv(rng, H, n_q, C, d)
    length = np.array([300, 250, 41], np.int32)
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        n_kb = (length[h] + BK - 1) // BK
        for b in range(n_qb):
            m = int(rng.integers(1, min(n_sel, n_kb) + 1))
            sel[h, b, :m] = np.sort(rng.choice(n_kb, size=m, replace=False))
            nsel[h, b] = m
    O, lse = oracle.sparse_attn_fwd(Q, K, V, None, length, sel, nsel, BQ, BK, 0.2)
    for h in range(H):
        L = length[h]
        mask = np.zeros((n_q, L), bool)
        for b in range(n_qb):
            for kb in sel[h, b, :nsel[h, b]]:
                mask[b * BQ:(b + 1) * BQ, kb * BK:min((kb + 1) * BK, L)] = True
        Od, lsed = dense_attention(Q[h], K[h, :L], V[h, :L], 0.2, mask=mask)
        assert np.abs(O[h] - Od).max() < 1e-12
        assert np.abs(lse[h] - lsed).max() < 1e-12


def test_lemma1_duplicate_keys_equal_grouped_attention_with_log_m_bias():
    # keys with exact duplicates: dense attention over all copies == attention over one
    # representative per group with multiplicity m_t (logit + log m_t) and the group's mean value
    rng = np.random.default_rng(2)
    g, d, n_q = 37, 64, 50
    reps = rng.standard_normal((g, d)).astype(np.float32)
    mult = rng.integers(1, 6, size=g)
    idx = np.repeat(np.arange(g), mult)
    perm = rng.permutation(idx.size)
    idx = idx[perm]
    K = reps[idx]
    V = rng.standard_normal((idx.size, d)).astype(np.float32)
    Q = rng.standard_normal((n_q, d)).astype(np.float32)
    Od, lsed = dense_attention(Q, K, V, d ** -0.5)
    Vmean = np.stack([V[idx == t].astype(np.float64).mean(axis=0) for t in range(g)])
    # grouped cache as the oracle sees it (fp32 storage of the mean value)
    C = 64
    Kc = np.zeros((1, C, d), np.float32); Kc[0, :g] = reps
    Vc = np.zeros((1, C, d), np.float32); Vc[0, :g] = Vmean.astype(np.float32)
    cnt = np.ones((1, C), np.int32); cnt[0, :g] = mult
    length = np.array([g], np.int32)
    sel, nsel = oracle.full_selection(1, n_q, 16, length, 8)
    O, lse = oracle.sparse_attn_fwd(Q[None], Kc, Vc, cnt, length, sel, nsel, 16, 8, d ** -0.5)
    assert np.abs(O[0] - Od).max() < 1e-5
    assert np.abs(lse[0] - lsed).max() < 1e-9
    # and without the bias / with plain (unweighted) values the identity must fail: guards a dropped term
    O_nobias, _ = oracle.sparse_attn_fwd(Q[None], Kc, Vc, None, length, sel, nsel, 16, 8, d ** -0.5)
    assert np.abs(O_nobias[0] - Od).max() > 1e-3


def test_unit_multiplicities_are_bitwise_the_unbiased_path():
    rng = np.random.default_rng(3)
    Q, K, V = rand_qkv(rng, 2, 40, 96, 32)
    length = np.array([96, 50], np.int32)
    sel, nsel = oracle.full_selection(2, 40, 8, length, 16)
    a = oracle.sparse_attn_fwd(Q, K, V, None, length, sel, nsel, 8, 16, 0.17)
    b = oracle.sparse_attn_fwd(Q, K, V, np.ones((2, 96), np.int32), length, sel, nsel, 8, 16, 0.17)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_bias_is_natural_log_added_after_scaling():
    # one query, two orthogonal unit keys, q = 0: logits are ln(cnt) alone -> weights cnt / sum(cnt)
    Q = np.zeros((1, 1, 4), np.float32)
    K = np.zeros((1, 2, 4), np.float32); K[0, 0, 0] = 1; K[0, 1, 1] = 1
    V = np.zeros((1, 2, 4), np.float32); V[0, 0, 0] = 1; V[0, 1, 1] = 1
    cnt = np.array([[3, 1]], np.int32)
    sel = np.array([[[0]]], np.int32); nsel = np.array([[1]], np.int32)
    O, lse = oracle.sparse_attn_fwd(Q, K, V, cnt, np.array([2], np.int32), sel, nsel, 1, 2, 123.0)
    assert np.allclose(O[0, 0], [0.75, 0.25, 0, 0], atol=1e-15)
    assert abs(lse[0, 0] - np.log(4.0)) < 1e-15


def test_empty_selection_gives_zero_output_and_minus_inf_lse():
    rng = np.random.default_rng(4)
    Q, K, V = rand_qkv(rng, 1, 10, 32, 16)
    sel = np.full((1, 2, 3), -1, np.int32)
    nsel = np.zeros((1, 2), np.int32)
    O, lse = oracle.sparse_attn_fwd(Q, K, V, None, np.array([32], np.int32), sel, nsel, 8, 8, 1.0)
    assert not O.any() and np.all(np.isneginf(lse))
    # a listed block that lies wholly beyond len contributes nothing either
    sel[0, :, 0] = 3
    nsel[:] = 1
    O, lse = oracle.sparse_attn_fwd(Q, K, V, None, np.array([20], np.int32), sel, nsel, 8, 8, 1.0)
    assert not O.any() and np.all(np.isneginf(lse))


def test_keys_beyond_len_are_invisible():
    rng = np.random.default_rng(5)
    Q, K, V = rand_qkv(rng, 1, 16, 64, 16)
    length = np.array([37], np.int32)
    sel, nsel = oracle.full_selection(1, 16, 8, length, 16)
    a = oracle.sparse_attn_fwd(Q, K, V, None, length, sel, nsel, 8, 16, 0.25)[0]
    K2, V2 = K.copy(), V.copy()
    K2[0, 37:] = 1e3; V2[0, 37:] = -1e3
    b = oracle.sparse_attn_fwd(Q, K2, V2, None, length, sel, nsel, 8, 16, 0.25)[0]
    assert np.array_equal(a, b)


def test_bf16_storage_is_read_as_its_exact_value():
    rng = np.random.default_rng(6)
    Q, K, V = rand_qkv(rng, 1, 24, 48, 32)
    Qb, Kb, Vb = (f32_to_bf16_bits(t) for t in (Q, K, V))
    length = np.array([48], np.int32)
    sel, nsel = oracle.full_selection(1, 24, 8, length, 16)
    a = oracle.sparse_attn_fwd(Qb, Kb, Vb, None, length, sel, nsel, 8, 16, 0.3)
    b = oracle.sparse_attn_fwd(bf16_bits_to_f32(Qb), bf16_bits_to_f32(Kb), bf16_bits_to_f32(Vb), None, length,
                               sel, nsel, 8, 16, 0.3)
    assert np.array_equal(a[0], b[0])


def test_recall_and_density_definitions():
    # recall = kept softmax mass of the dense attention; density = kept pairs / all pairs
    rng = np.random.default_rng(7)
    H, n_q, C, d, BQ, BK = 2, 32, 64, 16, 16, 8
    Q, K, V = rand_qkv(rng, H, n_q, C, d)
    length = np.array([64, 45], np.int32)
    cnt = rng.integers(1, 4, size=(H, C)).astype(np.int32)
    sel = np.array([[[0, 3, -1], [1, 2, 5]], [[0, 5, -1], [4, -1, -1]]], np.int32)
    nsel = np.array([[2, 3], [2, 1]], np.int32)
    rec, den = oracle.recall_density(Q, K, cnt, length, sel, nsel, BQ, BK, 0.5)
    r_sum, kept_pairs, all_pairs = 0.0, 0, 0
    for h in range(H):
        L = length[h]
        S = (Q[h].astype(np.float64) @ K[h, :L].astype(np.float64).T) * 0.5 + np.log(cnt[h, :L])[None]
        P = np.exp(S - logsumexp(S, axis=1)[:, None])
        for i in range(n_q):
            b = i // BQ
            m = np.zeros(L, bool)
            for kb in sel[h, b, :nsel[h, b]]:
                m[kb * BK:min((kb + 1) * BK, L)] = True
            r_sum += P[i, m].sum(); kept_pairs += m.sum(); all_pairs += L
    assert abs(rec - r_sum / (H * n_q)) < 1e-12
    assert abs(den - kept_pairs / all_pairs) < 1e-12
    full = oracle.full_selection(H, n_q, BQ, length, BK)
    rec, den = oracle.recall_density(Q, K, cnt, length, *full, BQ, BK, 0.5)
    assert abs(rec - 1) < 1e-12 and abs(den - 1) < 1e-12
