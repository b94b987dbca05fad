"""Pins for the oracle's Stage I saliency (Eq. 1) and TopK."""
import math

import numpy as np
import pytest
from scipy.special import softmax

import vitcop_inputs as I
from oracle import vitcop_oracle as O


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def small_case(seed, B=2, N=30, H=3, d=8):
    g = np.random.default_rng(seed)
    q = g.standard_normal((B, H, d)).astype(np.float32)
    k = g.standard_normal((B, N + 1, H, d)).astype(np.float32)
    return bits(q), bits(k)


@pytest.mark.parametrize("seed", range(3))
def test_equals_row0_of_textbook_attention(seed):
    # full (N+1)x(N+1) self-attention with a library softmax; Eq. 1 is its row 0
    qb, kb = small_case(seed)
    q = I.bf16_bits_to_f32(qb).astype(np.float64)
    k = I.bf16_bits_to_f32(kb).astype(np.float64)
    B, N1, H, d = k.shape
    g = np.random.default_rng(99)
    S = O.filter_scores(qb, kb)
    for b in range(B):
        acc = np.zeros(N1)
        for h in range(H):
            Q = g.standard_normal((N1, d))
            Q[0] = q[b, h]                       # only row 0 is the CLS query
            A = softmax(Q @ k[b, :, h, :].T / math.sqrt(d), axis=1)
            acc += A[0]
        assert np.allclose(S[b], acc[1:], rtol=1e-12, atol=1e-15)


def test_rows_sum_to_number_of_heads_when_cls_key_is_negligible():
    qb, kb = small_case(5, B=1, N=20, H=4, d=8)
    q = I.bf16_bits_to_f32(qb)
    k = I.bf16_bits_to_f32(kb).copy()
    k[0, 0] = -64.0 * q[0]                       # CLS logit hugely negative in every head
    S = O.filter_scores(qb, bits(k))
    assert abs(S.sum() - 4.0) < 1e-12


def test_uniform_keys_give_equal_scores_and_lowest_indices():
    H, d, N = 5, 16, 40
    q = np.random.default_rng(1).standard_normal((1, H, d)).astype(np.float32)
    k = np.tile(np.random.default_rng(2).standard_normal((1, 1, H, d)).astype(np.float32),
                (1, N + 1, 1, 1))
    S, idx = O.filter_visual(bits(q), bits(k), 9)
    assert np.allclose(S, H / (N + 1), rtol=1e-13)
    assert idx[0].tolist() == list(range(9))


def test_closed_form_one_hot_heads():
    # head 0 looks at patch a, head 1 at patch c; everything else has logit 0
    N, H, d = 10, 2, 4
    L = 8.0
    q = np.zeros((1, H, d), dtype=np.float32)
    q[0, :, 0] = L
    k = np.zeros((1, N + 1, H, d), dtype=np.float32)
    a, c = 3, 7                                    # patch indices (token = index + 1)
    k[0, a + 1, 0, 0] = 1.0
    k[0, c + 1, 1, 0] = 0.5
    S = O.filter_scores(bits(q), bits(k))[0]
    s = 1.0 / math.sqrt(d)
    za = math.exp(L * s) + N
    zc = math.exp(0.5 * L * s) + N
    exp = np.full(N, 1.0 / za + 1.0 / zc)
    exp[a] = math.exp(L * s) / za + 1.0 / zc
    exp[c] = 1.0 / za + math.exp(0.5 * L * s) / zc
    assert np.allclose(S, exp, rtol=1e-13)
    # explicit scale argument is honoured
    S2 = O.filter_scores(bits(q), bits(k), scale=0.25)[0]
    assert abs(S2[a] - (math.exp(2.0) / (math.exp(2.0) + N) + 1.0 / (math.exp(1.0) + N))) < 1e-13


def test_planted_patch_is_kept_and_cls_is_not_a_candidate():
    qb, kb = small_case(8, B=2, N=50, H=4, d=16)
    q = I.bf16_bits_to_f32(qb)
    k = I.bf16_bits_to_f32(kb).copy()
    k[:, 0] = 8.0 * q                              # CLS key grabs most attention itself
    k[0, 1 + 17] = 4.0 * q[0]
    k[1, 1 + 49] = 4.0 * q[1]
    S, idx = O.filter_visual(qb, bits(k), 1)
    assert idx.shape == (2, 1) and idx[0, 0] == 17 and idx[1, 0] == 49
    assert S.shape == (2, 50)


def test_config1_shape_counts():
    c = I.config1(B=2, N=64, C=128, H=4, d=32, n_centroids=8)
    S, idx = O.filter_visual(c["q_cls"], c["k"], c["keep"])
    assert idx.shape == (2, 32) and np.all(np.diff(idx, axis=1) > 0)
    assert idx.min() >= 0 and idx.max() < 64
