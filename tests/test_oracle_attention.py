"""Pins for the oracle's attention (exact causal softmax(QK^T)V)."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import vitcop_inputs as I
from oracle import vitcop_oracle as O


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def f64(b):
    return I.bf16_bits_to_f32(b).astype(np.float64)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (6, 2)])
def test_matches_library_sdpa(causal, Hq, Hkv):
    t = I.qkv_tensors(21, 2, 37, Hq, Hkv, 16)
    out, lse = O.attention(t["q"], t["k"], t["v"], None, causal)
    q = torch.from_numpy(f64(t["q"])).permute(0, 2, 1, 3)
    k = torch.from_numpy(f64(t["k"])).permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    v = torch.from_numpy(f64(t["v"])).permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=causal)
    assert np.allclose(out, ref.permute(0, 2, 1, 3).numpy(), rtol=1e-11, atol=1e-13)


def test_matches_scipy_softmax_and_logsumexp():
    t = I.qkv_tensors(22, 1, 19, 2, 1, 8)
    out, lse = O.attention(t["q"], t["k"], t["v"], 0.3, True)
    q, k, v = f64(t["q"]), f64(t["k"]), f64(t["v"])
    for h in range(2):
        s = q[0, :, h] @ k[0, :, 0].T * 0.3
        s[np.triu_indices(19, 1)] = -np.inf
        assert np.allclose(out[0, :, h], softmax(s, axis=1) @ v[0, :, 0], rtol=1e-12)
        assert np.allclose(lse[0, h], logsumexp(s, axis=1), rtol=1e-12, atol=1e-12)


def test_constant_values_and_first_row():
    t = I.qkv_tensors(23, 1, 25, 2, 2, 8)
    ones = bits(np.ones((1, 25, 2, 8)))
    out, _ = O.attention(t["q"], t["k"], ones, None, True)
    assert np.allclose(out, 1.0, rtol=0, atol=1e-14)
    out, _ = O.attention(t["q"], t["k"], t["v"], None, True)
    assert np.allclose(out[0, 0], f64(t["v"])[0, 0], rtol=1e-14)     # row 0 sees only key 0


def test_equal_keys_give_running_mean_of_values():
    t = I.qkv_tensors(24, 1, 12, 1, 1, 8)
    k = np.tile(f64(t["k"])[:, :1], (1, 12, 1, 1))
    out, lse = O.attention(t["q"], bits(k), t["v"], None, True)
    v = f64(t["v"])[0, :, 0]
    run = np.cumsum(v, axis=0) / np.arange(1, 13)[:, None]
    assert np.allclose(out[0, :, 0], run, rtol=1e-13)
    out_nc, _ = O.attention(t["q"], bits(k), t["v"], None, False)
    assert np.allclose(out_nc[0, :, 0], np.tile(v.mean(axis=0), (12, 1)), rtol=1e-13)


def test_two_token_closed_form():
    d = 4
    q = np.zeros((1, 2, 1, d)); k = np.zeros((1, 2, 1, d)); v = np.zeros((1, 2, 1, d))
    q[0, 1, 0, 0] = 2.0
    k[0, 0, 0, 0] = 1.0
    k[0, 1, 0, 0] = -1.0
    v[0, 0, 0] = [1, 2, 3, 4]
    v[0, 1, 0] = [-1, 0, 1, 2]
    out, lse = O.attention(bits(q), bits(k), bits(v), None, True)
    # logits of row 1: +2/sqrt(4) = 1 for key 0, -1 for key 1
    w0 = math.exp(1.0) / (math.exp(1.0) + math.exp(-1.0))
    assert np.allclose(out[0, 1, 0], w0 * np.array([1, 2, 3, 4]) + (1 - w0) * np.array([-1, 0, 1, 2]),
                       rtol=1e-14)
    assert abs(lse[0, 0, 1] - math.log(math.exp(1.0) + math.exp(-1.0))) < 1e-14
    assert abs(lse[0, 0, 0] - 0.0) < 1e-14


def test_gqa_head_mapping():
    # q-heads 0..2 read kv-head 0, q-heads 3..5 read kv-head 1
    t = I.qkv_tensors(25, 1, 9, 6, 2, 8)
    out, _ = O.attention(t["q"], t["k"], t["v"], None, True)
    for h in range(6):
        single, _ = O.attention(t["q"][:, :, h:h + 1], t["k"][:, :, h // 3:h // 3 + 1],
                                t["v"][:, :, h // 3:h // 3 + 1], None, True)
        assert np.array_equal(out[:, :, h], single[:, :, 0])


def test_row_sampler_agrees_with_full():
    t = I.qkv_tensors(26, 2, 33, 4, 2, 16)
    out, _ = O.attention(t["q"], t["k"], t["v"], None, True)
    rows = [0, 5, 32]
    got = O.attention_rows(t["q"], t["k"], t["v"], 1, 3, rows)
    assert np.allclose(got, out[1, rows, 3], rtol=1e-12, atol=1e-14)
