"""Pins for the oracle's K-norm saliency (Eq. 4) and Stage III selection."""
import numpy as np
import pytest

import vitcop_inputs as I
from oracle import vitcop_oracle as O


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_planted_powers_of_two():
    # rows g_i * e_1 with g_i a power of two: the norm is g_i exactly
    B, T, H, d = 1, 12, 4, 8
    k = np.zeros((B, T, H, d), dtype=np.float32)
    g = 2.0 ** np.array([3, -2, 0, 5, -4, 1, 2, -1, 4, -3, 6, -5], dtype=np.float32)
    k[0, :, 0, 0] = g
    n = O.k_norms(bits(k), 0, T)
    assert np.array_equal(n[0], g.astype(np.float64))
    # the 4 smallest gains sit at positions 1 (1/4), 4 (1/16), 9 (1/8), 11 (1/32)
    _, idx = O.knorm_select(bits(k), 0, T, 4)
    assert idx[0].tolist() == [1, 4, 9, 11]


def test_norm_spans_all_heads_and_takes_sqrt():
    # 3 in head 0 and 4 in head 5 -> norm 5 (a per-head or squared norm fails)
    k = np.zeros((1, 3, 6, 4), dtype=np.float32)
    k[0, 1, 0, 2] = 3.0
    k[0, 1, 5, 3] = -4.0
    k[0, 2, 2, 0] = 1.0
    k[0, 2, 3, 1] = 1.0
    n = O.k_norms(bits(k), 0, 3)[0]
    assert n[0] == 0.0 and n[1] == 5.0 and abs(n[2] - np.sqrt(2.0)) < 1e-15


def test_matches_library_norm():
    c = I.k_tensor_lognormal(5, 2, 50, 4, 16, 7, 30)
    n = O.k_norms(c["k"], 7, 30)
    rows = I.bf16_bits_to_f32(c["k"]).astype(np.float64).reshape(2, 50, -1)[:, 7:37]
    assert np.allclose(n, np.linalg.norm(rows, axis=2), rtol=1e-13, atol=0)


def test_only_visual_span_is_ranked():
    # text rows have the smallest norms but are not candidates; they are kept anyway
    B, T, H, d, vs, nv = 1, 20, 2, 8, 4, 10
    k = np.ones((B, T, H, d), dtype=np.float32)
    k[0, :vs] = 0.001
    k[0, vs + nv:] = 0.001
    k[0, vs + 3] = 0.5
    k[0, vs + 8] = 0.25
    nrm, idx = O.knorm_select(bits(k), vs, nv, 2)
    assert nrm.shape == (1, nv)
    assert idx[0].tolist() == [0, 1, 2, 3, vs + 3, vs + 8] + list(range(vs + nv, T))


@pytest.mark.parametrize("p", [-6, -1, 3, 9])
def test_power_of_two_scaling_leaves_selection_unchanged(p):
    c = I.k_tensor_lognormal(11, 2, 64, 2, 16, 3, 48)
    base = O.knorm_select(c["k"], 3, 48, 11)[1]
    scaled = bits(I.bf16_bits_to_f32(c["k"]) * np.float32(2.0 ** p))
    assert np.array_equal(O.knorm_select(scaled, 3, 48, 11)[1], base)


def test_pair_rotation_leaves_selection_unchanged_outside_band():
    # a RoPE-style rotation of (even, odd) pairs preserves every head's norm
    c = I.k_tensor_lognormal(12, 1, 80, 2, 16, 0, 80)
    k = I.bf16_bits_to_f32(c["k"]).astype(np.float64)
    g = np.random.default_rng(0)
    theta = g.random((1, 80, 2, 8)) * 2 * np.pi
    a, b = k[..., 0::2], k[..., 1::2]
    rot = np.empty_like(k)
    rot[..., 0::2] = a * np.cos(theta) - b * np.sin(theta)
    rot[..., 1::2] = a * np.sin(theta) + b * np.cos(theta)
    keep = 20
    n0, i0 = O.knorm_select(c["k"], 0, 80, keep)
    n1, i1 = O.knorm_select(bits(rot), 0, 80, keep)
    assert np.allclose(n0, n1, rtol=4e-3)           # bf16 re-rounding only
    band = O.tie_band(n0[0], keep, largest=False, rel=1e-2)
    s0 = set(i0[0].tolist()) - set(np.nonzero(band)[0].tolist())
    s1 = set(i1[0].tolist()) - set(np.nonzero(band)[0].tolist())
    assert s0 == s1 and len(i1[0]) == keep


def test_outliers_never_kept_on_schedule_shaped_input():
    c = I.k_tensor_lognormal(I.seed_for(2), 1, 640, 4, 32, 35, 576)
    assert c["outlier"].sum() == 29
    for keep in (192, 128, 64):
        _, idx = O.knorm_select(c["k"], 35, 576, keep)
        vis = idx[0, 35:35 + keep] - 35
        assert not c["outlier"][0, vis].any()
        # norms follow the planted gains: kept tokens have the smallest gains
        thr = np.sort(c["gain"][0])[keep - 1]
        assert np.mean(c["gain"][0, vis] <= thr * 1.1) > 0.9
