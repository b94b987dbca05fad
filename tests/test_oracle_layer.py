"""Pins for compaction, bf16 rounding, projections, the layer and the schedule."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O


def f64(b):
    return I.bf16_bits_to_f32(b).astype(np.float64)


def test_compact_is_index_select():
    g = np.random.default_rng(0)
    src = g.integers(0, 65535, size=(3, 20, 6), dtype=np.uint16)
    idx = np.sort(g.permuted(np.tile(np.arange(20), (3, 1)), axis=1)[:, :8], axis=1).astype(np.int32)
    got = O.compact(src, idx)
    assert np.array_equal(got, np.take_along_axis(src, idx[:, :, None].astype(np.int64), axis=1))
    ident = np.tile(np.arange(20, dtype=np.int32), (3, 1))
    assert np.array_equal(O.compact(src, ident), src)
    # composition of two compactions = compaction by composed indices
    idx2 = np.tile(np.array([0, 3, 7], dtype=np.int32), (3, 1))
    composed = np.take_along_axis(idx, idx2, axis=1)
    assert np.array_equal(O.compact(O.compact(src, idx), idx2), O.compact(src, composed))


def test_bf16_rounding_single_step():
    # agrees with the library's float32 -> bf16 rounding on float32 inputs
    g = np.random.default_rng(1)
    x = (g.standard_normal(20000) * np.exp(g.standard_normal(20000) * 3)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.f64_to_bf16_bits(x.astype(np.float64)), ref)
    assert np.array_equal(I.f32_to_bf16_bits(x), ref)
    # halfway cases go to even; just above halfway goes up even when a float32
    # detour would have landed exactly on the tie
    one = 1.0
    assert O.f64_to_bf16_bits(np.array([one + 2.0 ** -8]))[0] == 0x3F80          # tie -> even
    assert O.f64_to_bf16_bits(np.array([one + 3 * 2.0 ** -8]))[0] == 0x3F82      # tie -> even (up)
    assert O.f64_to_bf16_bits(np.array([one + 2.0 ** -8 + 2.0 ** -30]))[0] == 0x3F81
    assert O.f64_to_bf16_bits(np.array([-0.75]))[0] == 0xBF40
    assert np.array_equal(O.bf16_to_f64(np.array([0x3F80, 0xBF40, 0x4049], dtype=np.uint16)),
                          [1.0, -0.75, 3.140625])


def test_project_matches_library_matmul():
    c = I.layer_inputs(3, 2, 10, 32, 2, 2, 8, 0, 10)
    y = O.project(c["x"], c["wk"])
    ref = torch.from_numpy(f64(c["x"])) @ torch.from_numpy(f64(c["wk"])).T
    assert y.shape == (2, 10, 16) and np.allclose(y, ref.numpy(), rtol=1e-13, atol=1e-15)


def tiny_layer(seed=4, keep=6):
    c = I.layer_inputs(seed, 2, 24, 32, 4, 2, 8, 5, 12, w_std=0.2)
    return c, O.pruned_layer(c["x"], c["wq"], c["wk"], c["wv"], c["wo"], 4, 2, 8, 5, 12, keep)


def test_pruned_layer_with_full_budget_is_the_unpruned_layer():
    c = I.layer_inputs(4, 2, 24, 32, 4, 2, 8, 5, 12, w_std=0.2)
    p = O.pruned_layer(c["x"], c["wq"], c["wk"], c["wv"], c["wo"], 4, 2, 8, 5, 12, 12, residual=True)
    u = O.unpruned_layer(c["x"], c["wq"], c["wk"], c["wv"], c["wo"], 4, 2, 8, residual=True)
    assert np.array_equal(p["keep_idx"], np.tile(np.arange(24), (2, 1)))
    assert np.array_equal(p["y_bits"], u["y_bits"]) and np.array_equal(p["q"], u["q"])


def test_pruned_layer_equals_library_attention_on_gathered_rows():
    c, p = tiny_layer()
    idx = p["keep_idx"]
    assert idx.shape == (2, 24 - 12 + 6)
    x = torch.from_numpy(f64(c["x"]))
    xs = torch.stack([x[b, torch.from_numpy(idx[b].astype(np.int64))] for b in range(2)])

    def lin(t, w):
        y = t @ torch.from_numpy(f64(w)).T
        return y.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    # the library rounds through float32 (two rounding steps), so Q/K/V can differ
    # from the oracle's by one bf16 ulp: compare the attention output with a tolerance
    q = lin(xs, c["wq"]).reshape(2, 18, 4, 8).permute(0, 2, 1, 3)
    k = lin(xs, c["wk"]).reshape(2, 18, 2, 8).permute(0, 2, 1, 3).repeat_interleave(2, dim=1)
    v = lin(xs, c["wv"]).reshape(2, 18, 2, 8).permute(0, 2, 1, 3).repeat_interleave(2, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3)
    assert np.allclose(p["attn"], ref.numpy(), rtol=0, atol=0.05)
    assert np.abs(p["attn"] - ref.numpy()).mean() < 2e-3
    # K of survivors is gathered, not recomputed: identical bits
    assert np.array_equal(p["k_kept"], O.compact(p["k"], idx))
    # the ranking used this layer's own K
    n_ref = np.linalg.norm(f64(p["k"]).reshape(2, 24, -1)[:, 5:17], axis=2)
    assert np.allclose(p["norms"], n_ref, rtol=1e-13)


def test_schedule_counts_positions_and_unpruned_limit():
    cfg = I.layer_inputs(6, 1, 40, 32, 4, 2, 8, 4, 30, w_std=0.1)
    ws = {l: I.layer_inputs(60 + l, 1, 1, 32, 4, 2, 8, 0, 0, w_std=0.1) for l in range(5)}
    r = O.schedule_prefill(cfg["x"], lambda l: ws[l], 5, ((1, 20), (3, 8)), 4, 2, 8, 4, 30)
    lens = [lay["x_in"].shape[1] for lay in r["layers"]]
    assert lens == [40, 40, 30, 30, 18] and r["h"].shape == (1, 18, 32)
    pos = r["positions"][0]
    assert np.all(np.diff(pos) > 0) and pos[:4].tolist() == [0, 1, 2, 3]
    assert pos[-6:].tolist() == list(range(34, 40))
    # budgets equal to the current count change nothing: equals a chain of unpruned layers
    r2 = O.schedule_prefill(cfg["x"], lambda l: ws[l], 3, ((1, 30),), 4, 2, 8, 4, 30)
    h = cfg["x"]
    for l in range(3):
        h = O.unpruned_layer(h, ws[l]["wq"], ws[l]["wk"], ws[l]["wv"], ws[l]["wo"], 4, 2, 8,
                             residual=True)["y_bits"]
    assert np.array_equal(r2["h"], h)
    # second pruning ranks only the survivors of the first
    first = set(r["layers"][1]["keep_idx"][0].tolist())
    second_pos = r["layers"][1]["keep_idx"][0][r["layers"][3]["keep_idx"][0]]
    assert set(second_pos.tolist()) <= first and np.array_equal(second_pos, pos)
