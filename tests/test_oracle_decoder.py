"""Pins of the decoder-layer oracle against library routines and closed forms."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import vitcop_inputs as I
from oracle import decoder_oracle as Dc
from oracle import vitcop_oracle as O


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def f64(b):
    return O.bf16_to_f64(b)


def test_rmsnorm_matches_library():
    x = I.normal_bf16(1, 0, (5, 7, 96), 2.0)
    w = I.normal_bf16(1, 1, (96,), 1.0)
    got = Dc.rmsnorm(x, w, 1e-5)
    want = F.rms_norm(torch.from_numpy(f64(x)), (96,), torch.from_numpy(f64(w)), 1e-5).numpy()
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    # closed form: a constant row c with unit weight maps to c / sqrt(c^2 + eps)
    c = Dc.rmsnorm(bits(np.full((1, 8), 3.0)), bits(np.ones(8)), 0.25)
    assert np.allclose(c, 3.0 / np.sqrt(9.25))


def test_silu_mul_matches_library():
    g = I.normal_bf16(2, 0, (33, 40), 3.0)
    u = I.normal_bf16(2, 1, (33, 40), 1.0)
    want = (F.silu(torch.from_numpy(f64(g))) * torch.from_numpy(f64(u))).numpy()
    assert np.allclose(Dc.silu_mul(g, u), want, rtol=1e-13, atol=1e-15)


def test_rope_closed_forms_and_invariants():
    # d = 2: a single pair rotating by `position` radians (theta^0 = 1)
    x = bits(np.array([1.0, 0.0]).reshape(1, 1, 1, 2).repeat(4, axis=1))
    pos = np.array([[0, 1, 2, 7]])
    r = Dc.rope(x, pos, 10000.0)
    assert np.allclose(r[0, :, 0, 0], np.cos([0, 1, 2, 7])) and np.allclose(r[0, :, 0, 1], np.sin([0, 1, 2, 7]))
    # d = 4: channel 1 pairs with channel 3 and turns by position * theta^(-1/2)
    y = bits(np.array([0.0, 2.0, 0.0, 0.0]).reshape(1, 1, 1, 4))
    r = Dc.rope(y, np.array([[3]]), 100.0)
    assert np.allclose(r[0, 0, 0], [0.0, 2 * np.cos(0.3), 0.0, 2 * np.sin(0.3)])
    # position 0 is the identity; norms of pairs are preserved; scores depend on position differences only
    t = I.qkv_tensors(9, 2, 6, 3, 3, 64)
    pos = np.array([[0, 3, 4, 10, 11, 40], [5, 6, 7, 8, 9, 10]])
    q, k = Dc.rope(t["q"], pos, 10000.0), Dc.rope(t["k"], pos, 10000.0)
    assert np.array_equal(q[0, 0], f64(t["q"])[0, 0])
    assert np.allclose((q ** 2).sum(-1), (f64(t["q"]) ** 2).sum(-1), rtol=1e-12)
    q2, k2 = Dc.rope(t["q"], pos + 17, 10000.0), Dc.rope(t["k"], pos + 17, 10000.0)
    s1 = np.einsum("bnhd,bmhd->bhnm", q, k)
    s2 = np.einsum("bnhd,bmhd->bhnm", q2, k2)
    assert np.allclose(s1, s2, rtol=1e-9, atol=1e-9)


def torch_reference_layer(h, w, Hq, Hkv, d, positions, eps, theta):
    """The same layer with library ops in float64 and no intermediate rounding (no pruning)."""
    t = lambda b: torch.from_numpy(f64(b))
    B, T, D = h.shape
    x = t(h)
    a = F.rms_norm(x, (D,), t(w["ln1"]), eps)
    q = (a @ t(w["wq"]).T).reshape(B, T, Hq, d).transpose(1, 2)
    k = (a @ t(w["wk"]).T).reshape(B, T, Hkv, d).transpose(1, 2)
    v = (a @ t(w["wv"]).T).reshape(B, T, Hkv, d).transpose(1, 2)
    half = d // 2
    inv = theta ** (-torch.arange(half, dtype=torch.float64) * 2 / d)
    ang = torch.from_numpy(np.asarray(positions, dtype=np.float64))[:, None, :, None] * inv
    cos, sin = torch.cat([ang.cos(), ang.cos()], -1), torch.cat([ang.sin(), ang.sin()], -1)
    rot = lambda z: torch.cat([-z[..., half:], z[..., :half]], -1)
    q, k = q * cos + rot(q) * sin, k * cos + rot(k) * sin
    k = k.repeat_interleave(Hq // Hkv, dim=1)
    v = v.repeat_interleave(Hq // Hkv, dim=1)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B, T, Hq * d)
    h1 = x + o @ t(w["wo"]).T
    b = F.rms_norm(h1, (D,), t(w["ln2"]), eps)
    m = F.silu(b @ t(w["wg"]).T) * (b @ t(w["wu"]).T)
    return (h1 + m @ t(w["wd"]).T).numpy()


def test_unpruned_layer_matches_library_composition():
    c = I.decoder_inputs(77, 2, 40, 128, 4, 2, 64, 96)
    pos = np.tile(np.arange(40), (2, 1))
    r = Dc.decoder_layer(c["h"], c["w"], 4, 2, 64, 5, 30, 30, pos)
    want = torch_reference_layer(c["h"], c["w"], 4, 2, 64, pos, 1e-5, 10000.0)
    assert np.array_equal(r["keep_idx"], np.tile(np.arange(40), (2, 1)))
    # the oracle rounds every stored tensor to bf16 (relative 2^-9 each), the library route does not
    assert np.abs(r["y"] - want).max() <= 3e-2 * np.abs(want).max()
    assert np.mean(np.abs(r["y"] - want)) <= 4e-3 * np.mean(np.abs(want))


def test_pruned_layer_is_the_library_layer_on_the_survivors_prefix_property():
    # Pruning only tokens AFTER position p leaves the outputs of tokens <= p unchanged (causality):
    # compare the pruned layer's first rows with the unpruned layer's
    c = I.decoder_inputs(78, 1, 48, 128, 4, 4, 64, 96)
    pos = np.arange(48)[None]
    full = Dc.decoder_layer(c["h"], c["w"], 4, 4, 64, 20, 28, 28, pos)
    cut = Dc.decoder_layer(c["h"], c["w"], 4, 4, 64, 20, 28, 9, pos)
    assert cut["keep_idx"].shape == (1, 29) and np.array_equal(cut["keep_idx"][0, :20], np.arange(20))
    assert np.array_equal(cut["y_bits"][0, :20], full["y_bits"][0, :20])
    assert np.array_equal(cut["positions"], cut["keep_idx"])
    # and the kept visual tokens are the 9 smallest K-norms
    assert np.array_equal(cut["keep_idx"][0, 20:29] - 20, O.topk_smallest(full["norms"][0], 9))


def test_decode_attention_against_pinned_prefill_and_library():
    # the last row of a causal prefill IS a decode step over the same keys
    t = I.qkv_tensors(91, 2, 57, 6, 2, 64)
    full, full_lse = O.attention(t["q"], t["k"], t["v"])
    o, lse = Dc.decode_attention(t["q"][:, -1], t["k"], t["v"])
    assert np.allclose(o, full[:, -1], rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, full_lse[:, :, -1], rtol=1e-12)
    q = torch.from_numpy(f64(t["q"][:, -1]))[:, :, None, :]                     # [B,Hq,1,d]
    k = torch.from_numpy(f64(t["k"])).transpose(1, 2).repeat_interleave(3, dim=1)
    v = torch.from_numpy(f64(t["v"])).transpose(1, 2).repeat_interleave(3, dim=1)
    want = F.scaled_dot_product_attention(q, k, v)[:, :, 0].numpy()
    assert np.allclose(o, want, rtol=1e-12, atol=1e-14)
    # one cached key: the output is its value row; V == 1 gives 1
    o1, _ = Dc.decode_attention(t["q"][:, 0], t["k"][:, :1], t["v"][:, :1])
    assert np.array_equal(o1[:, 0], f64(t["v"])[:, 0, 0])
    ones = bits(np.ones((2, 57, 2, 64)))
    assert np.allclose(Dc.decode_attention(t["q"][:, 3], t["k"], ones)[0], 1.0)


def small_model(seed, n_layers, T, D=128, Hq=4, Hkv=2, d=64, F=96):
    layers = [I.decoder_inputs(seed + 1 + l, 1, T, D, Hq, Hkv, d, F)["w"] for l in range(n_layers)]
    return I.decoder_inputs(seed, 1, T, D, Hq, Hkv, d, F)["h"], layers


def test_vitcop_schedule_with_one_token_per_cluster_is_the_plain_schedule():
    # every token its own cluster and a budget below the number of clusters: no elites, every
    # "merged" token is the mean of one token, in token order: Stage II changes nothing
    h, layers = small_model(300, 3, 40)
    pos = (3 * np.arange(40))[None]
    s2 = {"layer": 1, "budget": 20, "xy": None, "d_c": 8.0, "tau": 0.6, "n_centers": 0}
    got = Dc.vitcop_schedule(h, layers, s2, (), 4, 2, 64, 6, 28, pos, labels=np.arange(28))
    want = Dc.decoder_schedule(h, layers, (), 4, 2, 64, 6, 28, pos)
    assert got["stage2"]["n_out"] == 28 and np.array_equal(got["stage2"]["index"], np.arange(28))
    assert np.array_equal(got["y_bits"], want["y_bits"]) and np.array_equal(got["positions"], pos)
    for (k1, v1), (k2, v2) in zip(got["caches"], want["caches"]):          # and leaves the same KV caches
        assert np.array_equal(k1, k2) and np.array_equal(v1, v2)


def test_vitcop_schedule_single_cluster_by_hand():
    # one cluster, budget 5: the 4 smallest K-norms stay as they are (in token order), the other 20
    # tokens become one token, their mean, at the position of the first of them; then layers 1, 2
    # run on 6 + 5 + 6 tokens.  Rebuilt here step by step from the pinned pieces.
    T, vs, n = 36, 6, 24
    h, layers = small_model(310, 3, T)
    pos = (2 * np.arange(T) + 1)[None]
    s2 = {"layer": 1, "budget": 5, "xy": None, "d_c": 8.0, "tau": 0.6, "n_centers": 0}
    got = Dc.vitcop_schedule(h, layers, s2, (), 4, 2, 64, vs, n, pos, labels=np.zeros(n, dtype=np.int64))
    h1 = Dc.decoder_layer(h, layers[0], 4, 2, 64, vs, n, n, pos)["y_bits"]
    norms = Dc.decoder_layer(h1, layers[1], 4, 2, 64, vs, n, n, pos)["norms"][0]        # layer 1's own K-norms
    elite = np.sort(O.topk_smallest(norms, 4))
    rest = np.setdiff1d(np.arange(n), elite)
    merged = f64(h1[0, vs + rest]).mean(axis=0)
    vis = np.concatenate([h1[0, vs + elite], O.f64_to_bf16_bits(merged)[None]], axis=0)
    h_new = np.concatenate([h1[:, :vs], vis[None], h1[:, vs + n:]], axis=1)
    pos_new = np.concatenate([pos[0, :vs], pos[0, vs + elite], pos[0, vs + rest[:1]], pos[0, vs + n:]])[None]
    assert got["stage2"]["n_out"] == 5 and np.array_equal(got["stage2"]["index"], np.append(elite, rest[0]))
    want = Dc.decoder_schedule(h_new, layers[1:], (), 4, 2, 64, vs, 5, pos_new)
    assert np.array_equal(got["y_bits"], want["y_bits"]) and np.array_equal(got["positions"], pos_new)


def test_vitcop_schedule_clusters_planted_regions_and_clamps_stage3():
    # visual hidden states = planted spatial regions: Stage II at layer 0 sees them untouched, finds the
    # regions, and leaves at most `budget` tokens; a Stage III budget above that keeps them all
    n, D = 60, 128
    v = I.vic_inputs(41, n, D, 12, 4, 0.1)
    h, layers = small_model(320, 2, 8 + n + 4, D=D)
    h = h.copy()
    h[0, 8:8 + n] = v["feats"]
    pos = np.arange(8 + n + 4)[None]
    s2 = {"layer": 0, "budget": 20, "xy": v["pos"], "d_c": 8.0, "tau": 0.6, "n_centers": 4}
    got = Dc.vitcop_schedule(h, layers, s2, ((1, 50),), 4, 2, 64, 8, n, pos)
    st = got["stage2"]
    assert np.array_equal(st["labels"], Dc.V.vic_cluster(v["feats"], v["pos"], 8.0, 0.6, 4)["labels"])
    assert st["n_out"] <= 20 and got["y"].shape[1] == 12 + st["n_out"]
    # the same call with the clustering and norms handed in decides the same
    again = Dc.vitcop_schedule(h, layers, s2, ((1, 50),), 4, 2, 64, 8, n, pos, labels=st["labels"], k_norms=st["norms"])
    assert np.array_equal(again["y_bits"], got["y_bits"])


def test_decode_step_is_the_last_row_of_the_prefill():
    # prefill of T tokens, last row == prefill of T-1 tokens (its caches) + one decoding step of token T:
    # every operation of a layer but the attention acts on rows independently, and the last row's
    # attention is the decoding step's (pinned above)
    T, D, Hq, Hkv, d, F = 30, 128, 4, 2, 64, 96
    h, layers = small_model(400, 3, T, D, Hq, Hkv, d, F)
    pos = (2 * np.arange(T) + 5)[None]
    full = Dc.decoder_schedule(h, layers, (), Hq, Hkv, d, 4, 20, pos)
    head = Dc.decoder_schedule(h[:, :T - 1], layers, (), Hq, Hkv, d, 4, 20, pos[:, :T - 1])
    step = Dc.decode_step(h[:, T - 1], layers, head["caches"], pos[:, T - 1], Hq, Hkv, d)
    assert np.allclose(step["y"][0], full["y"][0, T - 1], rtol=1e-9, atol=1e-11)
    assert np.array_equal(step["y_bits"][0], full["y_bits"][0, T - 1])
    for l in range(3):
        assert np.array_equal(step["appended"][l][0][0], full["caches"][l][0][0, T - 1])
        assert np.array_equal(step["appended"][l][1][0], full["caches"][l][1][0, T - 1])
    # after a pruned prefill the step attends over what each layer kept
    pr = Dc.decoder_schedule(h[:, :T - 1], layers, ((1, 6),), Hq, Hkv, d, 4, 20, pos[:, :T - 1])
    assert [c[0].shape[1] for c in pr["caches"]] == [29, 15, 15]
    st = Dc.decode_step(h[:, T - 1], layers, pr["caches"], pos[:, T - 1], Hq, Hkv, d)
    # ... and is again the last row of the same pruned prefill run over all T tokens: the K-norms of the
    # visual tokens do not depend on the text token after them, so both runs prune the same tokens
    full_pr = Dc.decoder_schedule(h, layers, ((1, 6),), Hq, Hkv, d, 4, 20, pos)
    assert np.array_equal(full_pr["keep_lists"][1][0, :-1], pr["keep_lists"][1][0])
    assert np.allclose(st["y"][0], full_pr["y"][0, -1], rtol=1e-9, atol=1e-11)
    assert np.array_equal(st["y_bits"][0], full_pr["y_bits"][0, -1])
    for l in range(3):
        assert np.array_equal(st["appended"][l][0][0], full_pr["caches"][l][0][0, -1])
        assert np.array_equal(st["appended"][l][1][0], full_pr["caches"][l][1][0, -1])


def test_decoder_schedule_with_pruning_is_a_chain_of_pruned_layers():
    # 5 layers, pruning on entry to layers 1 (20 -> 12 visual tokens) and 3 (12 -> 5).  Rebuilt by hand from
    # single layers: each stage ranks only the tokens still present, by the K-norms of ITS layer's input;
    # positions compose; the layers in between keep everything.  The keep lists themselves are re-derived
    # by a sort on norms recomputed from the layer input (RMSNorm, K projection, Eq. 4).
    T, vs, n, D, Hq, Hkv, d, F = 34, 6, 20, 128, 4, 2, 64, 96
    h, layers = small_model(330, 5, T, D, Hq, Hkv, d, F)
    pos = (3 * np.arange(T) + 2)[None]
    got = Dc.decoder_schedule(h, layers, ((1, 12), (3, 5)), Hq, Hkv, d, vs, n, pos)

    def own_list(h_in, w, n_now, keep):
        a = O.f64_to_bf16_bits(Dc.rmsnorm(h_in, w["ln1"], 1e-5))
        k = O.f64_to_bf16_bits(O.project(a, w["wk"]))[0, vs:vs + n_now]
        nrm = np.sqrt((f64(k) ** 2).sum(axis=1))
        kept = np.sort(np.lexsort((np.arange(n_now), nrm))[:keep])
        t_now = h_in.shape[1]
        return nrm, np.concatenate([np.arange(vs), vs + kept, np.arange(vs + n_now, t_now)])[None]

    cur, p_cur, n_now, caches = h, pos, n, []
    for l, w in enumerate(layers):
        keep = {1: 12, 3: 5}.get(l, n_now)
        nrm, idx = own_list(cur, w, n_now, keep)
        out = Dc.decoder_layer(cur, w, Hq, Hkv, d, vs, n_now, keep, p_cur, keep_idx=idx)
        if l in (1, 3):
            assert np.allclose(got["norms"][l][0], nrm, rtol=1e-12) and got["norms"][l].shape == (1, n_now)
            assert np.array_equal(got["keep_lists"][l], idx)
            p_cur = np.take_along_axis(p_cur, idx, axis=1)
        caches.append((out["k_rope"], out["v"]))
        cur, n_now = out["y_bits"], keep
    assert np.array_equal(got["y_bits"], cur) and np.array_equal(got["positions"], p_cur)
    assert [c[0].shape[1] for c in got["caches"]] == [34, 26, 26, 19, 19]
    for (k1, v1), (k2, v2) in zip(got["caches"], caches):
        assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    # positions compose: the second list indexes the sequence the first one left
    i1, i3 = got["keep_lists"][1][0], got["keep_lists"][3][0]
    assert np.array_equal(got["positions"][0], pos[0][i1][i3])
    assert set(i1[i3][vs:vs + 5]) <= set(i1[vs:vs + 12]) and len(i3) == 19
    # text tokens always survive, with their positions
    assert np.array_equal(got["positions"][0, :vs], pos[0, :vs])
    assert np.array_equal(got["positions"][0, vs + 5:], pos[0, vs + n:])
