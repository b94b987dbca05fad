"""CPU oracle for one full decoder layer of the prefill with pruning on entry.  TEST INFRASTRUCTURE ONLY.

The paper prunes inside the layers of LLaVA's language model (Sec. 4.1: LLaVA-1.5 / LLaVA-NeXT,
i.e. a LLaMA-family decoder) but does not restate that architecture.  This module writes out the
published pre-norm decoder layer (RMSNorm, rotary position embedding in the rotate-half
convention, grouped-query attention, SiLU-gated MLP, two residual adds) in NumPy float64, with
the pruning step of Alg. 1 (layer loop body) at its entry, and rounds to bf16 exactly where the
GPU path stores a bf16 tensor.  It imports only NumPy and the hot-path oracle next to it.

Readings: K-norms are taken before the rotary embedding (a per-pair rotation leaves them
unchanged, Sec. 3.2.2 / Eq. 4 does not say); survivors keep their original positions (the paper
is silent); pruning removes a token from the residual stream of this and all later layers.
"""
from __future__ import annotations

import numpy as np

from . import vic_oracle as V
from . import vitcop_oracle as O


def rmsnorm(x_bits, w_bits, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * w over the last axis, float64."""
    x = O.bf16_to_f64(x_bits)
    w = O.bf16_to_f64(w_bits)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(x_bits, positions, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: channel i < d/2 pairs with i + d/2, angle =
    position * theta^(-2i/d).  x_bits [B,N,H,d], positions [B,N] -> float64 [B,N,H,d]."""
    x = O.bf16_to_f64(x_bits)
    d = x.shape[-1]
    half = d // 2
    inv_freq = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = np.asarray(positions, dtype=np.float64)[:, :, None, None] * inv_freq        # [B,N,1,half]
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu_mul(gate_bits, up_bits) -> np.ndarray:
    """silu(gate) * up = gate / (1 + exp(-gate)) * up, float64."""
    g = O.bf16_to_f64(gate_bits)
    u = O.bf16_to_f64(up_bits)
    return g / (1.0 + np.exp(-g)) * u


def decoder_layer(h_bits, w: dict, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int, keep: int,
                  positions, eps: float = 1e-5, theta: float = 10000.0, keep_idx=None):
    """h [B,T,D] bits; w: bits of ln1, ln2 [D], wq [Hq d, D], wk, wv [Hkv d, D], wo [D, Hq d],
    wg, wu [F, D], wd [D, F]; positions [B,T].  Returns a dict with the output hidden states
    (float64 and bf16 bits), the keep list, the norms and the intermediates a staged check needs.
    ``keep_idx`` [B,T'] replaces the keep list computed here (for checking a pipeline whose own,
    separately validated, list differs among near-tied norms)."""
    B, T, D = h_bits.shape
    r16 = O.f64_to_bf16_bits
    a = r16(rmsnorm(h_bits, w["ln1"], eps))                                    # [B,T,D]
    k_all = r16(O.project(a, w["wk"])).reshape(B, T, Hkv, d)
    norms = O.k_norms(k_all, vis_start, n_vis)
    idx = O.keep_list(norms, T, vis_start, keep) if keep_idx is None else np.asarray(keep_idx)
    Tp = idx.shape[1]
    h_kept, a_kept, k_kept = O.compact(h_bits, idx), O.compact(a, idx), O.compact(k_all, idx)
    pos_kept = np.take_along_axis(np.asarray(positions), idx, axis=1)
    q = r16(O.project(a_kept, w["wq"])).reshape(B, Tp, Hq, d)
    v = r16(O.project(a_kept, w["wv"])).reshape(B, Tp, Hkv, d)
    q_r, k_r = r16(rope(q, pos_kept, theta)), r16(rope(k_kept, pos_kept, theta))
    attn, _ = O.attention(q_r, k_r, v)
    o = r16(attn).reshape(B, Tp, Hq * d)
    h1 = r16(O.bf16_to_f64(h_kept) + O.project(o, w["wo"]))
    b = r16(rmsnorm(h1, w["ln2"], eps))
    g, u = r16(O.project(b, w["wg"])), r16(O.project(b, w["wu"]))
    m = r16(silu_mul(g, u))
    y = O.bf16_to_f64(h1) + O.project(m, w["wd"])
    return {"y": y, "y_bits": r16(y), "keep_idx": idx, "norms": norms, "positions": pos_kept,
            "a": a, "q_rope": q_r, "k_rope": k_r, "v": v, "h1": h1, "m": m}


def decode_attention(q_bits, k_bits, v_bits, scale: float | None = None):
    """One decoding step over a (compacted) KV cache: for every sample and query head,
    o = softmax(scale * K q) V over ALL cached keys (the new token sees the whole cache).
    q [B,Hq,d], k, v [B,N,Hkv,d] bf16 bits -> (o float64 [B,Hq,d], lse float64 [B,Hq]).
    Query head h reads KV head h // (Hq // Hkv).  This is what the per-token cost of Table 5
    (decoding after a pruned prefill) is made of: one pass over the cache per layer."""
    q, k, v = O.bf16_to_f64(q_bits), O.bf16_to_f64(k_bits), O.bf16_to_f64(v_bits)
    B, Hq, d = q.shape
    Hkv = k.shape[2]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            s = k[b, :, hk, :] @ q[b, h] * scale
            m = s.max()
            p = np.exp(s - m)
            out[b, h] = p @ v[b, :, hk, :] / p.sum()
            lse[b, h] = m + np.log(p.sum())
    return out, lse


def decoder_schedule(h_bits, layer_weights, schedule, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int,
                     positions, eps: float = 1e-5, theta: float = 10000.0, keep_lists=None):
    """Whole-model prefill (layer loop of Alg. 1, Eq. 8): decoder layers in sequence, 0-indexed, pruning on
    entry to the scheduled layers by that layer's own K-norms; the hidden state is carried in bf16.
    ``schedule``: ((layer, keep), ...); ``keep_lists``: optional {layer: keep_idx} overriding the lists
    computed here.  Returns the final hidden state (float64, bits), positions, per pruning layer the
    keep list and the norms it was taken from, and per layer its KV cache (K after the rotary embedding, V;
    bf16 bits [B, T_l, Hkv, d])."""
    h = np.asarray(h_bits)
    pos = np.asarray(positions)
    stages = dict(schedule)
    cur_vis = n_vis
    kept, norms, caches = {}, {}, []
    out = None
    for l, w in enumerate(layer_weights):
        keep = stages.get(l, cur_vis)
        forced = None if keep_lists is None else keep_lists.get(l)
        out = decoder_layer(h, w, Hq, Hkv, d, vis_start, cur_vis, keep, pos, eps, theta, keep_idx=forced)
        caches.append((out["k_rope"], out["v"]))
        if l in stages:
            kept[l] = out["keep_idx"]
            norms[l] = out["norms"]
            pos = out["positions"]
            cur_vis = keep
        h = out["y_bits"]
    return {"y": out["y"], "y_bits": h, "positions": pos, "keep_lists": kept, "norms": norms, "caches": caches}


def vitcop_schedule(h_bits, layer_weights, stage2: dict, schedule, Hq: int, Hkv: int, d: int, vis_start: int,
                    n_vis: int, positions, eps: float = 1e-5, theta: float = 10000.0, labels=None, k_norms=None,
                    keep_lists=None):
    """The in-model procedure of Alg. 1 on ONE sample: decoder layers in sequence; on entry to layer
    ``stage2["layer"]`` the visual tokens are clustered (Alg. 2 on their hidden states and grid positions
    ``stage2["xy"]`` [n_vis, 2], with d_c, tau, n_centers) and replaced by the per-cluster elites and one
    merged token per cluster (Alg. 3 with budget ``stage2["budget"]`` and that layer's K-norms, Eq. 4);
    the Stage III rule (``schedule`` as in ``decoder_schedule``, layers after Stage II) prunes the rest.

    Readings: the clustering features are the hidden states entering the layer; the K-norms are those of
    the layer's own K projection of the normalised input, before the rotary embedding; the new visual
    block is laid out as ``collab_prune_merge`` returns it (elites in token order, then merged tokens in
    label order) between the unchanged text tokens; a merged token takes the position of the
    lowest-index token it absorbed and is stored in bf16; a Stage III budget above the number of visual
    tokens Stage II left keeps them all.

    ``labels`` [n_vis] and ``k_norms`` [n_vis] replace the clustering and the norms computed here (for
    checking a pipeline whose own, separately validated, values decide differently among near-ties).
    Returns the final hidden state, positions, what Stage II produced, and per layer the K (after the rotary
    embedding) and V of the tokens the layer attended over (the KV cache a decoding step continues from).
    """
    h = np.asarray(h_bits)
    pos = np.asarray(positions)
    assert h.shape[0] == 1, "one sample"
    r16 = O.f64_to_bf16_bits
    stages = dict(schedule)
    cur_vis = n_vis
    s2 = None
    out = None
    caches = []
    stage3 = {}          # per Stage III layer: the norms ranked there and the keep list taken
    for l, w in enumerate(layer_weights):
        if l == stage2["layer"]:
            T = h.shape[1]
            a = r16(rmsnorm(h, w["ln1"], eps))
            k_all = r16(O.project(a, w["wk"])).reshape(1, T, Hkv, d)
            norms = O.k_norms(k_all, vis_start, cur_vis)[0] if k_norms is None else np.asarray(k_norms)
            feats = h[0, vis_start:vis_start + cur_vis]
            if labels is None:
                lab = V.vic_cluster(feats, stage2["xy"], stage2["d_c"], stage2["tau"], stage2["n_centers"])["labels"]
            else:
                lab = np.asarray(labels)
            cm = V.collab_prune_merge(feats, lab, norms, stage2["budget"])
            n_out = len(cm["index"])
            new_vis = r16(cm["feats"]).reshape(n_out, h.shape[2])
            h = np.concatenate([h[:, :vis_start], new_vis[None], h[:, vis_start + cur_vis:]], axis=1)
            vis_pos = pos[0, vis_start + cm["index"].astype(np.int64)]
            pos = np.concatenate([pos[:, :vis_start], vis_pos[None], pos[:, vis_start + cur_vis:]], axis=1)
            s2 = {"labels": lab, "norms": norms, "index": cm["index"], "n_out": n_out, "elite": cm["elite"],
                  "feats": cm["feats"]}
            cur_vis = n_out
        keep = min(stages.get(l, cur_vis), cur_vis)
        forced = None if keep_lists is None else keep_lists.get(l)
        out = decoder_layer(h, w, Hq, Hkv, d, vis_start, cur_vis, keep, pos, eps, theta, keep_idx=forced)
        caches.append((out["k_rope"], out["v"]))
        if l in stages:
            stage3[l] = {"norms": out["norms"], "keep_idx": out["keep_idx"]}
            pos = out["positions"]
            cur_vis = keep
        h = out["y_bits"]
    return {"y": out["y"], "y_bits": h, "positions": pos, "stage2": s2, "stage3": stage3, "caches": caches}


def decode_step(h_bits, layer_weights, caches, positions, Hq: int, Hkv: int, d: int, eps: float = 1e-5,
                theta: float = 10000.0):
    """One decoding step of the whole model (what Table 5 times per generated token): the new token of
    every sample, ``h_bits`` [B, D], goes through all layers; layer l attends over its cache
    ``caches[l]`` = (K after the rotary embedding, V), bf16 bits [B, N_l, Hkv, d] (N_l differs between
    layers after a pruned prefill), extended by the token's own K and V.  ``positions`` [B]: the position
    id of the new token.  Rounds to bf16 where the prefill layer does.  Returns the output hidden state
    (float64, bits) and the per-layer rows appended to the caches."""
    h = np.asarray(h_bits)
    B, D = h.shape
    pos = np.asarray(positions).reshape(B, 1)
    r16 = O.f64_to_bf16_bits
    appended = []
    y = None
    for w, (k_cache, v_cache) in zip(layer_weights, caches):
        a = r16(rmsnorm(h, w["ln1"], eps))                                      # [B, D]
        q = r16(O.project(a, w["wq"])).reshape(B, 1, Hq, d)
        k = r16(O.project(a, w["wk"])).reshape(B, 1, Hkv, d)
        v = r16(O.project(a, w["wv"])).reshape(B, 1, Hkv, d)
        q_r, k_r = r16(rope(q, pos, theta)), r16(rope(k, pos, theta))
        keys = np.concatenate([np.asarray(k_cache), k_r], axis=1)
        vals = np.concatenate([np.asarray(v_cache), v], axis=1)
        attn, _ = decode_attention(q_r[:, 0], keys, vals)
        o = r16(attn).reshape(B, Hq * d)
        h1 = r16(O.bf16_to_f64(h) + O.project(o, w["wo"]))
        b = r16(rmsnorm(h1, w["ln2"], eps))
        g, u = r16(O.project(b, w["wg"])), r16(O.project(b, w["wu"]))
        m = r16(silu_mul(g, u))
        y = O.bf16_to_f64(h1) + O.project(m, w["wd"])
        h = r16(y)
        appended.append((k_r[:, 0], v[:, 0]))
    return {"y": y, "y_bits": h, "appended": appended}
