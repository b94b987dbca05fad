"""CPU oracle for the ViTCoP pruned-prefill hot path.  TEST INFRASTRUCTURE ONLY.

Plain NumPy, float64 arithmetic on the exact bf16 input bits, written from the
paper's definitions (arXiv 2601.17818).  Nothing here is tuned, blocked or
fused, and nothing is shared with the GPU library: this module imports only
NumPy.  Only the tests, the smoke check and the bench's ``cpu_baseline`` leg
may import it; the product path never does.

What is an exact definition and what is a reading
-------------------------------------------------
* ``filter_scores``      Eq. 1 (Sec. 3.1): attention from [CLS] to each token,
                         summed over heads.  Softmax scale 1/sqrt(d) is a
                         reading (the paper does not print it); [CLS] takes part
                         in the softmax but is not a candidate.
* ``topk_largest``       Alg. 1, Stage I TopK.  Ties -> lower index (reading;
                         the paper treats TopK as a set).
* ``k_norms``            Eq. 4 (Sec. 3.2.2): L2 norm of a token's K over all
                         (KV) heads.
* ``topk_smallest``      Alg. 1, Stage III: TopK of -K_norms, "smaller norm is
                         better" (Sec. 2.2, Key Insight 2).  Ties -> lower index.
* ``keep_list``          survivors in ascending original position, text tokens
                         always kept (reading: Alg. 1 only names the set).
* ``compact``            the gather implied by TopK(V_current, ...) in Alg. 1.
* ``attention``          exact causal softmax(Q K^T scale) V, which is what a
                         FlashAttention kernel computes (Sec. 1, Sec. 2.2).
* ``flops_layer`` etc.   Eq. 7-10 (App. E) as printed, plus the layer-count
                         reading that reproduces Table 7.

Every function is pinned by tests that do not re-type its formula: brute
force on tiny inputs, closed forms, planted inputs with results known a
priori, invariances, and the arithmetic of Table 7.  No function here is
"parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# storage-format helpers (bf16 bit pattern <-> float64)
# --------------------------------------------------------------------------


def bf16_to_f64(bits) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float64, exact."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """float64 -> bf16 bit pattern, one round-to-nearest-even step.

    Valid for finite values in the normal float32 range (asserted).
    """
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert np.all(np.isfinite(x))
    u = x.view(np.uint64)
    drop = np.uint64(52 - 7)                      # keep 7 explicit mantissa bits
    lsb = (u >> drop) & np.uint64(1)
    r = u + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + lsb
    r = (r >> drop) << drop
    y = r.view(np.float64)
    f = y.astype(np.float32)                      # exact: y has 8 significant bits
    ok = (f.astype(np.float64) == y) | (y == 0)
    assert np.all(ok), "value outside the normal float32 range"
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# selection (Alg. 1: TopK in Stage I and Stage III)
# --------------------------------------------------------------------------


def _ranks(scores: np.ndarray, largest: bool) -> np.ndarray:
    """rank_i = #(strictly better than i) + #(equal to i with a lower index)."""
    s = np.asarray(scores, dtype=np.float64)
    n = s.shape[0]
    rank = np.zeros(n, dtype=np.int64)
    step = 1024
    ar = np.arange(n)
    for lo in range(0, n, step):
        c = s[lo:lo + step, None]
        better = (s[None, :] > c) if largest else (s[None, :] < c)
        tie = (s[None, :] == c) & (ar[None, :] < ar[lo:lo + step, None])
        rank[lo:lo + step] = better.sum(axis=1) + tie.sum(axis=1)
    return rank


def topk_largest(scores, keep: int) -> np.ndarray:
    """Indices of the ``keep`` highest scores, ascending; ties -> lower index."""
    s = np.asarray(scores, dtype=np.float64)
    assert s.ndim == 1 and 0 <= keep <= s.shape[0] and np.all(np.isfinite(s))
    return np.nonzero(_ranks(s, True) < keep)[0].astype(np.int32)


def topk_smallest(scores, keep: int) -> np.ndarray:
    """Indices of the ``keep`` lowest scores, ascending; ties -> lower index."""
    s = np.asarray(scores, dtype=np.float64)
    assert s.ndim == 1 and 0 <= keep <= s.shape[0] and np.all(np.isfinite(s))
    return np.nonzero(_ranks(s, False) < keep)[0].astype(np.int32)


def tie_band(scores, keep: int, largest: bool, rel: float = 1e-3) -> np.ndarray:
    """Mask of candidates whose score is within ``rel`` (relative) of the k-th.

    Outside this band a float32 implementation must select exactly the same
    set as the float64 ranking; inside it may differ.
    """
    s = np.asarray(scores, dtype=np.float64)
    n = s.shape[0]
    if keep <= 0 or keep >= n:
        return np.zeros(n, dtype=bool)
    order = np.sort(s)
    theta = order[n - keep] if largest else order[keep - 1]
    return np.abs(s - theta) <= rel * abs(theta)


# --------------------------------------------------------------------------
# Stage I: [CLS]-attention saliency in the vision encoder (Sec. 3.1, Eq. 1)
# --------------------------------------------------------------------------


def filter_scores(q_cls, k, scale: float | None = None) -> np.ndarray:
    """S[b,i] = sum_h A^(h)[0, i+1] for the N patch tokens of each image.

    q_cls : [B,H,d]     bf16 bits, query of the [CLS] token
    k     : [B,N+1,H,d] bf16 bits, keys; token 0 is [CLS]
    The softmax of each head runs over all N+1 keys; the score of [CLS] itself
    is dropped.  Returns float64 [B,N].
    """
    q = bf16_to_f64(q_cls)
    kk = bf16_to_f64(k)
    B, H, d = q.shape
    assert kk.shape[0] == B and kk.shape[2] == H and kk.shape[3] == d
    N1 = kk.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    S = np.zeros((B, N1), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            logit = (kk[b, :, h, :] @ q[b, h, :]) * scale
            e = np.exp(logit - logit.max())
            S[b] += e / e.sum()
    return S[:, 1:]


def filter_visual(q_cls, k, keep: int, scale: float | None = None):
    """Stage I of Alg. 1: scores (Eq. 1) and the kept patch indices per image."""
    S = filter_scores(q_cls, k, scale)
    idx = np.stack([topk_largest(S[b], keep) for b in range(S.shape[0])])
    return S, idx.reshape(S.shape[0], keep)


# --------------------------------------------------------------------------
# In-LLM saliency: K-vector L2 norm (Sec. 3.2.2, Eq. 4) and Stage III TopK
# --------------------------------------------------------------------------


def k_norms(k, vis_start: int, n_vis: int) -> np.ndarray:
    """||K_i||_2 over all KV heads for the visual span.  k: [B,T,Hkv,d] bits."""
    kk = bf16_to_f64(k)
    B, T = kk.shape[0], kk.shape[1]
    assert 0 <= vis_start and vis_start + n_vis <= T
    rows = kk[:, vis_start:vis_start + n_vis].reshape(B, n_vis, kk.shape[2] * kk.shape[3])    # (n_vis may be 0)
    return np.sqrt((rows * rows).sum(axis=2))


def keep_list(norms, T: int, vis_start: int, keep: int) -> np.ndarray:
    """[B,T'] ascending positions: text before, kept visual, text after."""
    norms = np.asarray(norms, dtype=np.float64)
    B, n_vis = norms.shape
    out = []
    for b in range(B):
        kept = topk_smallest(norms[b], keep) + vis_start
        out.append(np.concatenate([np.arange(0, vis_start),
                                   kept,
                                   np.arange(vis_start + n_vis, T)]).astype(np.int32))
    return np.stack(out).reshape(B, T - n_vis + keep)


def knorm_select(k, vis_start: int, n_vis: int, keep: int):
    """Eq. 4 followed by the Stage III TopK of Alg. 1.  Returns (norms, keep_idx)."""
    k = np.asarray(k)
    nrm = k_norms(k, vis_start, n_vis)
    return nrm, keep_list(nrm, k.shape[1], vis_start, keep)


# --------------------------------------------------------------------------
# Token removal (implicit in TopK(V_current, ...) of Alg. 1)
# --------------------------------------------------------------------------


def compact(src, idx) -> np.ndarray:
    """dst[b,j,...] = src[b, idx[b,j], ...] (bit copy)."""
    src = np.asarray(src)
    idx = np.asarray(idx)
    B, T_out = idx.shape
    dst = np.empty((B, T_out) + src.shape[2:], dtype=src.dtype)
    for b in range(B):
        for j in range(T_out):
            dst[b, j] = src[b, idx[b, j]]
    return dst


# --------------------------------------------------------------------------
# Attention over the (shortened) sequence: exact softmax(Q K^T scale) V
# --------------------------------------------------------------------------


def attention(q, k, v, scale: float | None = None, causal: bool = True):
    """q: [B,N,Hq,d], k,v: [B,N,Hkv,d] bf16 bits.

    Query head h reads KV head h // (Hq // Hkv).  Causal: key j visible to
    query i iff j <= i, in the order the rows are given.
    Returns (out float64 [B,N,Hq,d], lse float64 [B,Hq,N]) with
    lse = log sum_j exp(scale * q_i . k_j) over visible keys.
    """
    qq, kk, vv = bf16_to_f64(q), bf16_to_f64(k), bf16_to_f64(v)
    B, N, Hq, d = qq.shape
    Hkv = kk.shape[2]
    assert Hq % Hkv == 0 and kk.shape == vv.shape == (B, N, Hkv, d)
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    g = Hq // Hkv
    out = np.empty((B, N, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq, N), dtype=np.float64)
    visible = np.tril(np.ones((N, N), dtype=bool)) if causal else np.ones((N, N), dtype=bool)
    for b in range(B):
        for h in range(Hq):
            s = (qq[b, :, h, :] @ kk[b, :, h // g, :].T) * scale
            s = np.where(visible, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            p = np.exp(s - m)
            z = p.sum(axis=1, keepdims=True)
            out[b, :, h, :] = (p / z) @ vv[b, :, h // g, :]
            lse[b, h, :] = (m + np.log(z))[:, 0]
    return out, lse


def attention_rows(q, k, v, b: int, h: int, rows, scale: float | None = None,
                   causal: bool = True) -> np.ndarray:
    """Same definition as ``attention`` for a few query rows of one (b, head).

    Used on full-size workloads where computing every row would take too long.
    Returns float64 [len(rows), d].
    """
    q, k, v = np.asarray(q), np.asarray(k), np.asarray(v)
    B, N, Hq, d = q.shape
    g = Hq // k.shape[2]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    kk = bf16_to_f64(k[b, :, h // g, :])
    vv = bf16_to_f64(v[b, :, h // g, :])
    res = np.empty((len(rows), d), dtype=np.float64)
    for r, i in enumerate(rows):
        last = i + 1 if causal else N
        s = (kk[:last] @ bf16_to_f64(q[b, i, h, :])) * scale
        p = np.exp(s - s.max())
        res[r] = (p / p.sum()) @ vv[:last]
    return res


# --------------------------------------------------------------------------
# Projections around the pruning point ("K vectors from the LLM's attention
# module", Sec. 3.2.2) and the pruned / unpruned layer
# --------------------------------------------------------------------------


def project(x, w) -> np.ndarray:
    """y = x @ w.T in float64.  x: [..., in] bits, w: [out, in] bits."""
    return bf16_to_f64(x) @ bf16_to_f64(w).T


def pruned_layer(x, wq, wk, wv, wo, Hq: int, Hkv: int, d: int, vis_start: int,
                 n_vis: int, keep: int, residual: bool = False) -> dict:
    """One attention layer with pruning on entry (Alg. 1, body of the layer loop).

    K is projected for every token of the layer input; the visual tokens are
    ranked by the norm of that K (Eq. 4) and the ``keep`` smallest survive;
    hidden states and K are compacted; Q and V are projected for survivors
    only; causal attention runs over the survivors; the output projection
    follows.  Every tensor the GPU stores as bf16 is rounded to bf16 here too.
    With ``residual`` the compacted hidden state is added to the output.
    """
    x = np.asarray(x)
    B, T, D = x.shape
    k_bits = f64_to_bf16_bits(project(x, wk)).reshape(B, T, Hkv, d)
    norms, idx = knorm_select(k_bits, vis_start, n_vis, keep)
    xs = compact(x, idx)                                     # [B,T',D]
    ks = compact(k_bits, idx)                                # [B,T',Hkv,d]
    Tp = idx.shape[1]
    q_bits = f64_to_bf16_bits(project(xs, wq)).reshape(B, Tp, Hq, d)
    v_bits = f64_to_bf16_bits(project(xs, wv)).reshape(B, Tp, Hkv, d)
    o, lse = attention(q_bits, ks, v_bits, None, True)
    o_bits = f64_to_bf16_bits(o).reshape(B, Tp, Hq * d)
    y = project(o_bits, wo)
    if residual:
        y = y + bf16_to_f64(xs)
    return {"k": k_bits, "norms": norms, "keep_idx": idx, "x_kept": xs, "k_kept": ks,
            "q": q_bits, "v": v_bits, "attn": o, "attn_bits": o_bits,
            "y": y, "y_bits": f64_to_bf16_bits(y)}


def unpruned_layer(x, wq, wk, wv, wo, Hq: int, Hkv: int, d: int,
                   residual: bool = False) -> dict:
    """The same layer without pruning (the vanilla prefill it is compared with)."""
    x = np.asarray(x)
    B, T, D = x.shape
    q_bits = f64_to_bf16_bits(project(x, wq)).reshape(B, T, Hq, d)
    k_bits = f64_to_bf16_bits(project(x, wk)).reshape(B, T, Hkv, d)
    v_bits = f64_to_bf16_bits(project(x, wv)).reshape(B, T, Hkv, d)
    o, lse = attention(q_bits, k_bits, v_bits, None, True)
    o_bits = f64_to_bf16_bits(o).reshape(B, T, Hq * d)
    y = project(o_bits, wo)
    if residual:
        y = y + bf16_to_f64(x)
    return {"q": q_bits, "k": k_bits, "v": v_bits, "attn": o, "attn_bits": o_bits,
            "y": y, "y_bits": f64_to_bf16_bits(y)}


def schedule_prefill(x, layer_weights, n_layers: int, schedule, Hq: int, Hkv: int,
                     d: int, vis_start: int, n_vis: int) -> dict:
    """Step-wise schedule (Alg. 1 layer loop; Eq. 8): 0-indexed layers, pruning
    on entry to a scheduled layer with that layer's own K, budgets counted in
    visual tokens.  ``layer_weights(l)`` returns the dict wq/wk/wv/wo of layer l.
    h <- h + attention block output; no MLP, no normalisation.

    Returns the final hidden state bits, the original positions of the
    surviving rows, and per-layer records (input bits, keep_idx or None).
    """
    h = np.asarray(x)
    B, T, _ = h.shape
    assert B == 1
    budgets = dict(schedule)
    positions = np.arange(T, dtype=np.int32)[None, :]
    cur_vis = n_vis
    layers = []
    for l in range(n_layers):
        w = layer_weights(l)
        if l in budgets:
            r = pruned_layer(h, w["wq"], w["wk"], w["wv"], w["wo"], Hq, Hkv, d,
                             vis_start, cur_vis, budgets[l], residual=True)
            positions = compact(positions[:, :, None], r["keep_idx"])[:, :, 0]
            cur_vis = budgets[l]
            layers.append({"x_in": h, "keep_idx": r["keep_idx"], "norms": r["norms"]})
        else:
            r = unpruned_layer(h, w["wq"], w["wk"], w["wv"], w["wo"], Hq, Hkv, d,
                               residual=True)
            layers.append({"x_in": h, "keep_idx": None, "norms": None})
        h = r["y_bits"]
    return {"h": h, "positions": positions, "layers": layers}


# --------------------------------------------------------------------------
# Accounting (App. E, Eq. 7-10; Table 7)
# --------------------------------------------------------------------------


def flops_layer(N: float, d: float) -> float:
    """Eq. 7: 4 N^2 d + 16 N d^2."""
    return 4.0 * N * N * d + 16.0 * N * d * d


def stage_layer_counts(l_s: int, l_d: int, n: int, zero_indexed: bool = True):
    """How many layers run at pi1, pi2, pi3.

    Eq. 9/10 as printed use (l_s - 1, l_d - l_s, n - l_d + 1).  Reading layer
    numbers as 0-indexed with pruning on entry gives (l_s, l_d - l_s, n - l_d),
    which is the only count that reproduces Table 7's ratios.
    """
    if zero_indexed:
        return (l_s, l_d - l_s, n - l_d)
    return (l_s - 1, l_d - l_s, n - l_d + 1)


def mean_retained_tokens(m: int, ratios, counts) -> float:
    """Layer-averaged visual token count (the quantity Eq. 10 averages)."""
    total = sum(c for c in counts)
    return sum(r * m * c for r, c in zip(ratios, counts)) / total


def cr_int(m: int, ratios, counts) -> float:
    """Eq. 10: integrated token compression ratio."""
    return 1.0 - mean_retained_tokens(m, ratios, counts) / m


def schedule_flops(m: int, n_text: int, d_model: int, ratios, counts) -> float:
    """Eq. 9 with the given per-stage layer counts."""
    return sum(c * flops_layer(r * m + n_text, d_model) for r, c in zip(ratios, counts))


def causal_attention_flops(B: int, N: int, Hq: int, d: int) -> float:
    """Multiply-adds that a causal attention must do, times two: 4 d per visible pair."""
    return 4.0 * d * Hq * B * N * (N + 1) / 2.0
