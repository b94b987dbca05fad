"""CPU oracle for Stage II: Visual Information Clustering (VIC) and collaborative pruning and
merging.  TEST INFRASTRUCTURE ONLY.

Plain NumPy float64 on the exact bf16 feature bits, written from Sec. 3.2.1
(Eq. 2, Eq. 3) and Alg. 2 of arXiv 2601.17818, step by step in the paper's
order and notation.  It imports only NumPy and shares nothing with the GPU
library.  Only tests, the smoke check and the bench's CPU leg may import it.

Steps and readings
------------------
* ``feature_distances``  D_feat[i,j] = ||f_i - f_j||_2 (Alg. 2, Step 1), from the
                         differences themselves (no Gram-matrix shortcut).
* ``spatial_distances``  D_spatial[i,j] = ||p_i - p_j||_2; positions are grid
                         coordinates normalised to [0,1]^2 (reading: the paper
                         gives tau = 0.6 without units).
* ``density``            Eq. 2: rho_i = sum_{j != i} exp(-(D_feat[i,j]/d_c)^2).
* ``parents``            Eq. 3 / Alg. 2 Step 2: delta_i = min D_feat[i,j] over
                         j with rho_j > rho_i (strictly) and D_spatial[i,j] <=
                         tau; N_i = the first j reaching that minimum (strict
                         "<" in the listing: ties -> lower index); none ->
                         delta_i = inf, N_i = -1.
* ``centers``            Step 3: gamma_i = rho_i * delta_i, the ``n_centers``
                         highest are centres (ties -> lower index).  Readings:
                         n_centers = ceil(n * alpha) is an argument (alpha is
                         never given); gamma_i = inf whenever delta_i = inf,
                         also for rho_i = 0.
* ``labels``             Step 4: centres get their own label; every other
                         token, in order of decreasing rho, takes the label of
                         its parent N_i.  Readings: a token that is not a
                         centre and has no parent (N_i = -1; the listing would
                         read L[-1]) becomes the root of its own cluster;
                         cluster labels are numbered 0..R-1 by the root's token
                         index (the listing numbers centres by gamma rank;
                         labels are names of sets, any numbering gives the
                         same partition).

Comparisons that decide integers (rho_j > rho_i, D <= tau, the minimum, the
TopK of gamma) are taken on the values handed in: callers that check a GPU
result pass the GPU's own float32 arrays, so both sides decide on identical
numbers.

``collab_prune_merge`` (Sec. 3.2.3, Eq. 5-6, Alg. 3) is described, with its
readings, above its definition at the end of this file.
"""
from __future__ import annotations

import math

import numpy as np


def _bf16_to_f64(bits) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def feature_distances(feat_bits, rows=None) -> np.ndarray:
    """feat_bits [n, D] bf16 bits -> D_feat [n, n] float64 (Alg. 2, Step 1); with ``rows`` only
    those rows of the matrix, [len(rows), n]."""
    f = _bf16_to_f64(feat_bits)
    n = f.shape[0]
    rows = range(n) if rows is None else list(rows)
    out = np.zeros((len(rows), n), dtype=np.float64)
    for r, i in enumerate(rows):
        diff = f - f[i]
        out[r] = np.sqrt(np.sum(diff * diff, axis=1))
    return out


def spatial_distances(pos) -> np.ndarray:
    """pos [n, 2] -> D_spatial [n, n] float64."""
    p = np.asarray(pos, dtype=np.float64)
    diff = p[:, None, :] - p[None, :, :]
    return np.sqrt(np.sum(diff * diff, axis=2))


def density(d_feat, d_c: float) -> np.ndarray:
    """Eq. 2: rho_i = sum over j != i of exp(-(D_feat[i,j] / d_c)^2)."""
    d = np.asarray(d_feat, dtype=np.float64)
    n = d.shape[0]
    rho = np.zeros(n, dtype=np.float64)
    for i in range(n):
        acc = 0.0
        for j in range(n):
            if j != i:
                acc += math.exp(-((d[i, j] / d_c) ** 2))
        rho[i] = acc
    return rho


def parents(d_feat, d_spatial, rho, tau: float):
    """Eq. 3 (Alg. 2 Step 2): delta_i = the smallest feature distance from token i to a token that is strictly
    denser and spatially within tau of it; N_i = that token (the lowest index among equal distances).
    Returns (delta [n], inf where no token qualifies; N [n] int32, -1 there)."""
    d_feat = np.asarray(d_feat, dtype=np.float64)
    d_spatial = np.asarray(d_spatial, dtype=np.float64)
    rho = np.asarray(rho, dtype=np.float64)
    n = len(rho)
    delta = np.full(n, np.inf, dtype=np.float64)
    parent = np.full(n, -1, dtype=np.int32)
    for i in range(n):
        allowed = (rho > rho[i]) & (d_spatial[i] <= tau)          # the set the minimum of Eq. 3 runs over
        if not allowed.any():
            continue
        masked = np.where(allowed, d_feat[i], np.inf)
        parent[i] = int(np.argmin(masked))                         # first occurrence of the minimum
        delta[i] = masked[parent[i]]
    return delta, parent


def importance(rho, delta) -> np.ndarray:
    """gamma = rho * delta (Step 3), inf wherever delta is inf."""
    rho = np.asarray(rho, dtype=np.float64)
    delta = np.asarray(delta, dtype=np.float64)
    gamma = np.empty_like(rho)
    for i in range(len(rho)):
        gamma[i] = np.inf if np.isinf(delta[i]) else rho[i] * delta[i]
    return gamma


def centers(gamma, n_centers: int) -> np.ndarray:
    """Indices of the n_centers highest gamma, ascending; ties -> lower index."""
    n = len(gamma)
    assert 0 <= n_centers <= n
    order = sorted(range(n), key=lambda i: (-gamma[i], i))      # inf sorts first; stable on index
    return np.array(sorted(order[:n_centers]), dtype=np.int32)


def labels(rho, parent, center_idx):
    """Step 4.  Returns (L [n] int32 in [0,R), roots [R] int32 ascending)."""
    n = len(rho)
    is_center = np.zeros(n, dtype=bool)
    is_center[np.asarray(center_idx, dtype=np.int64)] = True
    roots = [i for i in range(n) if is_center[i] or parent[i] < 0]
    L = np.full(n, -1, dtype=np.int32)
    for k, i in enumerate(roots):
        L[i] = k
    order = sorted(range(n), key=lambda i: (-rho[i], i))          # decreasing density
    for i in order:
        if L[i] == -1:
            assert L[parent[i]] != -1, "a parent is strictly denser, so it was labelled before"
            L[i] = L[parent[i]]
    return L, np.array(roots, dtype=np.int32)


def vic_cluster(feat_bits, pos, d_c: float, tau: float, n_centers: int):
    """Alg. 2 end to end for one image.  Returns a dict of every intermediate."""
    d_feat = feature_distances(feat_bits)
    d_sp = spatial_distances(pos)
    rho = density(d_feat, d_c)
    delta, parent = parents(d_feat, d_sp, rho, tau)
    gamma = importance(rho, delta)
    c = centers(gamma, n_centers)
    L, roots = labels(rho, parent, c)
    return {"d_feat": d_feat, "d_spatial": d_sp, "rho": rho, "delta": delta, "parent": parent,
            "gamma": gamma, "centers": c, "labels": L, "roots": roots}


def same_partition(a, b) -> bool:
    """True if two label arrays describe the same partition (labels are names)."""
    a = np.asarray(a)
    b = np.asarray(b)
    if a.shape != b.shape:
        return False
    fwd, bwd = {}, {}
    for x, y in zip(a.tolist(), b.tolist()):
        if fwd.setdefault(x, y) != y or bwd.setdefault(y, x) != x:
            return False
    return True


# ---------------------------------------------------------------------------
# Visual-textual collaborative pruning and merging (Sec. 3.2.3, Eq. 5-6; Alg. 3)
# ---------------------------------------------------------------------------
# Readings: B - N_c is taken as 0 when the budget is below the number of clusters (the listing
# would give negative quotas); "sort by K-norm ascending" is stable, so equal norms go to the
# lower index; the output set is laid out as the elites in ascending token index followed by the
# merged tokens in cluster-label order; a merged token is represented, for position purposes, by
# the lowest-index token it absorbed (the paper treats V_out as a set and says nothing of
# positions).  floor(|C_c| / n * (B - N_c)) is evaluated exactly, as an integer division.

def collab_prune_merge(feat_bits, labels, k_norms, budget: int):
    """Alg. 3 for one image.  feat_bits [n, D] bf16 bits, labels [n] in [0, N_c), k_norms [n].

    Returns a dict: ``quota`` [N_c], ``elite`` bool [n], ``feats`` float64 [n_out, D] (elites
    are the input rows, merged rows are the fp64 means of Eq. 6), ``index`` int32 [n_out]
    (elite: its token; merged: lowest-index absorbed token), ``assign`` int32 [n] (the output
    row every input token went to), ``n_elite``.
    """
    f = _bf16_to_f64(feat_bits)
    labels = np.asarray(labels, dtype=np.int64)
    norms = np.asarray(k_norms, dtype=np.float64)
    n = len(labels)
    n_c = int(labels.max()) + 1 if n else 0
    clusters = [[i for i in range(n) if labels[i] == c] for c in range(n_c)]      # GroupTokensByLabel
    assert all(len(c) > 0 for c in clusters), "labels must be the dense names 0..N_c-1"
    b_elites = max(0, budget - n_c)
    quota = np.zeros(n_c, dtype=np.int64)
    elite = np.zeros(n, dtype=bool)
    remaining = []
    for c, members in enumerate(clusters):
        quota[c] = (len(members) * b_elites) // n                                 # Eq. 5
        ranked = sorted(members, key=lambda i: (norms[i], i))                     # ascending K-norm
        for i in ranked[:quota[c]]:
            elite[i] = True
        remaining.append(sorted(ranked[quota[c]:]))
    elite_idx = [i for i in range(n) if elite[i]]
    rows, index = [f[i] for i in elite_idx], list(elite_idx)
    assign = np.full(n, -1, dtype=np.int32)
    for r, i in enumerate(elite_idx):
        assign[i] = r
    for c, rem in enumerate(remaining):
        if rem:
            rows.append(f[rem].sum(axis=0) / len(rem))                            # Eq. 6
            for i in rem:
                assign[i] = len(index)
            index.append(rem[0])
    feats = np.stack(rows) if rows else np.zeros((0, f.shape[1]))
    return {"quota": quota, "elite": elite, "feats": feats, "index": np.array(index, dtype=np.int32),
            "assign": assign, "n_elite": len(elite_idx)}
