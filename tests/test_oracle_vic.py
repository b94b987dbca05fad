"""Pins of the VIC oracle (Sec. 3.2.1, Eq. 2-3, Alg. 2) against things other than itself."""
import math

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import vitcop_inputs as I
from oracle import vic_oracle as V


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def line(points):
    """1-D features (exact in bf16) as [n,1] bits."""
    return bits(np.asarray(points, dtype=np.float32)[:, None])


def test_distances_match_library():
    c = I.vic_inputs(11, 40, 64)
    f = I.bf16_bits_to_f32(c["feats"]).astype(np.float64)
    assert np.allclose(V.feature_distances(c["feats"]), cdist(f, f), rtol=0, atol=1e-12)
    assert np.allclose(V.spatial_distances(c["pos"]), cdist(c["pos"].astype(np.float64), c["pos"].astype(np.float64)),
                       rtol=0, atol=1e-15)
    d = V.feature_distances(c["feats"])
    assert np.array_equal(d, d.T) and np.all(np.diag(d) == 0)


def test_density_closed_forms():
    # n identical tokens: every term is exp(0) = 1, the token itself excluded
    same = bits(np.ones((7, 5)))
    assert np.array_equal(V.density(V.feature_distances(same), 8.0), np.full(7, 6.0))
    # points 0, 1, 2.5, 10 on a line with d_c = 1 (Eq. 2 by hand)
    d = V.feature_distances(line([0, 1, 2.5, 10]))
    rho = V.density(d, 1.0)
    e = math.exp
    want = [e(-1) + e(-6.25) + e(-100), e(-1) + e(-2.25) + e(-81), e(-6.25) + e(-2.25) + e(-56.25),
            e(-100) + e(-81) + e(-56.25)]
    assert np.allclose(rho, want, rtol=1e-14)
    # d_c scales distances: doubling both leaves rho unchanged
    assert np.allclose(V.density(2.0 * d, 2.0), rho, rtol=1e-14)


def test_hand_example_parents_centres_labels():
    # same four points: densities order 1 > 0 > 2 > 3
    f = line([0, 1, 2.5, 10])
    pos = np.array([[0.1, 0.1], [0.1, 0.2], [0.2, 0.1], [0.2, 0.2]])
    r = V.vic_cluster(f, pos, 1.0, 10.0, 2)
    assert r["parent"].tolist() == [1, -1, 1, 2]
    assert r["delta"].tolist() == [1.0, np.inf, 1.5, 7.5]
    assert np.isinf(r["gamma"][1]) and r["gamma"][0] == r["rho"][0] * 1.0
    assert r["centers"].tolist() == [0, 1]                # gamma: inf, 0.3698, 0.1610, ~1e-24
    assert r["roots"].tolist() == [0, 1]
    assert r["labels"].tolist() == [0, 1, 1, 1]           # 2 -> 1, 3 -> 2 -> 1
    # one centre only: token 0 now follows its parent
    assert V.vic_cluster(f, pos, 1.0, 10.0, 1)["labels"].tolist() == [0, 0, 0, 0]
    # token 3 moved out of everyone's spatial reach: no parent, not a centre -> its own cluster
    far = pos.copy()
    far[3] = [0.9, 0.9]
    r = V.vic_cluster(f, far, 1.0, 0.6, 2)
    assert r["parent"].tolist() == [1, -1, 1, -1]
    assert r["centers"].tolist() == [1, 3]                # two infinite gammas
    assert r["labels"].tolist() == [0, 0, 0, 1]
    r = V.vic_cluster(f, far, 1.0, 0.6, 3)
    assert r["centers"].tolist() == [0, 1, 3] and r["labels"].tolist() == [0, 1, 1, 2]


def test_spatial_threshold_is_inclusive_and_density_strict():
    # two tokens exactly tau apart are neighbours; equal densities are never parents of each other
    f = line([0, 1, 2])
    pos = np.array([[0.0, 0.0], [0.0, 0.5], [0.0, 1.0]])
    d, ds = V.feature_distances(f), V.spatial_distances(pos)
    rho = V.density(d, 1.0)
    assert rho[0] == rho[2] < rho[1]
    delta, parent = V.parents(d, ds, rho, 0.5)
    assert parent.tolist() == [1, -1, 1]
    delta, parent = V.parents(d, ds, rho, 0.49)
    assert parent.tolist() == [-1, -1, -1]
    delta, parent = V.parents(d, ds, np.array([1.0, 1.0, 1.0]), 5.0)
    assert parent.tolist() == [-1, -1, -1]


def test_parents_against_independent_brute_force():
    # the definition walked pair by pair: a candidate replaces the current one only if it is strictly nearer
    c = I.vic_inputs(23, 60, 32, n_regions=5)
    d, ds = V.feature_distances(c["feats"]), V.spatial_distances(c["pos"])
    rho = V.density(d, 8.0)
    delta, parent = V.parents(d, ds, rho, 0.6)
    n_with = 0
    for i in range(60):
        best, arg = float("inf"), -1
        for j in range(60):
            if rho[j] > rho[i] and ds[i][j] <= 0.6 and d[i][j] < best:
                best, arg = d[i][j], j
        assert parent[i] == arg and (delta[i] == best or (arg < 0 and np.isinf(delta[i])))
        n_with += arg >= 0
    assert 0 < n_with < 60                                  # both branches were exercised


def test_equal_distance_candidates_go_to_the_lower_index():
    # token 2 sits exactly between two denser tokens
    f = line([0, 0.25, 2, 4, 3.75, -0.25, 4.25])
    pos = np.zeros((7, 2))
    d, ds = V.feature_distances(f), V.spatial_distances(pos)
    rho = V.density(d, 1.0)
    delta, parent = V.parents(d, ds, rho, 1.0)
    assert d[2, 0] == d[2, 3] and rho[0] > rho[2] and rho[3] > rho[2]
    assert parent[2] in (0, 1, 3, 4) and parent[2] == min(
        j for j in range(7) if rho[j] > rho[2] and d[2, j] == delta[2])


def balanced_regions(seed, n, regions, D=256):
    """First seed from ``seed`` on whose smallest region has more than a fifth of the largest
    one's tokens.  (A region's densest token scores about 0.7 (size-1) x 45, the runner-up inside
    a large region about 0.7 (size-1) x 4.5: density peaks only name every region if no region
    is tiny.)"""
    for s in range(seed, seed + 100):
        c = I.vic_inputs(s, n, D, n_regions=regions, noise=0.1)
        sizes = np.bincount(c["region"])
        sizes = sizes[sizes > 0]
        if sizes.min() >= 3 and sizes.min() - 1 > 0.2 * (sizes.max() - 1):
            return c
    raise AssertionError("no balanced seed")


@pytest.mark.parametrize("seed,n,regions", [(31, 150, 6), (32, 288, 12), (33, 172, 9)])
def test_recovers_planted_regions(seed, n, regions):
    # well separated regions, as many centres as regions: the partition must be the planted one
    c = balanced_regions(seed, n, regions)
    present = len(np.unique(c["region"]))
    r = V.vic_cluster(c["feats"], c["pos"], 8.0, 2.0, present)
    assert V.same_partition(r["labels"], c["region"])
    assert len(r["roots"]) == present


def test_structure_invariants_and_permutation():
    c = I.vic_inputs(41, 120, 64, n_regions=7, noise=0.3)
    r = V.vic_cluster(c["feats"], c["pos"], 8.0, 0.6, 10)
    L, parent, rho = r["labels"], r["parent"], r["rho"]
    roots = set(r["roots"].tolist())
    assert set(r["centers"].tolist()) <= roots and len(roots) >= 10
    assert [L[i] for i in sorted(roots)] == list(range(len(roots)))      # numbered by root index
    for i in range(120):
        if i not in roots:
            assert L[i] == L[parent[i]] and rho[parent[i]] > rho[i]
    # reordering the tokens reorders the labels: same partition
    perm = np.random.default_rng(5).permutation(120)
    rp = V.vic_cluster(c["feats"][perm], c["pos"][perm], 8.0, 0.6, 10)
    assert V.same_partition(rp["labels"], L[perm])
    # scaling the features and d_c together changes nothing
    f2 = I.f32_to_bf16_bits(I.bf16_bits_to_f32(c["feats"]) * np.float32(2.0))
    r2 = V.vic_cluster(f2, c["pos"], 16.0, 0.6, 10)
    assert np.array_equal(r2["labels"], L) and np.array_equal(r2["parent"], parent)


def test_centres_edge_counts():
    c = I.vic_inputs(51, 30, 16, n_regions=3)
    r0 = V.vic_cluster(c["feats"], c["pos"], 8.0, 0.6, 0)
    assert len(r0["centers"]) == 0 and set(r0["roots"].tolist()) == set(np.where(r0["parent"] < 0)[0].tolist())
    rn = V.vic_cluster(c["feats"], c["pos"], 8.0, 0.6, 30)
    assert rn["labels"].tolist() == list(range(30))
