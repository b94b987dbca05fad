"""Pins of the collaborative pruning and merging oracle (Sec. 3.2.3, Eq. 5-6, Alg. 3)."""
import numpy as np
import pytest

import vitcop_inputs as I
from oracle import vic_oracle as V
from oracle import vitcop_oracle as O


def bits(a):
    return I.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_hand_example():
    # 7 tokens, clusters {0,1,2,3}, {4,5}, {6}; budget 6 -> 3 elites to share: floor(4*3/7)=1, 0, 0
    feats = bits(np.arange(7)[:, None] * np.ones((1, 4)))           # token i = (i,i,i,i)
    labels = [0, 0, 0, 0, 1, 1, 2]
    norms = [5.0, 2.0, 9.0, 2.0, 1.0, 3.0, 7.0]
    r = V.collab_prune_merge(feats, labels, norms, 6)
    assert r["quota"].tolist() == [1, 0, 0]
    assert np.where(r["elite"])[0].tolist() == [1]                  # norms 2.0 at tokens 1 and 3: lower index
    assert r["index"].tolist() == [1, 0, 4, 6]                      # elite, then merged clusters 0, 1, 2
    want = [[1.0] * 4, [(0 + 2 + 3) / 3] * 4, [4.5] * 4, [6.0] * 4]
    assert np.allclose(r["feats"], want, rtol=0, atol=1e-15)
    assert r["assign"].tolist() == [1, 0, 1, 1, 2, 2, 3]
    # budget 10 -> 7 elites to share: 4, 2, 1: everybody is an elite, nothing is merged
    r = V.collab_prune_merge(feats, labels, norms, 10)
    assert r["quota"].tolist() == [4, 2, 1] and r["index"].tolist() == list(range(7))
    # budget below the number of clusters: no elites, one merged token per cluster
    r = V.collab_prune_merge(feats, labels, norms, 2)
    assert r["quota"].tolist() == [0, 0, 0] and r["index"].tolist() == [0, 4, 6]


def random_case(seed, n=150, D=32, n_c=9):
    g = np.random.default_rng(seed)
    labels = np.concatenate([np.arange(n_c), g.integers(0, n_c, n - n_c)])
    g.shuffle(labels)
    feats = bits(g.standard_normal((n, D)))
    norms = g.lognormal(0.0, 0.5, n).astype(np.float32)
    return feats, labels, norms


@pytest.mark.parametrize("budget", [9, 20, 64, 100, 150])
def test_counts_mass_and_order(budget):
    feats, labels, norms = random_case(3 + budget)
    n, n_c = len(labels), 9
    r = V.collab_prune_merge(feats, labels, norms, budget)
    sizes = np.bincount(labels, minlength=n_c)
    # Eq. 5 against real arithmetic done another way (exact fractions)
    from fractions import Fraction
    import math
    assert r["quota"].tolist() == [math.floor(Fraction(int(s), n) * (budget - n_c)) for s in sizes]
    n_merged = int(np.sum(sizes - r["quota"] > 0))
    assert len(r["index"]) == r["quota"].sum() + n_merged <= budget
    # elites beat every remaining token of their cluster
    for c in range(n_c):
        m = np.where(labels == c)[0]
        e, rest = m[r["elite"][m]], m[~r["elite"][m]]
        assert len(e) == r["quota"][c]
        if len(e) and len(rest):
            assert norms[e].max() <= norms[rest].min()
    # Eq. 6 conserves mass: sum of outputs weighted by how many tokens each absorbed = sum of inputs
    f = O.bf16_to_f64(feats)
    weight = np.bincount(r["assign"], minlength=len(r["index"]))
    assert np.allclose((r["feats"] * weight[:, None]).sum(0), f.sum(0), rtol=0, atol=1e-9)
    assert np.all(r["assign"] >= 0) and np.array_equal(r["feats"][: r["n_elite"]], f[r["index"][: r["n_elite"]]])
    assert np.all(np.diff(r["index"][: r["n_elite"]]) > 0)


def test_single_cluster_reduces_to_topk_smallest():
    # one cluster, budget B: B-1 elites by smallest norm (the pinned TopK) + the mean of the rest
    feats, _, norms = random_case(77, n=60, n_c=1)
    r = V.collab_prune_merge(feats, np.zeros(60, dtype=int), norms, 20)
    want = O.topk_smallest(norms.astype(np.float64), 19)
    assert r["index"][:-1].tolist() == want.tolist()
    rest = np.setdiff1d(np.arange(60), want)
    assert np.allclose(r["feats"][-1], O.bf16_to_f64(feats)[rest].mean(0), atol=1e-12)
    assert r["index"][-1] == rest.min()


def test_ties_go_to_the_lower_index():
    feats = bits(np.eye(6))
    r = V.collab_prune_merge(feats, [0] * 6, [1.0] * 6, 4)
    assert np.where(r["elite"])[0].tolist() == [0, 1, 2] and r["index"].tolist() == [0, 1, 2, 3]
