"""GPU parity: collaborative pruning and merging (Sec. 3.2.3, Eq. 5-6, Alg. 3) vs the oracle.

Quotas, elite sets, row layout and representatives are integer work on the given labels and fp32
norms: bit-exact.  Elite rows are bit copies; merged rows are means accumulated in fp32 and must
round to bf16 within half an ulp (plus the fp32 accumulation error) of the fp64 mean.
"""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vic_oracle as V
from oracle import vitcop_oracle as O
from gpu_util import dev, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def case(seed, n, D, n_c):
    g = np.random.default_rng(seed)
    labels = np.concatenate([np.arange(n_c), g.integers(0, n_c, n - n_c)]).astype(np.int32)
    g.shuffle(labels)
    feats = I.f32_to_bf16_bits(g.standard_normal((n, D)).astype(np.float32))
    norms = g.lognormal(0.0, 0.5, n).astype(np.float32)
    norms[g.integers(0, n, n // 10)] = norms[0]                 # some exact ties
    return feats, labels, norms


def run(vc, cases, budget):
    feats = dev(np.stack([c[0] for c in cases]))
    labels = torch.from_numpy(np.stack([c[1] for c in cases])).cuda()
    ncl = torch.tensor([int(c[1].max()) + 1 for c in cases], dtype=torch.int32, device="cuda")
    norms = torch.from_numpy(np.stack([c[2] for c in cases])).cuda()
    r = vc.vitcop_collab_prune_merge(feats, labels, ncl, norms, budget)
    torch.cuda.synchronize()
    return r


def check(r, b, c, budget):
    feats, labels, norms = c
    ref = V.collab_prune_merge(feats, labels, norms, budget)
    n_out = int(r["n_out"][b])
    assert n_out == len(ref["index"])
    assert np.array_equal(r["index"][b, :n_out].cpu().numpy(), ref["index"])
    assert np.array_equal(r["assign"][b].cpu().numpy(), ref["assign"])
    got = host_bits(r["feats"][b, :n_out])
    ne = ref["n_elite"]
    assert np.array_equal(got[:ne], feats[ref["index"][:ne]])                 # elites: bit copies
    want = ref["feats"][ne:]
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    err = np.abs(O.bf16_to_f64(got[ne:]) - want)
    assert np.all(err <= 0.5 * ulp + 1e-6 * np.maximum(np.abs(want), 1e-3)), "merged rows"


@pytest.mark.parametrize("n,D,n_c,budget", [(7, 8, 3, 6), (150, 64, 9, 64), (150, 64, 9, 9), (150, 64, 9, 4),
                                            (288, 4096, 29, 192), (288, 4096, 29, 400), (1856, 512, 186, 627),
                                            (65, 40, 1, 20), (64, 8, 64, 64)])
def test_matches_oracle(vc, n, D, n_c, budget):
    c = case(8000 + n + budget, n, D, n_c)
    check(run(vc, [c], budget), 0, c, budget)


def test_batch_and_empty(vc):
    cases = [case(8100 + b, 120, 128, 5 + b) for b in range(3)]
    r = run(vc, cases, 40)
    for b, c in enumerate(cases):
        check(r, b, c, 40)
    feats = torch.empty((2, 0, 64), dtype=torch.bfloat16, device="cuda")
    z = torch.zeros((2,), dtype=torch.int32, device="cuda")
    r = vc.vitcop_collab_prune_merge(feats, torch.empty((2, 0), dtype=torch.int32, device="cuda"), z,
                                     torch.empty((2, 0), dtype=torch.float32, device="cuda"), 10)
    torch.cuda.synchronize()
    assert r["n_out"].cpu().tolist() == [0, 0]


def test_after_vic_on_the_gpu(vc):
    # Stage II as the paper chains it: clusters from VIC, norms of the tokens, one budget
    c = I.vic_inputs(8200, 288, 1024, n_regions=12, noise=0.2)
    feats = dev(c["feats"][None])
    pos = torch.from_numpy(c["pos"][None]).cuda()
    v = vc.vitcop_vic_cluster(feats, pos, 8.0, 0.6, 29)
    norms = torch.from_numpy(np.random.default_rng(1).lognormal(0, 0.5, (1, 288)).astype(np.float32)).cuda()
    r = vc.vitcop_collab_prune_merge(feats, v["labels"], v["n_clusters"], norms, 192)
    torch.cuda.synchronize()
    labels = v["labels"][0].cpu().numpy()
    assert labels.max() + 1 == int(v["n_clusters"][0])
    check(r, 0, (c["feats"], labels, norms[0].cpu().numpy()), 192)
    assert int(r["n_out"][0]) <= 192


def test_deterministic(vc):
    c = case(8300, 500, 256, 40)
    a = run(vc, [c], 200)
    for _ in range(3):
        b = run(vc, [c], 200)
        n = int(a["n_out"][0])
        assert torch.equal(a["feats"][0, :n], b["feats"][0, :n]) and torch.equal(a["index"][0, :n], b["index"][0, :n])
