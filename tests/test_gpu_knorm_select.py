"""GPU parity: K-norm saliency + selection (Eq. 4, Alg. 1 Stage III) vs the oracle."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O
from gpu_util import assert_selection_matches, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def check(vc, kbits, vis_start, n_vis, keep, what):
    B, T = kbits.shape[:2]
    norms, idx = vc.vitcop_knorm_select(dev(kbits), vis_start, n_vis, keep)
    torch.cuda.synchronize()
    norms, idx = norms.cpu().numpy(), idx.cpu().numpy()
    ref_n, ref_idx = O.knorm_select(kbits, vis_start, n_vis, keep)
    assert np.allclose(norms, ref_n, rtol=2e-6, atol=0), what
    assert idx.shape == ref_idx.shape
    for b in range(B):
        assert np.array_equal(idx[b, :vis_start], np.arange(vis_start)), what
        assert np.array_equal(idx[b, vis_start + keep:], np.arange(vis_start + n_vis, T)), what
        assert_selection_matches(idx[b, vis_start:vis_start + keep] - vis_start, norms[b], ref_n[b],
                                 keep, False, f"{what} b={b}")


# (B, T, Hkv, d, vis_start, n_vis, keep): every row-length code path, ragged tails
SHAPES = [
    (1, 640, 32, 128, 35, 576, 64),     # config 0 (4096-element rows)
    (2, 301, 4, 128, 0, 290, 29),       # GQA rows of 512 elements, 8 rows per wavefront, ragged
    (3, 137, 8, 128, 5, 101, 50),       # 1024
    (2, 75, 16, 128, 3, 70, 7),         # 2048, 2 rows per wavefront, odd count
    (1, 50, 64, 128, 1, 47, 46),        # 8192
    (2, 90, 3, 64, 10, 61, 20),         # 192 elements: generic path
    (1, 70, 5, 128, 0, 70, 35),         # 640 elements: generic path
]


@pytest.mark.parametrize("shape", SHAPES)
def test_matches_oracle(vc, shape):
    B, T, Hkv, d, vs, nv, keep = shape
    c = I.k_tensor_lognormal(77 + T, B, T, Hkv, d, vs, nv)
    check(vc, c["k"], vs, nv, keep, str(shape))


def test_edge_budgets(vc):
    c = I.k_tensor_lognormal(5, 2, 40, 4, 128, 6, 30)
    for keep in (0, 1, 29, 30):
        check(vc, c["k"], 6, 30, keep, f"keep={keep}")
    # no visual tokens at all: the list is the identity
    norms, idx = vc.vitcop_knorm_select(dev(c["k"]), 10, 0, 0)
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(40), (2, 1)))


def test_exact_ties_go_to_the_lower_index(vc):
    # groups of identical rows: norms tie exactly; the cut falls inside a group
    g = np.random.default_rng(3)
    base = g.standard_normal((6, 4 * 128)).astype(np.float32)
    rows = base[g.integers(0, 6, size=200)]
    k = I.f32_to_bf16_bits(rows).reshape(1, 200, 4, 128)
    for keep in (10, 50, 100, 150):
        norms, idx = vc.vitcop_knorm_select(dev(k), 0, 200, keep)
        ref_n, ref_idx = O.knorm_select(k, 0, 200, keep)
        assert np.array_equal(idx.cpu().numpy(), ref_idx), keep      # bit-exact, ties included
    ones = I.f32_to_bf16_bits(np.ones((1, 64, 4, 128), np.float32))
    _, idx = vc.vitcop_knorm_select(dev(ones), 8, 48, 5)
    assert idx.cpu().numpy()[0].tolist() == list(range(8)) + [8, 9, 10, 11, 12] + list(range(56, 64))


def test_planted_norms_and_power_of_two_scaling(vc):
    k = np.zeros((1, 300, 4, 128), np.float32)
    g = np.random.default_rng(9)
    expo = g.permutation(300) % 40 - 20
    k[0, :, 0, 0] = 2.0 ** expo
    kb = I.f32_to_bf16_bits(k)
    norms, idx = vc.vitcop_knorm_select(dev(kb), 0, 300, 77)
    assert np.array_equal(norms.cpu().numpy()[0], (2.0 ** expo).astype(np.float32))
    assert np.array_equal(idx.cpu().numpy(), O.knorm_select(kb, 0, 300, 77)[1])
    c = I.k_tensor_lognormal(21, 1, 200, 4, 128, 0, 200)
    _, base = vc.vitcop_knorm_select(dev(c["k"]), 0, 200, 60)
    scaled = I.f32_to_bf16_bits(I.bf16_bits_to_f32(c["k"]) * np.float32(2.0 ** -7))
    _, idx2 = vc.vitcop_knorm_select(dev(scaled), 0, 200, 60)
    assert torch.equal(base, idx2)


def test_maximum_candidate_count(vc):
    n = vc.VITCOP_MAX_CANDIDATES
    c = I.k_tensor_lognormal(31, 1, n + 7, 1, 64, 3, n)
    check(vc, c["k"], 3, n, n // 10, "max candidates")
    with pytest.raises(vc.VitcopError):
        vc.vitcop_knorm_select(dev(c["k"][:, :8]), 0, 8, 9)


def test_strided_k_inside_fused_qkv_buffer(vc):
    B, T, Hkv, d, vs, nv, keep = 2, 100, 4, 128, 10, 80, 25
    c = I.k_tensor_lognormal(41, B, T, Hkv, d, vs, nv)
    row = Hkv * d
    fused = torch.zeros((B, T + 3, 3 * row), dtype=torch.bfloat16, device="cuda")
    fused[:, :T, row:2 * row] = dev(c["k"]).reshape(B, T, row)
    kview = fused[:, :, row:2 * row]
    norms, idx = vc.vitcop_knorm_select(kview, vs, nv, keep, shape=(B, T, Hkv, d),
                                        k_row_stride=3 * row, k_batch_stride=(T + 3) * 3 * row)
    ref_n, ref_idx = O.knorm_select(c["k"], vs, nv, keep)
    assert np.allclose(norms.cpu().numpy(), ref_n, rtol=2e-6)
    for b in range(B):
        assert_selection_matches(idx.cpu().numpy()[b, vs:vs + keep] - vs, norms.cpu().numpy()[b],
                                 ref_n[b], keep, False, "strided")


def test_precomputed_and_squared_norms(vc):
    g = np.random.default_rng(2)
    s = (g.random((3, 500)) * 10 + 0.1).astype(np.float32)
    T, vs, nv, keep = 520, 12, 500, 123
    n_in = torch.from_numpy(s).cuda()
    norms, idx = vc.vitcop_knorm_select(None, vs, nv, keep, norms=n_in.clone(), shape=(3, T, 4, 128),
                                        flags=vc.VITCOP_NORMS_PRECOMPUTED)
    assert np.array_equal(idx.cpu().numpy(), O.keep_list(s.astype(np.float64), T, vs, keep))
    sq = n_in * n_in
    norms2, idx2 = vc.vitcop_knorm_select(None, vs, nv, keep, norms=sq.clone(), shape=(3, T, 4, 128),
                                          flags=vc.VITCOP_NORMS_PRECOMPUTED | vc.VITCOP_NORMS_SQUARED)
    assert np.allclose(norms2.cpu().numpy(), s, rtol=3e-7)
    for b in range(3):
        assert_selection_matches(idx2.cpu().numpy()[b, vs:vs + keep] - vs, norms2.cpu().numpy()[b],
                                 s[b].astype(np.float64), keep, False, "squared")


def test_deterministic(vc):
    c = I.k_tensor_lognormal(51, 4, 640, 32, 128, 35, 576)
    k = dev(c["k"])
    n0, i0 = vc.vitcop_knorm_select(k, 35, 576, 64)
    for _ in range(10):
        n1, i1 = vc.vitcop_knorm_select(k, 35, 576, 64)
        assert torch.equal(n0, n1) and torch.equal(i0, i1)
