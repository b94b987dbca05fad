"""GPU parity: compaction (bit-exact) and the Stage I filter (Eq. 1 + TopK) vs the oracle."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O
from gpu_util import assert_selection_matches, dev, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


# ------------------------------------------------------------------ compaction

def test_compact_bit_exact_multi_tensor(vc):
    g = np.random.default_rng(0)
    B, T, To = 3, 211, 97
    hid = g.integers(0, 65536, size=(B, T, 4096), dtype=np.uint16)
    kv = g.integers(0, 65536, size=(B, T, 4, 128), dtype=np.uint16)
    odd = g.integers(0, 65536, size=(B, T, 6), dtype=np.uint16)          # 12-byte rows: 4-byte path
    pos = g.integers(0, 1 << 30, size=(B, T), dtype=np.int32)
    idx = np.stack([np.sort(g.permutation(T)[:To]) for _ in range(B)]).astype(np.int32)
    outs = vc.vitcop_compact([dev(hid), dev(kv), dev(odd), torch.from_numpy(pos).cuda()],
                             torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(outs[0]), O.compact(hid, idx))
    assert np.array_equal(host_bits(outs[1]), O.compact(kv, idx))
    assert np.array_equal(host_bits(outs[2]), O.compact(odd, idx))
    assert np.array_equal(outs[3].cpu().numpy(), O.compact(pos[:, :, None], idx)[:, :, 0])


def test_compact_identity_empty_and_repeats(vc):
    g = np.random.default_rng(1)
    src = g.integers(0, 65536, size=(2, 50, 256), dtype=np.uint16)
    ident = np.tile(np.arange(50, dtype=np.int32), (2, 1))
    (out,) = vc.vitcop_compact([dev(src)], torch.from_numpy(ident).cuda())
    assert np.array_equal(host_bits(out), src)
    (out,) = vc.vitcop_compact([dev(src)], torch.zeros((2, 0), dtype=torch.int32, device="cuda"))
    assert out.shape == (2, 0, 256)
    rep = np.array([[3, 3, 49, 0], [0, 0, 0, 1]], dtype=np.int32)       # a gather, not only a filter
    (out,) = vc.vitcop_compact([dev(src)], torch.from_numpy(rep).cuda())
    assert np.array_equal(host_bits(out), O.compact(src, rep))


def test_compact_composition(vc):
    c = I.k_tensor_lognormal(8, 2, 120, 4, 128, 0, 120)
    _, i1 = O.knorm_select(c["k"], 0, 120, 60)
    k1 = O.compact(c["k"], i1)
    _, i2 = O.knorm_select(k1, 0, 60, 20)
    (a,) = vc.vitcop_compact([dev(c["k"])], torch.from_numpy(i1).cuda())
    (b,) = vc.vitcop_compact([a], torch.from_numpy(i2).cuda())
    composed = np.take_along_axis(i1, i2, axis=1)
    (d,) = vc.vitcop_compact([dev(c["k"])], torch.from_numpy(composed).cuda())
    assert torch.equal(b, d) and np.array_equal(host_bits(b), O.compact(c["k"], composed))


# ---------------------------------------------------------------------- filter

def check_filter(vc, c, keep, what, scale=0.0):
    scores, idx = vc.vitcop_filter_visual(dev(c["q_cls"]), dev(c["k"]), keep, scale)
    torch.cuda.synchronize()
    scores, idx = scores.cpu().numpy(), idx.cpu().numpy()
    S, ref_idx = O.filter_visual(c["q_cls"], c["k"], keep, None if scale == 0.0 else scale)
    assert np.allclose(scores, S, rtol=2e-4, atol=1e-7), what
    for b in range(S.shape[0]):
        assert_selection_matches(idx[b], scores[b], S[b], keep, True, f"{what} b={b}")


@pytest.mark.parametrize("B,N,H,d", [(2, 64, 4, 64), (3, 197, 16, 64), (1, 50, 12, 64),
                                     (2, 100, 8, 128), (1, 33, 3, 128), (1, 300, 16, 128)])
def test_filter_shapes(vc, B, N, H, d):
    c = I.config1(B=B, N=N, C=256, H=H, d=d, n_centroids=16)
    check_filter(vc, c, N // 2, f"B{B} N{N} H{H} d{d}")
    check_filter(vc, c, 1, "keep 1")


def test_filter_config1_full(vc):
    c = I.config1()
    assert c["k"].shape == (8, 577, 16, 64)
    check_filter(vc, c, 288, "config 1")
    check_filter(vc, c, 0, "keep none")
    check_filter(vc, c, 576, "keep all")
    check_filter(vc, c, 100, "explicit scale", scale=0.07)


def test_filter_video_frames(vc):
    c = I.config4_frames(n_frames=6)
    check_filter(vc, c, c["keep"], "video frames")


def test_filter_uniform_and_planted(vc):
    H, d, N = 16, 64, 120
    g = np.random.default_rng(4)
    q = g.standard_normal((1, H, d)).astype(np.float32)
    k = np.tile(g.standard_normal((1, 1, H, d)).astype(np.float32), (1, N + 1, 1, 1))
    scores, idx = vc.vitcop_filter_visual(dev(I.f32_to_bf16_bits(q)), dev(I.f32_to_bf16_bits(k)), 17)
    assert idx.cpu().numpy()[0].tolist() == list(range(17))          # all tie -> lowest indices
    assert np.allclose(scores.cpu().numpy(), H / (N + 1), rtol=1e-5)
    k2 = g.standard_normal((1, N + 1, H, d)).astype(np.float32)
    k2[0, 1 + 77] = 3.0 * q[0]
    _, idx = vc.vitcop_filter_visual(dev(I.f32_to_bf16_bits(q)), dev(I.f32_to_bf16_bits(k2)), 1)
    assert idx.cpu().numpy()[0, 0] == 77
