"""GPU parity: causal prefill attention vs the oracle's exact softmax(QK^T)V."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O
from gpu_util import assert_attention_close, dev, host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def run(vc, t, causal=True, scale=0.0, lse=True):
    out, l = vc.vitcop_prefill_attn(dev(t["q"]), dev(t["k"]), dev(t["v"]), scale, causal, lse)
    torch.cuda.synchronize()
    return host_f64(out), (l.cpu().numpy().astype(np.float64) if lse else None)


# N spans: single row, inside one 32-row wavefront tile, exactly one key tile, ragged
# tails, several query blocks
@pytest.mark.parametrize("N", [1, 2, 31, 32, 33, 64, 65, 100, 127, 128, 129, 191, 300, 517])
def test_causal_sizes(vc, N):
    t = I.qkv_tensors(100 + N, 2, N, 3, 3, 128)
    out, lse = run(vc, t)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
    assert_attention_close(out, ref, f"N={N}")
    assert np.abs(lse - ref_lse).max() < 1e-3


# with few heads a wavefront owns one 32-query block at every length: block edges (128 queries per workgroup),
# ragged tails, several blocks, more key tiles than the ring has stages
@pytest.mark.parametrize("N", [320, 321, 384, 500, 511, 512, 513, 640, 784, 1024, 1025, 1087, 1280, 1500, 2100])
def test_causal_long(vc, N):
    t = I.qkv_tensors(150 + N, 1, N, 2, 2, 128)
    out, lse = run(vc, t)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
    assert_attention_close(out, ref, f"N={N}")
    assert np.abs(lse - ref_lse).max() < 1e-3


# enough (sample, head) pairs that 256-query workgroups fill the chip: from 512 tokens on a wavefront then owns
# two 32-query blocks.  Block edges, ragged first blocks, GQA, and the case just below the switch (one block)
@pytest.mark.parametrize("B,N,Hq,Hkv,causal", [
    (5, 512, 28, 4, True), (5, 513, 28, 4, True), (3, 777, 24, 24, True), (2, 1025, 28, 4, True),
    (2, 1300, 24, 8, True), (2, 1300, 24, 8, False), (5, 511, 28, 4, True), (1, 1025, 28, 4, True)])
def test_many_heads_two_query_blocks_per_wavefront(vc, B, N, Hq, Hkv, causal):
    t = I.qkv_tensors(170 + N + B, B, N, Hq, Hkv, 128)
    out, lse = run(vc, t, causal=causal)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], None, causal)
    assert_attention_close(out, ref, f"B={B} N={N} {Hq}/{Hkv} causal={causal}")
    assert np.abs(lse - ref_lse).max() < 1e-3


def test_long_gqa_batch_and_non_causal(vc):
    t = I.qkv_tensors(160, 2, 1111, 8, 2, 128)
    out, lse = run(vc, t)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
    assert_attention_close(out, ref, "long GQA")
    assert np.abs(lse - ref_lse).max() < 1e-3
    t = I.qkv_tensors(161, 1, 1300, 2, 1, 128)
    out, lse = run(vc, t, causal=False)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], None, False)
    assert_attention_close(out, ref, "long non-causal")
    assert np.abs(lse - ref_lse).max() < 1e-3


def test_long_large_logits(vc):
    # logits of order +-100 with outliers: exercises the deferred rescaling of the accumulators
    t = I.qkv_tensors(162, 1, 1200, 2, 2, 128, std=3.0)
    out, lse = run(vc, t, scale=0.11)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], 0.11)
    assert_attention_close(out, ref, "long large logits", v_scale=3.0)
    assert np.abs(lse - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("N,d,H", [(1500, 128, 2), (300, 128, 2), (700, 64, 2), (1040, 128, 56)])
def test_rising_scores_move_the_reference(vc, N, d, H):
    # scores that climb along the keys by several hundred in the exponent: the kernels raise their reference
    # maximum again and again (and rescale what they have accumulated), also inside diagonal tiles; softmax
    # weight sits on the last visible keys, so every row checks the state after all those moves
    # (56 heads: two query blocks per wavefront, each with a reference of its own)
    g = np.random.default_rng(77 + N)
    q = np.ones((1, N, H, d), np.float32) + 0.05 * g.standard_normal((1, N, H, d)).astype(np.float32)
    ramp = (np.arange(N, dtype=np.float32) / N * 6.0)[None, :, None, None]
    k = ramp * np.ones((1, N, H, d), np.float32) + 0.05 * g.standard_normal((1, N, H, d)).astype(np.float32)
    t = {"q": I.f32_to_bf16_bits(q), "k": I.f32_to_bf16_bits(k), "v": I.normal_bf16(78 + N, 3, (1, N, H, d))}
    out, lse = run(vc, t)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
    assert ref_lse.max() - ref_lse.min() > 40.0                  # the logits do span hundreds of bits
    assert_attention_close(out, ref, f"rising scores N={N} d={d}")
    assert np.abs(lse - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("N", [5, 64, 130, 257])
def test_non_causal(vc, N):
    t = I.qkv_tensors(200 + N, 1, N, 2, 2, 128)
    out, lse = run(vc, t, causal=False)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], None, False)
    assert_attention_close(out, ref, f"non-causal N={N}")
    assert np.abs(lse - ref_lse).max() < 1e-3


@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (8, 2), (6, 1)])
def test_gqa(vc, Hq, Hkv):
    t = I.qkv_tensors(300 + Hq, 1, 150, Hq, Hkv, 128)
    out, _ = run(vc, t)
    ref, _ = O.attention(t["q"], t["k"], t["v"])
    assert_attention_close(out, ref, f"GQA {Hq}/{Hkv}")


def test_explicit_scale_and_large_logits(vc):
    t = I.qkv_tensors(400, 1, 140, 2, 2, 128, std=3.0)       # logits of order +-100
    out, lse = run(vc, t, scale=0.11)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], 0.11)
    assert_attention_close(out, ref, "large logits", v_scale=3.0)
    assert np.abs(lse - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_structure_pins(vc):
    t = I.qkv_tensors(500, 1, 200, 2, 2, 128)
    ones = I.f32_to_bf16_bits(np.ones((1, 200, 2, 128), np.float32))
    out, _ = run(vc, dict(t, v=ones))
    assert np.abs(out - 1.0).max() < 1e-2                       # rows of softmax sum to 1
    out, _ = run(vc, t)
    v = I.bf16_bits_to_f32(t["v"]).astype(np.float64)
    assert np.array_equal(out[0, 0], v[0, 0])                   # row 0 sees key 0 only
    kk = np.tile(t["k"][:, :1], (1, 200, 1, 1))
    out, _ = run(vc, dict(t, k=kk))
    run_mean = np.cumsum(v[0], axis=0) / np.arange(1, 201)[:, None, None]
    assert np.abs(out[0] - run_mean).max() < 2e-2


def test_config0_pruned_shape_and_unpruned_shape(vc):
    for N in (128, 640):
        t = I.qkv_tensors(600 + N, 1, N, 32, 32, 128)
        out, lse = run(vc, t)
        ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
        assert_attention_close(out, ref, f"config0 N={N}")
        assert np.abs(lse - ref_lse).max() < 1e-3


# head dimension 64 (the vision encoder's, and small language models')
@pytest.mark.parametrize("N", [1, 33, 64, 65, 129, 300, 577, 1111])
def test_head_dim_64_causal(vc, N):
    t = I.qkv_tensors(800 + N, 2, N, 4, 2, 64)
    out, lse = run(vc, t)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"])
    assert_attention_close(out, ref, f"d=64 N={N}")
    assert np.abs(lse - ref_lse).max() < 1e-3


def test_head_dim_64_non_causal_and_scale(vc):
    t = I.qkv_tensors(850, 1, 577, 16, 16, 64)                  # one CLIP-L image: 576 patches + [CLS]
    out, lse = run(vc, t, causal=False)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], None, False)
    assert_attention_close(out, ref, "d=64 non-causal")
    assert np.abs(lse - ref_lse).max() < 1e-3
    t = I.qkv_tensors(851, 1, 200, 2, 2, 64, std=3.0)
    out, lse = run(vc, t, scale=0.2)
    ref, ref_lse = O.attention(t["q"], t["k"], t["v"], 0.2)
    assert_attention_close(out, ref, "d=64 large logits", v_scale=3.0)
    assert np.abs(lse - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_deterministic(vc):
    t = I.qkv_tensors(700, 2, 300, 4, 2, 128)
    q, k, v = dev(t["q"]), dev(t["k"]), dev(t["v"])
    a, _ = vc.vitcop_prefill_attn(q, k, v)
    for _ in range(5):
        b, _ = vc.vitcop_prefill_attn(q, k, v)
        assert torch.equal(a, b)
