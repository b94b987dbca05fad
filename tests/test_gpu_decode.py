"""GPU parity: one decoding step over a (compacted) KV cache vs the oracle's softmax(K q) V."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import decoder_oracle as Dc
from gpu_util import assert_attention_close, dev, host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def run(vc, t, scale=0.0):
    q = dev(t["q"][:, -1])
    o, lse = vc.vitcop_decode_attn(q, dev(t["k"]), dev(t["v"]), scale)
    torch.cuda.synchronize()
    return host_f64(o), lse.cpu().numpy().astype(np.float64)


# cache lengths: one key, inside one lane group, slice edges (64), ragged, several slices;
# head layouts: MHA, the video model's 28/4, a group above 8, d = 64
@pytest.mark.parametrize("B,N,Hq,Hkv,d", [(1, 1, 2, 2, 128), (2, 3, 4, 2, 128), (2, 64, 4, 4, 128), (1, 65, 6, 2, 64),
                                          (3, 384, 32, 32, 128), (1, 755, 28, 4, 128), (2, 1000, 20, 2, 128),
                                          (1, 2944, 8, 8, 128), (4, 224, 16, 16, 64), (1, 6400, 28, 4, 128)])
def test_matches_oracle(vc, B, N, Hq, Hkv, d):
    t = I.qkv_tensors(9500 + N + Hq, B, N, Hq, Hkv, d)
    out, lse = run(vc, t)
    ref, ref_lse = Dc.decode_attention(t["q"][:, -1], t["k"], t["v"])
    assert_attention_close(out, ref, f"decode N={N}")
    assert np.abs(lse - ref_lse).max() < 1e-3


def test_scale_large_logits_and_structure(vc):
    t = I.qkv_tensors(9600, 2, 300, 4, 2, 128, std=3.0)
    out, lse = run(vc, t, scale=0.11)
    ref, ref_lse = Dc.decode_attention(t["q"][:, -1], t["k"], t["v"], 0.11)
    assert_attention_close(out, ref, "decode large logits", v_scale=3.0)
    assert np.abs(lse - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())
    ones = I.f32_to_bf16_bits(np.ones((2, 300, 2, 128), np.float32))
    out, _ = run(vc, dict(t, v=ones))
    assert np.abs(out - 1.0).max() < 1e-2                         # softmax weights sum to 1


def test_decode_equals_last_row_of_prefill_and_is_deterministic(vc):
    t = I.qkv_tensors(9700, 2, 500, 8, 2, 128)
    q, k, v = dev(t["q"]), dev(t["k"]), dev(t["v"])
    full, _ = vc.vitcop_prefill_attn(q, k, v)
    o, _ = vc.vitcop_decode_attn(q[:, -1].contiguous(), k, v)
    torch.cuda.synchronize()
    assert (full[:, -1].float() - o.float()).abs().max().item() <= 2e-2
    for _ in range(3):
        o2, _ = vc.vitcop_decode_attn(q[:, -1].contiguous(), k, v)
        assert torch.equal(o, o2)
