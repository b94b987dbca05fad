"""GPU: the entry point that allocates nothing (vitcop_filter_visual_static) against the entry point it is a
variant of (vitcop_filter_visual), through the C ABI.  Both run the same kernels, so scores and indices must be
bit-identical; the oracle's check of those values is in test_gpu_compact_filter.py.  Two calls in a row share
the library's scratch array, the second on a smaller input."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def both(vc, f, keep):
    q, k = dev(f["q_cls"]), dev(f["k"])
    B, N = f["k"].shape[0], f["k"].shape[1] - 1
    want_scores, want_idx = vc.vitcop_filter_visual(q, k, keep)
    scores = torch.full((B, N), -1.0, dtype=torch.float32, device="cuda")
    idx = torch.full((B, keep), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    vc.vitcop_filter_visual_static(q, k, keep, scores, idx)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(scores, want_scores), "scores differ from vitcop_filter_visual"
    assert torch.equal(idx, want_idx), "indices differ from vitcop_filter_visual"


def test_static_filter_two_calls_second_smaller(vc):
    # config-1 shape (8 images x 577 tokens x 16 heads x 64), then a smaller and differently shaped input
    # (3 images x 101 tokens, d = 128) whose logits land in the part of the scratch the first call used
    both(vc, I.config1(), 288)
    both(vc, I.config1(trial=1, B=3, N=100, C=512, H=4, d=128, n_centroids=8), 37)
    # and back to a larger one
    both(vc, I.config1(trial=2, B=5, N=300, C=1024, H=16, d=64, n_centroids=16), 150)


def test_static_filter_rejects_what_does_not_fit(vc):
    # 64 images x 16 heads x 1025 tokens x 4 bytes = 4.2 MB of logits: above the built-in scratch
    q = torch.zeros((64, 16, 64), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((64, 1025, 16, 64), dtype=torch.bfloat16, device="cuda")
    scores = torch.empty((64, 1024), dtype=torch.float32, device="cuda")
    idx = torch.empty((64, 10), dtype=torch.int32, device="cuda")
    with pytest.raises(vc.VitcopError) as e:
        vc.vitcop_filter_visual_static(q, k, 10, scores, idx)
    assert e.value.code == vc.VITCOP_EUNSUPPORTED and "scratch" in str(e.value)
