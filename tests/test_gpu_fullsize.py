"""GPU parity at the full sizes of the workload configs, in the launch configuration bench.py times.

Where the oracle can compute everything in seconds the comparison is complete; for the
unpruned attention shapes it is on sampled query rows computed one by one.
"""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O
from gpu_util import assert_attention_close, assert_selection_matches, dev, host_f64
from test_gpu_layer import check_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def test_config3_bench_layer_keep320(vc):
    # the bench workload itself: B 4, T 2944, keep 320 of 2880 -> T' 384
    c = I.config3()
    check_layer(vc, c, 320, False, "config 3 keep 320")


@pytest.mark.parametrize("B,N,Hq,Hkv,seed", [(4, 2944, 32, 32, 3001), (1, 6400, 28, 4, 4001)])
def test_unpruned_attention_sampled_rows(vc, B, N, Hq, Hkv, seed):
    t = I.qkv_tensors(seed, B, N, Hq, Hkv, 128)
    out, lse = vc.vitcop_prefill_attn(dev(t["q"]), dev(t["k"]), dev(t["v"]), want_lse=True)
    torch.cuda.synchronize()
    out = host_f64(out)
    g = np.random.default_rng(seed)
    rows = sorted(set([0, 1, 31, 32, 63, 64, 255, 256, 257, N - 1, N - 2]
                      + g.integers(0, N, size=12).tolist()))
    for b, h in {(0, 0), (B - 1, Hq - 1), (int(g.integers(0, B)), int(g.integers(0, Hq)))}:
        ref = O.attention_rows(t["q"], t["k"], t["v"], b, h, rows)
        assert_attention_close(out[b, rows, h], ref, f"B{B} N{N} b{b} h{h}")


def test_config4_video_knorm_select_and_filter(vc):
    # vision side: 32 frames x 197 tokens, filter keeps 58 per frame
    fr = I.config4_frames()
    scores, idx = vc.vitcop_filter_visual(dev(fr["q_cls"]), dev(fr["k"]), fr["keep"])
    S, _ = O.filter_visual(fr["q_cls"], fr["k"], fr["keep"])
    scores, idx = scores.cpu().numpy(), idx.cpu().numpy()
    assert np.allclose(scores, S, rtol=2e-4, atol=1e-7)
    for b in range(fr["B"]):
        assert_selection_matches(idx[b], scores[b], S[b], fr["keep"], True, f"frame {b}")
    # LLM side: 6272 visual + 128 text tokens, GQA 4 KV heads x 128; keep 627 by K-norm
    c = I.config4_layer()
    k_bits = O.f64_to_bf16_bits(O.project(c["x"], c["wk"])).reshape(1, c["T"], 4, 128)
    norms, kidx = vc.vitcop_knorm_select(dev(k_bits), 0, 6272, c["keep"])
    ref_n, ref_idx = O.knorm_select(k_bits, 0, 6272, c["keep"])
    norms, kidx = norms.cpu().numpy(), kidx.cpu().numpy()
    assert np.allclose(norms, ref_n, rtol=2e-6)
    assert_selection_matches(kidx[0, :c["keep"]], norms[0], ref_n[0], c["keep"], False, "config 4")
    assert np.array_equal(kidx[0, c["keep"]:], np.arange(6272, 6400))


def test_config2_schedule_prefix_full_width(vc):
    # first four layers of the config-2 schedule at full width (D 4096, 32 x 128), budgets
    # 576 -> 192 -> 128 -> 64 brought forward to layers 1, 2, 3; each layer teacher-forced on
    # the oracle's input for that layer
    h2 = I.config2_hidden()
    sched = ((1, 192), (2, 128), (3, 64))
    ws = [I.config2_layer_weights(l) for l in range(4)]
    for w in ws:
        w["wo"] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w["wo"]) * np.float32(0.125))
    ref = O.schedule_prefill(h2["x"], lambda l: ws[l], 4, sched, 32, 32, 128, 35, 576)
    budgets, cur_vis = dict(sched), 576
    for l, lay in enumerate(ref["layers"]):
        keep = budgets.get(l, cur_vis)
        w = {n: dev(ws[l][n]) for n in ("wq", "wk", "wv", "wo")}
        r = vc.vitcop_layer_prefill(dev(lay["x_in"]), w["wq"], w["wk"], w["wv"], w["wo"], 32, 32, 128, 35,
                                    cur_vis, keep, residual=True)
        torch.cuda.synchronize()
        nxt = ref["layers"][l + 1]["x_in"] if l + 1 < 4 else ref["h"]
        same = True
        if lay["keep_idx"] is not None:
            idx, nr = r["keep_idx"].cpu().numpy(), r["norms"].cpu().numpy()
            assert_selection_matches(idx[0, 35:35 + keep] - 35, nr[0], lay["norms"][0], keep, False, f"layer {l}")
            vis = idx[0, 35:35 + keep] - 35
            # surviving rows carry small gains: none of the planted 4x outliers of the input survive layer 1
            same = np.array_equal(idx, lay["keep_idx"])
        if same:
            assert_attention_close(host_f64(r["y"]), O.bf16_to_f64(nxt), f"schedule layer {l}")
        cur_vis = keep
    assert ref["h"].shape == (1, 128, 4096)
