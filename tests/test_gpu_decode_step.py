"""GPU parity: the KV cache a prefill leaves behind and the whole-model decoding step over it."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import decoder_oracle as Dc
from oracle import vitcop_oracle as O
from gpu_util import assert_attention_close, assert_stream_close, dev, host_bits, host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def model(seed, n_layers, B, T, D, Hq, Hkv, d, F):
    layers = [I.decoder_inputs(seed + 1 + l, B, T, D, Hq, Hkv, d, F)["w"] for l in range(n_layers)]
    for w in layers:                       # small output projections keep the residual stream bounded
        for name in ("wo", "wd"):
            w[name] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w[name]) * np.float32(0.25))
    return I.decoder_inputs(seed, B, T, D, Hq, Hkv, d, F)["h"], layers


def cache_pair(B, cap, Hkv, d):
    return (torch.zeros((B, cap, Hkv, d), dtype=torch.bfloat16, device="cuda"),
            torch.zeros((B, cap, Hkv, d), dtype=torch.bfloat16, device="cuda"))


def rope_close(got_bits, ref_bits, what):
    """bf16 tensors that went through the fp32 rotary embedding: within one bf16 ulp of the pair's length."""
    got, ref = O.bf16_to_f64(got_bits), O.bf16_to_f64(ref_bits)
    scale = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1e-6)
    assert np.all(np.abs(got - ref) <= scale * 2.0 ** -7), what


def v_close(got, ref):
    """bf16 of an fp32 sum of a few hundred products against bf16 of the exact sum: one bf16 ulp of the
    entry, with a floor for entries near zero: the normalised input is itself rounded to bf16 from fp32
    on one side and from fp64 on the other, and one such rounding that falls the other way moves the sum
    by 2^-8 of one product (products here are around 0.05), whatever the size of the sum."""
    assert np.all(np.abs(got - ref) <= np.maximum(np.abs(ref), 5e-2) * 2.0 ** -7)


def test_prefill_leaves_the_kv_cache(vc):
    # one pruning layer: K (after the rotary embedding) and V of the kept tokens, rows [0,T') of the cache
    B, T, D, Hq, Hkv, d, F, vs, nv, keep, cap = 2, 150, 256, 4, 2, 128, 384, 10, 120, 50, 100
    c = I.decoder_inputs(7100, B, T, D, Hq, Hkv, d, F)
    pos = np.stack([np.sort(np.random.default_rng(5 + b).choice(3 * T, T, replace=False)) for b in range(B)])
    kc, vcache = cache_pair(B, cap, Hkv, d)
    w = {k: dev(v) for k, v in c["w"].items()}
    r = vc.vitcop_decoder_layer_prefill(dev(c["h"]), torch.from_numpy(pos.astype(np.int32)).cuda(), w, Hq, Hkv, d, vs,
                                        nv, keep, caches=(kc, vcache))
    torch.cuda.synchronize()
    idx = r["keep_idx"].cpu().numpy()
    ref = Dc.decoder_layer(c["h"], c["w"], Hq, Hkv, d, vs, nv, keep, pos, keep_idx=idx)
    Tp = T - nv + keep
    rope_close(host_bits(kc)[:, :Tp], ref["k_rope"], "K cache")
    v_got, v_ref = O.bf16_to_f64(host_bits(vcache)[:, :Tp]), O.bf16_to_f64(ref["v"])
    v_close(v_got, v_ref)
    assert not host_bits(kc)[:, Tp:].any() and not host_bits(vcache)[:, Tp:].any()           # nothing past T'


SMALL = (256, 4, 2, 128, 384)               # D, Hq, Hkv, d, F: below the streaming kernels' minimum width
RAGGED = (512, 4, 2, 128, 640)              # streaming kernels, F not a whole number of column blocks
CUT = (4160, 24, 6, 128, 2176)              # more row pairs than wavefronts: pairs cut between two of them
GATED_CUT = (2112, 4, 2, 128, 2304)
FULL = (4096, 32, 32, 128, 11008)           # the 7B shape bench.py times (two layers of it)


@pytest.mark.parametrize("B,n_cached,dims", [
    (1, (70, 40, 40), SMALL), (2, (1, 200, 64), SMALL), (6, (50, 20), RAGGED),
    (3, (33, 33, 9), RAGGED), (1, (5, 255), RAGGED), (4, (30, 17), CUT), (2, (17, 30), CUT), (1, (100, 10), GATED_CUT),
    (3, (9, 64), GATED_CUT), (4, (200, 115), FULL), (1, (115, 200), FULL)])
def test_decode_step_matches_oracle(vc, B, n_cached, dims):
    # layers whose caches have different lengths (as after a pruned prefill), capacity above them;
    # the caches are the oracle's (any bf16 values are a valid cache); one to four samples go through
    # the weight-streaming kernels, more through the few-row matrix-core kernels
    D, Hq, Hkv, d, F = dims
    cap = 256
    n_layers = len(n_cached)
    h, layers = model(7200 + B + D, n_layers, B, 1, D, Hq, Hkv, d, F)
    h = h[:, 0]
    pos = np.array([500 + 7 * b for b in range(B)], dtype=np.int32)
    caches_ref = [(I.normal_bf16(7300 + l, 0, (B, n, Hkv, d)), I.normal_bf16(7300 + l, 1, (B, n, Hkv, d)))
                  for l, n in enumerate(n_cached)]
    caches = []
    for (k, v), n in zip(caches_ref, n_cached):
        kc, vcache = cache_pair(B, cap, Hkv, d)
        kc[:, :n] = dev(k)
        vcache[:, :n] = dev(v)
        caches.append((kc, vcache))
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    plan = vc.DecoderDecodePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, caches, n_cached)
    y = plan.run()
    torch.cuda.synchronize()
    ref = Dc.decode_step(h, layers, caches_ref, pos, Hq, Hkv, d)
    assert_stream_close(host_f64(y), ref["y"], "decode step output")
    # layer 0's appended rows depend on the inputs alone: K after the rotary embedding, V
    rope_close(host_bits(caches[0][0])[:, n_cached[0]], ref["appended"][0][0], "appended K")
    v_got = O.bf16_to_f64(host_bits(caches[0][1])[:, n_cached[0]])
    v_ref = O.bf16_to_f64(ref["appended"][0][1])
    v_close(v_got, v_ref)
    for (kc, vcache), (k, v), n in zip(caches, caches_ref, n_cached):      # the cached rows are untouched
        assert np.array_equal(host_bits(kc)[:, :n], k) and np.array_equal(host_bits(vcache)[:, :n], v)
        assert not host_bits(kc)[:, n + 1:].any() and not host_bits(vcache)[:, n + 1:].any()


def test_prefill_then_decode_equals_longer_prefill(vc):
    # GPU only: a pruned prefill of T-1 tokens with cache export, then one decoding step of token T,
    # against the last row of the same pruned prefill over T tokens (same keep lists: the last token is text)
    B, T, D, Hq, Hkv, d, F, vs, nv = 1, 141, 256, 4, 2, 128, 384, 8, 100
    h, layers = model(7400, 3, B, T, D, Hq, Hkv, d, F)
    pos = (np.arange(T) * 2)[None].astype(np.int32)
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    schedule = ((1, 30),)
    caches = [cache_pair(B, 160, Hkv, d) for _ in range(3)]
    head = vc.DecoderSchedulePlan(dev(h[:, :T - 1]), torch.from_numpy(pos[:, :T - 1]).cuda(), wd, Hq, Hkv, d, vs, nv,
                                  schedule, caches=caches)
    head.run()
    full = vc.DecoderSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, nv, schedule)
    y_full = full.run()
    torch.cuda.synchronize()
    assert np.array_equal(full.positions.cpu().numpy()[0, :-1], head.positions.cpu().numpy()[0])
    n_cached = (T - 1, T - 1 - nv + 30, T - 1 - nv + 30)
    step = vc.DecoderDecodePlan(dev(h[:, T - 1]), torch.from_numpy(pos[:, T - 1]).cuda(), wd, Hq, Hkv, d, caches,
                                n_cached)
    y = step.run()
    torch.cuda.synchronize()
    assert_stream_close(host_f64(y), host_f64(y_full[:, -1]), "decode after prefill")


@pytest.mark.parametrize("B", [2, 6])
def test_decode_step_in_a_hip_graph(vc, B):
    # the step is kernel launches only (no allocation, synchronisation, copy or memset), on the streaming
    # path (B <= 4) and on the few-row matrix-core path: captured once and replayed, every replay gives the
    # eager result bit for bit, with eager work in between
    (D, Hq, Hkv, d, F), n_cached, cap = RAGGED, (40, 17, 90), 128
    h, layers = model(7600 + B, 3, B, 1, D, Hq, Hkv, d, F)
    pos = torch.tensor([300 + 111 * b for b in range(B)], dtype=torch.int32, device="cuda")
    caches = []
    for l, n in enumerate(n_cached):
        kc, vcache = cache_pair(B, cap, Hkv, d)
        kc[:, :n] = dev(I.normal_bf16(7700 + l, 0, (B, n, Hkv, d)))
        vcache[:, :n] = dev(I.normal_bf16(7700 + l, 1, (B, n, Hkv, d)))
        caches.append((kc, vcache))
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    plan = vc.DecoderDecodePlan(dev(h[:, 0]), pos, wd, Hq, Hkv, d, caches, n_cached)
    y_eager = plan.run().clone()
    rows_eager = [kc[:, n].clone() for (kc, _), n in zip(caches, n_cached)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.run()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        plan.y.zero_()
        for (kc, vcache), n in zip(caches, n_cached):          # eager work between the replays
            kc[:, n].zero_()
            vcache[:, n].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(plan.y, y_eager), f"replay {rep}"
        for (kc, _), n, row in zip(caches, n_cached, rows_eager):
            assert torch.equal(kc[:, n], row), f"replay {rep}: appended K"


@pytest.mark.parametrize("B,dims,lengths", [
    (3, RAGGED, ((40, 0, 17), (9, 33, 33))),                       # weight-streaming kernels; an empty cache
    (2, CUT, ((64, 65), (1, 200))),
    (6, RAGGED, ((50, 3, 0, 50, 21, 64), (20, 20, 19, 1, 7, 0)))])  # few-row matrix-core kernels
def test_decode_step_per_sample_cache_lengths(vc, B, dims, lengths):
    # every sample with a cache length of its own in every layer (what a batched Stage II leaves behind):
    # sample b's row of the output, and the rows it appends, against the oracle run on that sample alone
    D, Hq, Hkv, d, F = dims
    cap = 256
    n_layers = len(lengths)
    h, layers = model(7500 + B + D, n_layers, B, 1, D, Hq, Hkv, d, F)
    h = h[:, 0]
    pos = np.array([300 + 11 * b for b in range(B)], dtype=np.int32)
    filled = [(I.normal_bf16(7600 + l, 0, (B, cap, Hkv, d)), I.normal_bf16(7600 + l, 1, (B, cap, Hkv, d)))
              for l in range(n_layers)]
    caches = []
    for (k, v), ns in zip(filled, lengths):
        kc, vcache = cache_pair(B, cap, Hkv, d)
        for b, n in enumerate(ns):
            kc[b, :n] = dev(k[b, :n])
            vcache[b, :n] = dev(v[b, :n])
        caches.append((kc, vcache))
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    plan = vc.DecoderDecodePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, caches,
                                [list(ns) for ns in lengths])
    y = host_f64(plan.run())
    torch.cuda.synchronize()
    for b in range(B):
        own = [(k[b:b + 1, :ns[b]], v[b:b + 1, :ns[b]]) for (k, v), ns in zip(filled, lengths)]
        ref = Dc.decode_step(h[b:b + 1], layers, own, pos[b:b + 1], Hq, Hkv, d)
        assert_stream_close(y[b:b + 1], ref["y"], f"decode step output, sample {b}")
        n0 = lengths[0][b]
        rope_close(host_bits(caches[0][0])[b, n0], ref["appended"][0][0][0], f"appended K, sample {b}")
        v_close(O.bf16_to_f64(host_bits(caches[0][1])[b, n0]), O.bf16_to_f64(ref["appended"][0][1][0]))
        for (kc, vcache), (k, v), ns in zip(caches, filled, lengths):    # cached rows untouched, nothing past the new one
            n = ns[b]
            assert np.array_equal(host_bits(kc)[b, :n], k[b, :n]) and np.array_equal(host_bits(vcache)[b, :n], v[b, :n])
            assert not host_bits(kc)[b, n + 1:].any() and not host_bits(vcache)[b, n + 1:].any()
