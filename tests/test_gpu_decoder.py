"""GPU parity: RMSNorm, rotary embedding, SiLU gate and the full decoder layer with pruning on
entry, against the decoder-layer oracle."""
import numpy as np
import pytest
import torch

import vitcop_inputs as I
from oracle import decoder_oracle as Dc
from oracle import vic_oracle as V
from oracle import vitcop_oracle as O
from gpu_util import assert_stream_close, assert_selection_matches, dev, host_bits, host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vc():
    from paper_2601_17818_amd import binding
    return binding


def within_bf16(got_bits, ref, what, slack=1e-5):
    got = O.bf16_to_f64(got_bits)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
    assert np.all(np.abs(got - ref) <= 0.5 * ulp + slack * np.maximum(np.abs(ref), 1e-3)), what


@pytest.mark.parametrize("M,D", [(1, 8), (5, 96), (300, 4096), (130, 3584), (3, 8200)])
def test_rmsnorm(vc, M, D):
    x = I.normal_bf16(9000 + M, 0, (M, D), 2.0)
    w = I.f32_to_bf16_bits(1.0 + 0.1 * I.bf16_bits_to_f32(I.normal_bf16(9000 + M, 1, (D,))))
    y = vc.vitcop_rmsnorm(dev(x), dev(w), 1e-5)
    torch.cuda.synchronize()
    within_bf16(host_bits(y), Dc.rmsnorm(x, w, 1e-5), "rmsnorm")


@pytest.mark.parametrize("Hq,Hkv,d", [(4, 2, 128), (3, 3, 64), (28, 4, 128)])
def test_rope(vc, Hq, Hkv, d):
    t = I.qkv_tensors(9100 + Hq, 2, 37, Hq, Hkv, d)
    pos = np.stack([np.sort(np.random.default_rng(b).choice(3000, 37, replace=False)) for b in range(2)]).astype(np.int32)
    q, k = dev(t["q"]).clone(), dev(t["k"]).clone()
    vc.vitcop_rope(q, k, torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    # fp32 angles at positions up to 3000 are good to about 1e-3 rad (the ulp of the angle plus the
    # relative error of theta^(-2i/d)), which moves a rotated pair by that fraction of ITS length
    def check(got_bits, x_bits, what):
        ref = Dc.rope(x_bits, pos, 10000.0)
        x = O.bf16_to_f64(x_bits)
        half = d // 2
        pair = np.sqrt(x[..., :half] ** 2 + x[..., half:] ** 2)
        pair = np.concatenate([pair, pair], axis=-1)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
        assert np.all(np.abs(O.bf16_to_f64(got_bits) - ref) <= 0.5 * ulp + 2e-3 * pair), what

    check(host_bits(q), t["q"], "rope q")
    check(host_bits(k), t["k"], "rope k")
    k2 = dev(t["k"]).clone()
    vc.vitcop_rope(None, k2, torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    assert torch.equal(k2, k)


def test_silu_mul(vc):
    g = I.normal_bf16(9200, 0, (77, 1000), 3.0)
    u = I.normal_bf16(9200, 1, (77, 1000), 1.0)
    out = vc.vitcop_silu_mul(dev(g), dev(u))
    torch.cuda.synchronize()
    within_bf16(host_bits(out), Dc.silu_mul(g, u), "silu_mul", slack=2e-6)


def run_layer(vc, c, pos, vis_start, n_vis, keep):
    w = {k: dev(v) for k, v in c["w"].items()}
    r = vc.vitcop_decoder_layer_prefill(dev(c["h"]), torch.from_numpy(pos.astype(np.int32)).cuda(), w, c["Hq"], c["Hkv"],
                                        c["d"], vis_start, n_vis, keep)
    torch.cuda.synchronize()
    return r


@pytest.mark.parametrize("B,T,D,Hq,Hkv,d,F,vs,nv,keep", [(2, 200, 256, 4, 2, 128, 352, 20, 150, 60),
                                                       (1, 333, 512, 8, 8, 64, 704, 0, 300, 300),
                                                       (1, 420, 256, 4, 4, 64, 512, 10, 390, 0),
                                                       (1, 700, 512, 4, 4, 128, 1408, 0, 640, 320),
                                                       # 256 < rows <= 1024 and k >= 768: the split-K projections
                                                       # (K alone with norms, Q+V and gate+up as pairs, down)
                                                       (1, 400, 1024, 2, 2, 128, 768, 20, 300, 200),
                                                       (1, 320, 1024, 2, 2, 128, 768, 0, 300, 300),
                                                       # gate+up as 3 x 86 tiles: the trailing column tile of `up`
                                                       # goes out as a launch of its own
                                                       (1, 640, 1024, 2, 2, 128, 11008, 35, 576, 576),
                                                       # gate+up on the big tiles with the activation in their
                                                       # epilogue: 300 rows x 2 x 86 tiles of 192 x 256; 1400 rows
                                                       # on smaller tiles, whole and with a ragged last column tile
                                                       (1, 400, 1024, 2, 2, 128, 11008, 20, 300, 200),
                                                       (2, 700, 512, 4, 4, 128, 1408, 0, 640, 640),
                                                       (2, 700, 512, 4, 4, 128, 1376, 0, 640, 600)])
def test_decoder_layer_matches_oracle(vc, B, T, D, Hq, Hkv, d, F, vs, nv, keep):
    c = I.decoder_inputs(9300 + T, B, T, D, Hq, Hkv, d, F)
    pos = np.stack([np.sort(np.random.default_rng(10 + b).choice(2 * T, T, replace=False)) for b in range(B)])
    r = run_layer(vc, c, pos, vs, nv, keep)
    ref = Dc.decoder_layer(c["h"], c["w"], Hq, Hkv, d, vs, nv, keep, pos)
    norms, idx = r["norms"].cpu().numpy(), r["keep_idx"].cpu().numpy()
    assert np.allclose(norms, ref["norms"], rtol=2e-3)
    # RMSNorm gives every row the same scale, so the K-norms lie close together and the cut falls
    # among near-ties: the GPU's list must agree with the oracle's outside the tie band (and with
    # the tie rule on its own norms); the rest of the layer is then checked on the GPU's list
    for b in range(B):
        assert_selection_matches(idx[b, vs:vs + keep] - vs, norms[b], ref["norms"][b], keep, False, "decoder keep")
        assert np.array_equal(idx[b, :vs], np.arange(vs)) and np.array_equal(idx[b, vs + keep:], np.arange(vs + nv, T))
    if not np.array_equal(idx, ref["keep_idx"]):
        ref = Dc.decoder_layer(c["h"], c["w"], Hq, Hkv, d, vs, nv, keep, pos, keep_idx=idx)
    assert np.array_equal(r["positions"].cpu().numpy(), np.take_along_axis(pos, idx.astype(np.int64), axis=1))
    assert_stream_close(host_f64(r["y"]), ref["y"], "decoder layer output")


def test_decoder_layer_deterministic_and_prefix(vc):
    # rows before the visual span do not depend on what is pruned after them (causality)
    c = I.decoder_inputs(9400, 1, 300, 256, 4, 2, 128, 352)
    pos = np.arange(300)[None]
    full = run_layer(vc, c, pos, 40, 260, 260)
    cut = run_layer(vc, c, pos, 40, 260, 50)
    again = run_layer(vc, c, pos, 40, 260, 50)
    assert torch.equal(cut["y"], again["y"])
    # (equal up to the rounding order of the projections: few rows take the split-K path)
    a, b = host_f64(cut["y"][:, :40]), host_f64(full["y"][:, :40])
    assert_stream_close(a, b, "rows before the visual span")
    assert np.mean(a == b) > 0.9


def schedule_case(seed, B, T, D, Hq, Hkv, d, F, vs, nv, n_layers):
    """Layers whose K projection amplifies the first D/8 input channels, and visual rows that carry a
    log-normal share of their energy there: after RMSNorm the K-norms are spread, not concentrated."""
    layers = [I.decoder_inputs(seed + 1 + l, B, T, D, Hq, Hkv, d, F)["w"] for l in range(n_layers)]
    for w in layers:
        wk = I.bf16_bits_to_f32(w["wk"])
        wk[:, : D // 8] *= 4.0
        w["wk"] = I.f32_to_bf16_bits(wk)
        for name in ("wo", "wd"):          # small output projections keep the residual stream bounded
            w[name] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w[name]) * np.float32(0.25))
    h = I.bf16_bits_to_f32(I.decoder_inputs(seed, B, T, D, Hq, Hkv, d, F)["h"])
    gain, _ = I.lognormal_gains(seed, B, nv, sigma=1.0, outlier_frac=0.0)
    h[:, vs:vs + nv, : D // 8] *= gain[:, :, None].astype(np.float32)
    return I.f32_to_bf16_bits(h), layers


def test_decoder_schedule_matches_oracle(vc):
    # 6 layers, pruning on entry to layers 1 and 4.  Seeds are searched (on the oracle) for cuts
    # without near-ties at both stages; then positions and outputs must match the oracle's.
    B, T, D, Hq, Hkv, d, F, vs, nv = 1, 260, 256, 4, 2, 128, 352, 12, 230
    schedule = ((1, 120), (4, 40))
    pos = np.arange(T)[None].astype(np.int32)
    for seed in range(9830, 10000):
        h, layers = schedule_case(seed, B, T, D, Hq, Hkv, d, F, vs, nv, 6)
        ref = Dc.decoder_schedule(h, layers, schedule, Hq, Hkv, d, vs, nv, pos)
        if all(O.tie_band(ref["norms"][l][0], k, False, 4e-3).sum() <= 1 for l, k in schedule):
            break
    else:
        raise AssertionError("no seed with gap-free cuts")
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    plan = vc.DecoderSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, nv, schedule)
    plan.run()
    torch.cuda.synchronize()
    for s_, (l, k) in enumerate(schedule):        # every stage's record: the norms it ranked, the list it took
        got_n, got_idx = plan.stage_norms[s_].cpu().numpy(), plan.stage_keep_idx[s_].cpu().numpy()
        assert np.allclose(got_n, ref["norms"][l], rtol=2e-3)
        assert_selection_matches(got_idx[0, vs:vs + k] - vs, got_n[0], ref["norms"][l][0], k, False, f"stage {s_}")
        assert np.array_equal(got_idx, ref["keep_lists"][l])
    assert np.array_equal(plan.positions.cpu().numpy(), ref["positions"])
    assert_stream_close(host_f64(plan.y), ref["y"], "decoder schedule output")
    # the unpruned schedule has no decisions
    plan0 = vc.DecoderSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, nv, ())
    plan0.run()
    torch.cuda.synchronize()
    ref0 = Dc.decoder_schedule(h, layers, (), Hq, Hkv, d, vs, nv, pos)
    assert_stream_close(host_f64(plan0.y), ref0["y"], "unpruned decoder schedule")
    assert np.array_equal(plan0.positions.cpu().numpy(), pos)


@pytest.mark.parametrize("B,T,D,Hq,Hkv", [
    (1, 400, 1024, 2, 2),      # 256 < rows <= 768: K and the Q/V pair as split-K launches, finished in one launch
    (2, 180, 1024, 2, 2),      # the same with two samples' rows (and positions) side by side
    (1, 200, 1024, 2, 2),      # few rows: the three matrices in one launch, finished in one launch
    (2, 100, 512, 4, 4),
    (1, 400, 1024, 4, 2)])     # grouped-query heads: the plain sequence (projections, then the rotary kernel)
def test_layers_that_keep_all_tokens_finish_qkv_in_one_launch(vc, B, T, D, Hq, Hkv):
    # layers of a schedule that prune nothing project K, Q and V together and, where those projections leave
    # partial sums, add them up, round them and turn q and k by the rotary embedding in a single launch: the
    # caches (K after the embedding, V) of both layers and the output against the oracle
    d, F, vs, nv = 128, 768, 10, T - 40
    h, layers = schedule_case(9700 + T + D + Hq, B, T, D, Hq, Hkv, d, F, vs, nv, 2)
    pos = np.stack([np.sort(np.random.default_rng(40 + b).choice(4 * T, T, replace=False)) for b in range(B)]).astype(np.int32)
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    caches = [(torch.zeros((B, T, Hkv, d), dtype=torch.bfloat16, device="cuda"),
               torch.zeros((B, T, Hkv, d), dtype=torch.bfloat16, device="cuda")) for _ in range(2)]
    plan = vc.DecoderSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, nv, (), caches=caches)
    plan.run()
    torch.cuda.synchronize()
    ref = Dc.decoder_schedule(h, layers, (), Hq, Hkv, d, vs, nv, pos)
    # layer 0's K and V depend on the inputs alone: within one bf16 ulp of the head's largest entry (K: the
    # turn mixes a pair; both: a normalised input that rounds the other way on one side moves the fp32 sum
    # by 2^-8 of one product, whatever the size of the sum)
    for which, what in ((0, "K cache"), (1, "V cache")):
        got, want = O.bf16_to_f64(host_bits(caches[0][which])), O.bf16_to_f64(ref["caches"][0][which])
        assert np.all(np.abs(got - want) <= np.maximum(np.abs(want).max(axis=-1, keepdims=True), 1e-6) * 2.0 ** -7), what
    assert_stream_close(host_f64(plan.y), ref["y"], "two layers that keep all tokens")


def full_case(seed, vs, n, tail, D, Hq, Hkv, d, F, n_layers, grid, regions):
    """Text tokens ~ N(0,1); visual hidden states = planted spatial regions (vic_inputs); small output
    projections keep the residual stream close to the input, so the regions survive the first layers."""
    T = vs + n + tail
    layers = [I.decoder_inputs(seed + 1 + l, 1, T, D, Hq, Hkv, d, F)["w"] for l in range(n_layers)]
    for w in layers:
        for name in ("wo", "wd"):
            w[name] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w[name]) * np.float32(0.25))
    h = I.decoder_inputs(seed, 1, T, D, Hq, Hkv, d, F)["h"].copy()
    v = I.vic_inputs(seed, n, D, grid, regions, 0.15)
    h[0, vs:vs + n] = v["feats"]
    return h, layers, v["pos"]


@pytest.mark.parametrize("stage2_layer,schedule", [(1, ()), (0, ((2, 24),)), (2, ((3, 100),))])
def test_full_schedule_matches_oracle(vc, stage2_layer, schedule):
    # Alg. 1 end to end on one sample: decoder layers, Stage II (clustering + elites + merging) on entry
    # to one layer, Stage III (K-norm top-k) later.  The oracle is given the GPU's labels and norms (each
    # validated against the oracle's own below and in the Stage II tests), so its discrete steps decide
    # on the same numbers; the Stage III keep list and the norms it was taken from come out of the call
    # and are checked against the rule on the oracle's norms before the oracle continues with that list.
    D, Hq, Hkv, d, F, vs, n, tail = 256, 4, 2, 128, 352, 12, 150, 10
    T = vs + n + tail
    h, layers, xy = full_case(9900, vs, n, tail, D, Hq, Hkv, d, F, 4, 16, 6)
    pos = (2 * np.arange(T))[None].astype(np.int32)
    s2 = {"layer": stage2_layer, "budget": 60, "n_centers": 6, "d_c": 8.0, "tau": 0.6}
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    plan = vc.FullSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, n,
                               {**s2, "xy": torch.from_numpy(xy.astype(np.float32)[None]).cuda()}, schedule)
    y, p = plan.run()
    torch.cuda.synchronize()
    labels, norms = plan.labels[0].cpu().numpy(), plan.norms[0].cpu().numpy()
    # Stage II alone (no Stage III) with the oracle's own clustering and norms: same partition, close norms
    own = Dc.vitcop_schedule(h, layers[: stage2_layer + 1], {**s2, "xy": xy}, (), Hq, Hkv, d, vs, n, pos)
    assert V.same_partition(labels, own["stage2"]["labels"])
    assert np.allclose(norms, own["stage2"]["norms"], rtol=2e-3)
    # the whole run on the GPU's labels and norms
    ref = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, (), Hq, Hkv, d, vs, n, pos, labels=labels, k_norms=norms)
    st = ref["stage2"]
    assert plan.n_stage2 == [st["n_out"]] and st["n_out"] <= s2["budget"]
    assert plan.T_final_samples == [plan.T_final]
    assert np.array_equal(plan.out_index[0].cpu().numpy(), st["index"])
    got_pos = p.cpu().numpy()
    if schedule:
        (l3, k3), = schedule
        k3 = min(k3, st["n_out"])
        assert plan.T_final == T - n + k3
        # Stage III: the oracle's own decision on the sequence Stage II left, from its own K-norms of layer l3
        free = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, schedule, Hq, Hkv, d, vs, n, pos, labels=labels,
                                  k_norms=norms)
        norms3 = plan.stage_norms[0][0].cpu().numpy()
        idx = plan.stage_keep_idx[0][0].cpu().numpy()
        want3 = free["stage3"][l3]
        assert norms3.shape == want3["norms"][0].shape == (st["n_out"],)
        assert np.allclose(norms3, want3["norms"][0], rtol=2e-3)
        assert_selection_matches(idx[vs:vs + k3] - vs, norms3, want3["norms"][0], k3, False, "Stage III keep list")
        assert np.array_equal(idx[:vs], np.arange(vs))
        assert np.array_equal(idx[vs + k3:], np.arange(vs + st["n_out"], T - n + st["n_out"]))
        # the list is the rule's outside the band of near-ties: the oracle goes on with it
        ref = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, schedule, Hq, Hkv, d, vs, n, pos, labels=labels,
                                 k_norms=norms, keep_lists={l3: idx[None]})
    assert np.array_equal(got_pos, ref["positions"])
    assert_stream_close(host_f64(y), ref["y"], "full schedule output")


def test_full_schedule_caches_then_decode(vc):
    # the paper's whole procedure, then generation: prefill with Stage II on entry to layer 1 and Stage III on
    # entry to layer 3, every layer leaving its KV cache (three different lengths), then one decoding step over
    # those caches; oracle: the same procedure on the GPU's labels, norms and Stage III list, its caches, its step
    D, Hq, Hkv, d, F, vs, n, tail = 256, 4, 2, 128, 384, 12, 150, 10
    T = vs + n + tail
    h, layers, xy = full_case(9950, vs, n, tail, D, Hq, Hkv, d, F, 4, 16, 6)
    pos = (2 * np.arange(T))[None].astype(np.int32)
    s2 = {"layer": 1, "budget": 60, "n_centers": 6, "d_c": 8.0, "tau": 0.6}
    schedule = ((3, 20),)
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    cap = T + 8
    caches = [(torch.zeros((1, cap, Hkv, d), dtype=torch.bfloat16, device="cuda"),
               torch.zeros((1, cap, Hkv, d), dtype=torch.bfloat16, device="cuda")) for _ in layers]
    plan = vc.FullSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, n,
                               {**s2, "xy": torch.from_numpy(xy.astype(np.float32)[None]).cuda()}, schedule,
                               caches=caches)
    y, p = plan.run()
    torch.cuda.synchronize()
    labels, norms = plan.labels[0].cpu().numpy(), plan.norms[0].cpu().numpy()
    mid = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, (), Hq, Hkv, d, vs, n, pos, labels=labels, k_norms=norms)
    n2 = mid["stage2"]["n_out"]
    # Stage III list: checked against the rule on the oracle's own norms of that layer before the oracle uses it
    free = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, schedule, Hq, Hkv, d, vs, n, pos, labels=labels,
                              k_norms=norms)
    norms3, idx = plan.stage_norms[0][0].cpu().numpy(), plan.stage_keep_idx[0][0].cpu().numpy()
    assert np.allclose(norms3, free["stage3"][3]["norms"][0], rtol=2e-3)
    assert_selection_matches(idx[vs:vs + 20] - vs, norms3, free["stage3"][3]["norms"][0], 20, False, "Stage III")
    assert np.array_equal(idx[:vs], np.arange(vs)) and np.array_equal(idx[vs + 20:], np.arange(vs + n2, T - n + n2))
    ref = Dc.vitcop_schedule(h, layers, {**s2, "xy": xy}, schedule, Hq, Hkv, d, vs, n, pos, labels=labels,
                             k_norms=norms, keep_lists={3: idx[None]})
    assert np.array_equal(p.cpu().numpy(), ref["positions"])
    lengths = [T, T - n + n2, T - n + n2, T - n + 20]
    assert plan.T_final == lengths[-1] and plan.n_stage2 == [n2]
    assert plan.cache_len == [[L] for L in lengths]
    for (kc, vcache), (k_ref, v_ref), L in zip(caches, ref["caches"], lengths):
        assert k_ref.shape[1] == L
        assert_stream_close(host_f64(kc)[:, :L], O.bf16_to_f64(k_ref), "K cache after the full schedule")
        assert_stream_close(host_f64(vcache)[:, :L], O.bf16_to_f64(v_ref), "V cache after the full schedule")
        assert not host_bits(kc)[:, L:].any()
    # one decoding step from there: a new token at the next position
    h_new = I.decoder_inputs(9960, 1, 1, D, Hq, Hkv, d, F)["h"][:, 0]
    new_pos = np.array([2 * T], dtype=np.int32)
    step = vc.DecoderDecodePlan(dev(h_new), torch.from_numpy(new_pos).cuda(), wd, Hq, Hkv, d, caches, lengths)
    y1 = step.run()
    torch.cuda.synchronize()
    ref1 = Dc.decode_step(h_new, layers, ref["caches"], new_pos, Hq, Hkv, d)
    assert_stream_close(host_f64(y1), ref1["y"], "decoding step after the full schedule")


@pytest.mark.parametrize("seeds", [(9900, 9968, 9934), (9900, 9968, 9934, 9951, 10002, 10036)])
def test_full_schedule_batch_with_different_counts(vc, seeds):
    # Alg. 1 on a batch whose samples leave Stage II with different numbers of visual tokens: the library pads the
    # batch on the right; every sample's real rows must equal the one-sample procedure of the oracle (which knows
    # nothing of batches or padding).  First Stage III budget lies between the samples' counts (one sample keeps
    # all it has, the batch stays ragged), the second below all of them (the batch is dense again).
    D, Hq, Hkv, d, F, vs, n, tail = 256, 4, 2, 128, 384, 12, 150, 10
    T, B, n_layers = vs + n + tail, len(seeds), 5
    layers = None
    hs, xys = [], []
    for b, seed in enumerate(seeds):
        h_b, layers_b, xy_b = full_case(seed, vs, n, tail, D, Hq, Hkv, d, F, n_layers, 16, 6)
        layers = layers or layers_b                       # one model: the first sample's weights
        hs.append(h_b)
        xys.append(xy_b)
    h = np.concatenate(hs, axis=0)
    pos = np.stack([2 * np.arange(T) + 3 * b for b in range(B)]).astype(np.int32)
    s2 = {"layer": 1, "budget": 60, "n_centers": 6, "d_c": 8.0, "tau": 0.6}
    own = [Dc.vitcop_schedule(h[b:b + 1], layers[:2], {**s2, "xy": xys[b]}, (), Hq, Hkv, d, vs, n, pos[b:b + 1])
           for b in range(B)]
    counts = [o["stage2"]["n_out"] for o in own]
    assert len(set(counts)) == 3, counts                  # the case is about different counts
    k3a, k3b = sorted(set(counts))[1], 20
    schedule = ((2, k3a), (4, k3b))
    wd = [{k: dev(v) for k, v in w.items()} for w in layers]
    cap = T + 4
    caches = [(torch.zeros((B, cap, Hkv, d), dtype=torch.bfloat16, device="cuda"),
               torch.zeros((B, cap, Hkv, d), dtype=torch.bfloat16, device="cuda")) for _ in layers]
    xy_dev = torch.from_numpy(np.stack(xys).astype(np.float32)).cuda()
    plan = vc.FullSchedulePlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, n, {**s2, "xy": xy_dev},
                               schedule, caches=caches)
    y, p = plan.run()
    torch.cuda.synchronize()
    assert plan.n_stage2 == counts
    n_max = max(counts)
    T2 = T - n + n_max                                    # padded length after Stage II
    kept_a = [min(k3a, c) for c in counts]
    assert plan.T_final == T - n + k3b and plan.T_final_samples == [T - n + k3b] * B
    want_len = [[T] * B, [T - n + c for c in counts], [T - n + k for k in kept_a], [T - n + k for k in kept_a],
                [T - n + k3b] * B]
    assert plan.cache_len == want_len
    y_host, p_host = host_f64(y), p.cpu().numpy()
    # then one decoding step over those caches of different lengths (2 to 4 samples: the streaming matrix-vector
    # kernels; more: the few-row projections), every sample against the oracle's one-sample step
    h_new = I.decoder_inputs(9960, B, 1, D, Hq, Hkv, d, F)["h"][:, 0]
    new_pos = (2 * T + 5 * np.arange(B)).astype(np.int32)
    step = vc.DecoderDecodePlan(dev(h_new), torch.from_numpy(new_pos).cuda(), wd, Hq, Hkv, d, caches, plan.cache_len)
    y1 = host_f64(step.run())
    torch.cuda.synchronize()
    for b in range(B):
        labels, norms = plan.labels[b].cpu().numpy(), plan.norms[b].cpu().numpy()
        assert V.same_partition(labels, own[b]["stage2"]["labels"]), f"sample {b}"
        assert np.allclose(norms, own[b]["stage2"]["norms"], rtol=2e-3)
        one = dict(h_bits=h[b:b + 1], layer_weights=layers, stage2={**s2, "xy": xys[b]}, schedule=schedule, Hq=Hq,
                   Hkv=Hkv, d=d, vis_start=vs, n_vis=n, positions=pos[b:b + 1], labels=labels, k_norms=norms)
        free = Dc.vitcop_schedule(**one)
        c = counts[b]
        assert np.array_equal(plan.out_index[b, :c].cpu().numpy(), free["stage2"]["index"])
        # first Stage III stage: candidates are this sample's c tokens, it keeps min(k3a, c) of them
        ka = kept_a[b]
        got_n = plan.stage_norms[0][b].cpu().numpy()
        got_idx = plan.stage_keep_idx[0][b].cpu().numpy()
        want = free["stage3"][2]
        assert np.allclose(got_n[:c], want["norms"][0], rtol=2e-3) and not got_n[c:].any()
        assert_selection_matches(got_idx[vs:vs + ka] - vs, got_n[:c], want["norms"][0], ka, False, f"sample {b} stage a")
        assert np.array_equal(got_idx[:vs], np.arange(vs))
        assert np.array_equal(got_idx[vs + ka:vs + ka + tail], np.arange(vs + c, vs + c + tail))
        assert (got_idx[vs + ka + tail:] == T2 - 1).all()                      # padding rows
        list_a = got_idx[None, :vs + ka + tail]
        # second stage: the oracle continues with the first list, then its own norms decide
        mid = Dc.vitcop_schedule(**one, keep_lists={2: list_a})
        got_n = plan.stage_norms[1][b].cpu().numpy()
        got_idx = plan.stage_keep_idx[1][b].cpu().numpy()
        want = mid["stage3"][4]
        assert np.allclose(got_n[:ka], want["norms"][0], rtol=2e-3) and not got_n[ka:].any()
        assert_selection_matches(got_idx[vs:vs + k3b] - vs, got_n[:ka], want["norms"][0], k3b, False,
                                 f"sample {b} stage b")
        assert np.array_equal(got_idx[:vs], np.arange(vs))
        assert np.array_equal(got_idx[vs + k3b:], np.arange(vs + ka, vs + ka + tail))
        ref = Dc.vitcop_schedule(**one, keep_lists={2: list_a, 4: got_idx[None]})
        assert np.array_equal(p_host[b], ref["positions"][0])
        assert_stream_close(y_host[b:b + 1], ref["y"], f"sample {b} of the batch")
        for l, ((kc, vcache), (k_ref, v_ref)) in enumerate(zip(caches, ref["caches"])):
            L = want_len[l][b]
            assert k_ref.shape[1] == L
            assert_stream_close(host_f64(kc[b:b + 1, :L]), O.bf16_to_f64(k_ref), f"K cache, sample {b}, layer {l}")
            assert_stream_close(host_f64(vcache[b:b + 1, :L]), O.bf16_to_f64(v_ref), f"V cache, sample {b}, layer {l}")
        ref1 = Dc.decode_step(h_new[b:b + 1], layers, ref["caches"], new_pos[b:b + 1], Hq, Hkv, d)
        assert_stream_close(y1[b:b + 1], ref1["y"], f"decoding step, sample {b}")
        for l, ((kc, vcache), (k_row, v_row)) in enumerate(zip(caches, ref1["appended"])):
            L = want_len[l][b]                            # the step appended at the sample's own row
            assert_stream_close(host_f64(kc[b:b + 1, L]), O.bf16_to_f64(k_row), f"appended K, sample {b}, layer {l}")
            assert_stream_close(host_f64(vcache[b:b + 1, L]), O.bf16_to_f64(v_row), f"appended V, sample {b}, layer {l}")


def test_decoder_layer_right_padded_batch(vc):
    # a right-padded batch given directly to the layer: samples with all, some, one and none of the n_vis visual
    # tokens; every sample's real rows must equal the layer run on that sample alone (the oracle, on the sample's
    # own rows, with its own count and min(keep, count) survivors)
    B, D, Hq, Hkv, d, F, vs, nv, tail, keep = 4, 256, 4, 2, 128, 384, 7, 90, 9, 40
    counts = [90, 55, 1, 0]
    T = vs + nv + tail
    c = I.decoder_inputs(9700, B, T, D, Hq, Hkv, d, F)
    h = c["h"].copy()
    pos = np.stack([3 * np.arange(T) + b for b in range(B)]).astype(np.int32)
    for b, n_b in enumerate(counts):                     # text directly after the sample's own visual tokens
        real = vs + n_b + tail
        h[b, vs + n_b:real] = c["h"][b, vs + nv:]
        h[b, real:] = 0                                  # padding rows
        pos[b, vs + n_b:real] = pos[b, vs + nv:].copy()
        pos[b, real:] = 0
    wd = {k: dev(v) for k, v in c["w"].items()}
    plan = vc.DecoderLayerPlan(dev(h), torch.from_numpy(pos).cuda(), wd, Hq, Hkv, d, vs, nv, keep,
                               n_vis_samples=torch.tensor(counts, dtype=torch.int32, device="cuda"))
    plan.run()
    torch.cuda.synchronize()
    y, idx, p_out = host_f64(plan.y), plan.keep_idx.cpu().numpy(), plan.positions_out.cpu().numpy()
    norms = plan.norms.cpu().numpy()
    assert plan.n_vis_out.cpu().tolist() == [min(keep, n_b) for n_b in counts]
    assert y.shape[1] == T - nv + keep
    for b, n_b in enumerate(counts):
        real, k_b = vs + n_b + tail, min(keep, n_b)
        out_real = vs + k_b + tail
        ref = Dc.decoder_layer(h[b:b + 1, :real], c["w"], Hq, Hkv, d, vs, n_b, k_b, pos[b:b + 1, :real])
        assert np.allclose(norms[b, :n_b], ref["norms"][0], rtol=2e-3) and not norms[b, n_b:].any()
        if k_b:
            assert_selection_matches(idx[b, vs:vs + k_b] - vs, norms[b, :n_b], ref["norms"][0], k_b, False, f"sample {b}")
        assert np.array_equal(idx[b, :vs], np.arange(vs))
        assert np.array_equal(idx[b, vs + k_b:out_real], np.arange(vs + n_b, real))
        assert (idx[b, out_real:] == T - 1).all()
        if not np.array_equal(idx[b, :out_real], ref["keep_idx"][0]):
            ref = Dc.decoder_layer(h[b:b + 1, :real], c["w"], Hq, Hkv, d, vs, n_b, k_b, pos[b:b + 1, :real],
                                   keep_idx=idx[b:b + 1, :out_real])
        assert np.array_equal(p_out[b, :out_real], ref["positions"][0])
        assert_stream_close(y[b:b + 1, :out_real], ref["y"], f"right-padded batch, sample {b}")
