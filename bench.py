#!/usr/bin/env python3
"""Benchmark of the pruned-prefill hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--keep 320] [--no-schedule] [--no-cpu]

One step = one pass of the whole hot path over one batch of synthetic input:
  Stage I filter on the batch's 20 CLIP-shaped image tiles (scores, top-k, feature compaction)
  + one LLaVA-NeXT-7B-shaped attention layer with pruning on entry (batch 4, 2880 visual + 64
  text tokens): K projection of all tokens with the norm side output, selection, compaction of
  hidden states and K, Q/V projection of survivors, causal attention, output projection.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, vendor figure
# HBM-side bytes per launch of the K-projection GEMM at the bench shape, from two rocprofv3 --pmc
# runs (FETCH_SIZE, WRITE_SIZE) scaled by a plain 1 GiB copy: profiles/gemm_kproj_config3_hbm_traffic.txt
KPROJ_MEASURED_TRAFFIC_BYTES = 791.0e6


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=30)
    p.add_argument("--warmup", type=int, default=30,
                   help="untimed steps before the timed ones; the default spans the clock transient of the first "
                        "15 ms or so under load after idle (steps 5 to 20 run up to 15 %% slower than the steady state)")
    p.add_argument("--keep", type=int, default=320, help="visual budget of the timed layer (of 2880)")
    p.add_argument("--no-schedule", action="store_true", help="skip the 32-layer step-wise schedule leg")
    p.add_argument("--schedule", action="store_true", help="run the schedule leg even with --no-extras (profiling)")
    p.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    p.add_argument("--no-extras", action="store_true", help="only the headline step and its roofline")
    p.add_argument("--calib-copy", action="store_true",
                   help="also run one plain 1 GiB device copy (reference for scaling rocprofv3's "
                        "FETCH_SIZE / WRITE_SIZE counters)")
    p.add_argument("--mfma-kernels", type=int, default=0, metavar="N",
                   help="profiling mode: only N launches each of the matrix-core kernels at their bench shapes "
                        "(K projection on random and on zero operands, attention at 4 x 2944, at the video shape "
                        "and at the pruned 4 x 384, the Stage II clustering with its Gram launch), then one JSON "
                        "line of their times")
    p.add_argument("--traffic", type=float, default=None,
                   help="measured HBM bytes per launch of the dominant kernel (from rocprofv3 --pmc runs), "
                        "echoed in roofline.traffic")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import vitcop_inputs as I
    from paper_2601_17818_amd import binding as vc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    def ev_time(fn, reps, warm=3):
        """Average milliseconds per call, HIP events on the stream the kernels are launched on."""
        for _ in range(warm):
            fn()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    # ------------------------------------------------------------------ inputs
    c3 = I.config3()
    B, T, D, Hq, Hkv, d = c3["B"], c3["T"], c3["D"], c3["Hq"], c3["Hkv"], c3["d"]
    vs, nv = c3["vis_start"], c3["n_vis"]
    x = dev(c3["x"])
    wq, wk, wv, wo = (dev(c3[n]) for n in ("wq", "wk", "wv", "wo"))
    tiles = I.config1(B=5 * B)                       # 5 tiles per image, CLIP ViT-L/14-336 shape
    f_q, f_k, f_feat = dev(tiles["q_cls"]), dev(tiles["k"]), dev(tiles["feats"][:, 1:, :])
    f_keep = tiles["keep"]
    f_out = vc.vitcop_filter_visual(f_q, f_k, f_keep)
    f_bufs = (f_out[0], f_out[1], torch.empty(vc.lib.vitcop_filter_visual_workspace_bytes(
        5 * B, tiles["N"], tiles["H"], tiles["d"]), dtype=torch.uint8, device="cuda"))
    f_cmp = vc.vitcop_compact([f_feat], f_bufs[1])

    # original position ids of the tokens: gathered with the hidden states and K (the survivors keep them)
    pos3 = torch.arange(T, dtype=torch.int32, device="cuda").repeat(B, 1).contiguous()
    plans = {k: vc.LayerPlan(x, wq, wk, wv, wo, Hq, Hkv, d, vs, nv, k, want_norms=False, positions=pos3)
             for k in sorted(set(c3["keeps"]) | {args.keep, nv})}
    plan = plans[args.keep]
    Tp = T - nv + args.keep

    if args.mfma_kernels > 0:
        n_ = args.mfma_kernels
        kd_ = Hkv * d
        res = {}
        x2d = x.reshape(B * T, D)
        kb_ = vc.vitcop_project(x2d, wk, want_sumsq=True)
        res["kproj_random_ms"] = ev_time(lambda: vc.vitcop_project(x2d, wk, want_sumsq=True, out=kb_), n_)
        res["kproj_TFLOPs"] = 2.0 * B * T * kd_ * D / res["kproj_random_ms"] / 1e9
        for name, b_a, n_a, hq_a, hkv_a in (("attn_4x2944_mha32", B, T, Hq, Hkv), ("attn_1x6400_gqa28_4", 1, 6400, 28, 4),
                                             ("attn_4x384_mha32", B, Tp, Hq, Hkv)):
            qq = torch.randn((b_a, n_a, hq_a, d), dtype=torch.bfloat16, device="cuda")
            kk = torch.randn((b_a, n_a, hkv_a, d), dtype=torch.bfloat16, device="cuda")
            vv = torch.randn((b_a, n_a, hkv_a, d), dtype=torch.bfloat16, device="cuda")
            oo = torch.empty_like(qq)
            res[name + "_ms"] = ev_time(lambda: vc.vitcop_prefill_attn(qq, kk, vv, out=oo), n_, warm=3)
            res[name + "_TFLOPs"] = 4.0 * d * hq_a * b_a * n_a * (n_a + 1) / 2 / res[name + "_ms"] / 1e9
            del qq, kk, vv, oo
        cases = [I.vic_inputs(I.seed_for(1, 50 + j), 288, 4096, grid=24, n_regions=8, noise=0.2) for j in range(8)]
        vf = dev(np.stack([c["feats"] for c in cases]))
        vp = torch.from_numpy(np.stack([c["pos"] for c in cases])).cuda()
        res["vic_cluster_8x288x4096_ms"] = ev_time(lambda: vc.vitcop_vic_cluster(vf, vp, 8.0, 0.6, 29), n_)
        res["gram_GFLOP"] = 2.0 * 8 * 288 * 288 * 4096 / 1e9
        xz, wz = torch.zeros_like(x2d), torch.zeros_like(wk)
        res["kproj_zero_ms"] = ev_time(lambda: vc.vitcop_project(xz, wz, want_sumsq=True, out=kb_), n_)
        if args.calib_copy:
            src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "mfma-kernels", "launches_each": n_, **res}))
        return

    def step(kproj_events=None):
        vc.vitcop_filter_visual(f_q, f_k, f_keep, out=f_bufs)
        vc.vitcop_compact([f_feat], f_bufs[1], outs_in=f_cmp)
        plan.run(kproj_events)

    # HIP events around the dominant kernel (the K projection) of every timed step: the library
    # records them on the stream it launches on, right before and after that kernel
    kproj_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                    for _ in range(args.steps)]
    for a_, b_ in kproj_events:          # a first record creates the underlying handles
        a_.record()
        b_.record()

    # ------------------------------------------- measured ceilings (before the timed region)
    # Beside the vendor peaks: the SAME K-projection kernel and launch on all-zero operands (what the matrix
    # cores sustain when the data toggles no bits: the clock the chip holds under this kernel is power-limited
    # and depends on the operands), a plain 1 GiB device-to-device copy for HBM, and the launch back to back on
    # the bench operands.  They run first, so that the chip has also settled at the clock it holds under this
    # load when the warm-up steps begin (after idle the first 15 ms or so of the steps run up to 15 % slower).
    # (Left out with --no-extras, so that a profile of that command holds the K projection only as it runs
    # inside the steps.)
    kd, qd = Hkv * d, Hq * d
    kproj_flops = 2.0 * B * T * kd * D
    kbuf = vc.vitcop_project(x.reshape(B * T, D), wk, want_sumsq=True)
    t_kproj_alone, peak_measured = None, None
    if not args.no_extras:
        csrc_ = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        cdst_ = torch.empty_like(csrc_)
        t_copy = ev_time(lambda: cdst_.copy_(csrc_), 10)
        del csrc_, cdst_
        xz, wz = torch.zeros_like(x).reshape(B * T, D), torch.zeros_like(wk)
        zbuf = vc.vitcop_project(xz, wz, want_sumsq=True)
        t_kproj_zero = ev_time(lambda: vc.vitcop_project(xz, wz, want_sumsq=True, out=zbuf), 20)
        del xz, wz, zbuf
        t_kproj_alone = ev_time(lambda: vc.vitcop_project(x.reshape(B * T, D), wk, want_sumsq=True, out=kbuf), 20,
                                warm=30)
        peak_measured = {
            "mfma_TFLOPs_same_kernel_zero_operands": kproj_flops / (t_kproj_zero * 1e-3) / 1e12,
            "kproj_gemm_zero_operands_ms": t_kproj_zero,
            "kproj_gemm_random_operands_back_to_back_ms": t_kproj_alone,
            "hbm_copy_GBps": 2.0 * (1 << 30) / (t_copy * 1e-3) / 1e9,
        }

    # ------------------------------------------------------------ timed region
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = B * T / (ms_per_step * 1e-3)
    # the same K steps once more, now with the event pairs (kept out of the pass that is timed
    # for `value`, which they would lengthen by their own record calls)
    for i_ in range(args.steps):
        step(kproj_events[i_])
    torch.cuda.synchronize()
    t_kproj = sum(a_.elapsed_time(b_) for a_, b_ in kproj_events) / args.steps       # ms, inside the steps

    # ------------------------------------------- per-kernel durations (HIP events)
    reps = max(5, args.steps)
    roofline = {
        "kernel": "gemm_kernel<256,256> (K projection with squared-norm epilogue)",
        "bound": "mfma", "achieved": kproj_flops / (t_kproj * 1e-3) / 1e12,
        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "traffic": KPROJ_MEASURED_TRAFFIC_BYTES if args.keep == 320 else None,
    }
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["algorithmic_flops_per_launch"] = kproj_flops
    roofline["algorithmic_bytes_per_launch"] = 2.0 * (B * T * D + kd * D + B * T * kd)
    if args.traffic is not None:
        roofline["traffic"] = args.traffic
    if peak_measured is not None:
        roofline["peak_measured"] = peak_measured
    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "pruned_prefill_layer_tokens_per_s", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"config3: LLaVA-NeXT-7B-shaped layer, B={B}, T={T} (2880 visual + 64 text), "
                               f"keep {args.keep} of {nv} visual (T'={Tp}), D={D}, {Hq}x{d} MHA; "
                               f"plus Stage I filter on {5 * B} CLIP tiles (577x16x64, keep {f_keep})",
                   "seed": I.seed_for(3)},
        "roofline": roofline,
    }

    if not args.no_extras:
        kern = {}
        kern["kproj_gemm_ms"] = t_kproj
        kern["kproj_gemm_back_to_back_ms"] = t_kproj_alone
        # K-norm + select as its own call on the projected K (algorithmic bytes: K rows + norms + list)
        k_all = kbuf[0].reshape(B, T, Hkv, d)
        nbuf = torch.empty((B, nv), dtype=torch.float32, device="cuda")
        ibuf = torch.empty((B, Tp), dtype=torch.int32, device="cuda")
        t_ks = ev_time(lambda: vc.vitcop_knorm_select(k_all, vs, nv, args.keep, norms=nbuf, idx_out=ibuf), reps)
        ks_bytes = B * nv * (2 * kd + 4) + B * Tp * 4
        kern["knorm_select_ms"] = t_ks
        kern["knorm_select_GBps"] = ks_bytes / (t_ks * 1e-3) / 1e9
        # streaming measurement: many independent config-0-shaped samples, > 1 GiB of K
        R = 288
        kbig = torch.randn((R, 640, 32, 128), dtype=torch.bfloat16, device="cuda")
        nb2 = torch.empty((R, 576), dtype=torch.float32, device="cuda")
        ib2 = torch.empty((R, 128), dtype=torch.int32, device="cuda")
        t_s = ev_time(lambda: vc.vitcop_knorm_select(kbig, 35, 576, 64, norms=nb2, idx_out=ib2), 10)
        s_bytes = R * 576 * (2 * 4096 + 4) + R * 128 * 4
        kern["knorm_select_stream_GBps"] = s_bytes / (t_s * 1e-3) / 1e9
        kern["knorm_select_stream_frac_hbm"] = kern["knorm_select_stream_GBps"] / HBM_PEAK_GBPS
        idx_big = ib2
        cbig = torch.empty((R, 128, 32, 128), dtype=torch.bfloat16, device="cuda")
        t_c = ev_time(lambda: vc.vitcop_compact([kbig], idx_big, outs_in=[cbig]), 10)
        kern["compact_stream_GBps"] = (R * 128 * (2 * 8192 + 4)) / (t_c * 1e-3) / 1e9
        del kbig, cbig
        # filter (config 1 shape x 20 tiles)
        t_f = ev_time(lambda: vc.vitcop_filter_visual(f_q, f_k, f_keep, out=f_bufs), reps)
        f_bytes = 5 * B * (577 * 1024 * 2 + f_keep * 4)
        kern["filter_ms"] = t_f
        kern["filter_GBps"] = f_bytes / (t_f * 1e-3) / 1e9
        # attention (causal-useful FLOPs): the pruned and the unpruned shape of this layer, the same
        # unpruned shape with the batch raised to 24 workgroups per CU, and the video shape
        # (28 query heads on 4 KV heads) unpruned and at its pruned length
        for name, b_att, n_att, hq_att, hkv_att in (
                ("attn_pruned", B, Tp, Hq, Hkv), ("attn_unpruned", B, T, Hq, Hkv),
                ("attn_unpruned_batch16", 16, T, Hq, Hkv), ("attn_video_unpruned", 1, 6400, 28, 4),
                ("attn_video_pruned", 1, 755, 28, 4)):
            qq = torch.randn((b_att, n_att, hq_att, d), dtype=torch.bfloat16, device="cuda")
            kk = torch.randn((b_att, n_att, hkv_att, d), dtype=torch.bfloat16, device="cuda")
            vv = torch.randn((b_att, n_att, hkv_att, d), dtype=torch.bfloat16, device="cuda")
            oo = torch.empty_like(qq)
            t_a = ev_time(lambda: vc.vitcop_prefill_attn(qq, kk, vv, out=oo), 20, warm=10)
            fl = 4.0 * d * hq_att * b_att * n_att * (n_att + 1) / 2
            kern[name + "_ms"] = t_a
            kern[name + "_TFLOPs"] = fl / (t_a * 1e-3) / 1e12
            kern[name + "_frac_mfma"] = kern[name + "_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
            del qq, kk, vv, oo
        # Stage II (Sec. 3.2.1, 3.2.3): clustering of the Stage I survivors and per-cluster elites +
        # merging, at the image shape (8 images x 288 tokens, D 4096, 29 centres, budget 253) and at
        # the video shape (1856 tokens as one set, D 3584, 186 centres, budget 627)
        stage2 = {}
        for name, b2, n2, d2, nc2, bud2, grid2 in (("image_8x288", 8, 288, 4096, 29, 253, 24),
                                                   ("video_1x1856", 1, 1856, 3584, 186, 627, 44)):
            cases = [I.vic_inputs(I.seed_for(1, 50 + j), n2, d2, grid=grid2, n_regions=max(8, n2 // 40), noise=0.2)
                     for j in range(b2)]
            vf = dev(np.stack([c["feats"] for c in cases]))
            vp = torch.from_numpy(np.stack([c["pos"] for c in cases])).cuda()
            vnorm = torch.rand((b2, n2), dtype=torch.float32, device="cuda") + 0.5
            vr = vc.vitcop_vic_cluster(vf, vp, 8.0, 0.6, nc2)
            t_v = ev_time(lambda: vc.vitcop_vic_cluster(vf, vp, 8.0, 0.6, nc2), 10)
            t_m = ev_time(lambda: vc.vitcop_collab_prune_merge(vf, vr["labels"], vr["n_clusters"], vnorm, bud2), 10)
            stage2[name] = {"vic_ms": t_v, "collab_ms": t_m, "clusters": vr["n_clusters"].cpu().tolist(),
                            "gram_GFLOP": 2.0 * b2 * n2 * n2 * d2 / 1e9}
            del vf, vp, vr
        kern["stage2"] = stage2
        # one decoding step over the KV cache the prefill leaves behind (per layer): pruned and
        # unpruned cache length of this workload, and a streaming case (32 samples x 4096 keys,
        # 2.1 GB of K and V) for the HBM fraction; algorithmic bytes = K and V read once
        dec = {}
        for name, b_d, n_d in (("pruned", B, Tp), ("unpruned", B, T), ("stream", 32, 4096)):
            kk = torch.randn((b_d, n_d, Hkv, d), dtype=torch.bfloat16, device="cuda")
            vv = torch.randn((b_d, n_d, Hkv, d), dtype=torch.bfloat16, device="cuda")
            qq = torch.randn((b_d, Hq, d), dtype=torch.bfloat16, device="cuda")
            bufs = vc.vitcop_decode_attn(qq, kk, vv)
            bufs = (bufs[0], bufs[1], torch.empty(vc.lib.vitcop_decode_attn_workspace_bytes(b_d, n_d, Hq, Hkv, d),
                                                  dtype=torch.uint8, device="cuda"))
            t_d = ev_time(lambda: vc.vitcop_decode_attn(qq, kk, vv, out=bufs), 20, warm=5)
            dec[name + "_us"] = t_d * 1e3
            dec[name + "_GBps"] = 2.0 * b_d * n_d * Hkv * d * 2 / (t_d * 1e-3) / 1e9
            del kk, vv, qq, bufs
        dec["stream_frac_hbm"] = dec["stream_GBps"] / HBM_PEAK_GBPS
        dec["speedup_pruned_cache"] = dec["unpruned_us"] / dec["pruned_us"]
        kern["decode_step"] = dec
        # projections at the row counts pruning leaves in config 2 (128 rows; 4096x4096, the MLP's
        # 4096x11008 and 11008x4096): HBM-bound on the weights, which are rotated through more than
        # the 256 MB of cache so that every call streams them from HBM; per call = kernel + reduction
        few = {}
        for (N_, K_) in ((4096, 4096), (4096, 11008), (11008, 4096)):
            n_w = max(2, int(300e6 // (N_ * K_ * 2)) + 1)
            w_rot = [torch.randn((N_, K_), dtype=torch.bfloat16, device="cuda") * 0.02 for _ in range(n_w)]
            x_few = torch.randn((128, K_), dtype=torch.bfloat16, device="cuda")
            bufs = vc.vitcop_project(x_few, w_rot[0])
            ws_few = torch.empty(vc.lib.vitcop_project_workspace_bytes(128, N_, K_), dtype=torch.uint8, device="cuda")
            it = [0]

            def few_call():
                it[0] += 1
                vc.vitcop_project(x_few, w_rot[it[0] % n_w], out=bufs, scratch=ws_few)
            us = ev_time(few_call, 4 * n_w) * 1e3
            few[f"128x{N_}x{K_}"] = {"us": us, "weights_GBps": N_ * K_ * 2 / us / 1e3,
                                      "frac_hbm": N_ * K_ * 2 / us / 1e3 / HBM_PEAK_GBPS}
            del w_rot, x_few, bufs, ws_few
        kern["few_row_projection"] = few
        # a full decoder layer (RMSNorm, rotary embedding, gated MLP of width 11008 around the same
        # attention block) with pruning on entry, at the bench shape
        Fm = 11008
        dw = {"ln1": torch.ones(D, dtype=torch.bfloat16, device="cuda"),
              "ln2": torch.ones(D, dtype=torch.bfloat16, device="cuda"),
              "wq": wq, "wk": wk, "wv": wv, "wo": wo,
              "wg": torch.randn((Fm, D), dtype=torch.bfloat16, device="cuda") * 0.02,
              "wu": torch.randn((Fm, D), dtype=torch.bfloat16, device="cuda") * 0.02,
              "wd": torch.randn((D, Fm), dtype=torch.bfloat16, device="cuda") * 0.02}
        dpos = pos3
        dec_ms = {}
        for k_ in sorted(set(c3["keeps"]) | {args.keep, nv}):
            dp = vc.DecoderLayerPlan(x, dpos, dw, Hq, Hkv, d, vs, nv, k_)
            dec_ms["unpruned" if k_ == nv else f"keep{k_}"] = ev_time(dp.run, 10)
            del dp
        kern["decoder_layer_ms"] = dec_ms
        out["decoder_layer_speedup_vs_unpruned"] = {k_: dec_ms["unpruned"] / v_ for k_, v_ in dec_ms.items()
                                                    if k_ != "unpruned"}
        del dw
        # the layer alone at each keep ratio, and the unpruned layer
        layer_ms = {}
        for k_, p_ in plans.items():
            layer_ms[k_] = ev_time(p_.run, max(3, reps // 3))
        kern["layer_ms"] = {("unpruned" if k_ == nv else f"keep{k_}"): v_ for k_, v_ in layer_ms.items()}
        out["speedup_vs_unpruned"] = {f"keep{k_}": layer_ms[nv] / v_ for k_, v_ in layer_ms.items() if k_ != nv}
        out["layer_tokens_per_s"] = {("unpruned" if k_ == nv else f"keep{k_}"): B * T / (v_ * 1e-3)
                                     for k_, v_ in layer_ms.items()}
        # ---- the other workload configs at their own shapes: single-call latency (L) ----
        def layer_line(c, keeps, what):
            xs_ = dev(c["x"])
            ws_ = [dev(c[n]) for n in ("wq", "wk", "wv", "wo")]
            ps_ = torch.arange(c["T"], dtype=torch.int32, device="cuda").repeat(c["B"], 1).contiguous()
            ms = {}
            for k_ in keeps:
                pl_ = vc.LayerPlan(xs_, *ws_, c["Hq"], c["Hkv"], c["d"], c["vis_start"], c["n_vis"], k_,
                                   want_norms=False, positions=ps_)
                ms["unpruned" if k_ == c["n_vis"] else f"keep{k_}"] = ev_time(pl_.run, 20, warm=5)
                del pl_
            return {"workload": what, "layer_ms": ms,
                    "speedup_vs_unpruned": {k_: ms["unpruned"] / v_ for k_, v_ in ms.items() if k_ != "unpruned"},
                    "tokens_per_s": {k_: c["B"] * c["T"] / (v_ * 1e-3) for k_, v_ in ms.items()}}

        # config 0: one LLaVA-1.5-shaped sample, 640 tokens, keep 64 of 576 (launch-latency bound)
        c0 = I.config0()
        cfg0 = layer_line(c0, (64, 576), "config0: B=1, T=640 (35 + 576 + 29), keep 64 of 576, D=4096, 32x128 MHA")
        # compaction alone at that shape: hidden states, K and positions of the 128 survivors
        x0 = dev(c0["x"])
        k0 = torch.randn((1, 640, 32, 128), dtype=torch.bfloat16, device="cuda")
        p0 = torch.arange(640, dtype=torch.int32, device="cuda")[None].contiguous()
        i0 = torch.cat([torch.arange(35), 35 + torch.arange(64) * 9, torch.arange(611, 640)]).to(torch.int32).cuda()[None]
        o0 = vc.vitcop_compact([x0, k0, p0], i0)
        t_c0 = ev_time(lambda: vc.vitcop_compact([x0, k0, p0], i0, outs_in=o0), 50, warm=10)
        cfg0["compact_us"] = t_c0 * 1e3
        cfg0["compact_GBps"] = 128 * (2 * (8192 + 8192 + 4) + 4) / (t_c0 * 1e-3) / 1e9
        nb0 = torch.empty((1, 576), dtype=torch.float32, device="cuda")
        ib0 = torch.empty((1, 128), dtype=torch.int32, device="cuda")
        t_k0 = ev_time(lambda: vc.vitcop_knorm_select(k0, 35, 576, 64, norms=nb0, idx_out=ib0), 50, warm=10)
        cfg0["knorm_select_us"] = t_k0 * 1e3
        cfg0["knorm_select_GBps"] = (576 * (8192 + 4) + 128 * 4) / (t_k0 * 1e-3) / 1e9
        del x0, k0, p0, o0
        out["config0"] = cfg0
        # config 1 at its own batch: 8 images x 577 tokens, keep 288 of 576
        c1 = I.config1()
        q1, k1 = dev(c1["q_cls"]), dev(c1["k"])
        b1 = vc.vitcop_filter_visual(q1, k1, c1["keep"])
        b1 = (b1[0], b1[1], torch.empty(vc.lib.vitcop_filter_visual_workspace_bytes(8, 576, 16, 64),
                                       dtype=torch.uint8, device="cuda"))
        t_f1 = ev_time(lambda: vc.vitcop_filter_visual(q1, k1, c1["keep"], out=b1), 50, warm=10)
        out["config1"] = {"workload": "config1: 8 images x 577 tokens x 1024 (16x64), keep 288 of 576",
                          "filter_us": t_f1 * 1e3,
                          "filter_GBps": 8 * (577 * 1024 * 2 + 288 * 4) / (t_f1 * 1e-3) / 1e9,
                          "images_per_s": 8 / (t_f1 * 1e-3)}
        del q1, k1, b1
        # config 4: the video layer (GQA 28/4, D 3584).  (a) K-norm alone: 6272 -> 627 visual tokens;
        # (b) the chain: Stage I per frame (32 x 196 -> 58), compaction of the frame features, then the
        # layer on 1856 visual + 128 text tokens with keep 627; both against the unpruned 6400-token layer
        c4 = I.config4_layer()
        cfg4 = layer_line(c4, (627, 6272), "config4: B=1, T=6400 (32 frames x 196 + 128 text), keep 627 of 6272, "
                                           "D=3584, 28/4 GQA x128")
        fr = I.config4_frames()
        q4, k4, feat4 = dev(fr["q_cls"]), dev(fr["k"]), dev(np.ascontiguousarray(fr["feats"][:, 1:, :]))
        fo4 = vc.vitcop_filter_visual(q4, k4, fr["keep"])
        fb4 = (fo4[0], fo4[1], torch.empty(vc.lib.vitcop_filter_visual_workspace_bytes(32, 196, 16, 64),
                                          dtype=torch.uint8, device="cuda"))
        fc4 = vc.vitcop_compact([feat4], fb4[1])
        torch.cuda.synchronize()
        kept_bits = fc4[0].view(torch.int16).cpu().numpy().view(np.uint16).reshape(32 * fr["keep"], fr["C"])
        c4f = I.config4_layer(n_vis=32 * fr["keep"], vis_feats=I.bf16_bits_to_f32(kept_bits))
        x4f = dev(c4f["x"])
        w4 = [dev(c4f[n]) for n in ("wq", "wk", "wv", "wo")]
        p4f = torch.arange(c4f["T"], dtype=torch.int32, device="cuda")[None].contiguous()
        pl4 = vc.LayerPlan(x4f, *w4, 28, 4, 128, 0, c4f["n_vis"], 627, want_norms=False, positions=p4f)

        def chain4():
            vc.vitcop_filter_visual(q4, k4, fr["keep"], out=fb4)
            vc.vitcop_compact([feat4], fb4[1], outs_in=fc4)
            pl4.run()
        t_fl4 = ev_time(lambda: vc.vitcop_filter_visual(q4, k4, fr["keep"], out=fb4), 50, warm=10)
        t_l4 = ev_time(pl4.run, 20, warm=5)
        t_ch4 = ev_time(chain4, 20, warm=5)
        cfg4["filter_then_knorm"] = {
            "visual_tokens": [6272, 32 * fr["keep"], 627], "filter_us": t_fl4 * 1e3,
            "filter_GBps": 32 * (197 * 1024 * 2 + fr["keep"] * 4) / (t_fl4 * 1e-3) / 1e9,
            "layer_ms": t_l4, "chain_ms": t_ch4,
            "speedup_vs_unpruned": cfg4["layer_ms"]["unpruned"] / t_ch4,
            "tokens_per_s": 6400 / (t_ch4 * 1e-3)}
        del pl4, x4f, w4, q4, k4, feat4
        out["config4"] = cfg4
        out["knorm_select_GBps"] = kern["knorm_select_stream_GBps"]
        out["attn_bf16_TFLOPs"] = kern["attn_unpruned_TFLOPs"]
        out["attn_frac_of_peak"] = kern["attn_unpruned_frac_mfma"]
        out["attn_bf16_TFLOPs_batch16"] = kern["attn_unpruned_batch16_TFLOPs"]
        out["kernels"] = kern

    # -------------------------------------- step-wise schedule (config 2, 32 layers)
    if args.schedule or (not args.no_schedule and not args.no_extras):
        from concurrent.futures import ThreadPoolExecutor
        h2 = I.config2_hidden()
        with ThreadPoolExecutor(max_workers=8) as ex:
            w_host = list(ex.map(I.config2_layer_weights, range(I.CONFIG2_LAYERS)))
        for w in w_host:      # small output projection keeps the residual stream bounded without a norm
            w["wo"] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w["wo"]) * np.float32(0.125))
        w_dev = [{n: dev(w[n]) for n in ("wq", "wk", "wv", "wo")} for w in w_host]
        del w_host
        x2 = dev(h2["x"])
        sp = vc.SchedulePlan(x2, w_dev, 32, 32, 128, 35, 576, I.CONFIG2_SCHEDULE)
        up = vc.SchedulePlan(x2, w_dev, 32, 32, 128, 35, 576, ())
        t_sched = ev_time(sp.run, 5, warm=2)
        t_unpr = ev_time(up.run, 5, warm=2)
        out["schedule_config2"] = {"ms_pruned": t_sched, "ms_unpruned": t_unpr,
                                   "speedup": t_unpr / t_sched, "tokens_per_s": 640 / (t_sched * 1e-3),
                                   "layers": 32, "schedule": list(map(list, I.CONFIG2_SCHEDULE))}
        # the same schedule over full decoder layers (norms, rotary embedding, gated MLP with F = 11008);
        # the MLP weights are drawn on the device from a seeded generator
        gen = torch.Generator(device="cuda").manual_seed(2)
        F2 = 11008
        for w in w_dev:
            for n, shape, std in (("wg", (F2, 4096), 0.02), ("wu", (F2, 4096), 0.02), ("wd", (4096, F2), 0.0025)):
                w[n] = (torch.randn(shape, generator=gen, device="cuda") * std).to(torch.bfloat16)
            w["ln1"] = w["ln2"] = torch.ones(4096, dtype=torch.bfloat16, device="cuda")
        pos2 = torch.arange(640, dtype=torch.int32, device="cuda")[None].contiguous()
        dsp = vc.DecoderSchedulePlan(x2, pos2, w_dev, 32, 32, 128, 35, 576, I.CONFIG2_SCHEDULE)
        dup = vc.DecoderSchedulePlan(x2, pos2, w_dev, 32, 32, 128, 35, 576, ())
        t_dsched = ev_time(dsp.run, 6, warm=3)
        t_dunpr = ev_time(dup.run, 6, warm=3)
        out["decoder_schedule_config2"] = {"ms_pruned": t_dsched, "ms_unpruned": t_dunpr,
                                           "speedup": t_dunpr / t_dsched,
                                           "tokens_per_s": 640 / (t_dsched * 1e-3), "layers": 32, "F": F2}
        # the paper's own LLaVA-1.5 schedules (App. C, Table 7: Stage I keeps ratio r1 of the 576 visual
        # tokens before the language model, pruning on entry to layers 2 and 22 keeps r2 and r3) against
        # the unpruned 640-token prefill, with the FLOPs ratio Eq. 9 predicts (layer cost 4 n^2 d + 16 n d^2)
        def eq9_ratio(counts):
            cost = lambda n: 4.0 * n * n * 4096 + 16.0 * n * 4096 * 4096
            full = 32 * cost(640)
            return full / (2 * cost(counts[0]) + 20 * cost(counts[1]) + 10 * cost(counts[2]))
        paper = {}
        for name, (r1, r2, r3) in (("retain192", (0.5, 0.4394, 0.0879)), ("retain64", (0.3, 0.1343, 0.0269))):
            v1, v2, v3 = (int(round(576 * r)) for r in (r1, r2, r3))
            T1 = 64 + v1
            xp = x2[:, :T1].contiguous()          # (timing only: which visual tokens Stage I kept does not matter)
            pp = torch.arange(T1, dtype=torch.int32, device="cuda")[None].contiguous()
            plan = vc.DecoderSchedulePlan(xp, pp, w_dev, 32, 32, 128, 35, v1, ((2, v2), (22, v3)))
            t_p = ev_time(plan.run, 6, warm=3)
            paper[name] = {"visual_tokens": [v1, v2, v3], "ms": t_p, "speedup_vs_unpruned": t_dunpr / t_p,
                           "eq9_flops_ratio": eq9_ratio((64 + v1, 64 + v2, 64 + v3))}
            del plan, xp, pp
        # the same "retain 192" schedule on a batch of 8 prompts (2816 / 2536 / 920 rows per layer): the projections
        # are then matrix-core-bound on both sides and the speedup moves towards the FLOPs ratio
        x8 = x2.repeat(8, 1, 1).contiguous()
        p8 = pos2.repeat(8, 1).contiguous()
        u8 = vc.DecoderSchedulePlan(x8, p8, w_dev, 32, 32, 128, 35, 576, ())
        t_u8 = ev_time(u8.run, 3, warm=1)
        del u8
        r8 = vc.DecoderSchedulePlan(x8[:, :352].contiguous(), p8[:, :352].contiguous(), w_dev, 32, 32, 128, 35, 288,
                                    ((2, 253), (22, 51)))
        t_r8 = ev_time(r8.run, 3, warm=1)
        del r8, x8, p8
        paper["retain192_batch8"] = {"ms": t_r8, "ms_unpruned": t_u8, "speedup_vs_unpruned": t_u8 / t_r8,
                                     "unpruned_tokens_per_s": 8 * 640 / (t_u8 * 1e-3),
                                     "eq9_flops_ratio": paper["retain192"]["eq9_flops_ratio"]}
        out["decoder_schedule_paper_llava15"] = paper
        # the same "retain 192" setting with the paper's actual Stage II at layer 2 (clustering, elites,
        # merging; budget 253) and Stage III at layer 22; the 288 visual hidden states are planted spatial
        # regions so that the clustering has something to find; one host read-back inside
        vin = I.vic_inputs(2, 288, 4096, 24, 29, 0.15)
        xf = x2[:, :64 + 288].clone()
        xf[0, 35:35 + 288] = dev(vin["feats"])
        pf = torch.arange(64 + 288, dtype=torch.int32, device="cuda")[None].contiguous()
        xy = torch.from_numpy(vin["pos"].astype(np.float32)[None]).cuda()
        fplan = vc.FullSchedulePlan(xf, pf, w_dev, 32, 32, 128, 35, 288,
                                    {"layer": 2, "budget": 253, "n_centers": 29, "d_c": 8.0, "tau": 0.6, "xy": xy},
                                    ((22, 51),))
        t_f = ev_time(fplan.run, 5, warm=2)
        out["full_schedule_paper_llava15_retain192"] = {
            "ms": t_f, "speedup_vs_unpruned": t_dunpr / t_f, "visual_after_stage2": fplan.n_stage2[0],
            "tokens_final": fplan.T_final}
        del fplan, xf, pf, xy
        # the same on a batch of 8 prompts whose images differ (8 seeds of planted regions): Stage II leaves a
        # different number of visual tokens per sample, the batch runs right-padded to the longest
        xf8 = x2[:, :64 + 288].repeat(8, 1, 1).contiguous()
        xy8 = []
        for b in range(8):
            vin = I.vic_inputs(2 + b, 288, 4096, 24, 29, 0.15)
            xf8[b, 35:35 + 288] = dev(vin["feats"])
            xy8.append(vin["pos"].astype(np.float32))
        pf8 = torch.arange(64 + 288, dtype=torch.int32, device="cuda")[None].repeat(8, 1).contiguous()
        fplan8 = vc.FullSchedulePlan(xf8, pf8, w_dev, 32, 32, 128, 35, 288,
                                     {"layer": 2, "budget": 253, "n_centers": 29, "d_c": 8.0, "tau": 0.6,
                                      "xy": torch.from_numpy(np.stack(xy8)).cuda()}, ((22, 51),))
        t_f8 = ev_time(fplan8.run, 3, warm=1)
        out["full_schedule_paper_llava15_retain192"]["batch8"] = {
            "ms": t_f8, "speedup_vs_unpruned": paper["retain192_batch8"]["ms_unpruned"] / t_f8,
            "visual_after_stage2": fplan8.n_stage2, "tokens_final": fplan8.T_final}
        del fplan8, xf8, pf8, xy8
        # one decoding step (a new token per sample through all 32 layers) over the caches those prefills
        # leave: per-layer cache lengths of the unpruned prefill and of the paper's two schedules (Table 5's
        # time per generated token); a step streams every weight (12.95 GB) and every cached K and V once
        dec = {}
        w_bytes = 32 * (4 * 4096 * 4096 + 3 * 4096 * F2) * 2
        lens = {"unpruned": [640] * 32}
        for name, (r1, r2, r3) in (("retain192", (0.5, 0.4394, 0.0879)), ("retain64", (0.3, 0.1343, 0.0269))):
            v1, v2, v3 = (int(round(576 * r)) for r in (r1, r2, r3))
            lens[name] = [64 + v1] * 2 + [64 + v2] * 20 + [64 + v3] * 10
        for Bd in (1, 64):
            caches = [tuple(torch.empty((Bd, 704, 32, 128), dtype=torch.bfloat16, device="cuda").normal_(generator=gen)
                            for _ in range(2)) for _ in range(32)]
            hd = torch.empty((Bd, 4096), dtype=torch.bfloat16, device="cuda").normal_(generator=gen)
            pd = torch.full((Bd,), 700, dtype=torch.int32, device="cuda")
            for name, n_cached in lens.items():
                dplan = vc.DecoderDecodePlan(hd, pd, w_dev, 32, 32, 128, caches, n_cached)
                t_d = ev_time(dplan.run, 10, warm=3)
                moved = w_bytes + sum(n + 1 for n in n_cached) * Bd * 4096 * 2 * 2
                dec[f"batch{Bd}_{name}"] = {"ms_per_step": t_d, "tokens_per_s": Bd / (t_d * 1e-3),
                                            "GBps": moved / t_d / 1e6, "frac_hbm": moved / t_d / 1e6 / HBM_PEAK_GBPS}
                del dplan
            del caches, hd, pd
        out["decode_step_config2"] = dec
        del w_dev, sp, up, dsp, dup

    # ------------------------------------------------------ CPU oracle baseline
    if not args.no_cpu:
        from oracle import vitcop_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        t0 = time.perf_counter()
        n_cpu = 0
        while n_cpu == 0 or time.perf_counter() - t0 < 10.0:     # about 10 s of CPU work
            O.pruned_layer(c3["x"], c3["wq"], c3["wk"], c3["wv"], c3["wo"], Hq, Hkv, d, vs, nv, args.keep)
            O.filter_visual(tiles["q_cls"], tiles["k"], f_keep)
            n_cpu += 1
        t_cpu = (time.perf_counter() - t0) / n_cpu
        out["cpu_baseline"] = {"value": B * T / t_cpu, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{n_cpu} full steps of the same workload ({B} samples x {T} tokens, fp64 "
                                         f"pruned layer + filter on {5 * B} tiles), {t_cpu:.2f} s per step"}
        # the same oracle held to one thread, on one sample of the batch (a quarter of the step)
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                t0 = time.perf_counter()
                O.pruned_layer(c3["x"][:1], c3["wq"], c3["wk"], c3["wv"], c3["wo"], Hq, Hkv, d, vs, nv, args.keep)
                O.filter_visual(tiles["q_cls"][:5], tiles["k"][:5], f_keep)
                t_one = time.perf_counter() - t0
            out["cpu_baseline"]["single_thread"] = {
                "value": T / t_one, "unit": "tokens/s", "cores": 1,
                "sample": f"one sample ({T} tokens) + 5 tiles, {t_one:.2f} s"}
        except ImportError:
            pass

    print(json.dumps(out))


if __name__ == "__main__":
    main()
