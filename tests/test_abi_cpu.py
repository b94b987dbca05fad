"""The C-ABI library: loads, exports every declared symbol, validates on the host.

No compute call is made here; every call below must be rejected by the
argument checks that run before any HIP call.
"""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vitcop.h")

# a missing library is a failure here, not a skip: the boundary is what these tests are about
from paper_2601_17818_amd import binding  # noqa: E402

lib = binding.lib

A16 = 0x1000   # a fake, 16-byte aligned, non-null "device pointer" (never dereferenced)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vitcop_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_codes_match_header():
    text = open(HEADER).read()
    for name in ("VITCOP_OK", "VITCOP_EINVAL", "VITCOP_EUNSUPPORTED", "VITCOP_EWORKSPACE", "VITCOP_EHIP"):
        m = re.search(rf"#define\s+{name}\s+\(?(-?\d+)\)?", text)
        assert m and int(m.group(1)) == getattr(binding, name)
    m = re.search(r"#define\s+VITCOP_MAX_CANDIDATES\s+(\d+)", text)
    assert int(m.group(1)) == binding.VITCOP_MAX_CANDIDATES


def test_struct_sizes_match_c_layout():
    assert C.sizeof(binding.GatherT) == 40
    assert C.sizeof(binding.LayerT) == 10 * 4 + 12 * 8
    assert C.sizeof(binding.ScheduleT) == 10 * 4 + 9 * 8


def test_filter_validation():
    f = lib.vitcop_filter_visual
    assert f(A16, A16, 1, 10, 2, 64, 11, 0.0, None, A16, A16, 1 << 20, None) == binding.VITCOP_EINVAL
    assert "keep" in binding.vitcop_last_error()
    assert f(A16, A16, 1, 10, 2, 32, 5, 0.0, None, A16, A16, 1 << 20, None) == binding.VITCOP_EUNSUPPORTED
    assert f(None, A16, 1, 10, 2, 64, 5, 0.0, None, A16, A16, 1 << 20, None) == binding.VITCOP_EINVAL
    assert f(A16 + 2, A16, 1, 10, 2, 64, 5, 0.0, None, A16, A16, 1 << 20, None) == binding.VITCOP_EINVAL
    assert f(A16, A16, 1, 10, 2, 64, 5, 0.0, None, A16, A16, 8, None) == binding.VITCOP_EWORKSPACE
    assert f(A16, A16, 1, 10, 2, 64, 5, 0.0, None, A16, None, 0, None) == binding.VITCOP_EWORKSPACE
    assert f(A16, A16, 1, 20000, 2, 64, 5, 0.0, None, A16, A16, 1 << 30, None) == binding.VITCOP_EUNSUPPORTED
    assert f(A16, A16, -1, 10, 2, 64, 5, 0.0, None, A16, A16, 1 << 20, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_filter_visual_workspace_bytes(8, 576, 16, 64) >= 8 * 16 * 577 * 4
    # an empty batch is a no-op, not an error
    assert f(None, None, 0, 10, 2, 64, 5, 0.0, None, None, None, 0, None) == binding.VITCOP_OK


def test_filter_static_validation():
    # the variant without workspace: the same argument checks, then the size limit of its built-in scratch,
    # all before any HIP call
    f = lib.vitcop_filter_visual_static
    assert f(A16, A16, 1, 10, 2, 64, 11, 0.0, None, A16, None) == binding.VITCOP_EINVAL
    assert f(A16, A16, 1, 10, 2, 32, 5, 0.0, None, A16, None) == binding.VITCOP_EUNSUPPORTED
    assert f(None, A16, 1, 10, 2, 64, 5, 0.0, None, A16, None) == binding.VITCOP_EINVAL
    assert f(None, None, 0, 10, 2, 64, 5, 0.0, None, None, None) == binding.VITCOP_OK
    text = open(HEADER).read()
    limit = re.search(r"#define\s+VITCOP_FILTER_STATIC_MAX_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert int(limit.group(1)) << int(limit.group(2)) == binding.VITCOP_FILTER_STATIC_MAX_BYTES == 4 << 20
    # 64 x 16 x 1025 x 4 bytes of logits do not fit, 64 x 16 x 1024 x 4 would (rejected here for N > limit instead)
    assert f(A16, A16, 64, 1024, 16, 64, 5, 0.0, None, A16, None) == binding.VITCOP_EUNSUPPORTED
    assert "scratch" in binding.vitcop_last_error()


def test_knorm_select_validation():
    f = lib.vitcop_knorm_select

    def call(k=A16, rs=4096, bs=640 * 4096, B=1, T=640, Hkv=32, d=128, vs=35, nv=576, keep=64,
             norms=A16, idx=A16, flags=0):
        return f(k, rs, bs, B, T, Hkv, d, vs, nv, keep, norms, idx, flags, None, 0, None)

    assert call(keep=577) == binding.VITCOP_EINVAL
    assert call(vs=100, nv=576) == binding.VITCOP_EINVAL          # span leaves the sequence
    assert call(k=None) == binding.VITCOP_EINVAL
    assert call(k=A16 + 8) == binding.VITCOP_EINVAL
    assert call(rs=4095) == binding.VITCOP_EINVAL
    assert call(rs=2048) == binding.VITCOP_EINVAL                 # stride shorter than a row
    assert call(idx=None) == binding.VITCOP_EINVAL
    assert call(norms=None) == binding.VITCOP_EINVAL
    assert call(flags=8) == binding.VITCOP_EINVAL
    assert call(flags=binding.VITCOP_NORMS_SQUARED) == binding.VITCOP_EINVAL
    assert call(T=40000, nv=20000, vs=0, bs=40000 * 4096) == binding.VITCOP_EUNSUPPORTED
    assert call(Hkv=1, d=12, rs=16) == binding.VITCOP_EUNSUPPORTED  # row not a multiple of 8
    assert call(B=0) == binding.VITCOP_OK


def test_compact_validation():
    f = lib.vitcop_compact
    g = (binding.GatherT * 2)()
    g[0] = binding.GatherT(A16, A16 + 4096, 64, 64, 6400)
    g[1] = binding.GatherT(A16, A16, 64, 64, 6400)
    assert f(g, 2, A16, 1, 100, 10, None) == binding.VITCOP_EINVAL           # in place
    assert f(g, 9, A16, 1, 100, 10, None) == binding.VITCOP_EINVAL
    assert f(g, 1, None, 1, 100, 10, None) == binding.VITCOP_EINVAL
    g[0] = binding.GatherT(A16, A16 + 4096, 6, 64, 6400)
    assert f(g, 1, A16, 1, 100, 10, None) == binding.VITCOP_EINVAL           # row_bytes % 4
    g[0] = binding.GatherT(A16, A16 + 4096, 64, 32, 6400)
    assert f(g, 1, A16, 1, 100, 10, None) == binding.VITCOP_EINVAL           # stride < row
    g[0] = binding.GatherT(A16, A16 + 4096, 64, 64, 6400)
    assert f(g, 1, A16, 1, 0, 10, None) == binding.VITCOP_EINVAL             # rows from nothing
    assert f(g, 1, A16, 1, 100, 0, None) == binding.VITCOP_OK
    assert f(g, 0, None, 1, 100, 10, None) == binding.VITCOP_OK


def test_attn_validation():
    f = lib.vitcop_prefill_attn

    def call(q=A16, k=A16, v=A16, out=A16, B=1, N=128, Hq=32, Hkv=32, d=128, scale=0.0, causal=1):
        return f(q, k, v, out, None, B, N, Hq, Hkv, d, scale, causal, None, 0, None)

    assert call(Hq=28, Hkv=5) == binding.VITCOP_EINVAL
    assert call(d=96) == binding.VITCOP_EUNSUPPORTED
    assert call(d=64, N=0) == binding.VITCOP_OK                  # d = 64 passes validation
    assert call(causal=2) == binding.VITCOP_EINVAL
    assert call(scale=-1.0) == binding.VITCOP_EINVAL
    assert call(q=None) == binding.VITCOP_EINVAL
    assert call(out=A16 + 4) == binding.VITCOP_EINVAL
    assert call(N=0) == binding.VITCOP_OK and call(B=0) == binding.VITCOP_OK


def test_project_and_select_from_sumsq_validation():
    f = lib.vitcop_project
    assert f(A16, 4096, A16, A16, 4096, None, 0, 640, 4096, 4008, None, None, 0, None) == binding.VITCOP_EUNSUPPORTED
    assert f(A16, 4096, A16, A16, 4096, None, 0, 640, 4100, 4096, None, None, 0, None) == binding.VITCOP_EUNSUPPORTED
    assert f(A16, 1024, A16, A16, 4096, None, 0, 640, 4096, 4096, None, None, 0, None) == binding.VITCOP_EINVAL
    assert f(None, 4096, A16, A16, 4096, None, 0, 640, 4096, 4096, None, None, 0, None) == binding.VITCOP_EINVAL
    assert f(A16, 4096, A16, A16, 4096, A16, 8, 640, 4096, 4096, None, None, 0, None) == binding.VITCOP_EINVAL
    assert f(A16, 4096, A16, A16, 4096, None, 0, 0, 4096, 4096, None, None, 0, None) == binding.VITCOP_OK
    assert lib.vitcop_project_sumsq_parts(4096) == 32 and lib.vitcop_project_sumsq_parts(512) == 4
    # scratch of the few-row path: two fp32 partial tiles of 128 columns per workgroup
    assert lib.vitcop_project_workspace_bytes(128, 4096, 4096) == 2 * 256 * 128 * 128 * 4
    assert lib.vitcop_project_workspace_bytes(640, 4096, 4096) == 2 * 640 * 4096 * 4      # split-K: 4 x 32 tiles, 2 slices
    assert lib.vitcop_project_workspace_bytes(317, 4096, 4096) == 4 * 317 * 4096 * 4      # 2 x 32 tiles, 4 slices
    # 3 x 86 tiles of 256 x 256: the last column tile goes out on its own, in 16 slices
    assert lib.vitcop_project_workspace_bytes(640, 22016, 4096) == 16 * 640 * 256 * 4
    assert lib.vitcop_project_workspace_bytes(1536, 8192, 4096) == 0                       # 256 tiles: one whole round
    assert lib.vitcop_project_workspace_bytes(2000, 4096, 4096) == 0
    assert lib.vitcop_project_workspace_bytes(128, 4096, 96) == 0
    assert f(A16, 4096, A16, A16, 4096, None, 0, 128, 4096, 4096, None, A16 + 4, 1 << 30, None) == binding.VITCOP_EINVAL
    s = lib.vitcop_select_from_sumsq
    assert s(A16, 32, 640, 1, 640, 35, 576, 600, None, A16, None) == binding.VITCOP_EINVAL
    assert s(A16, 32, 100, 1, 640, 35, 576, 64, None, A16, None) == binding.VITCOP_EINVAL   # stride < B*T
    assert s(None, 32, 640, 1, 640, 35, 576, 64, None, A16, None) == binding.VITCOP_EINVAL
    assert s(A16, 0, 640, 1, 640, 35, 576, 64, None, A16, None) == binding.VITCOP_EINVAL


def layer_desc(**kw):
    base = dict(B=1, T=640, D=4096, Hq=32, Hkv=32, d=128, vis_start=35, n_vis=576, keep=64, residual=0,
                x=A16, wq=A16, wk=A16, wv=A16, wo=A16, y=A16, keep_idx=None, norms=None,
                positions_in=None, positions_out=None, ev_kproj_begin=None, ev_kproj_end=None)
    base.update(kw)
    return binding.LayerT(**base)


def test_layer_validation_and_workspace():
    ws = lib.vitcop_layer_workspace_bytes
    run = lib.vitcop_layer_prefill
    good = layer_desc()
    need = ws(C.byref(good))
    # K of all tokens + partials + survivors' x/K/Q/V/O
    assert need >= 640 * 4096 * 2 + 32 * 640 * 4 + 128 * 4096 * 2 * 5
    assert run(C.byref(good), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    assert run(C.byref(good), None, need, None) == binding.VITCOP_EWORKSPACE
    for bad in (layer_desc(keep=600), layer_desc(Hq=30), layer_desc(vis_start=100),
                layer_desc(x=None), layer_desc(positions_out=A16)):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    assert ws(C.byref(layer_desc(d=64, Hq=64, Hkv=64))) > 0
    assert ws(C.byref(layer_desc(d=96))) == 0
    assert run(C.byref(layer_desc(d=96)), A16, 1 << 40, None) == binding.VITCOP_EUNSUPPORTED
    assert run(C.byref(layer_desc(D=4100)), A16, 1 << 40, None) == binding.VITCOP_EUNSUPPORTED


def test_schedule_validation():
    n_layers = 4
    w = (C.c_void_p * n_layers)(*[A16] * n_layers)

    def desc(layers, keeps, **kw):
        pl = (C.c_int * max(1, len(layers)))(*layers)
        pk = (C.c_int * max(1, len(keeps)))(*keeps)
        base = dict(B=1, T=640, D=4096, Hq=32, Hkv=32, d=128, vis_start=35, n_vis=576,
                    n_layers=n_layers, n_stages=len(layers), prune_layer=pl, prune_keep=pk, x=A16,
                    wq=w, wk=w, wv=w, wo=w, y_out=A16, positions_out=None)
        base.update(kw)
        d = binding.ScheduleT(**base)
        d._keep = (pl, pk)
        return d

    run = lib.vitcop_schedule_prefill
    good = desc([1, 2], [192, 64])
    need = lib.vitcop_schedule_workspace_bytes(C.byref(good))
    assert need > 2 * 640 * 4096 * 2
    assert run(C.byref(good), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    assert run(C.byref(desc([2, 1], [192, 64])), A16, 1 << 40, None) == binding.VITCOP_EINVAL   # not ascending
    assert run(C.byref(desc([1, 2], [64, 192])), A16, 1 << 40, None) == binding.VITCOP_EINVAL   # budget grows
    assert run(C.byref(desc([1, 4], [192, 64])), A16, 1 << 40, None) == binding.VITCOP_EINVAL   # layer out of range
    assert run(C.byref(desc([1], [600])), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    assert run(C.byref(desc([1], [64], x=None)), A16, 1 << 40, None) == binding.VITCOP_EINVAL


def test_vic_validation():
    f = lib.vitcop_vic_cluster
    wsb = lib.vitcop_vic_cluster_workspace_bytes

    def call(feats=A16, rs=1024, bs=288 * 1024, pos=A16, B=1, n=288, D=1024, d_c=8.0, tau=0.6, nc=29,
             labels=A16, ncl=A16, ws=A16, ws_bytes=1 << 30):
        return f(feats, rs, bs, pos, B, n, D, d_c, tau, nc, labels, ncl, None, None, None, None, ws, ws_bytes, None)

    need = wsb(1, 288, 1024)
    assert need >= 288 * 288 * 4 + 5 * 288 * 4
    assert call(ws_bytes=need - 1) == binding.VITCOP_EWORKSPACE
    assert call(ws=None) == binding.VITCOP_EWORKSPACE
    assert call(n=8193, bs=8193 * 1024) == binding.VITCOP_EUNSUPPORTED and wsb(1, 8193, 1024) == 0
    assert call(D=1000, rs=1000) == binding.VITCOP_EUNSUPPORTED
    assert call(d_c=0.0) == binding.VITCOP_EINVAL
    assert call(tau=-1.0) == binding.VITCOP_EINVAL
    assert call(nc=289) == binding.VITCOP_EINVAL
    assert call(feats=None) == binding.VITCOP_EINVAL
    assert call(rs=1000) == binding.VITCOP_EINVAL
    assert call(feats=A16 + 2) == binding.VITCOP_EINVAL
    assert call(B=0) == binding.VITCOP_OK


def test_collab_validation():
    f = lib.vitcop_collab_prune_merge
    need = lib.vitcop_collab_prune_merge_workspace_bytes(1, 288)
    assert need >= 2 * 288 * 4

    def call(feats=A16, rs=4096, bs=288 * 4096, labels=A16, ncl=A16, norms=A16, B=1, n=288, D=4096, budget=192,
             out=A16, index=A16, n_out=A16, ws=A16, ws_bytes=1 << 20):
        return f(feats, rs, bs, labels, ncl, norms, B, n, D, budget, out, index, n_out, None, ws, ws_bytes, None)

    assert call(ws_bytes=need - 1) == binding.VITCOP_EWORKSPACE
    assert call(n=8193, bs=8193 * 4096) == binding.VITCOP_EUNSUPPORTED
    assert call(D=4100, rs=4104) == binding.VITCOP_EUNSUPPORTED
    assert call(budget=-1) == binding.VITCOP_EINVAL
    assert call(labels=None) == binding.VITCOP_EINVAL
    assert call(out=A16 + 8) == binding.VITCOP_EINVAL
    assert call(rs=4000) == binding.VITCOP_EINVAL
    assert call(B=0) == binding.VITCOP_OK


def test_decoder_validation():
    assert lib.vitcop_rmsnorm(A16, 4096, A16, 1e-5, A16, 4096, 10, 4100, None) == binding.VITCOP_EUNSUPPORTED
    assert lib.vitcop_rmsnorm(A16, 4000, A16, 1e-5, A16, 4096, 10, 4096, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_rmsnorm(None, 4096, A16, 1e-5, A16, 4096, 10, 4096, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_rmsnorm(None, 4096, None, 1e-5, None, 4096, 0, 4096, None) == binding.VITCOP_OK
    assert lib.vitcop_rope(A16, A16, A16, 1, 10, 4, 2, 100, 10000.0, None) == binding.VITCOP_EUNSUPPORTED
    assert lib.vitcop_rope(A16, A16, A16, 1, 10, 4, 2, 128, 1.0, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_rope(A16, A16, None, 1, 10, 4, 2, 128, 10000.0, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_rope(None, None, None, 1, 10, 4, 2, 128, 10000.0, None) == binding.VITCOP_OK
    assert lib.vitcop_silu_mul(A16, A16, A16, 12, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_silu_mul(A16, A16 + 2, A16, 16, None) == binding.VITCOP_EINVAL
    assert lib.vitcop_silu_mul(None, None, None, 0, None) == binding.VITCOP_OK
    assert C.sizeof(binding.DecoderLayerT) == 10 * 4 + 2 * 4 + 15 * 8 + 2 * 8 + 8 + 2 * 8      # caches, capacity (+ padding), per-sample counts

    def desc(**kw):
        base = dict(B=1, T=640, D=4096, Hq=32, Hkv=32, d=128, F=11008, vis_start=35, n_vis=576, keep=64,
                    eps=1e-5, theta=10000.0, h=A16, positions=A16, ln1=A16, ln2=A16, wq=A16, wk=A16, wv=A16,
                    wo=A16, wg=A16, wu=A16, wd=A16, y=A16, keep_idx=None, positions_out=None, norms=None,
                    k_cache=None, v_cache=None, cache_capacity=0)
        base.update(kw)
        return binding.DecoderLayerT(**base)

    ws = lib.vitcop_decoder_layer_workspace_bytes
    run = lib.vitcop_decoder_layer_prefill
    need = ws(C.byref(desc()))
    assert need >= 640 * 4096 * 2 * 2 + 128 * 11008 * 2 * 3
    assert run(C.byref(desc()), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    for bad in (desc(keep=600), desc(Hq=30), desc(theta=0.5), desc(wg=None), desc(positions=None)):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    assert run(C.byref(desc(F=11000)), A16, 1 << 40, None) == binding.VITCOP_EUNSUPPORTED
    assert ws(C.byref(desc(d=96))) == 0


def test_decoder_schedule_validation():
    # padding before the pointers and at the end
    assert C.sizeof(binding.DecoderScheduleT) == 11 * 4 + 2 * 4 + 4 + 15 * 8 + 2 * 8 + 8 + 2 * 8    # + stage records
    ptrs = (C.c_void_p * 4)(*[A16] * 4)

    def desc(layers=(1, 3), keeps=(128, 32), **kw):
        base = dict(B=1, T=640, D=4096, Hq=32, Hkv=32, d=128, F=11008, vis_start=35, n_vis=576, n_layers=4,
                    n_stages=len(layers), eps=1e-5, theta=10000.0,
                    prune_layer=(C.c_int * len(layers))(*layers), prune_keep=(C.c_int * len(keeps))(*keeps),
                    h=A16, positions=A16, y_out=A16, positions_out=None)
        base.update({n: C.cast(ptrs, C.POINTER(C.c_void_p)) for n in binding._DEC_WEIGHTS})
        base.update(kw)
        return binding.DecoderScheduleT(**base)

    ws = lib.vitcop_decoder_schedule_workspace_bytes
    run = lib.vitcop_decoder_schedule_prefill
    need = ws(C.byref(desc()))
    assert need >= 2 * 640 * 4096 * 2 + 640 * 4096 * 2 * 2
    assert run(C.byref(desc()), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    for bad in (desc(layers=(3, 1)), desc(layers=(1, 4)), desc(keeps=(32, 128)), desc(keeps=(600, 32)),
                desc(n_layers=0), desc(h=None), desc(wq=None), desc(Hq=30)):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    assert ws(C.byref(desc(layers=(3, 1)))) == 0
    assert ws(C.byref(desc(layers=(), keeps=()))) > 0


def test_full_schedule_validation():
    assert C.sizeof(binding.FullScheduleT) == C.sizeof(binding.DecoderScheduleT) + 3 * 4 + 2 * 4 + 4 + 8 * 8
    ptrs = (C.c_void_p * 4)(*[A16] * 4)
    t_final = C.c_int(0)

    def desc(B=1, layers=(3,), keeps=(32,), stage2_layer=1, budget=128, n_centers=20, d_c=8.0, tau=0.6, xy=A16,
             t_ptr=True, **kw):
        base = dict(B=B, T=640, D=4096, Hq=32, Hkv=32, d=128, F=11008, vis_start=35, n_vis=576, n_layers=4,
                    n_stages=len(layers), eps=1e-5, theta=10000.0,
                    prune_layer=(C.c_int * max(len(layers), 1))(*layers),
                    prune_keep=(C.c_int * max(len(keeps), 1))(*keeps),
                    h=A16, positions=A16, y_out=A16, positions_out=None)
        base.update({n: C.cast(ptrs, C.POINTER(C.c_void_p)) for n in binding._DEC_WEIGHTS})
        base.update(kw)
        return binding.FullScheduleT(binding.DecoderScheduleT(**base), stage2_layer, budget, n_centers, d_c, tau, xy,
                                     C.pointer(t_final) if t_ptr else None, None, None, None, None, None, None)

    ws = lib.vitcop_full_schedule_workspace_bytes
    run = lib.vitcop_full_schedule_prefill
    need = ws(C.byref(desc()))
    assert need > lib.vitcop_decoder_schedule_workspace_bytes(C.byref(desc().S)) + 576 * 576 * 4
    assert run(C.byref(desc()), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    assert ws(C.byref(desc(B=2))) > need + 2 * 640 * 4096 * 2                               # a batch needs more
    assert run(C.byref(desc(B=2)), A16, need, None) == binding.VITCOP_EWORKSPACE
    for bad in (desc(stage2_layer=4), desc(stage2_layer=3), desc(budget=600), desc(n_centers=600), desc(d_c=0.0),
                desc(tau=-1.0), desc(xy=None), desc(t_ptr=False), desc(layers=(3, 2), keeps=(32, 16))):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    assert ws(C.byref(desc(stage2_layer=3))) == 0          # Stage III must come after Stage II
    assert ws(C.byref(desc(layers=(), keeps=()))) > 0


def test_decode_validation():
    f = lib.vitcop_decode_attn
    need = lib.vitcop_decode_attn_workspace_bytes(4, 384, 32, 32, 128)
    assert need >= 4 * 32 * 128 * 4

    def call(q=A16, k=A16, v=A16, out=A16, B=4, N=384, Hq=32, Hkv=32, d=128, scale=0.0, ws=A16, ws_bytes=1 << 30):
        return f(q, k, v, out, None, B, N, Hq, Hkv, d, scale, ws, ws_bytes, None)

    assert call(ws_bytes=need - 1) == binding.VITCOP_EWORKSPACE
    assert call(N=0) == binding.VITCOP_EINVAL
    assert call(Hq=30) == binding.VITCOP_EINVAL
    assert call(d=96) == binding.VITCOP_EUNSUPPORTED
    assert call(scale=-1.0) == binding.VITCOP_EINVAL
    assert call(k=None) == binding.VITCOP_EINVAL
    assert call(out=A16 + 4) == binding.VITCOP_EINVAL
    assert call(B=0) == binding.VITCOP_OK
    assert lib.vitcop_decode_attn_workspace_bytes(4, 384, 32, 5, 128) == 0


def test_decoder_decode_validation():
    assert C.sizeof(binding.DecoderDecodeT) == 8 * 4 + 2 * 4 + 15 * 8 + 8       # + per-sample cache lengths
    ptrs = C.cast((C.c_void_p * 3)(*[A16] * 3), C.POINTER(C.c_void_p))

    def desc(n_cached=(352, 317, 115), **kw):
        counts = (C.c_int * 3)(*n_cached) if n_cached else None
        base = dict(B=1, D=4096, Hq=32, Hkv=32, d=128, F=11008, n_layers=3, cache_capacity=640, eps=1e-5,
                    theta=10000.0, n_cached=counts, h=A16, positions=A16, k_cache=ptrs, v_cache=ptrs, y_out=A16)
        base.update({n: ptrs for n in binding._DEC_WEIGHTS})
        base.update(kw)
        return binding.DecoderDecodeT(**base)

    ws = lib.vitcop_decoder_decode_workspace_bytes
    run = lib.vitcop_decoder_decode_step
    need = ws(C.byref(desc()))
    assert need >= 6 * 4096 * 2 + 3 * 11008 * 2
    assert ws(C.byref(desc(B=4))) > need
    assert run(C.byref(desc()), A16, need - 1, None) == binding.VITCOP_EWORKSPACE
    assert run(None, A16, 1 << 40, None) == binding.VITCOP_EINVAL
    for bad in (desc(B=0), desc(n_layers=0), desc(Hq=30), desc(n_cached=(352, 640, 115)), desc(n_cached=(-1, 1, 1)),
                desc(theta=1.0), desc(n_cached=None), desc(h=None), desc(k_cache=None), desc(wq=None)):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EINVAL
    for bad in (desc(d=96), desc(D=4100), desc(F=11000), desc(B=300)):
        assert run(C.byref(bad), A16, 1 << 40, None) == binding.VITCOP_EUNSUPPORTED
    assert ws(C.byref(desc(n_cached=(640, 1, 1)))) == 0        # a full cache has no row for the new token
