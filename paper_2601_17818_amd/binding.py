"""ctypes binding of libvitcop.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/vitcop.h).
Tensors are torch CUDA tensors (PyTorch is used for device memory and streams
only); bf16 tensors may be torch.bfloat16 or 16-bit integer bit patterns.
Calls enqueue on torch's current stream and do not synchronise.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvitcop.so")

VITCOP_OK = 0
VITCOP_EINVAL = -1
VITCOP_EUNSUPPORTED = -2
VITCOP_EWORKSPACE = -3
VITCOP_EHIP = -4
VITCOP_NORMS_PRECOMPUTED = 1
VITCOP_NORMS_SQUARED = 2
VITCOP_MAX_CANDIDATES = 16384

EXPORTS = (
    "vitcop_last_error", "vitcop_version",
    "vitcop_filter_visual_workspace_bytes", "vitcop_filter_visual",
    "vitcop_knorm_select_workspace_bytes", "vitcop_knorm_select",
    "vitcop_compact",
    "vitcop_prefill_attn_workspace_bytes", "vitcop_prefill_attn",
    "vitcop_project_sumsq_parts", "vitcop_project_workspace_bytes", "vitcop_project",
    "vitcop_select_from_sumsq",
    "vitcop_layer_workspace_bytes", "vitcop_layer_prefill",
    "vitcop_schedule_workspace_bytes", "vitcop_schedule_prefill",
    "vitcop_vic_cluster_workspace_bytes", "vitcop_vic_cluster",
    "vitcop_collab_prune_merge_workspace_bytes", "vitcop_collab_prune_merge",
    "vitcop_rmsnorm", "vitcop_rope", "vitcop_silu_mul",
    "vitcop_decoder_layer_workspace_bytes", "vitcop_decoder_layer_prefill",
    "vitcop_decode_attn_workspace_bytes", "vitcop_decode_attn",
    "vitcop_decoder_schedule_workspace_bytes", "vitcop_decoder_schedule_prefill",
    "vitcop_full_schedule_workspace_bytes", "vitcop_full_schedule_prefill",
    "vitcop_decoder_decode_workspace_bytes", "vitcop_decoder_decode_step",
    "vitcop_filter_visual_static",
)


class VitcopError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libvitcop error {code}: {msg}")
        self.code = code


class GatherT(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("row_bytes", C.c_int64),
                ("src_row_stride_bytes", C.c_int64), ("src_batch_stride_bytes", C.c_int64)]


class LayerT(C.Structure):
    _fields_ = [("B", C.c_int), ("T", C.c_int), ("D", C.c_int), ("Hq", C.c_int), ("Hkv", C.c_int),
                ("d", C.c_int), ("vis_start", C.c_int), ("n_vis", C.c_int), ("keep", C.c_int),
                ("residual", C.c_int),
                ("x", C.c_void_p), ("wq", C.c_void_p), ("wk", C.c_void_p), ("wv", C.c_void_p),
                ("wo", C.c_void_p), ("y", C.c_void_p), ("keep_idx", C.c_void_p),
                ("norms", C.c_void_p), ("positions_in", C.c_void_p), ("positions_out", C.c_void_p),
                ("ev_kproj_begin", C.c_void_p), ("ev_kproj_end", C.c_void_p)]


class DecoderLayerT(C.Structure):
    _fields_ = [("B", C.c_int), ("T", C.c_int), ("D", C.c_int), ("Hq", C.c_int), ("Hkv", C.c_int),
                ("d", C.c_int), ("F", C.c_int), ("vis_start", C.c_int), ("n_vis", C.c_int), ("keep", C.c_int),
                ("eps", C.c_float), ("theta", C.c_float),
                ("h", C.c_void_p), ("positions", C.c_void_p), ("ln1", C.c_void_p), ("ln2", C.c_void_p),
                ("wq", C.c_void_p), ("wk", C.c_void_p), ("wv", C.c_void_p), ("wo", C.c_void_p),
                ("wg", C.c_void_p), ("wu", C.c_void_p), ("wd", C.c_void_p), ("y", C.c_void_p),
                ("keep_idx", C.c_void_p), ("positions_out", C.c_void_p), ("norms", C.c_void_p),
                ("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("cache_capacity", C.c_int),
                ("n_vis_samples", C.c_void_p), ("n_vis_samples_out", C.c_void_p)]


_DEC_WEIGHTS = ("ln1", "ln2", "wq", "wk", "wv", "wo", "wg", "wu", "wd")


class DecoderScheduleT(C.Structure):
    _fields_ = ([(n, C.c_int) for n in ("B", "T", "D", "Hq", "Hkv", "d", "F", "vis_start", "n_vis",
                                         "n_layers", "n_stages")] +
                [("eps", C.c_float), ("theta", C.c_float),
                 ("prune_layer", C.POINTER(C.c_int)), ("prune_keep", C.POINTER(C.c_int)),
                 ("h", C.c_void_p), ("positions", C.c_void_p)] +
                [(n, C.POINTER(C.c_void_p)) for n in _DEC_WEIGHTS] +
                [("y_out", C.c_void_p), ("positions_out", C.c_void_p),
                 ("k_cache", C.POINTER(C.c_void_p)), ("v_cache", C.POINTER(C.c_void_p)), ("cache_capacity", C.c_int),
                 ("stage_norms", C.POINTER(C.c_void_p)), ("stage_keep_idx", C.POINTER(C.c_void_p))])


class DecoderDecodeT(C.Structure):
    _fields_ = ([(n, C.c_int) for n in ("B", "D", "Hq", "Hkv", "d", "F", "n_layers", "cache_capacity")] +
                [("eps", C.c_float), ("theta", C.c_float), ("n_cached", C.POINTER(C.c_int)),
                 ("h", C.c_void_p), ("positions", C.c_void_p)] +
                [(n, C.POINTER(C.c_void_p)) for n in _DEC_WEIGHTS] +
                [("k_cache", C.POINTER(C.c_void_p)), ("v_cache", C.POINTER(C.c_void_p)), ("y_out", C.c_void_p),
                 ("n_cached_samples", C.c_void_p)])


class FullScheduleT(C.Structure):
    _fields_ = [("S", DecoderScheduleT), ("stage2_layer", C.c_int), ("stage2_budget", C.c_int),
                ("n_centers", C.c_int), ("d_c", C.c_float), ("tau", C.c_float), ("vis_xy", C.c_void_p),
                ("T_final", C.POINTER(C.c_int)), ("n_stage2", C.POINTER(C.c_int)),
                ("labels", C.c_void_p), ("norms", C.c_void_p), ("out_index", C.c_void_p),
                ("T_final_samples", C.POINTER(C.c_int)), ("cache_len_samples", C.POINTER(C.c_int))]


class ScheduleT(C.Structure):
    _fields_ = [("B", C.c_int), ("T", C.c_int), ("D", C.c_int), ("Hq", C.c_int), ("Hkv", C.c_int),
                ("d", C.c_int), ("vis_start", C.c_int), ("n_vis", C.c_int),
                ("n_layers", C.c_int), ("n_stages", C.c_int),
                ("prune_layer", C.POINTER(C.c_int)), ("prune_keep", C.POINTER(C.c_int)),
                ("x", C.c_void_p),
                ("wq", C.POINTER(C.c_void_p)), ("wk", C.POINTER(C.c_void_p)),
                ("wv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("y_out", C.c_void_p), ("positions_out", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2601_17818_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f32, sz, u32 = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t, C.c_uint
    lib.vitcop_last_error.restype = C.c_char_p
    lib.vitcop_last_error.argtypes = []
    lib.vitcop_version.restype = i32
    lib.vitcop_filter_visual_workspace_bytes.restype = sz
    lib.vitcop_filter_visual_workspace_bytes.argtypes = [i32] * 4
    lib.vitcop_filter_visual.restype = i32
    lib.vitcop_filter_visual.argtypes = [vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.vitcop_filter_visual_static.restype = i32
    lib.vitcop_filter_visual_static.argtypes = [vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp]
    lib.vitcop_knorm_select_workspace_bytes.restype = sz
    lib.vitcop_knorm_select_workspace_bytes.argtypes = [i32, i32]
    lib.vitcop_knorm_select.restype = i32
    lib.vitcop_knorm_select.argtypes = [vp, i64, i64, i32, i32, i32, i32, i32, i32, i32, vp, vp, u32,
                                        vp, sz, vp]
    lib.vitcop_compact.restype = i32
    lib.vitcop_compact.argtypes = [C.POINTER(GatherT), i32, vp, i32, i32, i32, vp]
    lib.vitcop_prefill_attn_workspace_bytes.restype = sz
    lib.vitcop_prefill_attn_workspace_bytes.argtypes = [i32] * 5
    lib.vitcop_prefill_attn.restype = i32
    lib.vitcop_prefill_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, i32, vp, sz, vp]
    lib.vitcop_project_sumsq_parts.restype = i32
    lib.vitcop_project_sumsq_parts.argtypes = [i32]
    lib.vitcop_project.restype = i32
    lib.vitcop_project.argtypes = [vp, i64, vp, vp, i64, vp, i64, i32, i32, i32, vp, vp, sz, vp]
    lib.vitcop_project_workspace_bytes.restype = sz
    lib.vitcop_project_workspace_bytes.argtypes = [i32, i32, i32]
    lib.vitcop_select_from_sumsq.restype = i32
    lib.vitcop_select_from_sumsq.argtypes = [vp, i32, i64, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.vitcop_layer_workspace_bytes.restype = sz
    lib.vitcop_layer_workspace_bytes.argtypes = [C.POINTER(LayerT)]
    lib.vitcop_layer_prefill.restype = i32
    lib.vitcop_layer_prefill.argtypes = [C.POINTER(LayerT), vp, sz, vp]
    lib.vitcop_schedule_workspace_bytes.restype = sz
    lib.vitcop_schedule_workspace_bytes.argtypes = [C.POINTER(ScheduleT)]
    lib.vitcop_schedule_prefill.restype = i32
    lib.vitcop_schedule_prefill.argtypes = [C.POINTER(ScheduleT), vp, sz, vp]
    lib.vitcop_vic_cluster_workspace_bytes.restype = sz
    lib.vitcop_vic_cluster_workspace_bytes.argtypes = [i32, i32, i32]
    lib.vitcop_vic_cluster.restype = i32
    lib.vitcop_vic_cluster.argtypes = [vp, i64, i64, vp, i32, i32, i32, f32, f32, i32, vp, vp, vp, vp, vp, vp,
                                       vp, sz, vp]
    lib.vitcop_collab_prune_merge_workspace_bytes.restype = sz
    lib.vitcop_collab_prune_merge_workspace_bytes.argtypes = [i32, i32]
    lib.vitcop_collab_prune_merge.restype = i32
    lib.vitcop_collab_prune_merge.argtypes = [vp, i64, i64, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.vitcop_rmsnorm.restype = i32
    lib.vitcop_rmsnorm.argtypes = [vp, i64, vp, f32, vp, i64, i32, i32, vp]
    lib.vitcop_rope.restype = i32
    lib.vitcop_rope.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, vp]
    lib.vitcop_silu_mul.restype = i32
    lib.vitcop_silu_mul.argtypes = [vp, vp, vp, i64, vp]
    lib.vitcop_decoder_layer_workspace_bytes.restype = sz
    lib.vitcop_decoder_layer_workspace_bytes.argtypes = [C.POINTER(DecoderLayerT)]
    lib.vitcop_decoder_layer_prefill.restype = i32
    lib.vitcop_decoder_layer_prefill.argtypes = [C.POINTER(DecoderLayerT), vp, sz, vp]
    lib.vitcop_decode_attn_workspace_bytes.restype = sz
    lib.vitcop_decode_attn_workspace_bytes.argtypes = [i32] * 5
    lib.vitcop_decode_attn.restype = i32
    lib.vitcop_decode_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, sz, vp]
    lib.vitcop_decoder_schedule_workspace_bytes.restype = sz
    lib.vitcop_decoder_schedule_workspace_bytes.argtypes = [C.POINTER(DecoderScheduleT)]
    lib.vitcop_decoder_schedule_prefill.restype = i32
    lib.vitcop_decoder_schedule_prefill.argtypes = [C.POINTER(DecoderScheduleT), vp, sz, vp]
    lib.vitcop_full_schedule_workspace_bytes.restype = sz
    lib.vitcop_full_schedule_workspace_bytes.argtypes = [C.POINTER(FullScheduleT)]
    lib.vitcop_full_schedule_prefill.restype = i32
    lib.vitcop_full_schedule_prefill.argtypes = [C.POINTER(FullScheduleT), vp, sz, vp]
    lib.vitcop_decoder_decode_workspace_bytes.restype = sz
    lib.vitcop_decoder_decode_workspace_bytes.argtypes = [C.POINTER(DecoderDecodeT)]
    lib.vitcop_decoder_decode_step.restype = i32
    lib.vitcop_decoder_decode_step.argtypes = [C.POINTER(DecoderDecodeT), vp, sz, vp]
    return lib


lib = _load()


def vitcop_last_error() -> str:
    return lib.vitcop_last_error().decode()


def _check(rc: int) -> None:
    if rc != VITCOP_OK:
        raise VitcopError(rc, vitcop_last_error())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dense(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if t.element_size() != 2:
        raise ValueError(f"{name} must be a 16-bit (bf16) tensor")
    return t


def _ws(nbytes: int, like: torch.Tensor) -> torch.Tensor | None:
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=like.device)


# --------------------------------------------------------------------------


def vitcop_filter_visual(q_cls, k, keep: int, scale: float = 0.0, want_scores: bool = True,
                         out=None):
    """q_cls [B,H,d], k [B,N+1,H,d] -> (scores [B,N] fp32 or None, idx [B,keep] int32).

    ``out`` = (scores, idx, ws) reuses buffers from an earlier call (no allocation).
    """
    _dense(q_cls, "q_cls"); _dense(k, "k")
    B, N1, H, d = k.shape
    N = N1 - 1
    if out is not None:
        scores, idx, ws = out
    else:
        scores = torch.empty((B, N), dtype=torch.float32, device=k.device) if want_scores else None
        idx = torch.empty((B, max(keep, 0)), dtype=torch.int32, device=k.device)
        ws = _ws(lib.vitcop_filter_visual_workspace_bytes(B, N, H, d), k)
    _check(lib.vitcop_filter_visual(_ptr(q_cls), _ptr(k), B, N, H, d, keep, scale, _ptr(scores),
                                    _ptr(idx), _ptr(ws), ws.numel(), _stream()))
    return (scores, idx, ws) if out is not None else (scores, idx)


VITCOP_FILTER_STATIC_MAX_BYTES = 4 << 20


def vitcop_filter_visual_static(q_cls, k, keep: int, scores, idx, scale: float = 0.0) -> None:
    """vitcop_filter_visual without any allocation: ``scores`` [B,N] fp32 (or None) and ``idx`` [B,keep] int32
    are the caller's tensors, the logits go to the library's built-in scratch (B*H*(N+1)*4 bytes at most
    VITCOP_FILTER_STATIC_MAX_BYTES)."""
    _dense(q_cls, "q_cls"); _dense(k, "k")
    B, N1, H, d = k.shape
    _check(lib.vitcop_filter_visual_static(_ptr(q_cls), _ptr(k), B, N1 - 1, H, d, keep, scale, _ptr(scores),
                                           _ptr(idx), _stream()))


def vitcop_knorm_select(k, vis_start: int, n_vis: int, keep: int, *, norms=None, flags: int = 0,
                        k_row_stride: int | None = None, k_batch_stride: int | None = None,
                        shape=None, idx_out=None):
    """k [B,T,Hkv,d] -> (norms [B,n_vis] fp32, keep_idx [B,T'] int32).

    With ``flags & VITCOP_NORMS_PRECOMPUTED`` pass ``norms`` (and ``shape`` =
    (B,T,Hkv,d) when k is None).  Strides default to the dense layout.
    """
    if k is not None:
        B, T, Hkv, d = shape if shape is not None else k.shape
        if not k.is_cuda or k.element_size() != 2:
            raise ValueError("k must be a 16-bit CUDA tensor")
        dev = k.device
    else:
        B, T, Hkv, d = shape
        dev = norms.device
    rs = Hkv * d if k_row_stride is None else k_row_stride
    bs = T * rs if k_batch_stride is None else k_batch_stride
    if norms is None:
        norms = torch.empty((B, n_vis), dtype=torch.float32, device=dev)
    idx = idx_out if idx_out is not None else torch.empty(
        (B, max(T - n_vis + keep, 0)), dtype=torch.int32, device=dev)
    _check(lib.vitcop_knorm_select(_ptr(k), rs, bs, B, T, Hkv, d, vis_start, n_vis, keep,
                                   _ptr(norms), _ptr(idx), flags, None, 0, _stream()))
    return norms, idx


def vitcop_compact(srcs, idx, T_in: int | None = None, outs_in=None):
    """Each src [B,T_in,...] -> dst [B,T_out,...] gathered by idx [B,T_out] (int32)."""
    srcs = list(srcs)
    B, T_out = idx.shape
    arr = (GatherT * max(len(srcs), 1))()
    outs = []
    for i, s in enumerate(srcs):
        if not s.is_cuda or not s.is_contiguous():
            raise ValueError("sources must be contiguous CUDA tensors")
        row_bytes = s[0, 0].numel() * s.element_size() if s.dim() > 2 else s.element_size()
        dst = outs_in[i] if outs_in is not None else torch.empty(
            (B, T_out) + tuple(s.shape[2:]), dtype=s.dtype, device=s.device)
        arr[i] = GatherT(s.data_ptr(), dst.data_ptr(), row_bytes, row_bytes, s.shape[1] * row_bytes)
        outs.append(dst)
    t_in = srcs[0].shape[1] if (T_in is None and srcs) else (T_in or 0)
    _check(lib.vitcop_compact(arr, len(srcs), _ptr(idx), B, t_in, T_out, _stream()))
    return outs


def vitcop_prefill_attn(q, k, v, scale: float = 0.0, causal: bool = True, want_lse: bool = False,
                        out=None):
    """q [B,N,Hq,d], k,v [B,N,Hkv,d] -> (out [B,N,Hq,d] same dtype as q, lse [B,Hq,N] or None)."""
    _dense(q, "q"); _dense(k, "k"); _dense(v, "v")
    B, N, Hq, d = q.shape
    Hkv = k.shape[2]
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((B, Hq, N), dtype=torch.float32, device=q.device) if want_lse else None
    _check(lib.vitcop_prefill_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, N, Hq, Hkv, d,
                                   scale, 1 if causal else 0, None, 0, _stream()))
    return out, lse


def vitcop_project_sumsq_parts(N: int) -> int:
    return lib.vitcop_project_sumsq_parts(N)


def vitcop_project(x, w, residual=None, want_sumsq: bool = False, out=None, scratch=True):
    """x [M,K], w [N,K] -> (y [M,N], sumsq_parts [P,M] fp32 or None).

    ``out`` = (y, parts) reuses buffers from an earlier call; ``scratch`` = False withholds the
    workspace, so that a call with few rows also runs on the big tiles; a uint8 tensor of
    vitcop_project_workspace_bytes(M, N, K) or more is used as the workspace instead of a new one.
    """
    _dense(x, "x"); _dense(w, "w")
    M, K = x.shape
    N = w.shape[0]
    if out is not None:
        y, parts = out
    else:
        y = torch.empty((M, N), dtype=x.dtype, device=x.device)
        parts = None
        if want_sumsq:
            parts = torch.empty((vitcop_project_sumsq_parts(N), M), dtype=torch.float32, device=x.device)
    if residual is not None:
        _dense(residual, "residual")
    nb = lib.vitcop_project_workspace_bytes(M, N, K) if scratch is not False else 0
    if isinstance(scratch, torch.Tensor) and scratch.numel() >= nb:
        ws = scratch
    else:
        ws = _ws(nb, x) if nb else None
    _check(lib.vitcop_project(_ptr(x), K, _ptr(w), _ptr(y), N, _ptr(residual), N, M, N, K,
                              _ptr(parts), _ptr(ws), nb, _stream()))
    return y, parts


def vitcop_select_from_sumsq(parts, B: int, T: int, vis_start: int, n_vis: int, keep: int, out=None):
    """parts [P, B*T] fp32 -> (norms [B,n_vis], keep_idx [B,T'])."""
    P = parts.shape[0]
    if out is not None:
        norms, idx = out
    else:
        norms = torch.empty((B, n_vis), dtype=torch.float32, device=parts.device)
        idx = torch.empty((B, T - n_vis + keep), dtype=torch.int32, device=parts.device)
    _check(lib.vitcop_select_from_sumsq(_ptr(parts), P, parts.shape[1], B, T, vis_start, n_vis, keep,
                                        _ptr(norms), _ptr(idx), _stream()))
    return norms, idx


def vitcop_vic_cluster(feats, pos, d_c: float, tau: float, n_centers: int, want_dist: bool = False):
    """feats [B,n,D] bf16, pos [B,n,2] fp32 -> dict(labels [B,n], n_clusters [B], rho, delta, parent
    [B,n], and with ``want_dist`` the distance matrix [B,n,n4], n4 = n rounded up to 4)."""
    _dense(feats, "feats")
    B, n, D = feats.shape
    if not (pos.is_cuda and pos.is_contiguous() and pos.dtype == torch.float32 and tuple(pos.shape) == (B, n, 2)):
        raise ValueError("pos must be a contiguous CUDA float32 tensor [B,n,2]")
    dev = feats.device
    labels = torch.empty((B, n), dtype=torch.int32, device=dev)
    n_clusters = torch.empty((B,), dtype=torch.int32, device=dev)
    rho = torch.empty((B, n), dtype=torch.float32, device=dev)
    delta = torch.empty((B, n), dtype=torch.float32, device=dev)
    parent = torch.empty((B, n), dtype=torch.int32, device=dev)
    dist = torch.empty((B, n, (n + 3) // 4 * 4), dtype=torch.float32, device=dev) if want_dist else None
    need = lib.vitcop_vic_cluster_workspace_bytes(B, n, D)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
    _check(lib.vitcop_vic_cluster(_ptr(feats), D, n * D, _ptr(pos), B, n, D, d_c, tau, n_centers, _ptr(labels),
                                  _ptr(n_clusters), _ptr(rho), _ptr(delta), _ptr(parent), _ptr(dist), _ptr(ws),
                                  need, _stream()))
    return {"labels": labels, "n_clusters": n_clusters, "rho": rho, "delta": delta, "parent": parent,
            "dist": dist}


def vitcop_collab_prune_merge(feats, labels, n_clusters, k_norms, budget: int):
    """feats [B,n,D] bf16, labels [B,n] int32, n_clusters [B] int32, k_norms [B,n] fp32 ->
    dict(feats [B,n,D] (rows below n_out valid), index [B,n], n_out [B], assign [B,n])."""
    _dense(feats, "feats")
    B, n, D = feats.shape
    dev = feats.device
    out = torch.empty_like(feats)
    index = torch.empty((B, n), dtype=torch.int32, device=dev)
    n_out = torch.empty((B,), dtype=torch.int32, device=dev)
    assign = torch.empty((B, n), dtype=torch.int32, device=dev)
    need = lib.vitcop_collab_prune_merge_workspace_bytes(B, n)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
    _check(lib.vitcop_collab_prune_merge(_ptr(feats), D, n * D, _ptr(labels), _ptr(n_clusters), _ptr(k_norms),
                                         B, n, D, budget, _ptr(out), _ptr(index), _ptr(n_out), _ptr(assign),
                                         _ptr(ws), need, _stream()))
    return {"feats": out, "index": index, "n_out": n_out, "assign": assign}


def vitcop_rmsnorm(x, weight, eps: float = 1e-5):
    """x [M,D] bf16, weight [D] bf16 -> y [M,D]."""
    _dense(x, "x"); _dense(weight, "weight")
    M, D = x.shape
    y = torch.empty_like(x)
    _check(lib.vitcop_rmsnorm(_ptr(x), D, _ptr(weight), eps, _ptr(y), D, M, D, _stream()))
    return y


def vitcop_rope(q, k, positions, theta: float = 10000.0):
    """In place on q [B,N,Hq,d] and k [B,N,Hkv,d] (either may be None) with positions [B,N] int32."""
    t = q if q is not None else k
    B, N, _, d = t.shape
    Hq = q.shape[2] if q is not None else 0
    Hkv = k.shape[2] if k is not None else 0
    _check(lib.vitcop_rope(_ptr(q), _ptr(k), _ptr(positions), B, N, Hq, Hkv, d, theta, _stream()))
    return q, k


def vitcop_silu_mul(gate, up):
    _dense(gate, "gate"); _dense(up, "up")
    out = torch.empty_like(gate)
    _check(lib.vitcop_silu_mul(_ptr(gate), _ptr(up), _ptr(out), gate.numel(), _stream()))
    return out


def vitcop_decode_attn(q, k, v, scale: float = 0.0, want_lse: bool = True, out=None):
    """q [B,Hq,d], k, v [B,N,Hkv,d] -> (out [B,Hq,d], lse [B,Hq] or None).  ``out`` = (out, lse, ws) reuses buffers."""
    _dense(q, "q"); _dense(k, "k"); _dense(v, "v")
    B, Hq, d = q.shape
    N, Hkv = k.shape[1], k.shape[2]
    if out is not None:
        o, lse, ws = out
    else:
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device) if want_lse else None
        ws = _ws(max(lib.vitcop_decode_attn_workspace_bytes(B, N, Hq, Hkv, d), 16), q)
    _check(lib.vitcop_decode_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, N, Hq, Hkv, d, scale,
                                  _ptr(ws), ws.numel(), _stream()))
    return (o, lse, ws) if out is not None else (o, lse)


class DecoderLayerPlan:
    """Pre-marshalled vitcop_decoder_layer_prefill call.  ``w``: dict of device tensors ln1, ln2, wq, wk, wv,
    wo, wg, wu, wd."""

    def __init__(self, h, positions, w: dict, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int, keep: int,
                 eps: float = 1e-5, theta: float = 10000.0, caches=None, n_vis_samples=None):
        """``caches`` = (k_cache, v_cache) [B, capacity, Hkv, d]: the layer writes its KV cache there.
        ``n_vis_samples``: int32 device tensor [B] for a right-padded batch (sample b has that many of the
        n_vis visual tokens, its text follows them, the rest of its rows is padding); ``n_vis_out`` then holds
        the counts after the layer."""
        B, T, D = h.shape
        F = w["wg"].shape[0]
        Tp = T - n_vis + keep
        dev = h.device
        self.tensors = (h, positions, w, caches, n_vis_samples)
        self.n_vis_out = torch.empty((B,), dtype=torch.int32, device=dev) if n_vis_samples is not None else None
        kc, vc = caches if caches is not None else (None, None)
        self.y = torch.empty((B, Tp, D), dtype=h.dtype, device=dev)
        self.keep_idx = torch.empty((B, Tp), dtype=torch.int32, device=dev)
        self.positions_out = torch.empty((B, Tp), dtype=torch.int32, device=dev)
        self.norms = torch.empty((B, n_vis), dtype=torch.float32, device=dev)
        self.desc = DecoderLayerT(B, T, D, Hq, Hkv, d, F, vis_start, n_vis, keep, eps, theta, _ptr(h),
                                  _ptr(positions), _ptr(w["ln1"]), _ptr(w["ln2"]), _ptr(w["wq"]), _ptr(w["wk"]),
                                  _ptr(w["wv"]), _ptr(w["wo"]), _ptr(w["wg"]), _ptr(w["wu"]), _ptr(w["wd"]),
                                  _ptr(self.y), _ptr(self.keep_idx), _ptr(self.positions_out), _ptr(self.norms),
                                  _ptr(kc), _ptr(vc), kc.shape[1] if kc is not None else 0, _ptr(n_vis_samples),
                                  _ptr(self.n_vis_out))
        nb = lib.vitcop_decoder_layer_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, h)

    def run(self):
        _check(lib.vitcop_decoder_layer_prefill(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        return self.y


def vitcop_decoder_layer_prefill(h, positions, w, Hq, Hkv, d, vis_start, n_vis, keep, eps=1e-5, theta=10000.0,
                                 caches=None):
    """One full decoder layer with pruning on entry.  Returns dict(y, keep_idx, positions, norms)."""
    plan = DecoderLayerPlan(h, positions, w, Hq, Hkv, d, vis_start, n_vis, keep, eps, theta, caches)
    plan.run()
    return {"y": plan.y, "keep_idx": plan.keep_idx, "positions": plan.positions_out, "norms": plan.norms}


class LayerPlan:
    """Pre-marshalled vitcop_layer_prefill call (descriptor, outputs and workspace
    are created once; ``run`` only enqueues)."""

    def __init__(self, x, wq, wk, wv, wo, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int,
                 keep: int, residual: bool = False, want_idx: bool = True, want_norms: bool = True,
                 positions=None):
        B, T, D = x.shape
        Tp = T - n_vis + keep
        dev = x.device
        self.tensors = (x, wq, wk, wv, wo, positions)
        self.y = torch.empty((B, Tp, D), dtype=x.dtype, device=dev)
        self.keep_idx = torch.empty((B, Tp), dtype=torch.int32, device=dev) if want_idx else None
        self.norms = torch.empty((B, n_vis), dtype=torch.float32, device=dev) if want_norms else None
        self.positions_out = (torch.empty((B, Tp), dtype=torch.int32, device=dev)
                              if positions is not None else None)
        self.desc = LayerT(B, T, D, Hq, Hkv, d, vis_start, n_vis, keep, 1 if residual else 0,
                           _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo), _ptr(self.y),
                           _ptr(self.keep_idx), _ptr(self.norms), _ptr(positions),
                           _ptr(self.positions_out))
        nb = lib.vitcop_layer_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, x)

    def run(self, kproj_events=None):
        """``kproj_events`` = (begin, end): two torch.cuda.Event objects that have been recorded once
        (so that their handles exist); the library records them around the K projection."""
        if kproj_events is not None:
            self.desc.ev_kproj_begin = kproj_events[0].cuda_event
            self.desc.ev_kproj_end = kproj_events[1].cuda_event
        else:
            self.desc.ev_kproj_begin = None
            self.desc.ev_kproj_end = None
        _check(lib.vitcop_layer_prefill(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        return self.y


def vitcop_layer_prefill(x, wq, wk, wv, wo, Hq, Hkv, d, vis_start, n_vis, keep, residual=False,
                         positions=None):
    """One pruned attention layer.  Returns dict(y, keep_idx, norms, positions)."""
    plan = LayerPlan(x, wq, wk, wv, wo, Hq, Hkv, d, vis_start, n_vis, keep, residual,
                     positions=positions)
    plan.run()
    return {"y": plan.y, "keep_idx": plan.keep_idx, "norms": plan.norms,
            "positions": plan.positions_out}


def _cache_arrays(caches, n_layers: int):
    """(k pointer array, v pointer array, capacity) for a list of per-layer (k_cache, v_cache), or nulls."""
    if caches is None:
        return None, None, 0
    assert len(caches) == n_layers
    kc = (C.c_void_p * n_layers)(*[k.data_ptr() for k, _ in caches])
    vc = (C.c_void_p * n_layers)(*[v.data_ptr() for _, v in caches])
    return kc, vc, caches[0][0].shape[1]


class DecoderDecodePlan:
    """Pre-marshalled vitcop_decoder_decode_step call: one new token per sample through all layers.
    ``caches``: per layer (k_cache, v_cache) [B, capacity, Hkv, d]; ``n_cached``: tokens each layer's cache holds,
    one int per layer, or one list of B ints per layer when the samples' caches differ in length (those go to
    the device as an int32 tensor [n_layers, B], ``n_cached_samples``)."""

    def __init__(self, h, positions, weights, Hq: int, Hkv: int, d: int, caches, n_cached, eps: float = 1e-5,
                 theta: float = 10000.0):
        B, D = h.shape
        n_layers = len(weights)
        F = weights[0]["wg"].shape[0]
        self._kc, self._vc, cap = _cache_arrays(caches, n_layers)
        self.n_cached_samples = None
        if len(n_cached) and hasattr(n_cached[0], "__len__"):
            per = [[int(v) for v in row] for row in n_cached]
            if any(len(row) != B for row in per):
                raise ValueError("n_cached: one entry per sample in every layer")
            self.n_cached_samples = torch.tensor(per, dtype=torch.int32, device=h.device)
            n_cached = [max(row) for row in per]
        self.keepalive = (h, positions, weights, caches, self.n_cached_samples)
        self._n = (C.c_int * n_layers)(*[int(v) for v in n_cached])
        self._w = [(C.c_void_p * n_layers)(*[w[n].data_ptr() for w in weights]) for n in _DEC_WEIGHTS]
        self.y = torch.empty((B, D), dtype=h.dtype, device=h.device)
        self.desc = DecoderDecodeT(B, D, Hq, Hkv, d, F, n_layers, cap, eps, theta, self._n, _ptr(h), _ptr(positions),
                                   *self._w, self._kc, self._vc, _ptr(self.y), _ptr(self.n_cached_samples))
        nb = lib.vitcop_decoder_decode_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, h)

    def run(self):
        _check(lib.vitcop_decoder_decode_step(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        return self.y


class DecoderSchedulePlan:
    """Pre-marshalled vitcop_decoder_schedule_prefill call.  ``weights``: one dict per layer with the device
    tensors ln1, ln2, wq, wk, wv, wo, wg, wu, wd; ``schedule``: ((layer, keep), ...)."""

    def __init__(self, h, positions, weights, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int, schedule,
                 eps: float = 1e-5, theta: float = 10000.0, caches=None):
        """``caches``: per layer (k_cache, v_cache) [B, capacity, Hkv, d], filled by the prefill."""
        B, T, D = h.shape
        n_layers = len(weights)
        F = weights[0]["wg"].shape[0]
        self.keepalive = (h, positions, weights, caches)
        self._kc, self._vc, cap = _cache_arrays(caches, n_layers)
        layers = [int(s[0]) for s in schedule]
        keeps = [int(s[1]) for s in schedule]
        self._pl = (C.c_int * max(len(layers), 1))(*layers)
        self._pk = (C.c_int * max(len(keeps), 1))(*keeps)
        self._w = [(C.c_void_p * n_layers)(*[w[n].data_ptr() for w in weights]) for n in _DEC_WEIGHTS]
        T_final = T - n_vis + (keeps[-1] if keeps else n_vis)
        self.y = torch.empty((B, T_final, D), dtype=h.dtype, device=h.device)
        self.positions = torch.empty((B, T_final), dtype=torch.int32, device=h.device)
        # record of every stage's decision: the norms it ranked and the keep list it took
        present = [n_vis] + keeps[:-1]
        self.stage_norms = [torch.empty((B, n), dtype=torch.float32, device=h.device) for n in present]
        self.stage_keep_idx = [torch.empty((B, T - n_vis + k), dtype=torch.int32, device=h.device) for k in keeps]
        self._sn = (C.c_void_p * max(len(keeps), 1))(*[t.data_ptr() for t in self.stage_norms])
        self._sk = (C.c_void_p * max(len(keeps), 1))(*[t.data_ptr() for t in self.stage_keep_idx])
        self.desc = DecoderScheduleT(B, T, D, Hq, Hkv, d, F, vis_start, n_vis, n_layers, len(layers), eps, theta,
                                     self._pl, self._pk, _ptr(h), _ptr(positions), *self._w, _ptr(self.y),
                                     _ptr(self.positions), self._kc, self._vc, cap, self._sn, self._sk)
        nb = lib.vitcop_decoder_schedule_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, h)

    def run(self):
        _check(lib.vitcop_decoder_schedule_prefill(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        return self.y


class FullSchedulePlan:
    """Pre-marshalled vitcop_full_schedule_prefill call on a batch.  ``stage2``: dict with layer, budget,
    n_centers, d_c, tau and xy (device tensor [B, n_vis, 2] fp32); ``schedule``: the Stage III stages after it.
    ``run`` returns (y [B, T_final, D], positions [B, T_final]), right-padded: sample b's real rows are the
    first T_final_samples[b].  labels [B, n_vis], norms [B, n_vis], out_index [B, max count] and n_stage2 (list)
    hold what Stage II produced; stage_norms[s] [B, present] and stage_keep_idx[s] [B, kept rows] what Stage III
    stage s ranked and kept (padded like the batch); cache_len[l][b] the real rows of layer l's cache."""

    def __init__(self, h, positions, weights, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int, stage2: dict,
                 schedule, eps: float = 1e-5, theta: float = 10000.0, caches=None):
        B, T, D = h.shape
        n_layers = len(weights)
        F = weights[0]["wg"].shape[0]
        xy = stage2["xy"]
        if tuple(xy.shape) != (B, n_vis, 2):
            raise ValueError(f"stage2['xy'] must be [B, n_vis, 2] = {(B, n_vis, 2)}, got {tuple(xy.shape)}")
        self.keepalive = (h, positions, weights, xy, caches)
        self._kc, self._vc, cap = _cache_arrays(caches, n_layers)
        layers = [int(s[0]) for s in schedule]
        keeps = [int(s[1]) for s in schedule]
        self._pl = (C.c_int * max(len(layers), 1))(*layers)
        self._pk = (C.c_int * max(len(keeps), 1))(*keeps)
        self._w = [(C.c_void_p * n_layers)(*[w[n].data_ptr() for w in weights]) for n in _DEC_WEIGHTS]
        self._y = torch.empty((B * T * D,), dtype=h.dtype, device=h.device)
        self._pos = torch.empty((B * T,), dtype=torch.int32, device=h.device)
        self.labels = torch.empty((B, n_vis), dtype=torch.int32, device=h.device)
        self.norms = torch.empty((B, n_vis), dtype=torch.float32, device=h.device)
        self._out_index = torch.empty((B, n_vis), dtype=torch.int32, device=h.device)
        self._T_final = C.c_int(0)
        self._n2 = (C.c_int * B)()
        self._T_samples = (C.c_int * B)()
        self._cache_len = (C.c_int * (n_layers * B))()
        # record of every Stage III decision (sized for the counts before Stage II, cut in run)
        self._keeps, self._B, self._T, self._D, self._n_vis, self._n_layers = keeps, B, T, D, n_vis, n_layers
        self._stage_norms = [torch.empty((B * n_vis,), dtype=torch.float32, device=h.device) for _ in keeps]
        self._stage_keep_idx = [torch.empty((B * T,), dtype=torch.int32, device=h.device) for _ in keeps]
        self._sn = (C.c_void_p * max(len(keeps), 1))(*[t.data_ptr() for t in self._stage_norms])
        self._sk = (C.c_void_p * max(len(keeps), 1))(*[t.data_ptr() for t in self._stage_keep_idx])
        S = DecoderScheduleT(B, T, D, Hq, Hkv, d, F, vis_start, n_vis, n_layers, len(layers), eps, theta,
                             self._pl, self._pk, _ptr(h), _ptr(positions), *self._w, _ptr(self._y),
                             _ptr(self._pos), self._kc, self._vc, cap, self._sn, self._sk)
        self.desc = FullScheduleT(S, int(stage2["layer"]), int(stage2["budget"]), int(stage2["n_centers"]),
                                  float(stage2["d_c"]), float(stage2["tau"]), _ptr(xy),
                                  C.pointer(self._T_final), self._n2, _ptr(self.labels),
                                  _ptr(self.norms), _ptr(self._out_index), self._T_samples, self._cache_len)
        nb = lib.vitcop_full_schedule_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, h)

    def run(self):
        _check(lib.vitcop_full_schedule_prefill(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        B, T, D = self._B, self._T, self._D
        self.T_final = self._T_final.value
        self.n_stage2 = list(self._n2)
        self.T_final_samples = list(self._T_samples)
        self.cache_len = [[self._cache_len[l * B + b] for b in range(B)] for l in range(self._n_layers)]
        self.out_index = self._out_index[:, : max(self.n_stage2)]
        # stage s ranked the visual tokens present on entry (of the longest sample) and kept min(budget, present)
        present, text = max(self.n_stage2), T - self._n_vis
        self.stage_norms, self.stage_keep_idx = [], []
        for s, budget in enumerate(self._keeps):
            kept = min(budget, present)
            self.stage_norms.append(self._stage_norms[s][: B * present].view(B, present))
            self.stage_keep_idx.append(self._stage_keep_idx[s][: B * (text + kept)].view(B, text + kept))
            present = kept
        Tf = self.T_final
        return self._y[: B * Tf * D].view(B, Tf, D), self._pos[: B * Tf].view(B, Tf)


class SchedulePlan:
    """Pre-marshalled vitcop_schedule_prefill call."""

    def __init__(self, x, weights, Hq: int, Hkv: int, d: int, vis_start: int, n_vis: int, schedule):
        B, T, D = x.shape
        n_layers = len(weights)
        self.keepalive = (x, weights)
        layers = [int(s[0]) for s in schedule]
        keeps = [int(s[1]) for s in schedule]
        self._pl = (C.c_int * max(len(layers), 1))(*layers)
        self._pk = (C.c_int * max(len(keeps), 1))(*keeps)
        self._w = {n: (C.c_void_p * n_layers)(*[w[n].data_ptr() for w in weights])
                   for n in ("wq", "wk", "wv", "wo")}
        T_final = T - n_vis + (keeps[-1] if keeps else n_vis)
        self.y = torch.empty((B, T_final, D), dtype=x.dtype, device=x.device)
        self.positions = torch.empty((B, T_final), dtype=torch.int32, device=x.device)
        self.desc = ScheduleT(B, T, D, Hq, Hkv, d, vis_start, n_vis, n_layers, len(layers),
                              self._pl, self._pk, _ptr(x), self._w["wq"], self._w["wk"],
                              self._w["wv"], self._w["wo"], _ptr(self.y), _ptr(self.positions))
        nb = lib.vitcop_schedule_workspace_bytes(C.byref(self.desc))
        if nb == 0:
            raise VitcopError(VITCOP_EINVAL, vitcop_last_error())
        self.ws = _ws(nb, x)

    def run(self):
        _check(lib.vitcop_schedule_prefill(C.byref(self.desc), _ptr(self.ws), self.ws.numel(), _stream()))
        return self.y


def vitcop_schedule_prefill(x, weights, Hq, Hkv, d, vis_start, n_vis, schedule):
    plan = SchedulePlan(x, weights, Hq, Hkv, d, vis_start, n_vis, schedule)
    plan.run()
    return plan.y, plan.positions
