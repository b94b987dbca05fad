"""Helpers shared by the GPU parity tests (device transfer and comparison)."""
import numpy as np
import torch

import vitcop_inputs as I
from oracle import vitcop_oracle as O

ATTN_MAX_ABS = 2e-2      # bf16 attention output vs the fp64 oracle (stated tolerance)
ATTN_MEAN_REL = 1e-2
BAND_REL = 1e-3          # relative score gap below which the selection may differ


def dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit pattern -> torch.bfloat16 CUDA tensor (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 CUDA tensor -> uint16 bit pattern."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return I.bf16_bits_to_f32(host_bits(t)).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def _assert_close(got_f64, ref_f64, max_abs, what):
    err = np.abs(got_f64 - ref_f64)
    assert err.max() <= max_abs, f"{what}: max-abs {err.max():.4g} (bound {max_abs:.3g})"
    denom = max(float(np.abs(ref_f64).mean()), 1e-30)
    assert err.mean() / denom <= ATTN_MEAN_REL, f"{what}: mean-rel {err.mean() / denom:.4g}"


def assert_attention_close(got_f64: np.ndarray, ref_f64: np.ndarray, what="", v_scale: float = 1.0,
                           peaked: bool = False):
    """Outputs of the attention entry points (prefill and decoding): the stated tolerance as it is,
    2e-2 max-abs and 1e-2 mean-relative, for V drawn at unit scale (v ~ N(0,1), what the workloads
    and nearly every test use).  Attention is linear in V and both bf16 roundings behind the error
    (of the probabilities and of the output) are relative, so a test that draws V at ``v_scale``
    times the unit scale (the large-logit cases use 3) scales the max-abs bound by the same factor.
    ``peaked``: heavy-tailed projected inputs (log-normal row gains with 4x outliers) whose rows attend
    almost entirely to one outlier key; the output is then that key's value, and its two roundings
    (probability: 2^-9 relative, output: half an ulp) add up to one bf16 ulp of the largest output,
    which the bound is then not allowed to go below."""
    bound = ATTN_MAX_ABS * v_scale
    if peaked:
        bound = max(bound, 2.0 ** (np.floor(np.log2(float(np.abs(ref_f64).max()))) - 7))
    _assert_close(got_f64, ref_f64, bound, what)


def v_scale_of(v_bits) -> float:
    """Scale of a projected V relative to a unit-normal tensor, whose largest entry is about 5."""
    return max(1.0, float(np.abs(I.bf16_bits_to_f32(np.asarray(v_bits))).max()) / 5.0)


def assert_stream_close(got_f64: np.ndarray, ref_f64: np.ndarray, what=""):
    """Projected and residual-stream outputs (a layer's y, a schedule's hidden state, cache rows): the
    same bounds with the max-abs one scaled by max(1, |ref|_inf).  These tensors reach magnitudes of
    20 and more, where one bf16 rounding of the output alone is 0.06, so an absolute 2e-2 cannot hold."""
    _assert_close(got_f64, ref_f64, ATTN_MAX_ABS * max(1.0, float(np.abs(ref_f64).max())), what)


def assert_selection_matches(gpu_idx: np.ndarray, gpu_scores: np.ndarray, ref_scores: np.ndarray,
                             keep: int, largest: bool, what=""):
    """gpu_idx: ascending candidate indices chosen by the GPU for one sample.

    (1) exactly `keep` distinct ascending members;
    (2) bit-exact against the tie rule applied to the GPU's own fp32 scores;
    (3) equal to the oracle's set outside the band of near-ties around the k-th score.
    """
    n = len(ref_scores)
    assert gpu_idx.shape == (keep,), f"{what}: {gpu_idx.shape} vs keep {keep}"
    if keep:
        assert np.all(np.diff(gpu_idx) > 0) and gpu_idx[0] >= 0 and gpu_idx[-1] < n, what
    g32 = np.asarray(gpu_scores, dtype=np.float32)
    key = -g32 if largest else g32
    own = np.sort(np.lexsort((np.arange(n), key))[:keep])
    assert np.array_equal(gpu_idx, own), f"{what}: not the top-k of the GPU's own scores"
    ref = (O.topk_largest if largest else O.topk_smallest)(ref_scores, keep)
    band = O.tie_band(ref_scores, keep, largest, BAND_REL)
    outside = ~band
    a = np.zeros(n, bool); a[gpu_idx] = True
    b = np.zeros(n, bool); b[ref] = True
    assert np.array_equal(a[outside], b[outside]), f"{what}: differs from the oracle outside the tie band"
