"""Seeded synthetic inputs shaped like the paper's image and video workloads.

This module only draws random numbers and lays them out as bf16 bit patterns.
It holds none of the method's arithmetic (no scores, norms, selection or
attention), so both the CPU oracle's tests and the GPU path's tests and bench
may take their inputs from here: the same bits go to both sides.

All tensors are returned as numpy arrays; bf16 tensors are ``uint16`` arrays
holding the bf16 bit pattern (round-to-nearest-even from float32).

Linear weights use the ``[out_features, in_features]`` layout (y = x @ W.T),
so both GEMM operands are contiguous along the contraction index.

Workloads (the paper evaluates LLaVA-1.5 with 576 visual tokens per image,
LLaVA-NeXT with 2880 and LLaVA-NeXT-Video; Sec. 4.1-4.3):

  config 0  LLaVA-1.5-7B-shaped layer: 35 text + 576 visual + 29 text tokens
  config 1  CLIP ViT-L/14-336-shaped encoder output, clustered patches
  config 2  32-layer step-wise schedule, log-normal K-norms with outliers
  config 3  LLaVA-NeXT-7B-shaped high-resolution layer, batch 4
  config 4  video layer with grouped-query attention, AR(1) frames
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# bf16 bit helpers (storage format only)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit pattern -> float32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def seed_for(config: int, trial: int = 0) -> int:
    return 1000 * int(config) + 17 * int(trial)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    # one independent PCG64 stream per tensor, so shapes can change without
    # shifting the values of the other tensors
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def normal_bf16(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    x = _rng(seed, stream).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return f32_to_bf16_bits(x)


# --------------------------------------------------------------------------
# LLM-layer workloads (configs 0, 2, 3 and the LLM side of 4)
# --------------------------------------------------------------------------


def layer_inputs(seed: int, B: int, T: int, D: int, Hq: int, Hkv: int, d: int,
                 vis_start: int, n_vis: int, w_std: float = 0.02,
                 row_gain: np.ndarray | None = None) -> dict:
    """Hidden states X[B,T,D] ~ N(0,1) and Q/K/V/O weights ~ N(0, w_std).

    ``row_gain`` (optional, [B, n_vis] float32) scales the visual rows of X,
    which scales the K-vector norm of those tokens by the same factor.
    """
    x = _rng(seed, 0).standard_normal((B, T, D), dtype=np.float32)
    if row_gain is not None:
        x[:, vis_start:vis_start + n_vis, :] *= row_gain[:, :, None].astype(np.float32)
    out = {
        "B": B, "T": T, "D": D, "Hq": Hq, "Hkv": Hkv, "d": d,
        "vis_start": vis_start, "n_vis": n_vis,
        "x": f32_to_bf16_bits(x),
        "wq": normal_bf16(seed, 1, (Hq * d, D), w_std),
        "wk": normal_bf16(seed, 2, (Hkv * d, D), w_std),
        "wv": normal_bf16(seed, 3, (Hkv * d, D), w_std),
        "wo": normal_bf16(seed, 4, (D, Hq * d), w_std),
    }
    return out


def config0(trial: int = 0) -> dict:
    """LLaVA-1.5-7B-shaped decoder layer, batch 1, keep 64 of 576."""
    c = layer_inputs(seed_for(0, trial), B=1, T=640, D=4096, Hq=32, Hkv=32, d=128,
                     vis_start=35, n_vis=576)
    c["keep"] = 64
    return c


def lognormal_gains(seed: int, B: int, n_vis: int, sigma: float = 0.5,
                    outlier_frac: float = 0.05, outlier_gain: float = 4.0):
    """Per-token gains exp(sigma z), times outlier_gain on a seeded subset.

    Returns (gain [B,n_vis] float32, outlier mask [B,n_vis] bool).
    """
    g = _rng(seed, 10)
    z = g.standard_normal((B, n_vis), dtype=np.float32)
    gain = np.exp(np.float32(sigma) * z).astype(np.float32)
    n_out = int(round(outlier_frac * n_vis))
    mask = np.zeros((B, n_vis), dtype=bool)
    for b in range(B):
        mask[b, g.permutation(n_vis)[:n_out]] = True
    gain = np.where(mask, gain * np.float32(outlier_gain), gain).astype(np.float32)
    return gain, mask


# step-wise schedule of config 2: (layer index, visual budget entering that layer)
CONFIG2_SCHEDULE = ((2, 192), (8, 128), (16, 64))
CONFIG2_LAYERS = 32


def config2_hidden(trial: int = 0, T: int = 640, D: int = 4096,
                   vis_start: int = 35, n_vis: int = 576) -> dict:
    """Hidden states of config 2: visual rows scaled to log-normal norms."""
    seed = seed_for(2, trial)
    gain, mask = lognormal_gains(seed, 1, n_vis)
    x = _rng(seed, 0).standard_normal((1, T, D), dtype=np.float32)
    x[:, vis_start:vis_start + n_vis, :] *= gain[:, :, None]
    return {"B": 1, "T": T, "D": D, "Hq": 32, "Hkv": 32, "d": 128,
            "vis_start": vis_start, "n_vis": n_vis,
            "x": f32_to_bf16_bits(x), "gain": gain, "outlier": mask}


def config2_layer_weights(layer: int, trial: int = 0, D: int = 4096, Hq: int = 32,
                          Hkv: int = 32, d: int = 128, w_std: float = 0.02) -> dict:
    """Independent seeded Q/K/V/O weights of one layer of the schedule."""
    seed = seed_for(2, trial) + 100003 * (layer + 1)
    return {
        "wq": normal_bf16(seed, 1, (Hq * d, D), w_std),
        "wk": normal_bf16(seed, 2, (Hkv * d, D), w_std),
        "wv": normal_bf16(seed, 3, (Hkv * d, D), w_std),
        "wo": normal_bf16(seed, 4, (D, Hq * d), w_std),
    }


CONFIG3_KEEPS = (720, 320, 160)


def config3(trial: int = 0, B: int = 4) -> dict:
    """LLaVA-NeXT-7B-shaped layer: 2880 visual tokens first, then 64 text."""
    c = layer_inputs(seed_for(3, trial), B=B, T=2944, D=4096, Hq=32, Hkv=32, d=128,
                     vis_start=0, n_vis=2880)
    c["keeps"] = CONFIG3_KEEPS
    return c


# --------------------------------------------------------------------------
# Vision-encoder workloads (config 1 and the vision side of config 4)
# --------------------------------------------------------------------------


def _encoder_qk(seed: int, feats: np.ndarray, H: int, d: int):
    """Untimed stand-in for the scoring layer's Q/K projections.

    feats: [B, N+1, C] float32 (row 0 = CLS).  Returns bf16 bits of
    q_cls [B,H,d] and k [B,N+1,H,d].  Weights ~ N(0, 1/sqrt(C)) so that q and
    k have about unit variance.
    """
    B, N1, C = feats.shape
    std = 1.0 / np.sqrt(C)
    wq = _rng(seed, 21).standard_normal((C, H * d), dtype=np.float32) * np.float32(std)
    wk = _rng(seed, 22).standard_normal((C, H * d), dtype=np.float32) * np.float32(std)
    q_cls = feats[:, 0, :] @ wq
    k = feats.reshape(B * N1, C) @ wk
    return (f32_to_bf16_bits(q_cls.reshape(B, H, d)),
            f32_to_bf16_bits(k.reshape(B, N1, H, d)))


def config1(trial: int = 0, B: int = 8, N: int = 576, C: int = 1024, H: int = 16,
            d: int = 64, n_centroids: int = 64, noise: float = 0.1,
            keep: int | None = None) -> dict:
    """CLIP ViT-L/14-336-shaped encoder output with near-duplicate patches."""
    seed = seed_for(1, trial)
    g = _rng(seed, 0)
    feats = np.empty((B, N + 1, C), dtype=np.float32)
    assign = np.empty((B, N), dtype=np.int64)
    for b in range(B):
        cent = g.standard_normal((n_centroids, C), dtype=np.float32)
        a = g.integers(0, n_centroids, size=N)
        assign[b] = a
        feats[b, 1:] = cent[a] + np.float32(noise) * g.standard_normal((N, C), dtype=np.float32)
        feats[b, 0] = g.standard_normal(C, dtype=np.float32)
    q_cls, k = _encoder_qk(seed, feats, H, d)
    return {"B": B, "N": N, "C": C, "H": H, "d": d,
            "keep": (N // 2 if keep is None else keep),
            "feats": f32_to_bf16_bits(feats), "q_cls": q_cls, "k": k,
            "assign": assign}


def config4_frames(trial: int = 0, n_frames: int = 32, N: int = 196, C: int = 1024,
                   H: int = 16, d: int = 64, rho: float = 0.95) -> dict:
    """Vision side of the video workload: AR(1) drifting frame features."""
    seed = seed_for(4, trial)
    g = _rng(seed, 0)
    feats = np.empty((n_frames, N + 1, C), dtype=np.float32)
    cur = g.standard_normal((N, C), dtype=np.float32)
    innov = np.float32(np.sqrt(1.0 - rho * rho))
    for t in range(n_frames):
        if t > 0:
            cur = np.float32(rho) * cur + innov * g.standard_normal((N, C), dtype=np.float32)
        feats[t, 1:] = cur
        feats[t, 0] = cur.mean(axis=0) + np.float32(0.1) * g.standard_normal(C, dtype=np.float32)
    q_cls, k = _encoder_qk(seed, feats, H, d)
    return {"B": n_frames, "N": N, "C": C, "H": H, "d": d, "keep": int(N * 0.30),
            "feats": f32_to_bf16_bits(feats), "q_cls": q_cls, "k": k}


def config4_layer(trial: int = 0, n_vis: int = 6272, n_text: int = 128, D: int = 3584,
                  Hq: int = 28, Hkv: int = 4, d: int = 128,
                  vis_feats: np.ndarray | None = None) -> dict:
    """LLM side of the video workload (Qwen2-7B-style GQA 28/4, d 128).

    ``vis_feats`` ([n_vis, C] float32, e.g. the frame features that survive the
    filter) is mapped to the hidden width by a seeded random matrix standing in
    for the projector; without it the visual rows are the full AR(1) frames.
    """
    seed = seed_for(4, trial)
    if vis_feats is None:
        fr = config4_frames(trial)
        vis_feats = bf16_bits_to_f32(fr["feats"][:, 1:, :]).reshape(-1, fr["C"])
    assert vis_feats.shape[0] == n_vis
    C = vis_feats.shape[1]
    P = _rng(seed, 31).standard_normal((C, D), dtype=np.float32) * np.float32(1.0 / np.sqrt(C))
    T = n_vis + n_text
    x = np.empty((1, T, D), dtype=np.float32)
    x[0, :n_vis] = vis_feats.astype(np.float32) @ P
    x[0, n_vis:] = _rng(seed, 32).standard_normal((n_text, D), dtype=np.float32)
    return {
        "B": 1, "T": T, "D": D, "Hq": Hq, "Hkv": Hkv, "d": d,
        "vis_start": 0, "n_vis": n_vis, "keep": int(6272 * 0.1),
        "x": f32_to_bf16_bits(x),
        "wq": normal_bf16(seed, 1, (Hq * d, D), 0.02),
        "wk": normal_bf16(seed, 2, (Hkv * d, D), 0.02),
        "wv": normal_bf16(seed, 3, (Hkv * d, D), 0.02),
        "wo": normal_bf16(seed, 4, (D, Hq * d), 0.02),
    }


# --------------------------------------------------------------------------
# Direct Q/K/V tensors (attention and K-norm kernels in isolation)
# --------------------------------------------------------------------------


def qkv_tensors(seed: int, B: int, N: int, Hq: int, Hkv: int, d: int, std: float = 1.0) -> dict:
    return {"q": normal_bf16(seed, 41, (B, N, Hq, d), std),
            "k": normal_bf16(seed, 42, (B, N, Hkv, d), std),
            "v": normal_bf16(seed, 43, (B, N, Hkv, d), std)}


def k_tensor_lognormal(seed: int, B: int, T: int, Hkv: int, d: int, vis_start: int,
                       n_vis: int, sigma: float = 0.5) -> dict:
    """K[B,T,Hkv,d] ~ N(0,1) with visual rows scaled by log-normal gains + outliers."""
    gain, mask = lognormal_gains(seed, B, n_vis, sigma)
    k = _rng(seed, 42).standard_normal((B, T, Hkv * d), dtype=np.float32)
    k[:, vis_start:vis_start + n_vis, :] *= gain[:, :, None]
    return {"k": f32_to_bf16_bits(k.reshape(B, T, Hkv, d)), "gain": gain, "outlier": mask}


def vic_inputs(seed: int, n: int, D: int, grid: int = 24, n_regions: int = 12,
               noise: float = 0.1) -> dict:
    """Input of Visual Information Clustering (Sec. 3.2.1): the ``n`` patches that survived
    Stage I out of a ``grid`` x ``grid`` image, with features that are piecewise constant
    over spatial regions (the nearest of ``n_regions`` seeded sites) plus N(0, noise^2), and
    their positions as patch centres normalised to [0,1]^2.  With D = 1024 and noise 0.1,
    tokens of one region are about 4.5 apart and regions about 45 (the cutoff d_c is 8).
    Returns feature bits [n, D], pos float32 [n, 2], the region of every token and the
    ascending patch indices that were kept.
    """
    g = _rng(seed, 0)
    keep = np.sort(g.choice(grid * grid, size=n, replace=False))
    rows, cols = keep // grid, keep % grid
    pos = np.stack([(rows + 0.5) / grid, (cols + 0.5) / grid], axis=1).astype(np.float32)
    sites = g.random((n_regions, 2))
    region = np.argmin(((pos[:, None, :].astype(np.float64) - sites[None]) ** 2).sum(-1), axis=1)
    cent = g.standard_normal((n_regions, D), dtype=np.float32)
    feats = cent[region] + np.float32(noise) * g.standard_normal((n, D), dtype=np.float32)
    return {"n": n, "D": D, "feats": f32_to_bf16_bits(feats), "pos": pos,
            "region": region.astype(np.int64), "patch": keep.astype(np.int64)}


def decoder_inputs(seed: int, B: int, T: int, D: int, Hq: int, Hkv: int, d: int, F: int,
                   w_std: float | None = None, row_gain: np.ndarray | None = None,
                   vis_start: int = 0) -> dict:
    """Hidden states and the nine weight tensors of one pre-norm decoder layer (all bf16 bits):
    h [B,T,D] ~ N(0,1) (visual rows optionally scaled by ``row_gain`` [B,n]), norm weights
    ~ N(1, 0.1), projections ~ N(0, w_std) with w_std = 1/sqrt(fan_in) unless given."""
    g = _rng(seed, 0)
    h = g.standard_normal((B, T, D), dtype=np.float32)
    if row_gain is not None:
        n = row_gain.shape[1]
        h[:, vis_start:vis_start + n] *= row_gain[:, :, None].astype(np.float32)

    def lin(stream, out_f, in_f):
        std = w_std if w_std is not None else 1.0 / np.sqrt(in_f)
        return normal_bf16(seed, stream, (out_f, in_f), std)

    w = {"ln1": f32_to_bf16_bits(1.0 + 0.1 * _rng(seed, 1).standard_normal(D, dtype=np.float32)),
         "ln2": f32_to_bf16_bits(1.0 + 0.1 * _rng(seed, 2).standard_normal(D, dtype=np.float32)),
         "wq": lin(3, Hq * d, D), "wk": lin(4, Hkv * d, D), "wv": lin(5, Hkv * d, D),
         "wo": lin(6, D, Hq * d), "wg": lin(7, F, D), "wu": lin(8, F, D), "wd": lin(9, D, F)}
    return {"B": B, "T": T, "D": D, "Hq": Hq, "Hkv": Hkv, "d": d, "F": F, "h": f32_to_bf16_bits(h), "w": w}
