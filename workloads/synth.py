"""Seeded synthetic weights, activations and thresholds.

The paper evaluates on Llama-2/3 weights and real hidden states (Section 6.1); none of
those exist here, so every tensor is drawn from a distribution with the same shape and a
similar value profile: int4 codes uniform on {-8..7}, fp16 group scales uniform in a
small positive range, and zero-mean heavy-tailed activations (Gaussian, Laplace, or a
SwiGLU-like product), which is roughly what activation-sparsity work reports for hidden
states.  Kept positions are therefore iid - the worst case for locality.

This module only *draws and encodes inputs*.  It contains none of the method's steps.
"""
from __future__ import annotations

import numpy as np

GROUP = 128      # quantization group length along the input (K) dimension
TILE_ROWS = 256  # rows per zigzag tile (the paper's superblock height, Section 4.2.1)

TENSOR_IDS = {"w": 0, "q": 0, "k": 1, "v": 2, "o": 3, "gate": 4, "up": 5, "down": 6}
KIND_WEIGHTS, KIND_X, KIND_CALIB = 0, 50, 90

# (name, M, K, activation distribution) per benchmark configuration.
CONFIG_SHAPES = {
    1: [("w", 512, 1024, "normal")],
    2: [("q", 4096, 4096, "laplace")],
    3: [("gate", 11008, 4096, "laplace"), ("up", 11008, 4096, "laplace"),
        ("down", 4096, 11008, "silu_product")],
    4: [("q", 4096, 4096, "laplace"), ("k", 1024, 4096, "laplace"), ("v", 1024, 4096, "laplace"),
        ("o", 4096, 4096, "laplace"), ("gate", 14336, 4096, "laplace"),
        ("up", 14336, 4096, "laplace"), ("down", 4096, 14336, "laplace")],
    5: [("gate", 28672, 8192, "laplace"), ("up", 28672, 8192, "laplace"),
        ("down", 8192, 28672, "laplace")],
}
# fp16 scale range per configuration
CONFIG_SCALE_RANGE = {1: (0.005, 0.02), 2: (0.005, 0.02), 3: (0.005, 0.02),
                      4: (0.005, 0.02), 5: (0.003, 0.015)}


def seed_for(config: int, layer: int = 0, tensor: str | int = 0, kind: int = KIND_WEIGHTS) -> int:
    """One integer seed per (configuration, layer, tensor, kind of draw)."""
    tid = TENSOR_IDS[tensor] if isinstance(tensor, str) else int(tensor)
    return 0x5B07 * 1_000_000 + int(config) * 10_000 + int(layer) * 100 + tid + int(kind)


def make_weights(M: int, K: int, seed: int, scale_lo: float = 0.005, scale_hi: float = 0.02,
                 group: int = GROUP, want_q: bool = True) -> dict:
    """Row-major group-wise int4 source tensors.

    Returns a dict with
      q          int8  [M, K]       integer codes in [-8, 7] (only if want_q)
      q_rowmajor uint8 [M, K/2]     element (m, k) in byte k//2; even k in the low nibble,
                                    odd k in the high nibble; two's-complement 4-bit
      scales     float16 [M, K/group]
    """
    assert K % 2 == 0 and K % group == 0
    rng = np.random.default_rng(seed)
    q = rng.integers(-8, 8, size=(M, K), dtype=np.int8)
    scales = rng.uniform(scale_lo, scale_hi, size=(M, K // group)).astype(np.float16)
    lo = (q[:, 0::2].view(np.uint8) & 0x0F)
    hi = (q[:, 1::2].view(np.uint8) & 0x0F)
    q_rowmajor = np.ascontiguousarray(lo | (hi << 4)).astype(np.uint8)
    out = {"q_rowmajor": q_rowmajor, "scales": np.ascontiguousarray(scales)}
    if want_q:
        out["q"] = q
    return out


def make_fp_weights(M: int, K: int, seed: int, std: float = 0.02) -> np.ndarray:
    """Full-precision weights for the re-quantizing (column-block) path: fp32 N(0, std^2),
    with every 64th column scaled by 8 so that blocks see a spread of magnitudes."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((M, K)) * std).astype(np.float32)
    w[:, ::64] *= np.float32(8.0)
    return np.ascontiguousarray(w)


def _draw(rng: np.random.Generator, dist: str, shape) -> np.ndarray:
    if dist == "normal":
        v = rng.standard_normal(shape)
    elif dist == "laplace":
        v = rng.laplace(0.0, 1.0, shape)          # location 0, scale b = 1
    elif dist == "silu_product":
        g = rng.standard_normal(shape)
        u = rng.standard_normal(shape)
        v = g / (1.0 + np.exp(-g)) * u            # SiLU(g) * u, a SwiGLU-like hidden state
    elif dist == "laplace_clustered":
        # Laplace with a step envelope along the last axis: the first half of the columns is
        # scaled by 4, the second by 1/4, so at a 50 % threshold about 7 of 8 kept columns sit in
        # the first half - a pattern that starves half the workers of a static column partition.
        v = rng.laplace(0.0, 1.0, shape)
        K = shape[-1]
        v[..., : K // 2] *= 4.0
        v[..., K // 2:] *= 0.25
    else:
        raise ValueError(f"unknown distribution {dist!r}")
    return v


def make_x(K: int, dist: str, seed: int, batch: int = 1) -> np.ndarray:
    """Activations, drawn in fp64 and rounded to fp16; shape [batch, K]."""
    rng = np.random.default_rng(seed)
    return np.ascontiguousarray(_draw(rng, dist, (batch, K)).astype(np.float16))


def quantile_threshold(x: np.ndarray, sparsity: float) -> float:
    """Threshold that drops (about) a fraction `sparsity` of the entries of x.

    It is the element of rank floor(sparsity * n) of sorted |x| (so it is one of the data
    values and fp16-representable); sparsity 0 gives 0.0, which keeps every entry.  With
    ties in fp16 the achieved sparsity can fall slightly under the request.
    """
    a = np.sort(np.abs(x.astype(np.float32)).ravel())
    if sparsity <= 0.0:
        return 0.0
    r = int(np.floor(sparsity * a.size))
    if r >= a.size:
        return float("inf")
    return float(a[r])


def calibrated_threshold(K: int, dist: str, sparsity: float, seed: int, draws: int = 64) -> float:
    """Offline-style calibration: the quantile rule on a separate draw of draws*K samples
    from the same distribution, so run-time sparsity is near the request, not exactly it."""
    rng = np.random.default_rng(seed)
    cal = _draw(rng, dist, (draws * K,)).astype(np.float16)
    return quantile_threshold(cal, sparsity)


def make_case(config: int, tensor: str, layer: int = 0, batch: int = 1, want_q: bool = True) -> dict:
    """Weights + activations for one named tensor of one benchmark configuration."""
    for name, M, K, dist in CONFIG_SHAPES[config]:
        if name == tensor:
            break
    else:
        raise KeyError((config, tensor))
    lo, hi = CONFIG_SCALE_RANGE[config]
    w = make_weights(M, K, seed_for(config, layer, tensor, KIND_WEIGHTS), lo, hi, want_q=want_q)
    w["x"] = make_x(K, dist, seed_for(config, layer, tensor, KIND_X), batch)
    w.update(M=M, K=K, dist=dist, config=config, tensor=tensor, layer=layer)
    return w
