"""Seeded synthetic inputs for the hybrid dense / 2:4 tile linear layer.

This module only *draws inputs*: weights, activations, tile maps and 2:4 keep-masks with the shapes
and value distributions of the workloads the paper measures on (LLaMA / Qwen linear layers with
learned tile maps).  It holds none of the method's arithmetic (no mask merge, no packing, no
product) and is imported by both the GPU-side tests / benchmark and the CPU-oracle tests, so that both
sides see byte-identical inputs.  numpy only; bf16 tensors are uint16 bit patterns.

The learned masks of the paper are not available offline; a magnitude rule (keep the two largest
|w| of every 4 consecutive input features, lower index wins ties) stands in for the learned 2:4
mask, and an exact-count seeded shuffle stands in for the learned tile map.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _rng(seed: int, *tags) -> np.random.Generator:
    h = zlib.crc32(repr(tags).encode())
    return np.random.Generator(np.random.Philox(key=[(0x9A7C4 ^ h) & 0xFFFFFFFF, seed & 0xFFFFFFFF]))


def normal_bf16(seed: int, shape, std: float, *tags) -> np.ndarray:
    """N(0, std^2) drawn in float32, rounded to bf16; returned as uint16 bit patterns."""
    g = _rng(seed, "normal", *tags)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return f32_to_bf16_bits(a)


def n_sparse_tiles(T: int, f: float) -> int:
    """Exact number of 2:4 tiles for fraction f: round-half-up(f * T)."""
    return int(np.floor(f * T + 0.5))


def tile_map(seed: int, Tn: int, Tk: int, f: float, *tags) -> np.ndarray:
    """(Tn, Tk) uint8, 1 = dense tile, 0 = 2:4 tile; exactly n_sparse_tiles(T, f) zeros at shuffled spots."""
    T = Tn * Tk
    ns = n_sparse_tiles(T, f)
    g = _rng(seed, "tile_map", *tags)
    perm = g.permutation(T)
    m = np.ones(T, np.uint8)
    m[perm[:ns]] = 0
    return m.reshape(Tn, Tk)


def mask24_magnitude(W_bits: np.ndarray) -> np.ndarray:
    """(N, K) uint8 keep-mask with exactly two ones per group of 4 consecutive columns: the two
    largest |w| (compared on bf16 bit patterns & 0x7FFF, which is monotone in |w|); on ties the
    lower index is kept."""
    W_bits = np.ascontiguousarray(W_bits, dtype=np.uint16)
    N, K = W_bits.shape
    assert K % 4 == 0
    mag = (W_bits & np.uint16(0x7FFF)).reshape(N, K // 4, 4)
    # rank of element p = number of elements that beat it (larger magnitude, or equal magnitude at a
    # lower index); keep the elements of rank 0 and 1
    keep = np.empty((N, K // 4, 4), np.uint8)
    for p in range(4):
        beaten = np.zeros((N, K // 4), np.uint8)
        for o in range(4):
            if o == p:
                continue
            if o < p:
                beaten += mag[:, :, o] >= mag[:, :, p]
            else:
                beaten += mag[:, :, o] > mag[:, :, p]
        keep[:, :, p] = beaten < 2
    return keep.reshape(N, K)


@dataclass
class Case:
    name: str
    N: int
    K: int
    M: int
    tile: int
    f: float
    seed: int
    X: np.ndarray         # (M, K) bf16 bits, ~N(0, 1)
    W: np.ndarray         # (N, K) bf16 bits, ~N(0, 0.02^2), unmasked
    tile_map: np.ndarray  # (N/tile, K/tile) uint8, 1 = dense
    mask24: np.ndarray    # (N, K) uint8 2:4 keep-mask (meaningful in 2:4 tiles; defined everywhere)


def make_case(name: str, N: int, K: int, M: int, tile: int, f: float, seed: int = 0, with_mask=True) -> Case:
    assert N % tile == 0 and K % tile == 0
    X = normal_bf16(seed, (M, K), 1.0, name, "X", N, K, M)
    W = normal_bf16(seed, (N, K), 0.02, name, "W", N, K)
    tm = tile_map(seed, N // tile, K // tile, f, name, N, K, tile, f)
    m24 = mask24_magnitude(W) if with_mask else None
    return Case(name, N, K, M, tile, f, seed, X, W, tm, m24)


# The five workload configurations (shapes only; inputs are drawn by make_case).
CONFIGS = {
    "tiny": dict(shapes=[(512, 512)], tile=64, fs=[0.5], Ms=[16]),
    "qwen0p5b": dict(shapes=[(896, 896), (4864, 896), (896, 4864)], tile=128, fs=[0.0, 0.5, 1.0], Ms=[1, 64]),
    "llama7b_attn_decode": dict(shapes=[(4096, 4096)], tile=128, fs=[0.0, 0.25, 0.5, 0.75, 1.0], Ms=[1, 4, 16]),
    "llama7b_mlp_prefill": dict(shapes=[(11008, 4096), (4096, 11008)], tile=128, fs=[0.6], Ms=[2048, 4096]),
    "llama13b_stack": dict(shapes=[(5120, 5120)] * 4 + [(13824, 5120)] * 2 + [(5120, 13824)], tile=128,
                           layers=40, fs="U[0,1) per layer", Ms=[1, 512, 4096]),
}


def mask_logits(seed: int, N: int, K: int, tile: int, *tags):
    """Seeded stand-ins for learned mask logits: P_tile (N/tile, K/tile) and P_24 (6, N K / 4), fp32 N(0, 1), with a few
    exact ties, zeros and NaNs planted so that the tie and sign rules are exercised."""
    r = _rng(seed, "logits", N, K, tile, *tags)
    pt = r.standard_normal((N // tile, K // tile)).astype(np.float32)
    p24 = r.standard_normal((6, N * K // 4)).astype(np.float32)
    G = p24.shape[1]
    idx = r.integers(0, G, size=max(4, G // 50))
    p24[2, idx] = p24[4, idx] = np.maximum(p24[:, idx].max(axis=0), 0) + 1.0      # a tie for the maximum
    idx0 = r.integers(0, G, size=max(2, G // 200))
    p24[:, idx0] = 0.0                                                              # all six equal
    p24[r.integers(0, 6, size=3), r.integers(0, G, size=3)] = np.nan
    flat = pt.reshape(-1)
    flat[r.integers(0, flat.size, size=max(1, flat.size // 8))] = 0.0              # zero logit: the sparse class
    flat[r.integers(0, flat.size)] = np.nan
    return pt, p24


def layer_fractions(seed: int, n_layers: int = 40) -> np.ndarray:
    """One 2:4-tile fraction per decoder layer, U[0, 1) (non-uniform allocation across layers)."""
    return _rng(seed, "layer_fractions", n_layers).random(n_layers)


MATRICES = ("q", "k", "v", "o", "gate", "up", "down")


def matrix_fractions(n_layers: int, params, target: float = 0.5) -> np.ndarray:
    """2:4-tile fraction per (decoder layer, matrix), shape (n_layers, 7) in the order of MATRICES: a stand-in for the
    allocation the paper reports for a global sparsity target (Section 5, "Sparsity allocation", and the appendix with
    the per-matrix distributions; the figures' values are not reproduced, only their ordering): over depth the middle
    blocks take most of the sparsity, the first blocks less and the deepest blocks least; inside a block key and
    value stay dense, the output projection is pruned moderately, the query projection the most of the attention
    matrices, and gate / up / down take the bulk.  `params` = weights per matrix in the same order; the fractions are
    scaled so that their parameter-weighted mean is `target` (clipped to [0, 1])."""
    x = (np.arange(n_layers) + 0.5) / n_layers
    depth = np.sin(np.pi * x) * (1.0 - 0.5 * x)
    share = np.array([0.8, 0.0, 0.0, 0.4, 1.2, 1.2, 1.2])
    raw = depth[:, None] * share[None, :]
    w = np.asarray(params, dtype=np.float64)[None, :]
    lo, hi = 0.0, 64.0
    for _ in range(80):                     # bisection on the scale: the clipped mean is monotone in it
        c = 0.5 * (lo + hi)
        mean = float((np.clip(c * raw, 0.0, 1.0) * w).sum() / (w.sum() * n_layers))
        lo, hi = (c, hi) if mean < target else (lo, c)
    return np.clip(0.5 * (lo + hi) * raw, 0.0, 1.0)
