"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method (no quantiser, no product): it
only draws random tensors on the host with numpy, so that the CPU oracle and
the GPU library can be handed bit-identical inputs.  The layer shapes stand in
for the OPT and mixture-of-experts layers the paper measured (section 4.2.2's
micro-benchmarks of the QKV, attention-output and two FFN matrix multiplies;
section 4.3's expert FFNs); no checkpoint or dataset is read.
"""
from __future__ import annotations

import numpy as np

# (K, N) of the four matrix multiplies of an OPT-175B decoder layer
# (hidden 12288, FFN 49152).
OPT175B_LAYERS = {
    "qkv": (12288, 36864),
    "out_proj": (12288, 12288),
    "fc1": (12288, 49152),
    "fc2": (49152, 12288),
}

# Mixture-of-experts FFN used for the grouped product.
MOE = {"experts": 64, "d_model": 4096, "d_ff": 16384, "tokens": 2048, "top_k": 2, "zipf_a": 1.1}

# Heavy-tailed stress layer.
STRESS_LAYER = (8192, 28672)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable float32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    """float32 values of uint16 bf16 bit patterns."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def activations(M: int, K: int, dtype: str, seed: int) -> np.ndarray:
    """A ~ N(0,1).  dtype 'f16' -> float16 array; 'bf16' -> float32 array of bf16 values."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((M, K), dtype=np.float32)
    if dtype == "f16":
        return a.astype(np.float16)
    if dtype == "bf16":
        return round_to_bf16(a)
    raise ValueError("dtype must be 'f16' or 'bf16'")


def weights_gaussian(K: int, N: int, seed: int, sigma: float = 0.02,
                     outlier_prob: float = 0.0, outlier_scale: float = 20.0) -> np.ndarray:
    """W ~ N(0, sigma); a Bernoulli(outlier_prob) mask of entries is multiplied by outlier_scale."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(sigma)
    if outlier_prob > 0.0:
        # draw the outlier positions sparsely instead of a dense Bernoulli mask
        n_out = rng.binomial(K * N, outlier_prob)
        idx = rng.integers(0, K * N, size=n_out)
        flat = w.reshape(-1)
        flat[idx] *= np.float32(outlier_scale)
    return w.astype(np.float16)


def weights_heavy_tail(K: int, N: int, seed: int, nu: float = 3.0, sigma: float = 0.02,
                       col_prob: float = 0.01, col_scale: float = 50.0) -> np.ndarray:
    """W = sigma * Student-t(nu); a Bernoulli(col_prob) subset of columns is scaled by col_scale."""
    rng = np.random.default_rng(seed)
    w = rng.standard_t(nu, size=(K, N)).astype(np.float32)
    w *= np.float32(sigma)
    cols = rng.random(N) < col_prob
    w[:, cols] *= np.float32(col_scale)
    np.clip(w, -65504.0, 65504.0, out=w)
    return w.astype(np.float16)


def zipf_routing(tokens: int, experts: int, top_k: int, a: float, seed: int):
    """Top-k routing with expert popularity p_i ~ i^-a.

    Returns ``(offsets, expert_of_row)``: int32 offsets [experts+1] into the
    expert-sorted row list (tokens*top_k rows), and the expert id of each row.
    """
    rng = np.random.default_rng(seed)
    p = np.arange(1, experts + 1, dtype=np.float64) ** (-a)
    p /= p.sum()
    choice = np.empty((tokens, top_k), dtype=np.int64)
    for t in range(tokens):
        choice[t] = rng.choice(experts, size=top_k, replace=False, p=p)
    flat = np.sort(choice.reshape(-1), kind="stable")
    counts = np.bincount(flat, minlength=experts)
    offsets = np.zeros(experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return offsets, flat.astype(np.int32)


def config1(seed: int = 0):
    """M=4, K=N=1024 toy layer: fp16 A ~ N(0,1), fp16 W ~ N(0,0.02)."""
    return activations(4, 1024, "f16", seed), weights_gaussian(1024, 1024, seed + 1)


def opt175b_weight(layer: str, seed: int = 0, rows=None, cols=None) -> np.ndarray:
    """Weights of one OPT-175B-shaped layer: N(0,0.02) with 0.1 % of entries x20.

    ``rows`` / ``cols`` shrink the matrix (same recipe, smaller K / N) for
    cases the CPU oracle must finish quickly.
    """
    K, N = OPT175B_LAYERS[layer]
    K = rows or K
    N = cols or N
    lseed = seed * 1000 + list(OPT175B_LAYERS).index(layer)
    return weights_gaussian(K, N, lseed, outlier_prob=1e-3)
