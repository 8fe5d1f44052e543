"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO arithmetic of the method (no scales, codes or MBS words): it only draws
random tensors with numpy's PCG64 generator and rounds them to bf16.  Both the HIP path and the
test oracle are fed the same bytes produced here.  The tensors stand in for the activation and
weight tensors the paper dumps from Llama-3.1-8B / Qwen3-8B inference (Sec. 3.1), which are not
available: LLM layer shapes, heavy-tailed activations with a few outlier channels (Sec. 3.3,
4.3), small Gaussian weights.
"""
from __future__ import annotations

import math

import numpy as np


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def _outlier_columns(rng: np.random.Generator, K: int, count: int) -> np.ndarray:
    return rng.permutation(K)[:count]


def gaussian(rows: int, K: int, std: float, seed: int) -> np.ndarray:
    """Weights ~ N(0, std^2), bf16 bits [rows, K]."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, K), np.uint16)
    step = max(1, (1 << 22) // max(K, 1))
    for r0 in range(0, rows, step):  # chunked so the fp64 draw stays small
        r1 = min(rows, r0 + step)
        out[r0:r1] = to_bf16_bits(rng.standard_normal((r1 - r0, K)) * std)
    return out


def activations_normal(rows: int, K: int, n_outlier_cols: int, factor: float, seed: int) -> np.ndarray:
    """Activations ~ N(0,1) with `n_outlier_cols` seeded columns multiplied by `factor`."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K))
    x[:, _outlier_columns(rng, K, n_outlier_cols)] *= factor
    return to_bf16_bits(x)


def activations_student_t(rows: int, K: int, nu: float, outlier_frac: float, factor: float,
                          seed: int) -> np.ndarray:
    """Activations ~ Student-t(nu), ceil(outlier_frac*K) seeded channels multiplied by `factor`."""
    rng = np.random.default_rng(seed)
    cols = _outlier_columns(rng, K, math.ceil(outlier_frac * K))
    scale = np.ones(K)
    scale[cols] = factor
    out = np.empty((rows, K), np.uint16)
    step = max(1, (1 << 22) // max(K, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = to_bf16_bits(rng.standard_t(nu, (r1 - r0, K)) * scale)
    return out


def zipf_topk_routing(tokens: int, experts: int, top_k: int, exponent: float, seed: int):
    """Route each token to `top_k` distinct experts, P(e) ~ (e+1)^-exponent (Gumbel top-k).

    Returns (row_offsets [experts+1] int64, token_of_row [tokens*top_k] int64): rows grouped by
    expert, row_offsets[e]..row_offsets[e+1] are expert e's rows, token_of_row gives the source
    token of each grouped row.
    """
    rng = np.random.default_rng(seed)
    logp = -exponent * np.log(np.arange(1, experts + 1, dtype=np.float64))
    keys = logp[None, :] + rng.gumbel(size=(tokens, experts))
    choice = np.argsort(-keys, axis=1)[:, :top_k]                      # [tokens, top_k]
    flat_expert = choice.reshape(-1)
    flat_token = np.repeat(np.arange(tokens, dtype=np.int64), top_k)
    order = np.argsort(flat_expert, kind="stable")
    counts = np.bincount(flat_expert, minlength=experts).astype(np.int64)
    offsets = np.zeros(experts + 1, np.int64)
    np.cumsum(counts, out=offsets[1:])
    return offsets, flat_token[order]


# ---- the named workloads -------------------------------------------------------------------------
def tiny(seed: int = 0):
    """A 64x512 ~ N(0,1) with 4 outlier columns x50; W 256x512 ~ N(0, 0.02^2)."""
    return activations_normal(64, 512, 4, 50.0, seed), gaussian(256, 512, 0.02, seed + 1000)


def llama8b_ffn_up(rows_a: int = 4096, rows_w: int = 14336, K: int = 4096):
    """A ~ Student-t(4) with 1% channels x20 (seed 1); W ~ N(0, 0.02^2) (seed 2)."""
    return (activations_student_t(rows_a, K, 4.0, 0.01, 20.0, 1), gaussian(rows_w, K, 0.02, 2))


def decode_skinny(rows_w: int = 4096, K: int = 4096):
    """A 16xK as the prefill activations (seed 3); W ~ N(0, 0.02^2) (seed 2)."""
    return (activations_student_t(16, K, 4.0, 0.01, 20.0, 3), gaussian(rows_w, K, 0.02, 2))


def llama70b_ffn(rows_a: int = 8192, rows_w: int = 28672, K: int = 8192):
    """A ~ Student-t(3) with 0.5% channels x50 (seed 4); W ~ N(0, 0.015^2) (seed 5)."""
    return (activations_student_t(rows_a, K, 3.0, 0.005, 50.0, 4), gaussian(rows_w, K, 0.015, 5))


def moe(tokens: int = 8192, experts: int = 32, dim: int = 2880, top_k: int = 4):
    """Tokens as the prefill activations (seed 6); expert weights N(0,0.02^2) (seed 7);
    Zipf(1.1) top-k routing (seed 8).  Returns (x, W [experts*dim, dim], row_offsets, token_of_row)."""
    x = activations_student_t(tokens, dim, 4.0, 0.01, 20.0, 6)
    w = gaussian(experts * dim, dim, 0.02, 7)
    offsets, token_of_row = zipf_topk_routing(tokens, experts, top_k, 1.1, 8)
    return x, w, offsets, token_of_row
