"""Seeded synthetic inputs with the shapes of quantised LLM layers.

This module only draws numbers and shapes them; it holds no field arithmetic
and nothing of the proof system, so both the CPU oracle's tests and the GPU
path's tests can take their inputs from it without sharing any of the method.

The five workloads stand in for the linear layers of an 8B-class dense model
and an 8-expert MoE layer (the paper's own models and prompt sets are not
needed: the proven statement is a matrix product, whose cost depends only on
shape and operand width):

  tiny      A 64x64 int16 uniform, B 64x64 int8 uniform
  attn      A 512x4096 int16 Gaussian(sigma=2^10), B 4096x4096 int8 uniform
  ffn_up    A 2048x4096 int16 Gaussian,            B 4096x14336 int8 uniform
  moe       8 experts, top-2 routing of 4096 tokens, B_e 4096x14336 int8
  dense32   32 layers x {Wq, Wk, Wv, Wo, W_gate, W_up, W_down}, 1024 tokens

Activations are int16 (Gaussian samples rounded half-to-even and clipped),
weights are int8 uniform on [-128, 128).
"""
from __future__ import annotations

from typing import Iterator, List, Tuple

import numpy as np


def uniform_int8(shape, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(-128, 128, size=shape, dtype=np.int8)


def uniform_int16(shape, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(-(1 << 15), 1 << 15, size=shape, dtype=np.int16)


def gaussian_int16(shape, seed: int, sigma: float = 1024.0) -> np.ndarray:
    x = np.random.default_rng(seed).normal(0.0, sigma, size=shape)
    return np.clip(np.rint(x), -32768, 32767).astype(np.int16)


def exact_product_int64(A: np.ndarray, B: np.ndarray, row_block: int = 256) -> np.ndarray:
    """C = A.B as int64.  |C| < 2^15 * 2^7 * 2^14 = 2^36, far below 2^53, so a float64
    GEMM over row blocks is exact.  Input preparation only (C is a public input of the
    statement); it is never part of a timed prover region."""
    m, _ = A.shape
    Bf = B.astype(np.float64)
    C = np.empty((m, B.shape[1]), dtype=np.int64)
    for i0 in range(0, m, row_block):
        C[i0:i0 + row_block] = np.rint(A[i0:i0 + row_block].astype(np.float64) @ Bf).astype(np.int64)
    return C


def tiny() -> Tuple[np.ndarray, np.ndarray]:
    return uniform_int16((64, 64), 0), uniform_int8((64, 64), 1)


def attn_proj() -> Tuple[np.ndarray, np.ndarray]:
    return gaussian_int16((512, 4096), 2), uniform_int8((4096, 4096), 3)


def ffn_up(rows: int = 2048) -> Tuple[np.ndarray, np.ndarray]:
    return gaussian_int16((rows, 4096), 4), uniform_int8((4096, 14336), 5)


def moe_routing(tokens: int = 4096, experts: int = 8, top_k: int = 2, seed: int = 7) -> List[np.ndarray]:
    """Token indices (increasing) routed to each expert: top-k of uniform router scores,
    ties broken toward the lower expert index."""
    scores = np.random.default_rng(seed).random((tokens, experts))
    order = np.argsort(-scores, axis=1, kind="stable")[:, :top_k]
    return [np.sort(np.nonzero((order == e).any(axis=1))[0]) for e in range(experts)]


def moe_activations(tokens: int = 4096, hidden: int = 4096) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Shared token matrix X and the per-expert row index lists; A_e = X[idx_e]."""
    X = gaussian_int16((tokens, hidden), 6)
    return X, moe_routing(tokens)


def moe_expert_weight(e: int, hidden: int = 4096, ffn: int = 14336) -> np.ndarray:
    return uniform_int8((hidden, ffn), 8 + e)


DENSE_LAYER_SHAPES = (  # (name, d, n) with B of shape d x n
    ("Wq", 4096, 4096), ("Wk", 4096, 1024), ("Wv", 4096, 1024), ("Wo", 4096, 4096),
    ("W_gate", 4096, 14336), ("W_up", 4096, 14336), ("W_down", 14336, 4096),
)


def dense_layer(layer: int, tokens: int = 1024) -> Iterator[Tuple[str, np.ndarray, np.ndarray]]:
    """The seven (name, A, B) statements of one decoder layer, in proof order."""
    for idx, (name, d, n) in enumerate(DENSE_LAYER_SHAPES):
        A = gaussian_int16((tokens, d), 5000 + 7 * layer + idx)
        B = uniform_int8((d, n), 1000 + 7 * layer + idx)
        yield name, A, B


# --------------------------------------------------------------------------- logits for the distance step
def round_to_bfloat16(x: np.ndarray) -> np.ndarray:
    """Finite float32 values rounded to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.array(x, dtype=np.float32, order="C").view(np.uint32)
    bias = (u >> np.uint32(16)) & np.uint32(1)
    bias += np.uint32(0x7FFF)
    u += bias            # finite inputs cannot wrap: their exponent field is below 0xFF
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32).reshape(np.shape(x))


LOGITS_ROW_BLOCK = 64


def logits_pair(steps: int, vocab: int, seed: int, scale: float = 4.0, noise: float = 0.02, workers: int = 8):
    """(deployed, reference) float32 logits of `steps` decision steps over `vocab` entries.
    The reference is Gaussian with standard deviation `scale` (a moderately peaked softmax); the
    deployed logits are the reference rounded to bfloat16 plus small Gaussian noise, which is what a
    finite-precision serving stack does to them.  Every block of 64 rows has generators of its own,
    seeded by (seed, block, which), so the values do not depend on how many threads fill the blocks."""
    ref = np.empty((steps, vocab), dtype=np.float32)
    dep = np.empty((steps, vocab), dtype=np.float32)

    def fill(block: int) -> None:
        rows = slice(block * LOGITS_ROW_BLOCK, min(steps, (block + 1) * LOGITS_ROW_BLOCK))
        np.random.default_rng([seed, block, 0]).standard_normal(out=ref[rows], dtype=np.float32)
        ref[rows] *= np.float32(scale)
        np.random.default_rng([seed, block, 1]).standard_normal(out=dep[rows], dtype=np.float32)
        dep[rows] *= np.float32(noise)
        dep[rows] += round_to_bfloat16(ref[rows])

    blocks = range((steps + LOGITS_ROW_BLOCK - 1) // LOGITS_ROW_BLOCK)
    if workers > 1 and len(blocks) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(fill, blocks))
    else:
        for b in blocks:
            fill(b)
    return dep, ref


def topk_indices(logits: np.ndarray, k: int) -> np.ndarray:
    """Indices of k largest entries of every row, largest first (what a server would record), int32.
    Among equal values any choice is a valid top-k set; no particular one is promised."""
    part = np.argpartition(-logits, k - 1, axis=1)[:, :k]
    vals = np.take_along_axis(logits, part, axis=1)
    order = np.argsort(-vals, axis=1, kind="stable")
    return np.take_along_axis(part, order, axis=1).astype(np.int32)
