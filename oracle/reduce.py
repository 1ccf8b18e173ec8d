"""Receiver side of a reduce-scatter, by its definition. TEST INFRASTRUCTURE ONLY (see the package docstring).

GPU ``r`` of a GEMM -> reduce-scatter pair (paper Sec. II-A/B) ends up with row block ``r`` of the
sum of all GPUs' partial products: ``out = x_0 + x_1 + ... + x_{G-1}`` with ``x_j`` GPU j's partial
block. The paper does not fix the arithmetic (it leaves reduce-scatter out because DMA engines cannot
add); the reading taken here matches the GEMM: bf16 inputs widened exactly to fp32, added in fp32 in
ascending GPU order starting from ``x_0`` itself, one round-to-nearest-even to bf16. Every step is an
IEEE-754 operation with one correct result, so the GPU must reproduce the bits.
"""
from __future__ import annotations

import numpy as np


def widen_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest, ties to even; NaN stays a quiet NaN."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r[nan] = ((u[nan] >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16)
    return r


def rs_reduce(blocks) -> np.ndarray:
    """``blocks[j]`` = GPU j's partial block ``[rows, N]`` (bf16 bits), j ascending. Returns bf16 bits."""
    acc = widen_f32(blocks[0]).copy()
    for b in blocks[1:]:
        with np.errstate(over="ignore", invalid="ignore"):
            acc = (acc + widen_f32(b)).astype(np.float32)       # one fp32 addition per GPU, in order
    return round_bf16(acc)


def rs_reduce_f64(blocks) -> np.ndarray:
    """The same sum in fp64 without intermediate rounding (what the fp32 result approximates)."""
    acc = np.zeros(np.asarray(blocks[0]).shape, dtype=np.float64)
    for b in blocks:
        acc += widen_f32(b).astype(np.float64)
    return acc
