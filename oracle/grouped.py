"""Expert-parallel dispatch -> grouped expert GEMM, by its definition. TEST INFRASTRUCTURE ONLY.

A GPU hosts ``E`` experts with weights ``W_e [K, N]``; peer ``j`` sends it ``T[j][e]`` token rows for
expert ``e`` (paper Sec. II-A: expert parallelism disperses tokens all-to-all before the expert
layers; Sec. III-C: the amounts differ per pair of GPUs). The result is, for every token row ``a``
routed to expert ``e``, ``a @ W_e`` - whatever the transfer schedule.

Decomposition one level below the per-peer shard (Sec. III-A): the ``T[j][e]`` rows of a (peer, expert)
block are cut into ``c`` pieces as equal as integers allow (the first ``T mod c`` pieces one row
longer). Rows are laid out expert-major, then step, then peer, so that what arrives in step ``s`` for
expert ``e`` is contiguous: piece id ``i = (e*c + s)*G + j``, rows in id order.
"""
from __future__ import annotations

import numpy as np

from . import gemm as og


def piece_rows(T: int, c: int) -> list[int]:
    """Sizes of the ``c`` pieces of a block of ``T`` rows."""
    return [T // c + (1 if s < T % c else 0) for s in range(c)]


def layout(rows, c: int):
    """``rows[j][e]`` -> (piece_row0, piece_nrows, expert_row0, expert_nrows), pieces in id order
    ``(e*c + s)*G + j``."""
    rows = np.asarray(rows, dtype=np.int64)
    G, E = rows.shape
    n = E * c * G
    nr = np.zeros(n, dtype=np.int64)
    for e in range(E):
        for j in range(G):
            for s, r in enumerate(piece_rows(int(rows[j, e]), c)):
                nr[(e * c + s) * G + j] = r
    r0 = np.concatenate([[0], np.cumsum(nr)[:-1]])
    exp_n = rows.sum(axis=0)
    exp_0 = np.concatenate([[0], np.cumsum(exp_n)[:-1]])
    return r0, nr, exp_0, exp_n


def arrival_order(G: int, E: int, c: int, step_major: bool = True) -> list[int]:
    """Piece ids in issue order: step by step, every peer's pieces of that step (all-to-all), or peer
    by peer (one link at a time)."""
    if step_major:
        return [(e * c + s) * G + j for s in range(c) for j in range(G) for e in range(E)]
    return [(e * c + s) * G + j for j in range(G) for s in range(c) for e in range(E)]


def grouped_gemm(A, W, expert_nrows) -> np.ndarray:
    """fp64 ``[M, N]``: rows of ``A`` (bf16 bits, expert-major) times their expert's ``W[e]`` (bf16 bits)."""
    A = np.ascontiguousarray(A, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    out = np.zeros((A.shape[0], W.shape[2]), dtype=np.float64)
    r = 0
    for e, n in enumerate(int(x) for x in expert_nrows):
        if n:
            out[r:r + n] = og.ag_gemm([A[r:r + n]], W[e])
        r += n
    assert r == A.shape[0]
    return out
