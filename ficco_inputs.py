"""Seeded synthetic inputs for the all-gather -> GEMM path (and its mirror, GEMM -> reduce-scatter).

This module holds *no* arithmetic of the method itself: it only produces bf16 bit patterns
(``numpy.uint16``) of iid normal matrices and names the workload shapes. Both the CPU oracle's
tests and the GPU path's tests/bench draw their inputs from here, so that the two sides see the
same bits; neither side's code lives here.

Recipe (stands in for the model-derived GEMM shapes of the paper's Table I, at sizes one GPU can
hold): the activation ``A`` is the row-concatenation of ``G`` shards ``[M/G, K]`` with entries
~N(0, 1); the weight share ``W`` is ``[K, N]`` with entries ~N(0, 1/K) (second parameter is the
variance, so that ``A @ W`` has unit-variance entries). Every value is rounded once, to nearest
even, to bf16 on the host.

Generator: a counter-based 64-bit integer hash of (seed, tensor id, linear index) gives two
32-bit uniforms, which one Box-Muller branch turns into a standard normal in fp64. No state, so
any sub-block of a tensor can be produced on its own (``row0``/``rows``), and the values do not
depend on how the tensor is blocked.
"""
from __future__ import annotations

import os

import numpy as np

TENSOR_A = 0
TENSOR_W = 1
TENSOR_P = 2          # peers' partial output blocks (receiver side of a reduce-scatter)
TENSOR_T = 3          # token counts of an expert-parallel dispatch

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(x: np.ndarray) -> np.ndarray:
    """Bijective 64-bit finaliser (xor-shift-multiply rounds); ``x`` is uint64, wraps mod 2^64."""
    x = x.copy()
    x ^= x >> np.uint64(30)
    x *= np.uint64(0xBF58476D1CE4E5B9)
    x ^= x >> np.uint64(27)
    x *= np.uint64(0x94D049BB133111EB)
    x ^= x >> np.uint64(31)
    return x


def _key(seed: int, tensor_id: int) -> np.uint64:
    k = (int(seed) * 0x9E3779B97F4A7C15 + (int(tensor_id) + 1) * 0xD1B54A32D192ED03) & 0xFFFFFFFFFFFFFFFF
    return _mix64(np.array([k], dtype=np.uint64))[0]


def standard_normal_f64(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """``count`` iid N(0,1) fp64 values for linear indices ``start .. start+count-1`` of a tensor."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        h = _mix64((idx * np.uint64(0x9E3779B97F4A7C15)) ^ _key(seed, tensor_id))
    hi = (h >> np.uint64(32)).astype(np.float64)
    lo = (h & np.uint64(0xFFFFFFFF)).astype(np.float64)
    u1 = (hi + 1.0) * (1.0 / 4294967296.0)          # (0, 1]
    u2 = lo * (1.0 / 4294967296.0)                  # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (1-8-7), nearest even; returns the 16-bit patterns. Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, tensor_id: int, rows: int, cols: int, std: float = 1.0,
                row0: int = 0, block_rows: int = 0, workers: int = 0) -> np.ndarray:
    """bf16 bits ``[rows, cols]`` of rows ``row0 .. row0+rows-1`` of an iid N(0, std^2) tensor
    whose row length is ``cols``. Generated in row blocks to bound temporaries; big tensors spread
    their blocks over a few threads (the generator has no state, so the values do not change)."""
    out = np.empty((rows, cols), dtype=np.uint16)
    if block_rows <= 0:
        block_rows = max(1, (1 << 18) // max(cols, 1))      # blocks that stay in the caches

    def fill(r):
        nr = min(block_rows, rows - r)
        z = standard_normal_f64(seed, tensor_id, (row0 + r) * cols, nr * cols)
        out[r:r + nr] = f32_to_bf16_bits((z * std).astype(np.float32)).reshape(nr, cols)

    starts = range(0, rows, block_rows)
    if workers <= 0:
        workers = min(8, os.cpu_count() or 1) if rows * cols >= (1 << 24) else 1
    if workers > 1 and len(starts) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(fill, starts))
    else:
        for r in starts:
            fill(r)
    return out


def make_shards(seed: int, M: int, K: int, shards: int) -> list[np.ndarray]:
    """The G activation shards ``[M/G, K]`` (bf16 bits, ~N(0,1)); shard j is rows j*M/G.. of A."""
    assert M % shards == 0
    ms = M // shards
    return [normal_bf16(seed, TENSOR_A, ms, K, 1.0, row0=j * ms) for j in range(shards)]


def make_weight(seed: int, K: int, N: int) -> np.ndarray:
    """The resident weight share ``[K, N]`` (bf16 bits, ~N(0, 1/K))."""
    return normal_bf16(seed, TENSOR_W, K, N, float(K) ** -0.5)


# ---------------------------------------------------------------------------------------------
# Workloads. ``chunk_rows`` lists rows per chunk; chunks per shard c = (M/shards) / chunk_rows.
# ---------------------------------------------------------------------------------------------
CONFIGS = {
    # tiny case the oracle finishes in well under a second
    "cfg1_tiny": dict(M=512, K=1024, N=1024, shards=4, chunk_rows=[128, 32], seed=0,
                      direction="ag_gemm"),
    # Llama-3-8B QKV share at TP=8 (``k_slices``: the 2D decomposition is screened too; it needs no more
    # than a K-sliced staging layout on the sending side; ``k_widths``: column pieces of unequal width)
    "cfg2_qkv8b": dict(M=8192, K=4096, N=768, shards=8, chunk_rows=[1024, 512, 256], k_slices=[2, 4],
                       k_widths=[[3072, 1024]], seed=1, direction="ag_gemm"),
    # 70B-class FFN-up share
    "cfg3_ffn70b": dict(M=16384, K=8192, N=3584, shards=8, chunk_rows=[2048, 1024, 512, 256], seed=2,
                        direction="ag_gemm"),
    # GEMM -> reduce-scatter share (data movement half): output streamed out in 8 row blocks
    "cfg4_gemm_rs": dict(M=16384, K=3584, N=8192, shards=8, chunk_rows=[2048, 512, 256, 128], seed=3,
                         direction="gemm_rs"),
    # expert-parallel dispatch -> grouped expert GEMM: 8 peers send unequal token counts to 2 local experts
    # (Mixtral-like expert width: K = 4096, N = a quarter of the fused gate+up projection)
    "cfg7_ep_grouped": dict(K=4096, N=7168, shards=8, experts=2, tokens=16384, skew=0.6, pieces=[1, 2, 4, 8], seed=6,
                            direction="ep_grouped"),
    # M <= K share (row-parallel projection at a small token count): the shape the paper's rule sends
    # to the 2D decomposition; ``k_slices`` lists the slice counts exercised
    "cfg6_2d_proj": dict(M=4096, K=16384, N=4096, shards=8, chunk_rows=[512, 256, 128], k_slices=[2, 4, 8], seed=5,
                         direction="ag_gemm"),
}

# heuristic sweep (all-gather -> GEMM, 8 shards)
SWEEP = dict(M=[4096, 16384, 65536], K=[4096, 8192], N=[512, 1024, 3584, 14336], shards=8,
             chunks_per_shard=[1, 2, 4, 8, 16, 32], seed=4)


def make_partials(seed: int, peers: int, rows: int, N: int) -> np.ndarray:
    """``[peers, rows, N]`` bf16 bits ~N(0,1): the partial row blocks the GPUs of a reduce-scatter hold
    for one receiver (a GEMM output with unit-variance entries, like C of the configs)."""
    return normal_bf16(seed, TENSOR_P, peers * rows, N, 1.0).reshape(peers, rows, N)


def make_token_counts(seed: int, peers: int, experts: int, total: int, skew: float = 0.6) -> np.ndarray:
    """``[peers, experts]`` token counts that sum to ``total``: log-normal shares (sigma = ``skew``), the
    kind of imbalance a learned router produces; deterministic in the seed. ``skew`` 0 gives equal shares."""
    z = standard_normal_f64(seed, TENSOR_T, 0, peers * experts)
    w = np.exp(skew * z)
    share = w / w.sum() * total
    counts = np.floor(share).astype(np.int64)
    order = np.argsort(-(share - counts), kind="stable")
    counts[order[: total - int(counts.sum())]] += 1          # largest remainders get the leftover rows
    return counts.reshape(peers, experts)


def to_k_sliced(A: np.ndarray, slices: int) -> np.ndarray:
    """Layout change only: ``[M, K]`` row-major -> ``[slices, M, K/slices]``, slice s holding columns
    ``[s*K/slices, (s+1)*K/slices)`` of every row (the layout in which column pieces travel)."""
    M, K = A.shape
    assert K % slices == 0
    return np.ascontiguousarray(A.reshape(M, slices, K // slices).transpose(1, 0, 2))


def to_k_pieces(A: np.ndarray, widths) -> list[np.ndarray]:
    """Layout change only, for slices of unequal width: the list of ``[M, widths[s]]`` contiguous blocks,
    block s holding columns ``[sum(widths[:s]), sum(widths[:s+1]))`` of every row. Laid end to end
    (``np.concatenate([b.ravel() for b in blocks])``) they are the layout in which such pieces travel; with
    equal widths that is :func:`to_k_sliced`'s array."""
    M, K = A.shape
    assert sum(int(w) for w in widths) == K and all(int(w) > 0 for w in widths)
    edges = np.concatenate([[0], np.cumsum(np.asarray(widths, dtype=np.int64))])
    return [np.ascontiguousarray(A[:, edges[s]:edges[s + 1]]) for s in range(len(widths))]


def config_inputs(name: str):
    """(shards list, W) for a named workload."""
    c = CONFIGS[name]
    return make_shards(c["seed"], c["M"], c["K"], c["shards"]), make_weight(c["seed"], c["K"], c["N"])
