"""Decomposition rules, static descriptors and loss ratios of the overlap path, in plain Python.

TEST INFRASTRUCTURE ONLY (see the package docstring). Everything here is integer bookkeeping or a
one-line ratio taken from the paper's definitions; the HIP library has its own implementation
and the tests compare the two. The library's fitted schedule rules (piece count, communication
shape, slice cut) have no counterpart here: their constants are timing fits of one machine, not
something the paper defines, so the tests pin them by hand-worked cases instead.

Notation: G shards of ``ms = M/G`` rows; each shard cut into ``c`` sub-chunks of ``m = ms/c`` rows
(Sec. III-A: communication is decomposed one level below the shard); chunk id ``i = j*c + s`` is
sub-chunk ``s`` of shard ``j`` and covers rows ``[i*m, (i+1)*m)`` of the gathered activation.
"""
from __future__ import annotations

SERIAL = 0            # Fig. 3(b): gather every shard, then one GEMM
SHARD = 1             # Fig. 3(c): shard j arrives, GEMM on shard j
FINE_UNFUSED = 2      # Sec. V-A "unfused": one GEMM per received piece
FINE_FUSED = 3        # Sec. V-A "fused": one GEMM per step over every piece received in the step
FINE_PERSISTENT = 4   # one resident kernel whose tiles wait for their own piece (this build's design)
FINE_2D = 5           # Sec. V-A/B 2D decomposition: column pieces, step s moves k slice s of every shard

ORDER_STEP_MAJOR = 0  # Sec. III-B: step s moves sub-chunk s of every shard (all-to-all pattern)
ORDER_SHARD_MAJOR = 1 # all pieces of shard 0, then shard 1, ... (peer-to-peer pattern at finer grain)


def chunk_span(M: int, G: int, c: int, i: int) -> tuple[int, int]:
    """(first row, row count) of chunk ``i``."""
    assert M % (G * c) == 0
    m = M // (G * c)
    assert 0 <= i < G * c
    return i * m, m


def piece_span_2d(M: int, K: int, G: int, c: int, i: int, widths=None) -> tuple[int, int, int, int]:
    """(first row, rows, first column, columns) of column piece ``i = s*G + j``: k slice ``s`` of
    shard ``j`` (Sec. V-A: 2D decomposition cuts the shard along the contraction dimension).
    ``widths``: the c slice widths when they differ (they partition K in order); equal otherwise."""
    assert M % G == 0 and 0 <= i < G * c
    s, j = divmod(i, G)
    if widths is None:
        assert K % c == 0
        return j * (M // G), M // G, s * (K // c), K // c
    assert len(widths) == c and sum(widths) == K and min(widths) > 0
    return j * (M // G), M // G, sum(widths[:s]), widths[s]


def arrival_order_2d(G: int, c: int, order: int) -> list[int]:
    """Column-piece ids in issue order: slice by slice (step-major) or shard by shard."""
    if order == ORDER_STEP_MAJOR:
        return [s * G + j for s in range(c) for j in range(G)]
    if order == ORDER_SHARD_MAJOR:
        return [s * G + j for j in range(G) for s in range(c)]
    raise ValueError("order")


def arrival_order(G: int, c: int, order: int) -> list[int]:
    """Chunk ids in the order their transfers are issued."""
    if order == ORDER_STEP_MAJOR:
        return [j * c + s for s in range(c) for j in range(G)]
    if order == ORDER_SHARD_MAJOR:
        return [j * c + s for j in range(G) for s in range(c)]
    raise ValueError("order")


def plan(M: int, G: int, c: int, schedule: int, order: int | None = None) -> dict:
    """Transfers and GEMM launches of one schedule.

    Returns ``arrival`` (chunk ids in issue order), ``groups`` (one list of chunk ids per GEMM
    launch, in launch order; a launch starts when all its chunks have landed) and ``m``.
    """
    if schedule in (SERIAL, SHARD):
        if c != 1:
            raise ValueError("serial and shard-level schedules move whole shards (c = 1)")
        arr = list(range(G))
        groups = [arr[:]] if schedule == SERIAL else [[j] for j in arr]
    elif schedule in (FINE_UNFUSED, FINE_FUSED, FINE_PERSISTENT):
        arr = arrival_order(G, c, ORDER_STEP_MAJOR if order is None else order)
        if schedule == FINE_UNFUSED:
            groups = [[i] for i in arr]
        elif schedule == FINE_FUSED:
            groups = [arr[g * G:(g + 1) * G] for g in range(c)]     # one launch per step of G pieces
        else:
            groups = [arr[:]]                                       # one launch; waits are per tile
    elif schedule == FINE_2D:
        if M % G:
            raise ValueError("M must be a multiple of shards")
        arr = arrival_order_2d(G, c, ORDER_STEP_MAJOR if order is None else order)
        return dict(arrival=arr, groups=[arr[:]], m=M // G, n_chunks=G * c)
    else:
        raise ValueError("schedule")
    if M % (G * c):
        raise ValueError("M must be a multiple of shards*chunks")
    return dict(arrival=arr, groups=groups, m=M // (G * c), n_chunks=G * c)


# ------------------------------------------------------------------ static descriptors (Sec. IV)
def gemm_flops(m: int, N: int, K: int) -> int:
    return 2 * m * N * K


def mt_bytes(m: int, N: int, K: int, elem_bytes: int = 2) -> int:
    """Static memory traffic MT = MK + NK + MN of an (m, N, K) GEMM (Sec. IV-C), in bytes."""
    return elem_bytes * (m * K + N * K + m * N)


def otb(m: int, N: int, K: int, elem_bytes: int = 2) -> float:
    """Static op-to-byte ratio of the *resultant* (decomposed) GEMM (Sec. IV-B)."""
    return gemm_flops(m, N, K) / mt_bytes(m, N, K, elem_bytes)


# ------------------------------------------------------------------ loss ratios (Sec. IV-A..C)
def ideal_overlap_time(t_comm: float, t_gemm: float, n: int) -> float:
    """Ideal execution (Sec. IV-A): both operators split into ``n`` pieces whose times scale
    exactly with the split, piece p's GEMM depends on piece p's transfer, transfers run back to
    back on one engine and GEMMs back to back on the other."""
    assert n >= 1
    done_c = 0.0
    done_g = 0.0
    for _ in range(n):
        done_c += t_comm / n
        done_g = max(done_g, done_c) + t_gemm / n
    return done_g


def ideal_speedup(t_comm: float, t_gemm: float, n: int) -> float:
    return (t_comm + t_gemm) / ideal_overlap_time(t_comm, t_gemm, n)


def dil(t_pieces: list[float], t_whole: float) -> float:
    """Decomposition inefficiency loss: summed isolated time of the pieces over the time of the
    single large operation (Sec. IV-B)."""
    return sum(t_pieces) / t_whole


def cil(t_pieces_overlapped: list[float], t_pieces_isolated: list[float]) -> float:
    """Contention inefficiency loss: the decomposed operator run concurrently with the other
    operator, relative to the same decomposed operator in isolation (Sec. IV-C)."""
    return sum(t_pieces_overlapped) / sum(t_pieces_isolated)


# ------------------------------------------------------------------ heuristic (Sec. V-C)
def heuristic_paper(M: int, N: int, K: int, G: int, threshold: float, ratio: float = 5.0) -> str:
    """The paper's static decision rule. Shape first: 1D (row pieces) if M > K, else 2D. Among
    the 1D schedules the combined OTB-and-MT metric of the step GEMM is compared with a machine
    threshold: below it ``uniform-fused-1D``; above ``ratio`` times it ``hetero-unfused-1D``;
    otherwise ``hetero-fused-1D``. The paper does not print how OTB and MT are combined; the
    reading used here is their product (which is the step GEMM's flop count), with ``threshold``
    a fitted machine constant in the same unit."""
    if M <= K:
        return "uniform-fused-2D"
    ms = M // G
    x = otb(ms, N, K) * mt_bytes(ms, N, K)
    if x < threshold:
        return "uniform-fused-1D"
    if x > ratio * threshold:
        return "hetero-unfused-1D"
    return "hetero-fused-1D"
