"""Pins for the expert-parallel dispatch -> grouped GEMM oracle (``oracle/grouped.py``): the piece layout
checked against its wording by brute force, and the per-expert products against exact arithmetic and
weights that tell the experts apart."""
from fractions import Fraction

import numpy as np
import pytest

import ficco_inputs as fi
from oracle import grouped as ogr


def widen(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bits_of(x):
    return fi.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


@pytest.mark.parametrize("T,c", [(0, 4), (1, 4), (7, 3), (8, 4), (13, 5), (100, 1)])
def test_pieces_of_a_block_are_as_equal_as_integers_allow(T, c):
    r = ogr.piece_rows(T, c)
    assert len(r) == c and sum(r) == T and max(r) - min(r) <= 1 and r == sorted(r, reverse=True)


@pytest.mark.parametrize("rows,c", [([[3, 0], [5, 2], [0, 7]], 2), ([[4], [4], [4], [4]], 4), ([[1, 1, 1]], 3), ([[0, 0], [0, 0]], 1)])
def test_layout_places_every_token_once_expert_then_step_then_peer(rows, c):
    rows = np.asarray(rows)
    G, E = rows.shape
    r0, nr, e0, en = ogr.layout(rows, c)
    M = int(rows.sum())
    owner = -np.ones(M, dtype=np.int64)
    for i in range(E * c * G):
        assert np.all(owner[r0[i]:r0[i] + nr[i]] == -1)
        owner[r0[i]:r0[i] + nr[i]] = i
    assert np.all(owner >= 0)                                        # every row belongs to exactly one piece
    e_of, s_of, j_of = owner // (c * G), (owner // G) % c, owner % G
    key = (e_of * c + s_of) * G + j_of
    assert np.all(np.diff(key) >= 0)                                 # expert-major, then step, then peer
    for e in range(E):
        assert np.array_equal(np.flatnonzero(e_of == e), np.arange(e0[e], e0[e] + en[e]))    # an expert's rows are contiguous
        for j in range(G):
            assert int(np.sum((e_of == e) & (j_of == j))) == rows[j, e]                      # peer j's count for expert e
    for step_major in (True, False):
        arr = ogr.arrival_order(G, E, c, step_major)
        assert sorted(arr) == list(range(E * c * G))
    arr = ogr.arrival_order(G, E, c, True)
    steps = [(i // G) % c for i in arr]
    assert steps == sorted(steps)                                    # step by step; within a step every peer, every expert
    assert [i % G for i in ogr.arrival_order(G, E, c, False)] == sorted(i % G for i in arr)


def test_grouped_product_exact_rational_brute_force():
    rng = np.random.default_rng(3)
    en = [3, 0, 2]
    K, N = 5, 4
    A = bits_of(rng.integers(-6, 7, size=(5, K)).astype(np.float32))
    W = bits_of(rng.integers(-6, 7, size=(3, K, N)).astype(np.float32))
    out = ogr.grouped_gemm(A, W, en)
    expert_of_row = [0, 0, 0, 2, 2]
    for i in range(5):
        for n in range(N):
            s = sum(Fraction(float(widen(A[i, k]))) * Fraction(float(widen(W[expert_of_row[i], k, n]))) for k in range(K))
            assert Fraction(float(out[i, n])) == s


def test_experts_are_told_apart_by_their_weights():
    # W_e = (e + 1) * identity: every row must come back scaled by its own expert's factor
    K = 8
    en = [2, 3, 1]
    A = fi.normal_bf16(5, fi.TENSOR_A, 6, K)
    W = np.stack([bits_of((e + 1) * np.eye(K, dtype=np.float32)) for e in range(3)])
    out = ogr.grouped_gemm(A, W, en)
    factor = np.repeat([1.0, 2.0, 3.0], en)[:, None]
    assert np.array_equal(out, widen(A) * factor)


def test_token_counts_are_deterministic_and_sum_to_the_total():
    a = fi.make_token_counts(6, 8, 2, 16384, 0.6)
    assert a.shape == (8, 2) and a.sum() == 16384 and np.array_equal(a, fi.make_token_counts(6, 8, 2, 16384, 0.6))
    assert a.max() > 2 * a.min()                                     # visibly unequal
    even = fi.make_token_counts(6, 4, 2, 800, 0.0)
    assert np.all(even == 100)
