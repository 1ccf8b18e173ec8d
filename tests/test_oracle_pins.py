"""Pins for the CPU oracle: it is checked against things other than itself - a hand-worked
instance, exact rational brute force, closed forms, a library routine, and metamorphic
properties - chosen so that a dropped term, a swapped index or a transposed operand fails."""
import os
from fractions import Fraction

import numpy as np
import pytest

import ficco_inputs as fi
from oracle import gemm as og


def widen(bits):
    """Independent bf16 -> fp64 widening (numpy bit shift), not the oracle's."""
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bits_of(x):
    return fi.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_widening_known_patterns():
    # bf16 is the high half of fp32: sign 1, exponent 8, mantissa 7
    assert widen([0x3F80, 0xC000, 0x3F00, 0x0000, 0x8000, 0x4049])[:4].tolist() == [1.0, -2.0, 0.5, 0.0]
    assert widen([0x4049])[0] == 3.140625
    # the oracle's own widening, observed through W = I: C must equal A exactly
    a = np.array([[0x3F80, 0xC000, 0x4049, 0x3DCD]], dtype=np.uint16)
    eye = bits_of(np.eye(4))
    assert np.array_equal(og.ag_gemm([a], eye), widen(a))


def test_hand_worked_golden(repo_root):
    shards, W, ref = [], [], []
    with open(os.path.join(repo_root, "tests", "golden", "tiny_gemm.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0].startswith("I"):
                shards.append(np.array([[int(x, 16) for x in t[1:]]], dtype=np.uint16))
            elif t[0] == "W":
                W.append([int(x, 16) for x in t[1:]])
            elif t[0] == "REF":
                ref.append([float(x) for x in t[1:]])
    out = og.ag_gemm(shards, np.array(W, dtype=np.uint16))
    assert np.array_equal(out, np.array(ref))


@pytest.mark.parametrize("G,ms,K,N,seed", [(1, 1, 1, 1, 0), (2, 3, 5, 4, 1), (4, 2, 8, 7, 2), (3, 1, 7, 8, 3)])
def test_exact_rational_brute_force(G, ms, K, N, seed):
    shards = fi.make_shards(seed, G * ms, K, G)
    W = fi.make_weight(seed, K, N)
    out = og.ag_gemm(shards, W)
    A = np.concatenate(shards, 0)
    for i in range(G * ms):
        for j in range(N):
            s = Fraction(0)
            for k in range(K):
                s += Fraction(float(widen(A[i, k]))) * Fraction(float(widen(W[k, j])))
            # sums this small are exact in fp64, so equality is exact
            assert Fraction(float(out[i, j])) == s, (i, j)


def test_identity_returns_gathered_activation():
    G, ms, K = 4, 16, 64
    shards = fi.make_shards(5, G * ms, K, G)
    out = og.ag_gemm(shards, bits_of(np.eye(K)))
    assert np.array_equal(out, widen(np.concatenate(shards, 0)))
    # rectangular: W = [I_N ; 0] selects the first N columns
    N = 24
    Wsel = np.zeros((K, N), dtype=np.float32)
    Wsel[:N, :N] = np.eye(N)
    assert np.array_equal(og.ag_gemm(shards, bits_of(Wsel)), widen(np.concatenate(shards, 0))[:, :N])


@pytest.mark.parametrize("K", [1, 7, 1024, 3584])
def test_all_ones_gives_K(K):
    one = np.full((3, K), 0x3F80, dtype=np.uint16)
    W = np.full((K, 5), 0x3F80, dtype=np.uint16)
    assert np.array_equal(og.ag_gemm([one, one], W), np.full((6, 5), float(K)))


def test_row_selector_places_rows():
    # A[i,:] = e_{i mod K}  =>  C[i,:] = W[i mod K,:]; W is random and not symmetric, so a
    # transposed operand, a wrong shard order or an off-by-one row all show up.
    G, ms, K, N = 4, 6, 5, 9
    M = G * ms
    A = np.zeros((M, K), dtype=np.float32)
    A[np.arange(M), np.arange(M) % K] = 1.0
    Ab = bits_of(A)
    W = fi.make_weight(9, K, N)
    out = og.ag_gemm([Ab[j * ms:(j + 1) * ms] for j in range(G)], W)
    assert np.array_equal(out, widen(W)[np.arange(M) % K])


def test_shard_order_is_row_order():
    # shard j is the constant j+1: row block j of the result is (j+1) * column sums of W
    G, ms, K, N = 4, 3, 8, 6
    shards = [bits_of(np.full((ms, K), float(j + 1))) for j in range(G)]
    W = bits_of(np.arange(K * N, dtype=np.float32).reshape(K, N) % 13 - 6)
    out = og.ag_gemm(shards, W)
    cs = widen(W).sum(0)
    for j in range(G):
        assert np.array_equal(out[j * ms:(j + 1) * ms], np.tile((j + 1) * cs, (ms, 1)))


def test_power_of_two_scaling_is_exact():
    shards = fi.make_shards(11, 32, 48, 2)
    W = fi.make_weight(11, 48, 20)
    base = og.ag_gemm(shards, W)
    twice = [bits_of(2.0 * widen(s)) for s in shards]
    assert np.array_equal(og.ag_gemm(twice, W), 2.0 * base)
    assert np.array_equal(og.ag_gemm(shards, bits_of(0.25 * widen(W))), 0.25 * base)


def test_matches_library_matmul_fp64():
    # the definition reduces to a plain fp64 matrix product of the widened inputs
    G, ms, K, N = 4, 40, 300, 70
    shards = fi.make_shards(13, G * ms, K, G)
    W = fi.make_weight(13, K, N)
    out = og.ag_gemm(shards, W)
    lib = widen(np.concatenate(shards, 0)) @ widen(W)
    assert np.max(np.abs(out - lib)) <= 1e-12 * (1 + np.max(np.abs(lib)))
    # a transposed or row-reversed weight is far outside that
    bad = widen(np.concatenate(shards, 0)) @ widen(W)[::-1]
    assert np.max(np.abs(out - bad)) > 1e-3


def test_rows_variant_equals_full():
    G, ms, K, N = 4, 10, 33, 17
    shards = fi.make_shards(17, G * ms, K, G)
    W = fi.make_weight(17, K, N)
    full = og.ag_gemm(shards, W)
    rows = np.array([0, 39, 10, 9, 25, 25], dtype=np.int64)
    assert np.array_equal(og.ag_gemm_rows(shards, W, rows), full[rows])
    with pytest.raises(RuntimeError):
        og.ag_gemm_rows(shards, W, np.array([40]))


def test_empty_and_degenerate_shapes():
    W = fi.make_weight(1, 8, 4)
    assert og.ag_gemm([np.zeros((0, 8), np.uint16)] * 2, W).shape == (0, 4)
    # K = 0: an empty sum is zero
    assert np.array_equal(og.ag_gemm([np.zeros((2, 0), np.uint16)], np.zeros((0, 3), np.uint16)), np.zeros((2, 3)))


def test_gemm_rs_blocks_concatenate_to_product():
    A = fi.normal_bf16(3, fi.TENSOR_A, 16, 12)
    W = fi.make_weight(3, 12, 8)
    blocks = og.gemm_rs_blocks(A, W, 8)
    assert len(blocks) == 8 and all(b.shape == (2, 8) for b in blocks)
    assert np.array_equal(np.concatenate(blocks, 0), widen(A) @ widen(W))   # tiny: exact in fp64


def test_acceptance_metric_definition():
    ref = np.array([[0.0, 3.0], [-1.0, 100.0]])
    gpu = ref + np.array([[0.5, 0.0], [0.0, -1.01]])
    assert og.rel_err(gpu, ref) == pytest.approx(0.5)
    assert og.rel_err(ref, ref) == 0.0


def test_generator_statistics_and_determinism():
    a = fi.normal_bf16(0, fi.TENSOR_A, 256, 512)
    b = fi.normal_bf16(0, fi.TENSOR_A, 64, 512, row0=64)
    assert np.array_equal(a[64:128], b)                      # blocking-independent
    x = widen(a)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    w = widen(fi.make_weight(0, 1024, 64))
    assert abs(w.std() * 32.0 - 1.0) < 0.02                  # variance 1/K
    assert not np.array_equal(fi.normal_bf16(1, fi.TENSOR_A, 4, 4), fi.normal_bf16(0, fi.TENSOR_A, 4, 4))
    assert not np.array_equal(fi.normal_bf16(0, fi.TENSOR_W, 4, 4), fi.normal_bf16(0, fi.TENSOR_A, 4, 4))


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is halfway between 1.0 (even mantissa) and 1 + 2^-7: ties go to even
    assert fi.f32_to_bf16_bits(np.float32(1.0 + 2.0 ** -8)) == 0x3F80
    assert fi.f32_to_bf16_bits(np.float32(1.0 + 3 * 2.0 ** -8)) == 0x3F82
    assert fi.f32_to_bf16_bits(np.float32(1.0 + 2.0 ** -8 + 2.0 ** -20)) == 0x3F81


# ------------------------------------------------------------------ 2D decomposition (Sec. V-A/B)
def test_k_sliced_layout_is_a_column_partition():
    A = np.arange(6 * 8, dtype=np.uint16).reshape(6, 8)
    S = fi.to_k_sliced(A, 4)
    assert S.shape == (4, 6, 2)
    for s in range(4):
        assert np.array_equal(S[s], A[:, 2 * s:2 * s + 2])
    assert np.array_equal(fi.to_k_sliced(A, 1)[0], A)


@pytest.mark.parametrize("G,ms,K,N,c,seed", [(2, 2, 8, 3, 2, 0), (4, 1, 12, 5, 3, 1), (1, 3, 4, 2, 4, 2)])
def test_2d_steps_exact_rational_brute_force(G, ms, K, N, c, seed):
    """Small-integer inputs: every partial sum is an integer far below 2^53, so accumulating slice
    by slice is exact and must equal the rational row-times-column sums of the unsliced matrix."""
    rng = np.random.default_rng(seed)
    A = bits_of(rng.integers(-8, 9, size=(G * ms, K)).astype(np.float32))
    W = bits_of(rng.integers(-8, 9, size=(K, N)).astype(np.float32))
    out = og.ag_gemm_2d(fi.to_k_sliced(A, c), W, G)
    for i in range(G * ms):
        for j in range(N):
            s = sum(Fraction(float(widen(A[i, k]))) * Fraction(float(widen(W[k, j]))) for k in range(K))
            assert Fraction(float(out[i, j])) == s, (i, j)


def test_2d_steps_pick_the_matching_weight_rows():
    """A = [1 0 ... | 0 ... 1 ...]: one 1 per row in a known column; the result row must be that row
    of W. A slice paired with the wrong rows of W, or a transposed slice, fails."""
    K, N, M, G, c = 16, 5, 8, 4, 4
    W = fi.make_weight(7, K, N)
    cols = [(5 * i + 3) % K for i in range(M)]
    A = np.zeros((M, K), dtype=np.float32)
    A[np.arange(M), cols] = 1.0
    out = og.ag_gemm_2d(fi.to_k_sliced(bits_of(A), c), W, G)
    assert np.array_equal(out, widen(W)[cols])


def test_2d_steps_equal_whole_product_on_random_inputs():
    G, M, K, N, c = 4, 64, 256, 24, 4
    shards = fi.make_shards(11, M, K, G)
    W = fi.make_weight(11, K, N)
    A = np.concatenate(shards, 0)
    whole = og.ag_gemm(shards, W)
    steps = og.ag_gemm_2d(fi.to_k_sliced(A, c), W, G)
    # same terms, another association of the fp64 sums
    assert np.max(np.abs(whole - steps)) <= 1e-12 * K
    assert np.array_equal(og.ag_gemm_2d(fi.to_k_sliced(A, 1), W, G), whole)


# ------------------------------------------------------------------ column pieces of unequal width
def test_k_pieces_layout_partitions_the_columns_in_order():
    A = np.arange(5 * 12, dtype=np.uint16).reshape(5, 12)
    blocks = fi.to_k_pieces(A, [6, 2, 4])
    assert [b.shape for b in blocks] == [(5, 6), (5, 2), (5, 4)]
    assert np.array_equal(np.concatenate(blocks, 1), A)
    assert all(b.flags["C_CONTIGUOUS"] for b in blocks)
    # equal widths give the bytes of the [c, M, K/c] layout
    flat = np.concatenate([b.ravel() for b in fi.to_k_pieces(A, [4, 4, 4])])
    assert np.array_equal(flat, fi.to_k_sliced(A, 3).ravel())


@pytest.mark.parametrize("G,ms,widths,N,seed", [(2, 2, [6, 2], 3, 0), (4, 1, [1, 8, 3], 5, 1), (1, 3, [2, 1, 1, 4], 2, 2)])
def test_2d_unequal_steps_exact_rational_brute_force(G, ms, widths, N, seed):
    """As the equal-width brute force: small integers, every partial sum exact, so the slice-by-slice
    result must equal the rational sums over the unsliced matrix whatever the widths."""
    K = sum(widths)
    rng = np.random.default_rng(seed)
    A = bits_of(rng.integers(-8, 9, size=(G * ms, K)).astype(np.float32))
    W = bits_of(rng.integers(-8, 9, size=(K, N)).astype(np.float32))
    out = og.ag_gemm_2d(fi.to_k_pieces(A, widths), W, G)
    for i in range(G * ms):
        for j in range(N):
            s = sum(Fraction(float(widen(A[i, k]))) * Fraction(float(widen(W[k, j]))) for k in range(K))
            assert Fraction(float(out[i, j])) == s, (i, j)


def test_2d_unequal_steps_pick_the_matching_weight_rows():
    """One 1 per row of A in a known column: the result row must be that row of W. A slice paired with
    rows of W that start at the equal-width offset instead of the running sum of widths fails."""
    K, N, M, G = 16, 5, 8, 4
    widths = [2, 9, 1, 4]
    W = fi.make_weight(7, K, N)
    cols = [(5 * i + 3) % K for i in range(M)]
    A = np.zeros((M, K), dtype=np.float32)
    A[np.arange(M), cols] = 1.0
    out = og.ag_gemm_2d(fi.to_k_pieces(bits_of(A), widths), W, G)
    assert np.array_equal(out, widen(W)[cols])
