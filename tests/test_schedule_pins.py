"""Pins for the decomposition rules, static descriptors and loss ratios in ``oracle/schedule.py``:
brute force from the paper's wording, hand-computed values, closed forms and limits."""
import itertools

import pytest

from oracle import schedule as sch


@pytest.mark.parametrize("G,c", [(4, 1), (4, 4), (8, 2), (8, 32), (3, 5)])
def test_chunks_tile_the_gathered_rows(G, c):
    M = G * c * 16
    spans = [sch.chunk_span(M, G, c, i) for i in range(G * c)]
    assert spans[0][0] == 0 and spans[-1][0] + spans[-1][1] == M
    for (r0, n0), (r1, _) in zip(spans, spans[1:]):
        assert r0 + n0 == r1 and n0 == M // (G * c)
    # chunk j*c+s lies inside shard j (rows [j*M/G, (j+1)*M/G)) and is its s-th piece
    for j, s in itertools.product(range(G), range(c)):
        r0, n = sch.chunk_span(M, G, c, j * c + s)
        assert r0 == j * (M // G) + s * n


@pytest.mark.parametrize("G,c", [(4, 4), (8, 2), (2, 3)])
def test_step_major_is_all_to_all_order(G, c):
    # Sec. III-B in words: in step s every shard contributes its s-th piece
    arr = sch.arrival_order(G, c, sch.ORDER_STEP_MAJOR)
    assert sorted(arr) == list(range(G * c))
    for s in range(c):
        step = arr[s * G:(s + 1) * G]
        assert [i % c for i in step] == [s] * G            # piece index s ...
        assert [i // c for i in step] == list(range(G))    # ... of every shard, once
    assert sch.arrival_order(G, c, sch.ORDER_SHARD_MAJOR) == list(range(G * c))


def test_plans_by_schedule():
    M, G = 512, 4
    p = sch.plan(M, G, 1, sch.SERIAL)
    assert p["arrival"] == [0, 1, 2, 3] and p["groups"] == [[0, 1, 2, 3]] and p["m"] == 128
    p = sch.plan(M, G, 1, sch.SHARD)
    assert p["groups"] == [[0], [1], [2], [3]]
    p = sch.plan(M, G, 4, sch.FINE_UNFUSED)
    assert p["arrival"][:5] == [0, 4, 8, 12, 1] and p["groups"][:2] == [[0], [4]] and p["m"] == 32
    p = sch.plan(M, G, 4, sch.FINE_FUSED)
    assert p["groups"] == [[0, 4, 8, 12], [1, 5, 9, 13], [2, 6, 10, 14], [3, 7, 11, 15]]
    p = sch.plan(M, G, 4, sch.FINE_PERSISTENT, sch.ORDER_SHARD_MAJOR)
    assert p["groups"] == [list(range(16))]
    for s in (sch.SERIAL, sch.SHARD):
        with pytest.raises(ValueError):
            sch.plan(M, G, 2, s)
    with pytest.raises(ValueError):
        sch.plan(500, G, 4, sch.FINE_FUSED)


@pytest.mark.parametrize("schedule", [sch.SERIAL, sch.SHARD, sch.FINE_UNFUSED, sch.FINE_FUSED, sch.FINE_PERSISTENT])
def test_groups_partition_the_arrivals(schedule):
    c = 1 if schedule in (sch.SERIAL, sch.SHARD) else 4
    p = sch.plan(1024, 8, c, schedule)
    flat = [i for g in p["groups"] for i in g]
    assert flat == p["arrival"] and sorted(flat) == list(range(8 * c))


def test_static_descriptors_hand_values():
    # (1,1,1): 2 flops over 3 elements of 2 bytes
    assert sch.mt_bytes(1, 1, 1) == 6 and sch.otb(1, 1, 1) == pytest.approx(1 / 3)
    # M=512, N=K=1024: MT = 2*(512Ki + 1Mi + 512Ki) = 4 MiB, flops = 2^30, OTB = 256
    assert sch.mt_bytes(512, 1024, 1024) == 4 << 20
    assert sch.gemm_flops(512, 1024, 1024) == 1 << 30
    assert sch.otb(512, 1024, 1024) == 256.0
    # cube of side n: OTB = 2n^3 / (6 n^2) = n/3
    assert sch.otb(300, 300, 300) == pytest.approx(100.0)
    # OTB of the decomposed GEMM falls with the row count, MT is dominated by the weight
    assert sch.otb(128, 1024, 1024) < sch.otb(512, 1024, 1024)
    # OTB x MT is the flop count
    assert sch.otb(64, 768, 4096) * sch.mt_bytes(64, 768, 4096) == pytest.approx(sch.gemm_flops(64, 768, 4096))


def test_ideal_overlap_closed_form_and_limits():
    # n = 1 is serial execution
    assert sch.ideal_overlap_time(3.0, 5.0, 1) == 8.0
    assert sch.ideal_speedup(3.0, 5.0, 1) == 1.0
    # pipeline closed form: first transfer and last GEMM are exposed, the longer operator fills the rest
    for tc, tg, n in [(3.0, 5.0, 4), (5.0, 3.0, 8), (2.0, 2.0, 64), (1.0, 10.0, 3)]:
        closed = (tc + tg) / n + (n - 1) / n * max(tc, tg)
        assert sch.ideal_overlap_time(tc, tg, n) == pytest.approx(closed)
    # balanced operators approach 2x as the pieces shrink; never exceed it
    assert sch.ideal_speedup(1.0, 1.0, 1 << 16) == pytest.approx(2.0, rel=1e-4)
    # bell curve in the GEMM/communication ratio with its top at balance
    xs = [0.1, 0.3, 1.0, 3.0, 10.0]
    sp = [sch.ideal_speedup(1.0, x, 64) for x in xs]
    assert sp.index(max(sp)) == 2 and sp[0] < sp[1] < sp[2] > sp[3] > sp[4]
    assert sch.ideal_speedup(1.0, 0.25, 64) == pytest.approx(sch.ideal_speedup(0.25, 1.0, 64))
    # more pieces never hurt in the ideal model
    ts = [sch.ideal_overlap_time(4.0, 6.0, n) for n in (1, 2, 4, 8, 64)]
    assert all(a >= b for a, b in zip(ts, ts[1:]))


def test_loss_ratios():
    assert sch.dil([1.0] * 8, 8.0) == 1.0
    assert sch.dil([1.25] * 8, 8.0) == 1.25
    assert sch.cil([1.1] * 4, [1.0] * 4) == pytest.approx(1.1)
    assert sch.cil([1.0, 2.0], [1.0, 2.0]) == 1.0


def test_heuristic_rule_structure():
    T = 1e9
    assert sch.heuristic_paper(4096, 1024, 8192, 8, T) == "uniform-fused-2D"     # M <= K
    assert sch.heuristic_paper(8192, 1024, 8192, 8, T) == "uniform-fused-2D"
    # Sec. IV-B/C by hand for the step GEMM (2048 x 512 x 4096, bf16): ops 2*2048*512*4096 = 8 589 934 592;
    # bytes 2*(2048*4096 + 512*4096 + 2048*512) = 23 068 672; OTB = 372.36...; OTB x MT = the op count
    M, N, K = 16384, 512, 4096
    x = 8589934592
    assert sch.mt_bytes(M // 8, N, K) == 23068672 and sch.otb(M // 8, N, K) == pytest.approx(372.3636, rel=1e-6)
    assert sch.heuristic_paper(M, N, K, 8, x * 1.01) == "uniform-fused-1D"
    assert sch.heuristic_paper(M, N, K, 8, x / 2) == "hetero-fused-1D"
    assert sch.heuristic_paper(M, N, K, 8, x / 5.01) == "hetero-unfused-1D"
    assert sch.heuristic_paper(M, N, K, 8, x / 2, ratio=1.5) == "hetero-unfused-1D"


@pytest.mark.parametrize("G,c", [(4, 1), (4, 4), (8, 2), (3, 5)])
def test_column_pieces_tile_the_activation(G, c):
    # Sec. V-A in words: the 2D decomposition cuts every shard along k; step s moves slice s of each shard
    M, K = G * 6, c * 10
    cover = [[0] * K for _ in range(M)]
    for i in range(G * c):
        r0, nr, k0, nk = sch.piece_span_2d(M, K, G, c, i)
        assert nr == M // G and nk == K // c
        for r in range(r0, r0 + nr):
            for k in range(k0, k0 + nk):
                cover[r][k] += 1
    assert all(v == 1 for row in cover for v in row)
    arr = sch.arrival_order_2d(G, c, sch.ORDER_STEP_MAJOR)
    for s in range(c):
        step = arr[s * G:(s + 1) * G]
        spans = [sch.piece_span_2d(M, K, G, c, i) for i in step]
        assert [sp[2] for sp in spans] == [s * (K // c)] * G           # one k slice per step ...
        assert [sp[0] for sp in spans] == [j * (M // G) for j in range(G)]   # ... from every shard
    by_shard = sch.arrival_order_2d(G, c, sch.ORDER_SHARD_MAJOR)
    assert sorted(by_shard) == list(range(G * c))
    assert [sch.piece_span_2d(M, K, G, c, i)[0] for i in by_shard] == [j * (M // G) for j in range(G) for _ in range(c)]
    p = sch.plan(M, G, c, sch.FINE_2D)
    assert p["arrival"] == arr and p["groups"] == [arr] and p["m"] == M // G and p["n_chunks"] == G * c


@pytest.mark.parametrize("G,widths", [(4, [7, 1, 2]), (2, [3, 3]), (3, [1, 2, 4, 8])])
def test_column_pieces_of_unequal_width_tile_the_activation(G, widths):
    # the slices partition k in order whatever their widths; rows are still the shard's
    M, K, c = G * 5, sum(widths), len(widths)
    cover = [[0] * K for _ in range(M)]
    for i in range(G * c):
        r0, nr, k0, nk = sch.piece_span_2d(M, K, G, c, i, widths)
        assert (r0, nr) == ((i % G) * (M // G), M // G) and nk == widths[i // G] and k0 == sum(widths[:i // G])
        for r in range(r0, r0 + nr):
            for k in range(k0, k0 + nk):
                cover[r][k] += 1
    assert all(v == 1 for row in cover for v in row)
    if len(set(widths)) == 1:
        assert all(sch.piece_span_2d(M, K, G, c, i, widths) == sch.piece_span_2d(M, K, G, c, i) for i in range(G * c))
