"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-side logic (plans, arrival lists, groups, static descriptors, ideal-overlap model, shape
rules) agrees with the oracle's plain-Python rules. No kernel is launched."""
import os
import re

import pytest

import paper_2512_10236_amd as ficco
from oracle import schedule as sch


def test_library_exports_every_declared_symbol(repo_root):
    text = open(os.path.join(repo_root, "include", "ficco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ficco_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    lib = ficco.load()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in ficco.h but not exported"
    assert declared == set(ficco.EXPORTS)
    assert "gfx950" in ficco.ficco_version()


def test_enum_values_match_header(repo_root):
    text = open(os.path.join(repo_root, "include", "ficco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for name, val in re.findall(r"\b(FICCO_[A-Z0-9_x]+)\s*=\s*(-?\d+)", text):
        assert getattr(ficco, name) == int(val), name


SCHEDS = [(ficco.FICCO_SERIAL, sch.SERIAL), (ficco.FICCO_SHARD, sch.SHARD),
          (ficco.FICCO_FINE_UNFUSED, sch.FINE_UNFUSED), (ficco.FICCO_FINE_FUSED, sch.FINE_FUSED),
          (ficco.FICCO_FINE_PERSISTENT, sch.FINE_PERSISTENT)]


@pytest.mark.parametrize("G,c", [(4, 1), (4, 4), (8, 2), (8, 32), (3, 5)])
@pytest.mark.parametrize("lib_s,ora_s", SCHEDS)
@pytest.mark.parametrize("order", [ficco.FICCO_ORDER_STEP_MAJOR, ficco.FICCO_ORDER_SHARD_MAJOR])
def test_plan_lists_match_oracle(G, c, lib_s, ora_s, order):
    if lib_s in (ficco.FICCO_SERIAL, ficco.FICCO_SHARD):
        c = 1
    M = G * c * 16
    plan = ficco.ficco_plan(M, 64, 8, G, c, lib_s)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_ORDER, order)
        arrival, group_ids = ficco.ficco_plan_arrival(plan)
        info = ficco.ficco_plan_info(plan)
    finally:
        ficco.ficco_destroy(plan)
    ref = sch.plan(M, G, c, ora_s, order)
    assert arrival == ref["arrival"]
    groups = [[] for _ in range(info.n_groups)]
    for chunk, g in zip(arrival, group_ids):
        groups[g].append(chunk)
    assert groups == ref["groups"]
    assert info.chunk_rows == ref["m"] and info.n_chunks == ref["n_chunks"]


def test_chaining_takes_two_different_plans():
    a = ficco.ficco_plan(512, 128, 8, 4, 2, ficco.FICCO_FINE_PERSISTENT)
    b = ficco.ficco_plan(512, 128, 8, 4, 2, ficco.FICCO_FINE_2D)
    g = ficco.ficco_plan_grouped(128, 8, [[3, 4], [5, 6]], 1, ficco.FICCO_FINE_PERSISTENT)
    try:
        ficco.ficco_plan_chain(a, b)
        ficco.ficco_plan_chain(b, a)
        ficco.ficco_plan_chain(a, None)
        ficco.ficco_plan_chain(g, a)          # grouped plans chain like the others
        ficco.ficco_plan_chain(g, None)
        for plan in (a, g):
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_plan_chain(plan, plan)
    finally:
        ficco.ficco_destroy(b)          # the plan in front goes first: the link outlives it
        ficco.ficco_destroy(a)
        ficco.ficco_destroy(g)


def test_2d_default_slices_are_as_equal_as_whole_k_tiles_allow():
    # 11 k-tiles in 4 slices: 3, 3, 3, 2 tiles
    plan = ficco.ficco_plan(64, 64 * 11, 8, 4, 4, ficco.FICCO_FINE_2D)
    try:
        k0, w = ficco.ficco_plan_slices(plan)
    finally:
        ficco.ficco_destroy(plan)
    assert w == [192, 192, 192, 128] and k0 == [0, 192, 384, 576]


def test_2d_slice_widths_are_validated_and_reported():
    M, K, G, c = 64, 64 * 8, 4, 4
    plan = ficco.ficco_plan(M, K, 8, G, c, ficco.FICCO_FINE_2D)
    rows = ficco.ficco_plan(M, K, 8, G, 2, ficco.FICCO_FINE_PERSISTENT)
    try:
        k0, w = ficco.ficco_plan_slices(plan)
        assert w == [K // c] * c and k0 == [s * (K // c) for s in range(c)]
        widths = [64 * 4, 64, 64 * 2, 64]
        ficco.ficco_plan_set_slice_widths(plan, widths)
        k0, w = ficco.ficco_plan_slices(plan)
        assert w == widths and k0 == [sum(widths[:s]) for s in range(c)]
        for s in range(c):
            for j in range(G):
                assert sch.piece_span_2d(M, K, G, c, s * G + j, widths)[2:] == (k0[s], w[s])
        # the arrival list does not depend on the widths
        assert ficco.ficco_plan_arrival(plan)[0] == sch.arrival_order_2d(G, c, sch.ORDER_STEP_MAJOR)
        for bad in (widths[:-1], [w_ + 64 for w_ in widths], [widths[0] - 32, widths[1] + 32] + widths[2:],
                    [0] + [widths[0] + widths[1]] + widths[2:]):
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_plan_set_slice_widths(plan, bad)
        assert ficco.ficco_plan_slices(plan)[1] == widths          # a rejected list changes nothing
        ficco.ficco_plan_set_slice_widths(plan, None)
        assert ficco.ficco_plan_slices(plan)[1] == [K // c] * c
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set_slice_widths(rows, [K // 2, K // 2])     # row pieces have no slices
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_slices(rows)
    finally:
        ficco.ficco_destroy(plan)
        ficco.ficco_destroy(rows)


@pytest.mark.parametrize("G,c", [(4, 1), (4, 4), (8, 2), (3, 5)])
@pytest.mark.parametrize("order", [ficco.FICCO_ORDER_STEP_MAJOR, ficco.FICCO_ORDER_SHARD_MAJOR])
def test_2d_plan_lists_match_oracle(G, c, order):
    M, K = G * 16, 64 * c
    plan = ficco.ficco_plan(M, K, 8, G, c, ficco.FICCO_FINE_2D)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_ORDER, order)
        arrival, group_ids = ficco.ficco_plan_arrival(plan)
        info = ficco.ficco_plan_info(plan)
        for opt, val in [(ficco.FICCO_OPT_LOCAL_SHARD, 1), (ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)]:
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_plan_set(plan, opt, val)
    finally:
        ficco.ficco_destroy(plan)
    ref = sch.plan(M, G, c, sch.FINE_2D, order)
    assert arrival == ref["arrival"] and set(group_ids) == {0}
    assert info.n_groups == 1 and info.chunk_rows == ref["m"] and info.n_chunks == ref["n_chunks"]
    # descriptors of one column piece: an (M/G, N, K/c) GEMM
    assert info.mt_bytes == sch.mt_bytes(M // G, 8, K // c)


def test_packing_is_an_option_of_the_fused_schedule_only():
    for sched, c, ok in [(ficco.FICCO_FINE_FUSED, 2, True), (ficco.FICCO_FINE_UNFUSED, 2, False),
                         (ficco.FICCO_FINE_PERSISTENT, 2, False), (ficco.FICCO_SERIAL, 1, False), (ficco.FICCO_FINE_2D, 2, False)]:
        plan = ficco.ficco_plan(512, 128, 8, 4, c, sched)
        try:
            if ok:
                ficco.ficco_plan_set(plan, ficco.FICCO_OPT_PACKING, 1)
                ficco.ficco_plan_set(plan, ficco.FICCO_OPT_PACKING, 0)
                with pytest.raises(ficco.FiccoError):
                    ficco.ficco_plan_set(plan, ficco.FICCO_OPT_PACKING, 2)
            else:
                with pytest.raises(ficco.FiccoError):
                    ficco.ficco_plan_set(plan, ficco.FICCO_OPT_PACKING, 1)
        finally:
            ficco.ficco_destroy(plan)


def test_tile_order_options_take_powers_of_two_up_to_eight():
    plan = ficco.ficco_plan(512, 128, 8, 4, 2, ficco.FICCO_FINE_PERSISTENT)
    try:
        for opt in (ficco.FICCO_OPT_TILE_GROUP, ficco.FICCO_OPT_TILE_COLUMN_LISTS):
            for v in (0, 1, 2, 4, 8):
                ficco.ficco_plan_set(plan, opt, v)
            for v in (-1, 3, 5, 6, 7, 16):
                with pytest.raises(ficco.FiccoError):
                    ficco.ficco_plan_set(plan, opt, v)
    finally:
        ficco.ficco_destroy(plan)


def test_custom_arrival_and_local_shard():
    plan = ficco.ficco_plan(512, 64, 8, 4, 4, ficco.FICCO_FINE_FUSED)
    try:
        rev = list(range(15, -1, -1))
        ficco.ficco_plan_set_arrival(plan, rev)
        arrival, gids = ficco.ficco_plan_arrival(plan)
        assert arrival == rev and gids == [q // 4 for q in range(16)]
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set_arrival(plan, [0] * 16)          # not a permutation
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set_arrival(plan, list(range(8)))    # wrong length
    finally:
        ficco.ficco_destroy(plan)
    plan = ficco.ficco_plan(512, 64, 8, 4, 2, ficco.FICCO_FINE_UNFUSED)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_LOCAL_SHARD, 2)
        arrival, _ = ficco.ficco_plan_arrival(plan)
        # the local shard's pieces (ids 4, 5) move to the front, the rest keep step-major order
        assert arrival == [4, 5, 0, 2, 6, 1, 3, 7]
    finally:
        ficco.ficco_destroy(plan)


@pytest.mark.parametrize("args", [
    (0, 64, 8, 4, 1, 0), (512, 0, 8, 4, 1, 0), (512, 64, 0, 4, 1, 0),     # empty dimensions
    (512, 64, 8, 0, 1, 0), (512, 64, 8, 4, 0, 2),                          # no shards / no pieces
    (500, 64, 8, 4, 2, 2),                                                  # M not divisible
    (512, 96, 8, 4, 1, 0), (512, 64, 12, 4, 1, 0),                          # K % 64, N % 8
    (512, 64, 8, 4, 2, 0), (512, 64, 8, 4, 2, 1),                           # pieces with serial / shard
    (1 << 20, 64, 8, 8192, 1, 2),                                           # too many pieces
    (512, 192, 8, 4, 4, 5), (510, 128, 8, 4, 2, 5),                         # 2D: more slices than k-tiles, M % shards
])
def test_shape_rules(args):
    with pytest.raises(ficco.FiccoError) as e:
        ficco.ficco_plan(*args)
    assert e.value.status == ficco.FICCO_ERR_SHAPE


def test_argument_errors():
    with pytest.raises(ficco.FiccoError) as e:
        ficco.ficco_plan(512, 64, 8, 4, 1, 9)
    assert e.value.status == ficco.FICCO_ERR_ARG
    plan = ficco.ficco_plan(512, 64, 8, 4, 1, ficco.FICCO_SHARD)
    try:
        for opt, val in [(ficco.FICCO_OPT_DIRECTION, 5), (ficco.FICCO_OPT_MODE, 9), (ficco.FICCO_OPT_TILE, 99),
                         (ficco.FICCO_OPT_LOCAL_SHARD, 4), (99, 0), (ficco.FICCO_OPT_SPIN_LIMIT_US, 0)]:
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_plan_set(plan, opt, val)
        with pytest.raises(ficco.FiccoError) as e:
            ficco.ficco_query_stats(plan)
        assert e.value.status == ficco.FICCO_ERR_STATE
    finally:
        ficco.ficco_destroy(plan)
    assert ficco.ficco_strerror(ficco.FICCO_ERR_TIMEOUT).startswith("resident")
    ficco.ficco_destroy(None)


@pytest.mark.parametrize("m,N,K", [(1, 1, 1), (512, 1024, 1024), (64, 768, 4096), (2048, 3584, 8192)])
def test_static_descriptors_match_oracle(m, N, K):
    otb, mt = ficco.ficco_static_descriptors(m, N, K)
    assert mt == sch.mt_bytes(m, N, K)
    assert otb == pytest.approx(sch.otb(m, N, K), rel=1e-15)


@pytest.mark.parametrize("tc,tg,n", [(3.0, 5.0, 1), (3.0, 5.0, 4), (5.0, 3.0, 8), (2.0, 2.0, 64), (1200.0, 30.0, 32)])
def test_ideal_overlap_matches_oracle(tc, tg, n):
    assert ficco.ficco_ideal_overlap_us(tc, tg, n) == pytest.approx(sch.ideal_overlap_time(tc, tg, n), rel=1e-14)


# The fitted rules of the library (Sec. V-C read for this machine) are pinned by cases worked out by hand
# from the rule as the header states it; no second implementation is consulted.
#
# Row pieces (ficco_pick_schedule): the resident schedule; pieces per shard c = the power of two up to 32 that
# divides the shard, keeps pieces of at least 256 rows and minimises
#     T(c) = max(Tc + 16 c, Tg + 8 c) + min(Tc, Tg) / c      [us]
# with Tc = (M/shards) * K * 2 B / 58e3 B/us (one shard over one link) and Tg = 2 M N K / 1.2e9 flop/us.
ROW_PIECE_CASES = [
    # Tc = 2048*8192*2/58e3 = 578.5, Tg = 801.7: T(1) = 801.7+8+578.5 = 1388.3, T(2) = 1107.0, T(4) = 978.4,
    # T(8) = 865.7+72.3 = 938.0; 16 pieces would have 128 rows
    ((16384, 8192, 3584, 8), 8),
    # Tc = 72.3, Tg = 14.3: T(1) = 88.3+14.3 = 102.6, T(2) = 104.3+7.2 = 111.5 (256-row pieces are the limit)
    ((4096, 4096, 512, 8), 1),
    # Tc = 2314.1, Tg = 12827.6: T(8) = 12891.6+289.3 = 13180.9, T(16) = 12955.6+144.6 = 13100.3, T(32) = 13156.0
    ((65536, 8192, 14336, 8), 16),
    # the 128-row shard is below the 256-row minimum -> 1 piece
    ((512, 1024, 1024, 4), 1),
    # Tc = 433.9, Tg = 171.8: T(1) = 621.7, T(2) = 465.9+85.9 = 551.8, T(4) = 497.9+43.0 = 540.8, T(8) = 583.4
    ((24576, 4096, 1024, 8), 4),
    # Tc = 144.6, Tg = 42.9: T(1) = 160.6+42.9 = 203.6, T(2) = 176.6+21.5 = 198.1, T(4) = 208.6+10.7 = 219.4
    ((8192, 4096, 768, 8), 2),
    # Tc = 289.3, Tg = 400.9: T(4) = 432.9+72.3 = 505.2, T(8) = 464.9+36.2 = 501.0
    ((16384, 4096, 3584, 8), 8),
    # Tc = 72.3, Tg = 400.9: T(1) = 408.9+72.3 = 481.2, T(2) = 416.9+36.2 = 453.0; 4 pieces would have 128 rows
    ((4096, 4096, 14336, 8), 2),
    # transfers and GEMM level (Tc = 144.6, Tg = 143.2): T(1) = 303.8, T(2) = 248.2, T(4) = 208.6+35.8 = 244.4
    ((8192, 4096, 2560, 8), 4),
    # Tc = 1157.0, Tg = 229.1: T(2) = 1189.0+114.6 = 1303.6, T(4) = 1221.0+57.3 = 1278.3, T(8) = 1285.0+28.6 = 1313.7
    ((65536, 4096, 512, 8), 4),
]


@pytest.mark.parametrize("shape,pieces", ROW_PIECE_CASES)
def test_pick_schedule_hand_cases(shape, pieces):
    assert ficco.ficco_pick_schedule(*shape) == (ficco.FICCO_FINE_PERSISTENT, pieces)


def test_pick_schedule_returns_a_valid_plan():
    for M in (4096, 16384, 65536):
        for K in (4096, 8192):
            for N in (512, 1024, 3584, 14336):
                s, c = ficco.ficco_pick_schedule(M, K, N, 8)
                assert s == ficco.FICCO_FINE_PERSISTENT
                assert 1 <= c <= 32 and (M // 8) % c == 0 and (c == 1 or M // 8 // c >= 256)
                plan = ficco.ficco_plan(M, K, N, 8, 1, ficco.FICCO_AUTO)
                info = ficco.ficco_plan_info(plan)
                ficco.ficco_destroy(plan)
                assert (info.schedule, info.chunks) == (s, c)


# Communication shape. Column pieces need an output of at most 256 tiles of 256x256 (one round over 256 CUs:
# ceil(M/256) * ceil(N/256) <= 256) and at least two k-tiles of 64. For a sender that holds its slices K-sliced
# (ficco_pick_schedule_layout, K_SLICED) that is all: slices 2 when N*shards <= 8192 (the transfers are the longer
# side), else 2 below 1e11 flop, 4 below 4e11, 8 from there, never more than K/64. For the caller's row-major
# matrix (ficco_pick_schedule_any = layout ROW_MAJOR) the step pays for the re-layout, so column pieces also need
# N*shards > 8192 and at least 2e11 flop: 4 slices below 4e11 flop, 8 from there. Otherwise the row-piece answer.
K_SLICED_CASES = [
    # 8192*768 = 6.3e6 outputs; N*G = 6144 -> 2 slices
    ((8192, 4096, 768, 8), (ficco.FICCO_FINE_2D, 2)),
    # 4096*4096 = 1.7e7 outputs; N*G = 32768; 2*4096*4096*16384 = 5.5e11 flop -> 8 slices
    ((4096, 16384, 4096, 8), (ficco.FICCO_FINE_2D, 8)),
    # 4096*3584 = 1.5e7 outputs; 2*4096*3584*8192 = 2.4e11 flop -> 4 slices
    ((4096, 8192, 3584, 8), (ficco.FICCO_FINE_2D, 4)),
    # 16384*3584 = 5.9e7 outputs: several rounds of tiles -> row pieces, 8 per shard (worked above)
    ((16384, 8192, 3584, 8), (ficco.FICCO_FINE_PERSISTENT, 8)),
    # 4096*14336 = 5.9e7 outputs -> row pieces, 2 per shard (worked above)
    ((4096, 4096, 14336, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # one k-tile: nothing to slice; Tc = 1.1, Tg = 0.2: T(1) = 17.1+0.2 = 17.4, T(2) = 33.2 -> 1 piece
    ((4096, 64, 512, 8), (ficco.FICCO_FINE_PERSISTENT, 1)),
    # two k-tiles, N*G = 4096 -> 2 slices
    ((4096, 128, 512, 8), (ficco.FICCO_FINE_2D, 2)),
    # 1.7e7 outputs, 1.4e11 flop, but N*G = 8192: the transfers are the longer side -> 2 slices
    ((16384, 4096, 1024, 8), (ficco.FICCO_FINE_2D, 2)),
    # 4096*4096 outputs, N*G = 32768, 2*4096*4096*2048 = 6.9e10 flop -> 2 slices
    ((4096, 2048, 4096, 8), (ficco.FICCO_FINE_2D, 2)),
    # either side of the limit: 16 x 16 = 256 tiles, 2*4096*4096*8192 = 2.7e11 flop -> 4 slices ...
    ((4096, 8192, 4096, 8), (ficco.FICCO_FINE_2D, 4)),
    # ... 16 x 17 = 272 tiles -> row pieces; Tc = 144.6, Tg = 229.5: T(1) = 382.1, T(2) = 245.5+72.3 = 317.8 -> 2
    ((4096, 8192, 4104, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
]
ROW_MAJOR_CASES = [
    # N*G = 6144: transfer-bound -> row pieces, 2 per shard (worked above)
    ((8192, 4096, 768, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # N*G = 32768, 5.5e11 flop -> 8 slices
    ((4096, 16384, 4096, 8), (ficco.FICCO_FINE_2D, 8)),
    # N*G = 28672, 2.4e11 flop -> 4 slices
    ((4096, 8192, 3584, 8), (ficco.FICCO_FINE_2D, 4)),
    # N*G = 28672 but 2*4096*3584*4096 = 1.2e11 flop: too little GEMM to hide the re-layout -> row pieces;
    # Tc = 72.3, Tg = 100.2: T(1) = 108.2+72.3 = 180.5, T(2) = 116.2+36.2 = 152.4 -> 2 pieces
    ((4096, 4096, 3584, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # N*G = 8192 counts as transfer-bound -> row pieces; Tc = 289.3, Tg = 114.5: T(1) = 419.8, T(2) = 321.3+57.3 =
    # 378.5, T(4) = 353.3+28.6 = 381.9 -> 2 pieces
    ((16384, 4096, 1024, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # 6.9e10 flop -> row pieces; Tc = 36.2, Tg = 57.3: T(1) = 65.3+36.2 = 101.4, T(2) = 73.3+18.1 = 91.3 -> 2 pieces
    ((4096, 2048, 4096, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # large outputs stay with row pieces whatever the layout
    ((16384, 8192, 3584, 8), (ficco.FICCO_FINE_PERSISTENT, 8)),
    ((4096, 4096, 14336, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # either side of the output limit (256 and 272 tiles) at 2.7e11 flop
    ((4096, 8192, 4096, 8), (ficco.FICCO_FINE_2D, 4)),
    ((4096, 8192, 4104, 8), (ficco.FICCO_FINE_PERSISTENT, 2)),
    # the tiny configuration: 512 x 1024 x 1024 on 4 shards, 1e9 flop -> row pieces, 1 per shard (worked above)
    ((512, 1024, 1024, 4), (ficco.FICCO_FINE_PERSISTENT, 1)),
]


@pytest.mark.parametrize("shape,answer", K_SLICED_CASES)
def test_pick_schedule_k_sliced_source_hand_cases(shape, answer):
    assert ficco.ficco_pick_schedule_layout(*shape, ficco.FICCO_LAYOUT_K_SLICED) == answer


@pytest.mark.parametrize("shape,answer", ROW_MAJOR_CASES)
def test_pick_schedule_any_hand_cases(shape, answer):
    assert ficco.ficco_pick_schedule_any(*shape) == answer
    assert ficco.ficco_pick_schedule_layout(*shape, ficco.FICCO_LAYOUT_ROW_MAJOR) == answer


# The cut of the k range (ficco_pick_slice_widths): two slices of a transfer-bound shape (N*shards <= 8192)
# take three quarters and one quarter of the k-tiles (first = (3*kt + 2) // 4 k-tiles, at least one tile
# each); everything else as even as whole k-tiles allow, the first kt mod slices one tile wider.
SLICE_WIDTH_CASES = [
    ((8192, 4096, 768, 8, 2), [3072, 1024]),               # kt = 64 -> 48 + 16 tiles
    ((4096, 128, 512, 8, 2), [64, 64]),                    # kt = 2 -> (6+2)//4 = 2, capped at kt-1 = 1 tile
    ((4096, 192, 512, 8, 2), [128, 64]),                   # kt = 3 -> (9+2)//4 = 2 tiles + 1
    ((4096, 4096, 3584, 8, 4), [1024] * 4),
    ((4096, 4096, 3584, 8, 2), [2048, 2048]),              # N*G = 28672: not transfer-bound
    ((64, 704, 8, 8, 4), [192, 192, 192, 128]),            # kt = 11 = 4*2 + 3: three slices of 3 tiles, one of 2
    ((4096, 8192, 1024, 8, 2), [6144, 2048]),              # N*G = 8192 counts as transfer-bound; kt = 128 -> 96 + 32
]


@pytest.mark.parametrize("args,widths", SLICE_WIDTH_CASES)
def test_pick_slice_widths_hand_cases(args, widths):
    assert ficco.ficco_pick_slice_widths(*args) == widths


def test_pick_slice_widths_rejects_bad_arguments():
    for bad in ((4096, 4096, 512, 8, 0), (4096, 100, 512, 8, 1), (4096, 128, 512, 8, 3)):
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_pick_slice_widths(*bad)


def test_pick_schedule_any_gives_valid_plans_with_its_own_cut():
    for M in (512, 4096, 8192, 16384, 65536):
        for K in (64, 128, 4096, 8192, 16384):
            for N in (8, 512, 768, 1024, 3584, 4096, 14336):
                s, c = ficco.ficco_pick_schedule_any(M, K, N, 8)
                plan = ficco.ficco_plan(M, K, N, 8, c, s)          # whatever it answers can be planned
                ficco.ficco_destroy(plan)
                plan = ficco.ficco_plan(M, K, N, 8, 1, ficco.FICCO_AUTO_ANY)
                info = ficco.ficco_plan_info(plan)
                widths = ficco.ficco_plan_slices(plan)[1] if s == ficco.FICCO_FINE_2D else None
                ficco.ficco_destroy(plan)
                assert (info.schedule, info.chunks) == (s, c)
                if s == ficco.FICCO_FINE_2D:
                    assert -(-M // 256) * -(-N // 256) <= 256 and 2 <= c <= K // 64 and N * 8 > 8192 and 2.0 * M * N * K >= 2e11
                    assert widths == ficco.ficco_pick_slice_widths(M, K, N, 8, c)
                    assert len(widths) == c and sum(widths) == K and all(w > 0 and w % 64 == 0 for w in widths)
                else:
                    assert (s, c) == ficco.ficco_pick_schedule(M, K, N, 8)


RS_PIECE_CASES = [
    # reduce-scatter direction: a link carries (M/G) x N output elements. M 16384, K 3584, N 8192, G 8:
    # Tc = 2048*8192*2/58e3 = 578.5 us, Tg = 2*16384*8192*3584/1.2e9 = 801.6 us;
    # T(1) = 809.6 + 578.5 = 1388.1, T(2) = 817.6 + 289.3 = 1106.9, T(4) = 833.6 + 144.6 = 978.2,
    # T(8) = 865.6 + 72.3 = 937.9; 16 pieces would be 128 rows each (< 256) -> 8
    ((16384, 3584, 8192, 8), 8),
    # M 8192, K 4096, N 768: Tc = 1024*768*2/58e3 = 27.1 us, Tg = 43.0 us;
    # T(1) = 51.0 + 27.1 = 78.1, T(2) = max(59.1, 59.0) + 13.6 = 72.7, T(4) = max(91.1, 75.0) + 6.8 = 97.9 -> 2
    ((8192, 4096, 768, 8), 2),
]


@pytest.mark.parametrize("shape,pieces", RS_PIECE_CASES)
def test_reduce_scatter_piece_rule_hand_cases(shape, pieces):
    assert ficco.ficco_pick_schedule_rs(*shape) == (ficco.FICCO_FINE_PERSISTENT, pieces)
    M, K, N, G = shape
    assert (M // G) % pieces == 0


def test_host_resident_row_major_shards_never_get_column_pieces():
    """Strided rectangles out of pinned host memory all go through one engine: the rule keeps row pieces, the
    answer of ficco_pick_schedule, for every shape; a plan does not take the hint as an option (the run sees
    where A_src lives)."""
    for shape, _ in ROW_MAJOR_CASES + K_SLICED_CASES:
        assert ficco.ficco_pick_schedule_layout(*shape, ficco.FICCO_LAYOUT_ROW_MAJOR_HOST) == ficco.ficco_pick_schedule(*shape)
    plan = ficco.ficco_plan(4096, 8192, 3584, 8, 4, ficco.FICCO_FINE_2D)
    try:
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_ROW_MAJOR_HOST)
    finally:
        ficco.ficco_destroy(plan)
    with pytest.raises(ficco.FiccoError):
        ficco.ficco_pick_schedule_layout(4096, 8192, 3584, 8, 3)


def test_source_layout_option_belongs_to_column_pieces():
    plan = ficco.ficco_plan(512, 1024, 1024, 4, 2, ficco.FICCO_FINE_2D)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_ROW_MAJOR)
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, 2)
    finally:
        ficco.ficco_destroy(plan)
    plan = ficco.ficco_plan(512, 1024, 1024, 4, 2, ficco.FICCO_FINE_PERSISTENT)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_ROW_MAJOR)
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
    finally:
        ficco.ficco_destroy(plan)


# ------------------------------------------------------------------ expert-parallel (grouped) plans
from oracle import grouped as ogr  # noqa: E402


@pytest.mark.parametrize("rows,c,sched", [([[3, 0], [5, 2], [0, 7]], 2, ficco.FICCO_FINE_PERSISTENT),
                                          ([[40], [13], [0], [91]], 4, ficco.FICCO_FINE_PERSISTENT),
                                          ([[10, 20, 30], [5, 0, 1]], 1, ficco.FICCO_SHARD),
                                          ([[10, 20], [7, 9]], 1, ficco.FICCO_SERIAL)])
def test_grouped_plan_layout_and_arrival_match_oracle(rows, c, sched):
    G, E = len(rows), len(rows[0])
    plan = ficco.ficco_plan_grouped(64, 8, rows, c, sched)
    try:
        r0, nr = ficco.ficco_plan_pieces(plan)
        arrival, gids = ficco.ficco_plan_arrival(plan)
        info = ficco.ficco_plan_info(plan)
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)
        by_peer, _ = ficco.ficco_plan_arrival(plan)
        for opt, val in [(ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS), (ficco.FICCO_OPT_LOCAL_SHARD, 0),
                         (ficco.FICCO_OPT_PACKING, 1), (ficco.FICCO_OPT_TIMING, 1)]:
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_plan_set(plan, opt, val)
    finally:
        ficco.ficco_destroy(plan)
    o_r0, o_nr, _, _ = ogr.layout(rows, c)
    assert r0 == list(o_r0) and nr == list(o_nr)
    assert info.M == sum(map(sum, rows)) and info.n_chunks == G * E * c and info.shards == G and set(gids) == {0}
    assert arrival == ogr.arrival_order(G, E, c, step_major=sched != ficco.FICCO_SHARD)
    assert by_peer == ogr.arrival_order(G, E, c, step_major=False)


@pytest.mark.parametrize("args,status", [
    ((64, 8, [[0, 0]], 1, 4), "SHAPE"), ((64, 8, [[-1, 2]], 1, 4), "SHAPE"), ((96, 8, [[4]], 1, 4), "SHAPE"),
    ((64, 12, [[4]], 1, 4), "SHAPE"), ((64, 8, [[4]], 2, 0), "SHAPE"), ((64, 8, [[4]] * 70, 64, 4), "SHAPE"),
    ((64, 8, [[4]], 1, 2), "ARG"), ((64, 8, [[4]], 1, 3), "ARG"), ((64, 8, [[4]], 1, 5), "ARG")])
def test_grouped_plan_rules(args, status):
    with pytest.raises(ficco.FiccoError) as e:
        ficco.ficco_plan_grouped(*args)
    assert e.value.status == getattr(ficco, "FICCO_ERR_" + status)


def test_library_path_can_be_overridden_for_measuring_builds(monkeypatch, tmp_path):
    """FICCO_LIBRARY names a measuring build (see _build.build_variant); without it the in-tree library is used,
    and a path that does not exist is an error, not a fallback."""
    from paper_2512_10236_amd import _build, binding
    monkeypatch.delenv("FICCO_LIBRARY", raising=False)
    assert binding.library_path() == _build.LIB
    other = str(tmp_path / "libficco_other.so")
    monkeypatch.setenv("FICCO_LIBRARY", other)
    assert binding.library_path() == other
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(RuntimeError):
        binding.load()


def test_row_strides_beyond_the_loaders_reach_are_refused():
    """The kernels address a tile's rows with 32-bit byte offsets: K (the row stride of A and of the packed
    weight) is limited to 2^22 elements, and a plan beyond that is a shape error, not a launch."""
    K = (1 << 22) + 64
    with pytest.raises(ficco.FiccoError):
        ficco.ficco_plan(1024, K, 256, 8, 1, ficco.FICCO_SERIAL)
    plan = ficco.ficco_plan(1024, 1 << 22, 256, 8, 1, ficco.FICCO_SERIAL)
    ficco.ficco_destroy(plan)
