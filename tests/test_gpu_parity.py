"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
seeded inputs; plus bit-equality across schedules, dependency checks (NaN-poisoned destination,
delayed and reordered transfers) and the error path of the resident kernel's bounded wait.

Tolerance: max |gpu - ref| / (|ref| + 1) <= 8e-3 (one bf16 output rounding is <= 2^-8 relative;
fp32 accumulation over K <= 8192 unit-variance products adds far less)."""
import numpy as np
import pytest

import ficco_inputs as fi
import paper_2512_10236_amd as ficco
from oracle import gemm as og

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 8e-3
NAN_BF16 = 0x7FC0
STREAM, ENGINES = ficco.FICCO_COPY_STREAM, ficco.FICCO_COPY_ENGINES
BACKENDS = [STREAM, ENGINES]
ALL_SCHEDULES = [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1), (ficco.FICCO_FINE_UNFUSED, 4),
                 (ficco.FICCO_FINE_FUSED, 4), (ficco.FICCO_FINE_PERSISTENT, 4)]


def as_i16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))


def widen(bits):
    return fi.bf16_bits_to_f32(bits).astype(np.float64)


def run_ag(gpu, shards, W, schedule, c, *, src="pinned", opts=(), arrival=None, delay_copy=False,
           timing=0, allow_timeout=False, runs=1, local_shard=None, backend=None, widths=None, row_major=False):
    """One all-gather -> GEMM through the C ABI; returns (C bits, stats). ``widths``: column pieces of
    these widths (FICCO_FINE_2D, ``c`` = their number) instead of equal ones. Column pieces travel out of a
    K-sliced source (FICCO_LAYOUT_K_SLICED) unless ``row_major`` asks for the caller's own layout."""
    dev = gpu["dev"]
    A = np.concatenate(shards, 0)
    M, K = A.shape
    N = W.shape[1]
    G = len(shards)
    k_sliced = schedule == ficco.FICCO_FINE_2D and not row_major
    if k_sliced:
        if widths is None and K % c == 0:
            A = fi.to_k_sliced(A, c).reshape(M, K)         # same bytes, column pieces contiguous
        else:
            if widths is None:                             # the library's own cut into whole k-tiles
                probe = ficco.ficco_plan(M, K, N, G, c, schedule)
                widths = ficco.ficco_plan_slices(probe)[1]
                ficco.ficco_destroy(probe)
                assert sum(widths) == K and len(widths) == c and max(widths) - min(widths) <= 64
            assert len(widths) == c
            A = np.concatenate([b.ravel() for b in fi.to_k_pieces(A, widths)]).reshape(M, K)
    A_src = as_i16(A).pin_memory() if src == "pinned" else as_i16(A).to(dev)
    W_dev = as_i16(W).to(dev)
    A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)     # poison: unread rows show up as NaN
    C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    ms = M // G

    def place_local():
        if local_shard is not None:                     # the local shard is already in place, nothing moves it
            A_dev[local_shard * ms:(local_shard + 1) * ms] = as_i16(A[local_shard * ms:(local_shard + 1) * ms]).to(dev)

    place_local()
    torch.cuda.synchronize()
    plan = ficco.ficco_plan(M, K, N, G, c, schedule)
    try:
        if local_shard is not None:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_LOCAL_SHARD, local_shard)
        if backend is not None:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_COPY_BACKEND, backend)
        for o, v in opts:
            ficco.ficco_plan_set(plan, o, v)
        if widths is not None:
            ficco.ficco_plan_set_slice_widths(plan, widths)
        if k_sliced:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
        if arrival is not None:
            ficco.ficco_plan_set_arrival(plan, arrival)
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_TIMING, timing)
        for r in range(runs):
            if r:
                A_dev.fill_(NAN_BF16)
                place_local()
                torch.cuda.synchronize()
            if delay_copy:
                with torch.cuda.stream(gpu["xs"]):
                    torch.cuda._sleep(40_000_000)          # tens of ms before the first transfer may start
            ficco.ficco_run(plan, A_src, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
            st = ficco.ficco_query_stats(plan, allow_timeout=allow_timeout)
        info = ficco.ficco_plan_info(plan)
    finally:
        ficco.ficco_destroy(plan)
    torch.cuda.synchronize()
    return C_dev.cpu().numpy().view(np.uint16), st, info


def check(bits, ref, what=""):
    out = widen(bits)
    assert np.isfinite(out).all(), f"{what}: non-finite output (a tile ran before its rows landed?)"
    err = og.rel_err(out, ref)
    assert err <= TOL, f"{what}: rel err {err}"
    return err


# ------------------------------------------------------------------------------------------------
def test_cfg1_all_schedules_match_oracle_and_each_other(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    ref = og.ag_gemm(shards, W)
    base = None
    for backend in BACKENDS + [None]:
        for sched, c in ALL_SCHEDULES + [(ficco.FICCO_FINE_UNFUSED, 1), (ficco.FICCO_FINE_PERSISTENT, 1)]:
            bits, st, info = run_ag(gpu, shards, W, sched, c, backend=backend)
            check(bits, ref, ficco.SCHEDULE_NAMES[sched])
            if base is None:
                base = bits
            assert np.array_equal(bits, base), f"{ficco.SCHEDULE_NAMES[sched]} c={c} backend {backend} differs bitwise from serial"
            assert st.n_copies == info.n_chunks and st.copy_bytes == 512 * 1024 * 2
            assert st.wall_us > 0 and st.flops == 2 * 512 * 1024 * 1024
            # without a request the library moves the pieces with the copy engines
            assert info.copy_backend == (backend if backend is not None else ENGINES)


@pytest.mark.parametrize("tile", [ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_256x128,
                                  ficco.FICCO_TILE_128x256, ficco.FICCO_TILE_64x256, ficco.FICCO_TILE_32x256,
                                  ficco.FICCO_TILE_128x128_DEEP, ficco.FICCO_TILE_128x192, ficco.FICCO_TILE_256x192])
def test_every_tile_shape_ragged(gpu, tile):
    # 3 shards x 2 pieces of 88 rows (no tile height divides it), N = 328 (not a tile width), K = 192
    G, c, m, K, N = 3, 2, 88, 192, 328
    shards = fi.make_shards(21, G * c * m, K, G)
    W = fi.make_weight(21, K, N)
    ref = og.ag_gemm(shards, W)
    outs = []
    for sched, cc, backend in [(ficco.FICCO_SERIAL, 1, STREAM), (ficco.FICCO_FINE_FUSED, c, STREAM), (ficco.FICCO_FINE_FUSED, c, ENGINES),
                               (ficco.FICCO_FINE_PERSISTENT, c, ENGINES)]:
        bits, _, info = run_ag(gpu, shards, W, sched, cc, opts=[(ficco.FICCO_OPT_TILE, tile)], backend=backend)
        check(bits, ref, f"tile {tile} sched {sched}")
        outs.append(bits)
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    test_every_tile_shape_ragged.results = getattr(test_every_tile_shape_ragged, "results", []) + [outs[0]]
    # tile shape must not change the bits either
    assert np.array_equal(test_every_tile_shape_ragged.results[0], outs[0])


@pytest.mark.parametrize("seed", [101, 102, 103, 104, 105, 106])
def test_seeded_random_shapes_schedules_and_options(gpu, seed):
    """Shapes, piece counts, schedules, tiles, tile orders, sources, backends, arrival orders and slice widths
    drawn from a seeded generator (the same cases every run): whatever the combination, the result is within
    tolerance of the oracle and bitwise that of the serial schedule."""
    rng = np.random.default_rng(seed)
    tiles = [ficco.FICCO_TILE_AUTO, ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_256x128, ficco.FICCO_TILE_128x256,
             ficco.FICCO_TILE_64x256, ficco.FICCO_TILE_32x256, ficco.FICCO_TILE_128x128_DEEP, ficco.FICCO_TILE_128x192, ficco.FICCO_TILE_256x192]
    G = int(rng.choice([1, 2, 3, 4, 8]))
    c = int(rng.choice([1, 2, 3, 4, 6]))
    m = int(rng.choice([8, 24, 40, 72, 136, 264]))            # rows of a piece: below, across and above the tile heights
    kt = int(rng.integers(1, 9))                              # k-tiles of 64
    K, N = 64 * kt, 8 * int(rng.integers(1, 90))
    shards = fi.make_shards(seed, G * c * m, K, G)
    W = fi.make_weight(seed, K, N)
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    check(base, ref, f"serial G={G} c={c} m={m} K={K} N={N}")
    for case in range(5):
        sched = int(rng.choice([ficco.FICCO_SHARD, ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT, ficco.FICCO_FINE_2D]))
        opts = [(ficco.FICCO_OPT_TILE, int(rng.choice(tiles)))]
        if rng.random() < 0.5:
            opts.append((ficco.FICCO_OPT_TILE_GROUP, int(rng.choice([1, 2, 4, 8]))))
        src = "device" if rng.random() < 0.5 else "pinned"
        backend = None if sched == ficco.FICCO_FINE_2D or rng.random() < 0.6 else int(rng.choice([STREAM, ENGINES]))
        kw = {}
        cc = 1 if sched == ficco.FICCO_SHARD else c
        if sched == ficco.FICCO_FINE_2D:
            n_sl = int(rng.integers(1, min(kt, 5) + 1))
            cuts = np.sort(rng.choice(np.arange(1, kt), size=n_sl - 1, replace=False)) if n_sl > 1 else np.array([], dtype=int)
            edges = np.concatenate([[0], cuts, [kt]])
            kw["widths"] = [int(64 * (edges[i + 1] - edges[i])) for i in range(n_sl)]
            cc = n_sl
        elif rng.random() < 0.4:
            opts.append((ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR))
        if rng.random() < 0.3 and sched != ficco.FICCO_SHARD:
            n_pieces = G * cc
            kw["arrival"] = [int(i) for i in rng.permutation(n_pieces)]
        what = f"seed {seed} case {case}: G={G} c={cc} m={m} K={K} N={N} sched={sched} opts={opts} src={src} backend={backend} {kw}"
        bits, st, _ = run_ag(gpu, shards, W, sched, cc, src=src, opts=opts, backend=backend, runs=2, **kw)
        assert np.array_equal(bits, base), what
        assert st.copy_bytes == G * c * m * K * 2, what


@pytest.mark.parametrize("seed", [111, 112, 113, 114])
def test_seeded_random_gemm_rs(gpu, seed):
    """GEMM -> reduce-scatter (data movement half) over shapes, piece counts, schedules, tiles, tile orders, peer
    kinds and backends drawn from a seeded generator: every peer receives its row block of the oracle's
    product, bitwise what the serial schedule delivers."""
    dev = gpu["dev"]
    rng = np.random.default_rng(seed)
    tiles = [ficco.FICCO_TILE_AUTO, ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_256x128, ficco.FICCO_TILE_128x256,
             ficco.FICCO_TILE_64x256, ficco.FICCO_TILE_32x256, ficco.FICCO_TILE_128x128_DEEP, ficco.FICCO_TILE_128x192, ficco.FICCO_TILE_256x192]
    G = int(rng.choice([1, 2, 4, 8]))
    c = int(rng.choice([1, 2, 3, 4]))
    m = int(rng.choice([8, 24, 72, 136, 264]))
    K, N = 64 * int(rng.integers(1, 7)), 8 * int(rng.integers(1, 90))
    M = G * c * m
    A = fi.normal_bf16(seed, fi.TENSOR_A, M, K)
    W = fi.make_weight(seed, K, N)
    blocks = og.gemm_rs_blocks(A, W, G)
    A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
    base = None
    cases = [(ficco.FICCO_SERIAL, 1, "device", None, [])]
    for _ in range(5):
        sched = int(rng.choice([ficco.FICCO_SHARD, ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT]))
        kind = "device" if rng.random() < 0.6 else "pinned"
        backend = None if rng.random() < 0.5 else int(rng.choice([STREAM, ENGINES]))
        if sched == ficco.FICCO_FINE_PERSISTENT and backend == STREAM:
            backend = ENGINES                                  # the kernel releases copy-engine transfers
        opts = [(ficco.FICCO_OPT_TILE, int(rng.choice(tiles)))]
        if rng.random() < 0.5:
            opts.append((ficco.FICCO_OPT_TILE_GROUP, int(rng.choice([1, 2, 4, 8]))))
        cases.append((sched, 1 if sched == ficco.FICCO_SHARD else c, kind, backend, opts))
    for sched, cc, kind, backend, opts in cases:
        what = f"seed {seed}: G={G} c={cc} m={m} K={K} N={N} sched={sched} peers={kind} backend={backend} opts={opts}"
        C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
        peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16, device=dev) if kind == "device"
                 else torch.full((M // G, N), NAN_BF16, dtype=torch.int16).pin_memory() for _ in range(G)]
        torch.cuda.synchronize()
        plan = ficco.ficco_plan(M, K, N, G, cc, sched)
        try:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
            if backend is not None:
                ficco.ficco_plan_set(plan, ficco.FICCO_OPT_COPY_BACKEND, backend)
            for o, v in opts:
                ficco.ficco_plan_set(plan, o, v)
            for rep_ in range(2):
                for p_ in peers:
                    p_.fill_(NAN_BF16)
                torch.cuda.synchronize()
                ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, peers, gpu["cs"], gpu["xs"])
                st = ficco.ficco_query_stats(plan)
        finally:
            ficco.ficco_destroy(plan)
        torch.cuda.synchronize()
        got = np.concatenate([p_.cpu().numpy().view(np.uint16) for p_ in peers], 0)
        if base is None:
            for j in range(G):
                check(got[j * (M // G):(j + 1) * (M // G)], blocks[j], what)
            base = got
        assert np.array_equal(got, base), what
        assert np.array_equal(got, C_dev.cpu().numpy().view(np.uint16)), what
        assert st.copy_bytes == M * N * 2, what


def test_every_tile_order_gives_the_same_bits(gpu):
    # 42 row tiles x 9 column tiles of 32x256 (both ragged): more tiles than workgroups that fit, so the
    # resident kernels draw tickets and steal, and the one-launch kernel loops
    G, c, m, K, N = 3, 2, 200, 192, 2104
    shards = fi.make_shards(27, G * c * m, K, G)
    W = fi.make_weight(27, K, N)
    ref = og.ag_gemm(shards, W)
    tile = [(ficco.FICCO_OPT_TILE, ficco.FICCO_TILE_32x256)]
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, opts=tile)
    check(base, ref, "serial")
    for g in (1, 2, 4, 8):
        order = tile + [(ficco.FICCO_OPT_TILE_GROUP, g)]
        for sched, cc in ((ficco.FICCO_SERIAL, 1), (ficco.FICCO_FINE_FUSED, c)):
            bits, _, _ = run_ag(gpu, shards, W, sched, cc, opts=order)
            assert np.array_equal(bits, base), f"group {g} sched {sched}"
        for cl in (1, 2, 4, 8):
            lists = order + [(ficco.FICCO_OPT_TILE_COLUMN_LISTS, cl)]
            bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_PERSISTENT, c, src="device", opts=lists)
            assert np.array_equal(bits, base), f"resident, group {g}, {cl} column lists"
            bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, 3, src="device", opts=lists)
            assert np.array_equal(bits, base), f"column pieces, group {g}, {cl} column lists"
    # more column lists than column tiles (1024 columns are 4 tiles of 256): refused when the run is enqueued
    shards, W = fi.config_inputs("cfg1_tiny")
    with pytest.raises(ficco.FiccoError):
        run_ag(gpu, shards, W, ficco.FICCO_FINE_PERSISTENT, 4, src="device",
               opts=[(ficco.FICCO_OPT_TILE, ficco.FICCO_TILE_256x256), (ficco.FICCO_OPT_TILE_COLUMN_LISTS, 8)])


def test_closed_forms_on_gpu(gpu):
    G, ms, K = 4, 96, 256
    M = G * ms
    # identity: C == A bit for bit
    shards = fi.make_shards(5, M, K, G)
    eye = fi.f32_to_bf16_bits(np.eye(K, dtype=np.float32))
    for sched, c in ALL_SCHEDULES:
        bits, _, _ = run_ag(gpu, shards, eye, sched, c)
        assert np.array_equal(bits, np.concatenate(shards, 0)), sched
    # all ones: every entry equals K exactly (K is representable in bf16)
    one = [np.full((ms, K), 0x3F80, np.uint16)] * G
    Wone = np.full((K, 64), 0x3F80, np.uint16)
    bits, _, _ = run_ag(gpu, one, Wone, ficco.FICCO_FINE_PERSISTENT, 2)
    assert np.array_equal(widen(bits), np.full((M, 64), float(K)))
    # row selector: C[i,:] = W[i mod K,:] bit for bit - a misplaced piece cannot hide
    A = np.zeros((M, K), np.float32)
    A[np.arange(M), np.arange(M) % K] = 1.0
    Ab = fi.f32_to_bf16_bits(A)
    W = fi.make_weight(9, K, 136)
    for sched, c in ALL_SCHEDULES:
        bits, _, _ = run_ag(gpu, [Ab[j * ms:(j + 1) * ms] for j in range(G)], W, sched, c)
        assert np.array_equal(bits, W[np.arange(M) % K]), sched
    # power-of-two scaling is exact
    b1, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SHARD, 1)
    twice = [fi.f32_to_bf16_bits(2.0 * fi.bf16_bits_to_f32(s)) for s in shards]
    b2, _, _ = run_ag(gpu, twice, W, ficco.FICCO_SHARD, 1)
    assert np.array_equal(widen(b2), 2.0 * widen(b1))


def test_arrival_order_and_delay_do_not_change_bits(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    n = 16
    rng = np.random.default_rng(0)
    orders = [list(range(n - 1, -1, -1)), list(rng.permutation(n))]
    for sched in (ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT):
        for backend in BACKENDS:
            for arr in orders:
                bits, _, _ = run_ag(gpu, shards, W, sched, 4, arrival=arr, backend=backend)
                assert np.array_equal(bits, base), (sched, arr, backend)
            bits, _, _ = run_ag(gpu, shards, W, sched, 4, opts=[(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)], backend=backend)
            assert np.array_equal(bits, base)
        # transfers held back for tens of ms on the copy stream: the GEMM must wait for them (poison would show)
        bits, st, _ = run_ag(gpu, shards, W, sched, 4, delay_copy=True, backend=STREAM)
        assert np.array_equal(bits, base), sched


def test_repeated_runs_and_timing_spans(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    for backend in BACKENDS:
        for sched, c in ALL_SCHEDULES:
            bits, st, info = run_ag(gpu, shards, W, sched, c, timing=1, runs=3, backend=backend)
            assert np.array_equal(bits, base)
            assert st.run_index == 3 and st.n_launches == info.n_groups
            assert 0 < st.gemm_busy_us <= st.wall_us * 1.05
            assert 0 < st.copy_span_us <= st.wall_us * 1.05


def test_flag_written_by_stream_write_value(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    stream = (ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)
    for fw in (0, 1):
        bits, _, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_PERSISTENT, 4, opts=[stream, (ficco.FICCO_OPT_FLAG_WRITE, fw)], runs=2)
        assert np.array_equal(bits, base) and info.copy_backend == ficco.FICCO_COPY_STREAM


def test_device_staging_source(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    for sched, c in ALL_SCHEDULES:
        bits, _, _ = run_ag(gpu, shards, W, sched, c, src="device")
        assert np.array_equal(bits, base)


def test_local_shard_needs_no_transfer(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    ref = og.ag_gemm(shards, W)
    dev = gpu["dev"]
    A = np.concatenate(shards, 0)
    M, K, N, G = 512, 1024, 1024, 4
    for sched, backend in [(s_, b_) for s_ in (ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT)
                           for b_ in BACKENDS]:
        A_src = as_i16(A).pin_memory()
        A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
        A_dev[256:384] = as_i16(A[256:384]).to(dev)            # shard 2 is already here
        C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
        W_dev = as_i16(W).to(dev)
        torch.cuda.synchronize()
        plan = ficco.ficco_plan(M, K, N, G, 4, sched)
        try:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_LOCAL_SHARD, 2)
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_COPY_BACKEND, backend)
            ficco.ficco_run(plan, A_src, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
            st = ficco.ficco_query_stats(plan)
        finally:
            ficco.ficco_destroy(plan)
        assert st.n_copies == 12 and st.copy_bytes == 384 * 1024 * 2
        check(C_dev.cpu().numpy().view(np.uint16), ref, f"local shard, sched {sched}")


def test_gemm_rs_streams_row_blocks_to_peers(gpu):
    dev = gpu["dev"]
    M, K, N, G = 1024, 256, 512, 8
    A = fi.normal_bf16(3, fi.TENSOR_A, M, K)
    W = fi.make_weight(3, K, N)
    blocks = og.gemm_rs_blocks(A, W, G)
    base = None
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1), (ficco.FICCO_FINE_UNFUSED, 4), (ficco.FICCO_FINE_FUSED, 2),
                     (ficco.FICCO_FINE_PERSISTENT, 4), (ficco.FICCO_FINE_PERSISTENT, 1)]:
        for kind, backend in (("device", None), ("pinned", STREAM), ("pinned", ENGINES)):
            if sched == ficco.FICCO_FINE_PERSISTENT and backend == STREAM:
                continue                                   # the kernel releases copy-engine transfers: engine backend only
            A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
            C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
            if kind == "device":
                peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16, device=dev) for _ in range(G)]
            else:
                peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16).pin_memory() for _ in range(G)]
            torch.cuda.synchronize()
            plan = ficco.ficco_plan(M, K, N, G, c, sched)
            try:
                ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
                if backend is not None:
                    ficco.ficco_plan_set(plan, ficco.FICCO_OPT_COPY_BACKEND, backend)
                for rep_ in range(2):                     # twice: the per-piece tile counters are never reset
                    for p_ in peers:
                        p_.fill_(NAN_BF16)
                    torch.cuda.synchronize()
                    ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, peers, gpu["cs"], gpu["xs"])
                    st = ficco.ficco_query_stats(plan)
            finally:
                ficco.ficco_destroy(plan)
            torch.cuda.synchronize()
            got = [p.cpu().numpy().view(np.uint16) for p in peers]
            for j in range(G):
                check(got[j], blocks[j], f"peer {j} {kind} sched {sched}")
            allbits = np.concatenate(got, 0)
            assert np.array_equal(allbits, C_dev.cpu().numpy().view(np.uint16))
            if base is None:
                base = allbits
            assert np.array_equal(allbits, base)
            assert st.copy_bytes == M * N * 2 and st.n_copies == G * c


@pytest.mark.parametrize("tile", [ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_256x128,
                                  ficco.FICCO_TILE_128x256, ficco.FICCO_TILE_64x256, ficco.FICCO_TILE_32x256,
                                  ficco.FICCO_TILE_128x128_DEEP, ficco.FICCO_TILE_128x192, ficco.FICCO_TILE_256x192])
def test_gemm_rs_resident_every_tile_shape_ragged(gpu, tile):
    # the resident kernel's own epilogue (row segments through LDS, written through the caches) on pieces
    # of 88 rows and 328 columns: no tile height or width divides them
    dev = gpu["dev"]
    G, c, m, K, N = 3, 2, 88, 192, 328
    M = G * c * m
    A = fi.normal_bf16(31, fi.TENSOR_A, M, K)
    W = fi.make_weight(31, K, N)
    blocks = og.gemm_rs_blocks(A, W, G)
    outs = []
    for sched in (ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT):
        A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
        C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
        peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16, device=dev) for _ in range(G)]
        torch.cuda.synchronize()
        plan = ficco.ficco_plan(M, K, N, G, c, sched)
        try:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_TILE, tile)
            for _ in range(2):
                ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, peers, gpu["cs"], gpu["xs"])
                ficco.ficco_query_stats(plan)
        finally:
            ficco.ficco_destroy(plan)
        torch.cuda.synchronize()
        got = np.concatenate([p.cpu().numpy().view(np.uint16) for p in peers], 0)
        for j in range(G):
            check(got[j * c * m:(j + 1) * c * m], blocks[j], f"peer {j} tile {tile} sched {sched}")
        assert np.array_equal(got, C_dev.cpu().numpy().view(np.uint16))
        outs.append(got)
    assert np.array_equal(outs[0], outs[1])


def test_resident_kernel_gives_up_when_flags_never_arrive(gpu):
    # host-forced: the transfers are issued but the ready flags are withheld; the kernel's bounded
    # wait must expire, every workgroup must drain, and the run must report a timeout
    shards, W = fi.config_inputs("cfg1_tiny")
    bits, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_PERSISTENT, 4,
                         opts=[(ficco.FICCO_OPT_HOLD_FLAGS, 1), (ficco.FICCO_OPT_SPIN_LIMIT_US, 20000)],
                         allow_timeout=True)
    assert st.timed_out == 1
    assert 15000 < st.wall_us < 2_000_000
    # and the library is healthy afterwards
    base, st2, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_PERSISTENT, 4)
    assert st2.timed_out == 0
    check(base, og.ag_gemm(shards, W))


def test_run_rejects_bad_arguments(gpu):
    dev = gpu["dev"]
    t = torch.zeros((512, 1024), dtype=torch.int16, device=dev)
    w = torch.zeros((1024, 1024), dtype=torch.int16, device=dev)
    host_unpinned = torch.zeros((512, 1024), dtype=torch.int16)
    plan = ficco.ficco_plan(512, 1024, 1024, 4, 1, ficco.FICCO_SHARD)
    try:
        for args in [(None, t, w, t, None), (host_unpinned, t, w, t, None), (t, None, w, t, None),
                     (t, t, w, t, [t] * 4), (t, host_unpinned, w, t, None)]:
            with pytest.raises(ficco.FiccoError) as e:
                ficco.ficco_run(plan, *args, gpu["cs"], gpu["xs"])
            assert e.value.status == ficco.FICCO_ERR_ARG
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_run(plan, t, t, w, t, None, gpu["cs"], gpu["cs"])       # same stream twice
    finally:
        ficco.ficco_destroy(plan)


def test_cfg2_full_compare(gpu):
    cfg = fi.CONFIGS["cfg2_qkv8b"]
    shards, W = fi.config_inputs("cfg2_qkv8b")
    ref = og.ag_gemm(shards, W)
    base = None
    ms = cfg["M"] // cfg["shards"]
    cases = [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1)]
    for rows in cfg["chunk_rows"]:
        for sched in (ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT):
            cases.append((sched, ms // rows))
    cases += [(ficco.FICCO_FINE_2D, c) for c in cfg["k_slices"]]       # the bench screens column pieces here too
    cases += [(ficco.FICCO_FINE_2D, tuple(w)) for w in cfg["k_widths"]]
    for sched, c in cases:
        # device staging source for the resident schedules, as the bench times them
        src = "device" if sched in (ficco.FICCO_FINE_PERSISTENT, ficco.FICCO_FINE_2D) else "pinned"
        widths = list(c) if isinstance(c, tuple) else None
        bits, st, _ = run_ag(gpu, shards, W, sched, len(c) if widths else c, src=src, widths=widths)
        if base is None:
            check(bits, ref, "cfg2 serial")
            base = bits
        assert np.array_equal(bits, base), (sched, c)
    # the configuration the bench times: two plans of the unequal column cut chained behind each other, taking
    # steps in turn from the device staging source
    dev = gpu["dev"]
    widths = cfg["k_widths"][0]
    A = np.concatenate(shards, 0)
    M, K, N, G = cfg["M"], cfg["K"], cfg["N"], cfg["shards"]
    src = as_i16(np.concatenate([b.ravel() for b in fi.to_k_pieces(A, widths)]).reshape(M, K)).to(dev)
    W_dev = as_i16(W).to(dev)
    A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
    outs = [torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev) for _ in range(2)]
    plans = [ficco.ficco_plan(M, K, N, G, len(widths), ficco.FICCO_FINE_2D) for _ in range(2)]
    try:
        for p_ in plans:
            ficco.ficco_plan_set_slice_widths(p_, widths)
            ficco.ficco_plan_set(p_, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
        ficco.ficco_plan_chain(plans[0], plans[1])
        ficco.ficco_plan_chain(plans[1], plans[0])
        for i in range(10):
            ficco.ficco_run(plans[i % 2], src, A_dev, W_dev, outs[i % 2], None, gpu["cs"], gpu["xs"])
        for p_ in plans:
            ficco.ficco_query_stats(p_)
        for o in outs:
            assert np.array_equal(o.cpu().numpy().view(np.uint16), base), "cfg2, chained plans"
    finally:
        for p_ in plans:
            ficco.ficco_destroy(p_)
    torch.cuda.synchronize()


def test_cfg3_sampled_rows(gpu):
    cfg = fi.CONFIGS["cfg3_ffn70b"]
    shards, W = fi.config_inputs("cfg3_ffn70b")
    M, G = cfg["M"], cfg["shards"]
    rng = np.random.default_rng(3)
    m = 512
    rows = np.unique(np.concatenate([rng.integers(0, M, 32), np.arange(0, M, m), np.arange(m - 1, M, m)]))
    ref = og.ag_gemm_rows(shards, W, rows)
    base = None
    S, E = ficco.FICCO_COPY_STREAM, ficco.FICCO_COPY_ENGINES
    for sched, c, src, backend in [(ficco.FICCO_SERIAL, 1, "pinned", S), (ficco.FICCO_SHARD, 1, "pinned", S),
                                   (ficco.FICCO_FINE_FUSED, 4, "pinned", S), (ficco.FICCO_FINE_UNFUSED, 2, "device", E),
                                   (ficco.FICCO_FINE_PERSISTENT, 4, "pinned", S),      # full grid minus the helper-kernel headroom
                                   (ficco.FICCO_FINE_PERSISTENT, 4, "pinned", E), (ficco.FICCO_FINE_PERSISTENT, 2, "device", E),
                                   (ficco.FICCO_FINE_PERSISTENT, 8, "device", E),      # what ficco_pick_schedule answers for this shape
                                   (ficco.FICCO_SERIAL, 1, "device", E)]:
        bits, st, info = run_ag(gpu, shards, W, sched, c, src=src, opts=[(ficco.FICCO_OPT_COPY_BACKEND, backend)])
        assert info.copy_backend == backend
        if base is None:
            check(bits[rows], ref, "cfg3 sampled rows")
            base = bits
        assert np.array_equal(bits, base), (sched, c, src)


# ------------------------------------------------------------------ copy-engine (SDMA) backend
def test_engines_backend_pinned_and_device_sources(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    for src in ("pinned", "device"):
        for sched, c in ALL_SCHEDULES:
            # links: engines side by side; fw 0: kernels watch the transfers' completion signals when
            # the runtime reports them reachable, fw 2: a 4-byte flag copy behind every transfer
            for links, fw in ((0, 0), (1, 0), (3, 2), (0, 2)):
                bits, st, info = run_ag(gpu, shards, W, sched, c, src=src, runs=2,
                                        opts=[(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_ENGINES),
                                              (ficco.FICCO_OPT_LINKS, links), (ficco.FICCO_OPT_FLAG_WRITE, fw)])
                assert np.array_equal(bits, base), (src, sched, c, links)
                assert info.copy_backend == ficco.FICCO_COPY_ENGINES
                assert info.links == (4 if links == 0 else links)
                assert st.n_copies == info.n_chunks and st.copy_span_us > 0


def test_engines_backend_orders_and_local_shard(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    eng = [(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_ENGINES)]
    rng = np.random.default_rng(1)
    for sched in (ficco.FICCO_FINE_UNFUSED, ficco.FICCO_FINE_FUSED, ficco.FICCO_FINE_PERSISTENT):
        bits, _, _ = run_ag(gpu, shards, W, sched, 4, src="device", arrival=list(rng.permutation(16)), opts=eng)
        assert np.array_equal(bits, base)
        bits, _, _ = run_ag(gpu, shards, W, sched, 4, src="device",
                            opts=eng + [(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)])
        assert np.array_equal(bits, base)


def test_engines_links_run_side_by_side(gpu):
    # 8 shards of 8 MiB from a device staging buffer: all links at once must be several times
    # faster than one transfer at a time (the peer-to-peer pattern of shard-level overlap)
    M, K, N, G = 8192, 4096, 256, 8
    shards = fi.make_shards(7, M, K, G)
    W = fi.make_weight(7, K, N)
    _, st_all, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device", runs=3)
    _, st_one, _ = run_ag(gpu, shards, W, ficco.FICCO_SHARD, 1, src="device", runs=3)
    assert st_all.copy_bytes == st_one.copy_bytes == M * K * 2
    assert st_one.copy_span_us > 3.0 * st_all.copy_span_us, (st_one.copy_span_us, st_all.copy_span_us)


def test_engines_bounded_wait_in_per_launch_kernels(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    _, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_FUSED, 4, src="device", allow_timeout=True,
                      opts=[(ficco.FICCO_OPT_HOLD_FLAGS, 1), (ficco.FICCO_OPT_SPIN_LIMIT_US, 20000)])
    assert st.timed_out == 1
    bits, st2, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_FUSED, 4, src="device")
    assert st2.timed_out == 0
    check(bits, og.ag_gemm(shards, W))


# ------------------------------------------------------------------------------------------------
# 2D decomposition: column pieces, one resident kernel accumulating slice by slice
def test_2d_matches_oracle_and_serial_bits(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    A = np.concatenate(shards, 0)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    for c in (1, 2, 4, 16):
        ref = og.ag_gemm_2d(fi.to_k_sliced(A, c), W, len(shards))
        for src, opts in [("pinned", [(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)]),
                          ("pinned", [(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_ENGINES)]),
                          ("device", [(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)]),
                          ("device", [(ficco.FICCO_OPT_FLAG_WRITE, 2)]),
                          ("device", [])]:
            bits, st, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src=src, opts=opts, runs=2)
            check(bits, ref, f"2D c={c} {src} {opts}")
            assert np.array_equal(bits, base), f"2D c={c} {src} {opts}: differs bitwise from serial"
            assert st.n_copies == 4 * c and st.copy_bytes == 512 * 1024 * 2 and st.n_launches == 1
            assert info.n_groups == 1 and info.chunk_rows == 128


@pytest.mark.parametrize("tile", [ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_256x128,
                                  ficco.FICCO_TILE_128x256, ficco.FICCO_TILE_64x256, ficco.FICCO_TILE_32x256,
                                  ficco.FICCO_TILE_128x128_DEEP, ficco.FICCO_TILE_128x192, ficco.FICCO_TILE_256x192])
def test_2d_every_tile_shape_ragged(gpu, tile):
    # 3 shards of 88 rows (tiles straddle shards), N = 328, K = 3 slices of 128
    G, ms, K, N, c = 3, 88, 384, 328, 3
    shards = fi.make_shards(23, G * ms, K, G)
    W = fi.make_weight(23, K, N)
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, opts=[(ficco.FICCO_OPT_TILE, tile)])
    bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src="device", opts=[(ficco.FICCO_OPT_TILE, tile)])
    check(bits, ref, f"2D tile {tile}")
    assert np.array_equal(bits, base)


def test_2d_unequal_slices_match_oracle_and_serial_bits(gpu):
    """Column pieces of unequal width (narrow first, narrow last, one k-tile, the library's own cut of a k range
    that the slice count does not divide): the bits are those of the serial schedule."""
    G, ms, K, N = 4, 160, 1024, 328
    shards = fi.make_shards(31, G * ms, K, G)
    W = fi.make_weight(31, K, N)
    A = np.concatenate(shards, 0)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    check(base, og.ag_gemm(shards, W), "serial")
    for widths in ([768, 256], [64, 64, 128, 256, 512], [512, 448, 64], [64] * 16, [1024]):
        ref = og.ag_gemm_2d(fi.to_k_pieces(A, widths), W, G)
        for src, opts in [("pinned", [(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)]),
                          ("device", [(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)]),
                          ("device", [(ficco.FICCO_OPT_FLAG_WRITE, 2)]),
                          ("device", [])]:
            bits, st, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, len(widths), src=src, opts=opts, runs=2, widths=widths)
            check(bits, ref, f"2D widths={widths} {src} {opts}")
            assert np.array_equal(bits, base), f"2D widths={widths} {src} {opts}: differs bitwise from serial"
            assert st.n_copies == G * len(widths) and st.copy_bytes == G * ms * K * 2
    # 16 k-tiles in 3, 5 and 7 slices: the first slices are one k-tile wider
    for c in (3, 5, 7):
        bits, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src="device")
        assert np.array_equal(bits, base), f"2D c={c}"
        assert st.n_copies == G * c and st.copy_bytes == G * ms * K * 2
    # reversed arrival with unequal widths: a tile still takes the slices in k order
    rev = list(range(G * 3 - 1, -1, -1))
    bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, 3, src="device", arrival=rev, widths=[128, 640, 256])
    assert np.array_equal(bits, base)


def test_2d_more_slices_than_the_kernels_slice_table_holds(gpu):
    # 80 slices of one k-tile each, then 70 of unequal width: the kernel keeps 64 boundaries in LDS and reads the rest from memory
    G, ms, N = 2, 96, 72
    K = 64 * 80
    shards = fi.make_shards(33, G * ms, K, G)
    W = fi.make_weight(33, K, N)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    check(base, og.ag_gemm(shards, W), "serial")
    bits, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, 80, src="device", runs=2)
    assert np.array_equal(bits, base) and st.n_copies == G * 80
    widths = [64] * 60 + [128] * 10
    bits, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, len(widths), src="device", widths=widths)
    assert np.array_equal(bits, base) and st.n_copies == G * 70


def test_chained_plans_take_turns_on_one_a_dev_without_host_waits(gpu):
    """Two plans chained behind each other run in turn, the host never waiting between steps: they share A_dev,
    read different sources and write different outputs, so a transfer of the next step that started before
    the previous step's kernel had finished would put the wrong rows under that kernel."""
    dev = gpu["dev"]
    G, ms, K, N = 4, 512, 2048, 4096
    M = G * ms
    sh1, sh2 = fi.make_shards(41, M, K, G), fi.make_shards(42, M, K, G)
    W = fi.make_weight(41, K, N)
    base1, _, _ = run_ag(gpu, sh1, W, ficco.FICCO_SERIAL, 1)
    base2, _, _ = run_ag(gpu, sh2, W, ficco.FICCO_SERIAL, 1)
    rows = np.arange(0, M, 37)
    check(base1[rows], og.ag_gemm_rows(sh1, W, rows), "serial, first source")
    check(base2[rows], og.ag_gemm_rows(sh2, W, rows), "serial, second source")
    widths = [1536, 512]
    A1 = np.concatenate(sh1, 0)
    A2 = np.concatenate([b.ravel() for b in fi.to_k_pieces(np.concatenate(sh2, 0), widths)]).reshape(M, K)
    src1, src2 = as_i16(A1).to(dev), as_i16(A2).to(dev)
    W_dev = as_i16(W).to(dev)
    A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
    C1 = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    C2 = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    pa = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_PERSISTENT)
    pb = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_2D)
    try:
        ficco.ficco_plan_set_slice_widths(pb, widths)
        ficco.ficco_plan_set(pb, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
        ficco.ficco_plan_chain(pa, pb)
        ficco.ficco_plan_chain(pb, pa)
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_plan_chain(pa, pa)
        for it in range(8):
            ficco.ficco_run(pa, src1, A_dev, W_dev, C1, None, gpu["cs"], gpu["xs"])
            ficco.ficco_run(pb, src2, A_dev, W_dev, C2, None, gpu["cs"], gpu["xs"])
            if it in (2, 5):                              # outputs of a step in the middle, while later steps are queued
                sa, sb = ficco.ficco_query_stats(pa), ficco.ficco_query_stats(pb)
                assert np.array_equal(C1.cpu().numpy().view(np.uint16), base1), f"step {it}: first plan"
                assert np.array_equal(C2.cpu().numpy().view(np.uint16), base2), f"step {it}: second plan"
                assert sa.n_copies == 2 * G and sb.n_copies == 2 * G and sa.n_launches == 1
                C1.fill_(0x7FFF); C2.fill_(0x7FFF); torch.cuda.synchronize()
        ficco.ficco_query_stats(pa); ficco.ficco_query_stats(pb)
        assert np.array_equal(C1.cpu().numpy().view(np.uint16), base1)
        assert np.array_equal(C2.cpu().numpy().view(np.uint16), base2)
        # the plan in front is destroyed first: the one behind it runs on, with nothing left to wait for
        ficco.ficco_destroy(pa)
        pa = None
        C2.fill_(0x7FFF)
        ficco.ficco_run(pb, src2, A_dev, W_dev, C2, None, gpu["cs"], gpu["xs"])
        ficco.ficco_query_stats(pb)
        assert np.array_equal(C2.cpu().numpy().view(np.uint16), base2)
        # chained plans need the copy engines
        pc = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_FUSED)
        try:
            ficco.ficco_plan_set(pc, ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)
            ficco.ficco_plan_chain(pc, pb)
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_run(pc, as_i16(A1).pin_memory(), A_dev, W_dev, C1, None, gpu["cs"], gpu["xs"])
            ficco.ficco_plan_chain(pc, None)
        finally:
            ficco.ficco_destroy(pc)
        # ... and are defined for the transfers into A_dev only
        pr = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_FUSED)
        try:
            ficco.ficco_plan_set(pr, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
            ficco.ficco_plan_chain(pr, pb)
            peers = [torch.zeros((ms, N), dtype=torch.int16, device=dev) for _ in range(G)]
            with pytest.raises(ficco.FiccoError):
                ficco.ficco_run(pr, None, A_dev, W_dev, C1, peers, gpu["cs"], gpu["xs"])
        finally:
            ficco.ficco_destroy(pr)
    finally:
        if pa is not None:
            ficco.ficco_destroy(pa)
        ficco.ficco_destroy(pb)
    torch.cuda.synchronize()


def test_chained_plan_is_let_go_when_the_run_in_front_gives_up(gpu):
    """The plan in front never sees its flags (forced from the host) and its kernel gives up after the spin
    limit; the run still ends by releasing the plan behind it, whose result must be complete and right."""
    dev = gpu["dev"]
    shards, W = fi.config_inputs("cfg1_tiny")
    A = np.concatenate(shards, 0)
    M, K = A.shape
    N, G = W.shape[1], len(shards)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    src, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
    A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
    C1 = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    C2 = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    for sched in (ficco.FICCO_FINE_PERSISTENT, ficco.FICCO_FINE_FUSED):     # released by the kernel itself / by the release kernel
        pa = ficco.ficco_plan(M, K, N, G, 2, sched)
        pb = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_PERSISTENT)
        try:
            ficco.ficco_plan_set(pa, ficco.FICCO_OPT_HOLD_FLAGS, 1)
            ficco.ficco_plan_set(pa, ficco.FICCO_OPT_SPIN_LIMIT_US, 2000)
            ficco.ficco_plan_chain(pb, pa)
            C2.fill_(0x7FFF)
            torch.cuda.synchronize()
            ficco.ficco_run(pa, src, A_dev, W_dev, C1, None, gpu["cs"], gpu["xs"])
            ficco.ficco_run(pb, src, A_dev, W_dev, C2, None, gpu["cs"], gpu["xs"])
            sa = ficco.ficco_query_stats(pa, allow_timeout=True)
            sb = ficco.ficco_query_stats(pb)
            assert sa.timed_out == 1 and sb.timed_out == 0
            assert np.array_equal(C2.cpu().numpy().view(np.uint16), base), f"plan behind a run that gave up (schedule {sched})"
        finally:
            ficco.ficco_destroy(pa)
            ficco.ficco_destroy(pb)
    torch.cuda.synchronize()


def test_auto_any_plan_runs_from_the_callers_row_major_matrix(gpu):
    """FICCO_AUTO_ANY may answer with column pieces; A_src stays the caller's row-major matrix, in device memory
    (the sender-side re-layout kernel releases each piece's transfer) and in pinned host memory (rectangular
    engine copies), and a sender that holds its slices K-sliced already can say so."""
    dev = gpu["dev"]
    M, K, N, G = 4096, 8192, 3584, 8                       # a sweep shape the rule sends to column pieces
    shards = fi.make_shards(fi.SWEEP["seed"], M, K, G)
    W = fi.make_weight(fi.SWEEP["seed"], K, N)
    A = np.concatenate(shards, 0)
    rows = np.unique(np.concatenate([np.arange(0, M, 193), [0, M // G - 1, M // G, M - 1]]))
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device")
    check(base[rows], og.ag_gemm_rows(shards, W, rows), "serial")
    W_dev = as_i16(W).to(dev)
    assert ficco.ficco_pick_schedule_any(M, K, N, G) == (ficco.FICCO_FINE_2D, 4)
    for kind in ("device", "pinned", "k_sliced"):
        plan = ficco.ficco_plan(M, K, N, G, 1, ficco.FICCO_AUTO_ANY)
        try:
            info = ficco.ficco_plan_info(plan)
            assert (info.schedule, info.chunks) == (ficco.FICCO_FINE_2D, 4)
            _, widths = ficco.ficco_plan_slices(plan)
            want = np.concatenate([b.ravel() for b in fi.to_k_pieces(A, widths)])
            if kind == "k_sliced":
                ficco.ficco_plan_set(plan, ficco.FICCO_OPT_SOURCE_LAYOUT, ficco.FICCO_LAYOUT_K_SLICED)
                src = as_i16(want.reshape(M, K)).to(dev)
            else:
                src = as_i16(A).to(dev) if kind == "device" else as_i16(A).pin_memory()
            for run in range(3):                              # signals, counters and the staging copy are reused
                A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
                C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
                torch.cuda.synchronize()
                ficco.ficco_run(plan, src, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
                st = ficco.ficco_query_stats(plan)
                assert st.n_copies == 4 * G and st.copy_bytes == M * K * 2
                assert np.array_equal(C_dev.cpu().numpy().view(np.uint16), base), (kind, run)
                # the landing buffer holds the K-sliced matrix
                assert np.array_equal(A_dev.cpu().numpy().view(np.uint16).ravel(), want), (kind, run)
        finally:
            ficco.ficco_destroy(plan)
    torch.cuda.synchronize()


@pytest.mark.parametrize("src", ["device", "pinned"])
def test_2d_from_row_major_source_ragged_and_unequal(gpu, src):
    # 3 shards of 88 rows (no tile height divides it), K = 5 k-tiles cut 128 + 64 + 128, N not a tile width;
    # then equal slices, reversed arrival, shard-major order (transfers one after the other)
    G, ms, K, N = 3, 88, 320, 328
    shards = fi.make_shards(33, G * ms, K, G)
    W = fi.make_weight(33, K, N)
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    check(base, ref, "serial")
    for widths, arrival, opts in [([128, 64, 128], None, ()), (None, None, ()), ([64, 192, 64], list(range(3 * G))[::-1], ()),
                                  (None, None, [(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)])]:
        c = len(widths) if widths else 5
        bits, st, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src=src, widths=widths, arrival=arrival, opts=opts,
                                runs=2, row_major=True)
        assert info.copy_backend == ENGINES and st.n_copies == c * G
        assert np.array_equal(bits, base), (src, widths, arrival, opts)


def test_2d_row_major_source_is_refused_on_the_stream_backend(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    with pytest.raises(ficco.FiccoError) as e:
        run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, 2, backend=STREAM, row_major=True)
    assert e.value.status == ficco.FICCO_ERR_ARG


def test_cfg2_and_cfg6_2d_from_row_major_device_source(gpu):
    for name, c, widths in [("cfg2_qkv8b", 2, [3072, 1024]), ("cfg6_2d_proj", 8, None)]:
        cfg = fi.CONFIGS[name]
        shards, W = fi.config_inputs(name)
        rows = np.unique(np.concatenate([np.arange(0, cfg["M"], 257), [0, cfg["M"] // 8 - 1, cfg["M"] // 8, cfg["M"] - 1]]))
        ref = og.ag_gemm_rows(shards, W, rows)
        base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device")
        check(base[rows], ref, f"{name} serial")
        bits, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src="device", widths=widths, runs=2, row_major=True)
        assert np.array_equal(bits, base), f"{name}: column pieces out of the row-major source differ bitwise from serial"


def test_2d_waits_for_late_and_reordered_slices(gpu):
    G, ms, K, N, c = 4, 256, 1024, 512, 4
    shards = fi.make_shards(24, G * ms, K, G)
    W = fi.make_weight(24, K, N)
    ref = og.ag_gemm(shards, W)
    rev = list(range(G * c - 1, -1, -1))                  # last slice lands first: tiles must still wait for slice 0
    bits_rev, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, src="device", arrival=rev)
    check(bits_rev, ref, "2D reversed arrival")
    bits_late, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, c, delay_copy=True,
                             opts=[(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)])
    check(bits_late, ref, "2D delayed transfers")
    assert np.array_equal(bits_rev, bits_late)


def test_2d_timeout_is_reported_not_hung(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    # flags are never raised: every waiting tile must give up after the spin limit and the run must end
    _, st, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, 2, src="device",
                      opts=[(ficco.FICCO_OPT_HOLD_FLAGS, 1), (ficco.FICCO_OPT_SPIN_LIMIT_US, 2000)], allow_timeout=True)
    assert st.timed_out == 1


def test_cfg6_2d_full_size_sampled_rows(gpu):
    cfg = fi.CONFIGS["cfg6_2d_proj"]
    shards, W = fi.config_inputs("cfg6_2d_proj")
    rows = np.unique(np.concatenate([np.arange(0, cfg["M"], 331), [0, 255, 256, 511, 512, cfg["M"] - 1]]))
    ref = og.ag_gemm_rows(shards, W, rows)
    base, st0, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device")
    check(base[rows], ref, "cfg6 serial")
    for c in cfg["k_slices"] + [(1024, 3072, 4096, 4096, 4096)]:      # equal slices, then a narrow first one
        widths = list(c) if isinstance(c, tuple) else None
        bits, st, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_2D, len(c) if widths else c, src="device", runs=2, widths=widths)
        check(bits[rows], ref, f"cfg6 2D c={c}")
        assert np.array_equal(bits, base), f"cfg6 2D c={c} differs bitwise from serial"


# ------------------------------------------------------------------------------------------------
# fused schedule with explicit Gather / Scatter copies on the copy engines
def test_packed_fused_matches_in_place_fused(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    pk = (ficco.FICCO_OPT_PACKING, 1)
    for c, src, opts, local in [(4, "device", [pk], None), (1, "device", [pk], None), (4, "pinned", [pk], None),
                                (4, "device", [pk], 2),
                                (2, "device", [pk, (ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR), (ficco.FICCO_OPT_LINKS, 3)], None)]:
        bits, st, info = run_ag(gpu, shards, W, ficco.FICCO_FINE_FUSED, c, src=src, opts=opts, runs=2, local_shard=local)
        check(bits, ref, f"packed c={c} {src} {opts} local={local}")
        assert np.array_equal(bits, base), f"packed c={c} {src} {opts}: differs bitwise from serial"
        n = 4 * c
        assert st.n_copies == 3 * n - (c if local is not None else 0) and st.n_launches == info.n_groups
        assert info.copy_backend == ficco.FICCO_COPY_ENGINES


def test_packed_fused_ragged_pieces(gpu):
    G, c, m, K, N = 3, 2, 88, 192, 328
    shards = fi.make_shards(25, G * c * m, K, G)
    W = fi.make_weight(25, K, N)
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    rev = list(range(G * c - 1, -1, -1))
    for arrival in (None, rev):
        bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_FUSED, c, src="device", arrival=arrival,
                            opts=[(ficco.FICCO_OPT_PACKING, 1)], timing=1)
        check(bits, ref, "packed ragged")
        assert np.array_equal(bits, base)


# ------------------------------------------------------------------------------------------------
# HIP graph of one run of the per-launch schedules (stream backend, pinned far side)
def test_graph_replays_match_eager_runs(gpu):
    shards, W = fi.config_inputs("cfg1_tiny")
    ref = og.ag_gemm(shards, W)
    dev = gpu["dev"]
    A = np.concatenate(shards, 0)
    M, K = A.shape
    N, G = W.shape[1], len(shards)
    A_src = as_i16(A).pin_memory()
    W_dev = as_i16(W).to(dev)
    A_dev = torch.empty((M, K), dtype=torch.int16, device=dev)
    C_dev = torch.empty((M, N), dtype=torch.int16, device=dev)
    eager, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1)
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1), (ficco.FICCO_FINE_UNFUSED, 4), (ficco.FICCO_FINE_FUSED, 4)]:
        plan = ficco.ficco_plan(M, K, N, G, c, sched)
        try:
            with pytest.raises(ficco.FiccoError) as e:
                ficco.ficco_graph_launch(plan, gpu["cs"])
            assert e.value.status == ficco.FICCO_ERR_STATE
            ficco.ficco_graph_capture(plan, A_src, A_dev, W_dev, C_dev, None)
            info = ficco.ficco_plan_info(plan)
            for replay in range(4):
                # the program's own eager work and a synchronisation between replays
                A_dev.fill_(NAN_BF16)
                C_dev.fill_(0x7FFF)
                torch.cuda.synchronize()
                if replay == 2:                 # an eager run of the same plan between two replays
                    ficco.ficco_run(plan, A_src, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
                    ficco.ficco_query_stats(plan)
                    A_dev.fill_(NAN_BF16)
                    C_dev.fill_(0x7FFF)
                    torch.cuda.synchronize()
                ficco.ficco_graph_launch(plan, gpu["cs"])
                st = ficco.ficco_query_stats(plan)
                torch.cuda.synchronize()
                bits = C_dev.cpu().numpy().view(np.uint16)
                check(bits, ref, f"graph sched {sched} replay {replay}")
                assert np.array_equal(bits, eager), f"graph sched {sched} replay {replay}: differs from the eager run"
                assert st.n_copies == info.n_chunks and st.n_launches == info.n_groups and st.wall_us > 0
        finally:
            ficco.ficco_destroy(plan)


def test_graph_of_gemm_rs_and_argument_checks(gpu):
    dev = gpu["dev"]
    M, K, N, G = 1024, 256, 512, 8
    A = fi.normal_bf16(3, fi.TENSOR_A, M, K)
    W = fi.make_weight(3, K, N)
    blocks = og.gemm_rs_blocks(A, W, G)
    A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
    C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
    peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16).pin_memory() for _ in range(G)]
    plan = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_FUSED)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
        ficco.ficco_graph_capture(plan, None, A_dev, W_dev, C_dev, peers)
        for replay in range(3):
            for p_ in peers:
                p_.fill_(NAN_BF16)
            C_dev.zero_()
            torch.cuda.synchronize()
            ficco.ficco_graph_launch(plan, gpu["cs"])
            ficco.ficco_query_stats(plan)
            torch.cuda.synchronize()
            for j in range(G):
                check(peers[j].numpy().view(np.uint16), blocks[j], f"graph RS peer {j} replay {replay}")
    finally:
        ficco.ficco_destroy(plan)
    # what a graph cannot hold is refused
    dev_peers = [torch.zeros((M // G, N), dtype=torch.int16, device=dev) for _ in range(G)]
    for sched, c, opts, args in [
            (ficco.FICCO_FINE_PERSISTENT, 2, [], (as_i16(A).pin_memory(), A_dev, W_dev, C_dev, None)),     # waits inside the kernel
            (ficco.FICCO_FINE_FUSED, 2, [], (A_dev.clone(), A_dev, W_dev, C_dev, None)),                  # device source: copy kernels
            (ficco.FICCO_FINE_FUSED, 2, [(ficco.FICCO_OPT_COPY_BACKEND, ENGINES)], (as_i16(A).pin_memory(), A_dev, W_dev, C_dev, None)),
            (ficco.FICCO_FINE_FUSED, 2, [(ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)], (None, A_dev, W_dev, C_dev, dev_peers))]:
        plan = ficco.ficco_plan(M, K, N, G, c, sched)
        try:
            for o, v in opts:
                ficco.ficco_plan_set(plan, o, v)
            with pytest.raises(ficco.FiccoError) as e:
                ficco.ficco_graph_capture(plan, *args)
            assert e.value.status == ficco.FICCO_ERR_ARG
        finally:
            ficco.ficco_destroy(plan)


# ------------------------------------------------------------------------------------------------
# full sizes of the remaining workload and the largest piece count the plan accepts
def test_cfg4_gemm_rs_full_size_sampled_rows(gpu):
    cfg = fi.CONFIGS["cfg4_gemm_rs"]
    dev = gpu["dev"]
    M, K, N, G = cfg["M"], cfg["K"], cfg["N"], cfg["shards"]
    A = fi.normal_bf16(cfg["seed"], fi.TENSOR_A, M, K)
    W = fi.make_weight(cfg["seed"], K, N)
    rows = np.unique(np.concatenate([np.arange(0, M, 1021), [0, M // G - 1, M // G, M - 1]]))
    ref = og.ag_gemm_rows([A], W, rows)
    A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
    base = None
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_FINE_FUSED, 4), (ficco.FICCO_FINE_PERSISTENT, 8)]:   # what bench.py screens
        C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
        peers = [torch.full((M // G, N), NAN_BF16, dtype=torch.int16, device=dev) for _ in range(G)]
        torch.cuda.synchronize()
        plan = ficco.ficco_plan(M, K, N, G, c, sched)
        try:
            ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
            ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, peers, gpu["cs"], gpu["xs"])
            st = ficco.ficco_query_stats(plan)
        finally:
            ficco.ficco_destroy(plan)
        torch.cuda.synchronize()
        got = torch.cat(peers, 0).cpu().numpy().view(np.uint16)
        check(got[rows], ref, f"cfg4 sched {sched}")
        assert st.copy_bytes == M * N * 2
        if base is None:
            base = got
        assert np.array_equal(got, base)


def test_largest_piece_count(gpu):
    # shards * pieces = 4096, the most a plan accepts: one-row pieces
    G, c, K, N = 8, 512, 64, 16
    M = G * c
    shards = fi.make_shards(26, M, K, G)
    W = fi.make_weight(26, K, N)
    ref = og.ag_gemm(shards, W)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device")
    check(base, ref, "serial")
    for sched in (ficco.FICCO_FINE_PERSISTENT, ficco.FICCO_FINE_FUSED):
        bits, st, info = run_ag(gpu, shards, W, sched, c, src="device")
        assert info.n_chunks == 4096 and st.n_copies == 4096
        assert np.array_equal(bits, base), sched
    with pytest.raises(ficco.FiccoError):
        ficco.ficco_plan(2 * M, K, N, G, 2 * c, ficco.FICCO_FINE_PERSISTENT)
