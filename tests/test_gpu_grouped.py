"""GPU parity of the expert-parallel path (ficco_plan_grouped + ficco_run) against the oracle, element
by element within the GEMM tolerance, and bit-equality across schedules, piece counts and orders."""
import numpy as np
import pytest

import ficco_inputs as fi
import paper_2512_10236_amd as ficco
from oracle import gemm as og
from oracle import grouped as ogr

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 8e-3
NAN_BF16 = 0x7FC0


def as_i16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))


def widen(bits):
    return fi.bf16_bits_to_f32(bits).astype(np.float64)


def run_grouped(gpu, A, W, rows, c, sched, *, src="device", opts=(), arrival=None, runs=1, allow_timeout=False):
    dev = gpu["dev"]
    M, K = A.shape
    N = W.shape[2]
    A_src = as_i16(A).pin_memory() if src == "pinned" else as_i16(A).to(dev)
    W_dev = as_i16(W).to(dev)
    A_dev = torch.full((M, K), NAN_BF16, dtype=torch.int16, device=dev)
    C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()
    plan = ficco.ficco_plan_grouped(K, N, rows, c, sched)
    try:
        for o, v in opts:
            ficco.ficco_plan_set(plan, o, v)
        if arrival is not None:
            ficco.ficco_plan_set_arrival(plan, arrival)
        for r in range(runs):
            if r:
                A_dev.fill_(NAN_BF16)
                C_dev.fill_(0x7FFF)
                torch.cuda.synchronize()
            ficco.ficco_run(plan, A_src, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
            st = ficco.ficco_query_stats(plan, allow_timeout=allow_timeout)
        info = ficco.ficco_plan_info(plan)
    finally:
        ficco.ficco_destroy(plan)
    torch.cuda.synchronize()
    return C_dev.cpu().numpy().view(np.uint16), st, info


def make_case(seed, rows, K, N):
    rows = np.asarray(rows)
    M, E = int(rows.sum()), rows.shape[1]
    A = fi.normal_bf16(seed, fi.TENSOR_A, M, K)
    W = np.stack([fi.normal_bf16(seed + 100 + e, fi.TENSOR_W, K, N, float(K) ** -0.5) for e in range(E)])
    return A, W, rows.sum(axis=0)


def check(bits, ref, what):
    out = widen(bits)
    assert np.isfinite(out).all(), f"{what}: non-finite output (a tile ran before its rows landed, or a row was never written?)"
    err = og.rel_err(out, ref)
    assert err <= TOL, f"{what}: rel err {err}"


@pytest.mark.parametrize("rows", [
    [[40, 13], [0, 77], [91, 5], [300, 0]],               # unequal, zero blocks, segments that are no tile multiple
    [[128] * 3] * 4,                                       # equal shares
    [[1, 0, 2]],                                           # a handful of tokens from one peer
    [[700], [20], [0], [333], [5], [64], [1], [257]],      # one expert, strongly skewed peers
])
def test_grouped_matches_oracle_in_every_schedule(gpu, rows):
    K, N = 256, 328
    A, W, en = make_case(41, rows, K, N)
    ref = ogr.grouped_gemm(A, W, en)
    base = None
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1), (ficco.FICCO_FINE_PERSISTENT, 1),
                     (ficco.FICCO_FINE_PERSISTENT, 3), (ficco.FICCO_FINE_PERSISTENT, 8)]:
        for src in ("device", "pinned"):
            bits, st, info = run_grouped(gpu, A, W, rows, c, sched, src=src, runs=2)
            check(bits, ref, f"sched {sched} c={c} {src}")
            if base is None:
                base = bits
            assert np.array_equal(bits, base), f"sched {sched} c={c} {src}: bits differ from the serial schedule"
            _, nr, _, _ = ogr.layout(rows, c)
            assert st.n_copies == int(np.count_nonzero(nr)) and st.copy_bytes == A.size * 2 and st.n_launches == 1
            assert st.flops == 2 * A.shape[0] * N * K


def test_chained_grouped_plans_take_turns_on_one_a_dev(gpu):
    """Two expert-parallel plans with different token tables, sources and outputs, chained behind each other on
    one A_dev (sized for the larger), run in turn without host waits: the dispatch of the next step may only
    start when the previous step's kernel has finished."""
    dev = gpu["dev"]
    K, N = 1024, 2048
    rows1 = [[300, 211], [512, 40], [0, 700], [129, 256]]
    rows2 = [[700, 5], [64, 333], [257, 1], [90, 402]]
    A1, W, en1 = make_case(51, rows1, K, N)
    A2, _, en2 = make_case(52, rows2, K, N)
    ref1, ref2 = ogr.grouped_gemm(A1, W, en1), ogr.grouped_gemm(A2, W, en2)
    base1, _, _ = run_grouped(gpu, A1, W, rows1, 1, ficco.FICCO_SERIAL)
    base2, _, _ = run_grouped(gpu, A2, W, rows2, 1, ficco.FICCO_SERIAL)
    check(base1, ref1, "serial, first table")
    check(base2, ref2, "serial, second table")
    M1, M2 = A1.shape[0], A2.shape[0]
    src1, src2, W_dev = as_i16(A1).to(dev), as_i16(A2).to(dev), as_i16(W).to(dev)
    A_dev = torch.full((max(M1, M2), K), NAN_BF16, dtype=torch.int16, device=dev)
    C1 = torch.full((M1, N), 0x7FFF, dtype=torch.int16, device=dev)
    C2 = torch.full((M2, N), 0x7FFF, dtype=torch.int16, device=dev)
    pa = ficco.ficco_plan_grouped(K, N, rows1, 2, ficco.FICCO_FINE_PERSISTENT)
    pb = ficco.ficco_plan_grouped(K, N, rows2, 3, ficco.FICCO_FINE_PERSISTENT)
    try:
        ficco.ficco_plan_chain(pa, pb)
        ficco.ficco_plan_chain(pb, pa)
        for it in range(6):
            ficco.ficco_run(pa, src1, A_dev, W_dev, C1, None, gpu["cs"], gpu["xs"])
            ficco.ficco_run(pb, src2, A_dev, W_dev, C2, None, gpu["cs"], gpu["xs"])
        ficco.ficco_query_stats(pa)
        ficco.ficco_query_stats(pb)
        assert np.array_equal(C1.cpu().numpy().view(np.uint16), base1)
        assert np.array_equal(C2.cpu().numpy().view(np.uint16), base2)
    finally:
        ficco.ficco_destroy(pa)
        ficco.ficco_destroy(pb)
    torch.cuda.synchronize()


def test_grouped_experts_use_their_own_weights(gpu):
    # W_e = (e + 1) * identity: every output row is its input row times its expert's factor, exactly
    K = N = 128
    rows = [[5, 9, 2], [17, 0, 30]]
    A = fi.normal_bf16(42, fi.TENSOR_A, 63, K)
    W = np.stack([fi.f32_to_bf16_bits((e + 1) * np.eye(K, dtype=np.float32)) for e in range(3)])
    bits, _, _ = run_grouped(gpu, A, W, rows, 2, ficco.FICCO_FINE_PERSISTENT)
    factor = np.repeat([1.0, 2.0, 3.0], np.asarray(rows).sum(axis=0))[:, None]
    want = fi.f32_to_bf16_bits((widen(A) * factor).astype(np.float32))
    assert np.array_equal(bits, want)


@pytest.mark.parametrize("tile", [ficco.FICCO_TILE_256x256, ficco.FICCO_TILE_128x128, ficco.FICCO_TILE_128x256, ficco.FICCO_TILE_32x256,
                                  ficco.FICCO_TILE_128x192])
def test_grouped_tiles_orders_and_flag_modes(gpu, tile):
    rows = [[300, 41], [77, 500], [0, 129], [260, 3]]
    K, N = 192, 264
    A, W, en = make_case(43, rows, K, N)
    ref = ogr.grouped_gemm(A, W, en)
    t = (ficco.FICCO_OPT_TILE, tile)
    base, _, _ = run_grouped(gpu, A, W, rows, 1, ficco.FICCO_SERIAL, opts=[t])
    check(base, ref, f"tile {tile} serial")
    n = 4 * 2 * 4
    for opts, arrival in [([t], None), ([t, (ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)], None),
                          ([t, (ficco.FICCO_OPT_FLAG_WRITE, 2)], None), ([t, (ficco.FICCO_OPT_LINKS, 3)], None),
                          ([t], list(range(n - 1, -1, -1)))]:
        bits, _, _ = run_grouped(gpu, A, W, rows, 4, ficco.FICCO_FINE_PERSISTENT, opts=opts, arrival=arrival)
        assert np.array_equal(bits, base), (tile, opts, arrival is not None)


def test_grouped_full_size_sampled_rows(gpu):
    cfg = fi.CONFIGS["cfg7_ep_grouped"]
    rows = fi.make_token_counts(cfg["seed"], cfg["shards"], cfg["experts"], cfg["tokens"], cfg["skew"])
    K, N = cfg["K"], cfg["N"]
    A, W, en = make_case(cfg["seed"], rows, K, N)
    sample = np.unique(np.concatenate([np.arange(0, A.shape[0], 397), [0, int(en[0]) - 1, int(en[0]), A.shape[0] - 1]]))
    expert_of = np.repeat(np.arange(len(en)), en)
    ref = np.stack([og.ag_gemm_rows([A], W[expert_of[r]], [r])[0] for r in sample])
    base = None
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_FINE_PERSISTENT, 4)]:
        bits, _, _ = run_grouped(gpu, A, W, rows.tolist(), c, sched)
        check(bits[sample], ref, f"cfg7 sched {sched} c={c}")
        if base is None:
            base = bits
        assert np.array_equal(bits, base)


def test_grouped_timeout_and_bad_arguments(gpu):
    rows = [[64, 64], [64, 64]]
    A, W, en = make_case(44, rows, 128, 64)
    _, st, _ = run_grouped(gpu, A, W, rows, 2, ficco.FICCO_FINE_PERSISTENT, allow_timeout=True,
                           opts=[(ficco.FICCO_OPT_HOLD_FLAGS, 1), (ficco.FICCO_OPT_SPIN_LIMIT_US, 5000)])
    assert st.timed_out == 1
    bits, st2, _ = run_grouped(gpu, A, W, rows, 2, ficco.FICCO_FINE_PERSISTENT)
    assert st2.timed_out == 0
    check(bits, ogr.grouped_gemm(A, W, en), "after timeout")
    with pytest.raises(ficco.FiccoError):
        run_grouped(gpu, A, W, rows, 2, ficco.FICCO_FINE_PERSISTENT, opts=[(ficco.FICCO_OPT_COPY_BACKEND, ficco.FICCO_COPY_STREAM)])
