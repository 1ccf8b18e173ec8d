"""GPU parity of the reduce-scatter receiver (ficco_rs_reduce) against the oracle: bit-exact, since the
sum is defined operation by operation (fp32, ascending GPU order, one rounding)."""
import numpy as np
import pytest

import ficco_inputs as fi
import paper_2512_10236_amd as ficco
from oracle import gemm as og
from oracle import reduce as orr

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

NAN_BF16 = 0x7FC0


def as_i16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))


def reduce_once(gpu, x, block, sched, c, *, src="device", opts=(), runs=1, allow_timeout=False):
    """x: [G, rows, N] bf16 bits, x[block] is the receiver's own partial block. Returns (out bits, stats)."""
    dev = gpu["dev"]
    G, rows, N = x.shape
    P_src = as_i16(x).pin_memory() if src == "pinned" else as_i16(x).to(dev)
    if src == "device":
        P_src[block].fill_(NAN_BF16)                     # the receiver's slot of the source is never read
    P_dev = torch.full((G, rows, N), NAN_BF16, dtype=torch.int16, device=dev)
    own = as_i16(x[block]).to(dev)
    out = torch.full((rows, N), 0x7FFF, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()
    plan = ficco.ficco_plan(G * rows, 64, N, G, c, sched)
    try:
        for o, v in opts:
            ficco.ficco_plan_set(plan, o, v)
        for r in range(runs):
            if r:
                P_dev.fill_(NAN_BF16)
                out.fill_(0x7FFF)
                torch.cuda.synchronize()
            ficco.ficco_rs_reduce(plan, block, P_src, P_dev, own, out, gpu["cs"])
            st = ficco.ficco_query_stats(plan, allow_timeout=allow_timeout)
    finally:
        ficco.ficco_destroy(plan)
    torch.cuda.synchronize()
    assert np.array_equal(P_dev[block].cpu().numpy().view(np.uint16), np.full((rows, N), NAN_BF16, np.uint16)), "own slot was written"
    return out.cpu().numpy().view(np.uint16), st


CASES = [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_SHARD, 1), (ficco.FICCO_FINE_FUSED, 4), (ficco.FICCO_FINE_PERSISTENT, 8)]


@pytest.mark.parametrize("G,rows,N,block", [(4, 64, 256, 1), (8, 96, 328, 7), (3, 40, 8, 0), (1, 16, 64, 0)])
def test_reduce_is_bit_exact_for_every_schedule(gpu, G, rows, N, block):
    x = fi.make_partials(31, G, rows, N)
    want = orr.rs_reduce(list(x))
    for sched, c in CASES:
        if rows % c:
            c = 1 if sched in (ficco.FICCO_SERIAL, ficco.FICCO_SHARD) else 2
        for src in ("device", "pinned"):
            got, st = reduce_once(gpu, x, block, sched, c, src=src, runs=2)
            assert np.array_equal(got, want), f"G={G} rows={rows} N={N} sched={sched} c={c} {src}"
            assert st.n_copies == (G - 1) * c and st.copy_bytes == (G - 1) * rows * N * 2 and st.n_launches == 1
            assert st.flops == (G - 1) * rows * N


def test_reduce_orders_flag_modes_and_links(gpu):
    G, rows, N, block = 8, 256, 512, 3
    x = fi.make_partials(32, G, rows, N)
    want = orr.rs_reduce(list(x))
    for opts in ([(ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)], [(ficco.FICCO_OPT_FLAG_WRITE, 2)],
                 [(ficco.FICCO_OPT_LINKS, 3)], [(ficco.FICCO_OPT_LINKS, 1), (ficco.FICCO_OPT_ORDER, ficco.FICCO_ORDER_SHARD_MAJOR)]):
        got, _ = reduce_once(gpu, x, block, ficco.FICCO_FINE_FUSED, 4, opts=opts, runs=2)
        assert np.array_equal(got, want), opts


def test_reduce_hand_cases_on_gpu(gpu):
    # the order and rounding cases the oracle is pinned with, replicated over a tile and a ragged tail
    def b(v):
        return (np.float32(v).view(np.uint32) >> 16).astype(np.uint16)
    rows, N = 33, 264                                   # 8712 elements: one full tile of 8192 and a tail
    cases = [([2.0 ** 24, 1.0, -(2.0 ** 24)], 0.0), ([2.0 ** 24, -(2.0 ** 24), 1.0], 1.0), ([1.0, 2.0 ** -8, 0.0], 1.0),
             ([1.0 + 2.0 ** -7, 2.0 ** -8, 0.0], 1.0 + 2.0 ** -6), ([-0.0, -0.0, -0.0], -0.0)]
    for vals, want in cases:
        x = np.stack([np.full((rows, N), b(v), dtype=np.uint16) for v in vals])
        for block in range(3):
            got, _ = reduce_once(gpu, x, block, ficco.FICCO_FINE_FUSED, 3)
            assert np.array_equal(got, np.full((rows, N), b(want), dtype=np.uint16)), (vals, block)
            assert np.array_equal(got, orr.rs_reduce(list(x)))


def test_reduce_after_gemm_rs_completes_the_pair(gpu):
    # this GPU's partial product (a GEMM_RS run) supplies `own`; the peers' partials are synthetic
    dev = gpu["dev"]
    M, K, N, G, block = 1024, 256, 512, 8, 5
    A = fi.normal_bf16(3, fi.TENSOR_A, M, K)
    W = fi.make_weight(3, K, N)
    x = fi.make_partials(33, G, M // G, N)
    A_dev, W_dev = as_i16(A).to(dev), as_i16(W).to(dev)
    C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
    peers = [torch.zeros((M // G, N), dtype=torch.int16, device=dev) for _ in range(G)]
    P_src = as_i16(x).to(dev)
    P_dev = torch.full((G, M // G, N), NAN_BF16, dtype=torch.int16, device=dev)
    out = torch.zeros((M // G, N), dtype=torch.int16, device=dev)
    torch.cuda.synchronize()
    plan = ficco.ficco_plan(M, K, N, G, 2, ficco.FICCO_FINE_FUSED)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_DIRECTION, ficco.FICCO_DIR_GEMM_RS)
        ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, peers, gpu["cs"], gpu["xs"])
        ficco.ficco_query_stats(plan)
        ficco.ficco_rs_reduce(plan, block, P_src, P_dev, C_dev[block * (M // G):(block + 1) * (M // G)], out, gpu["cs"])
        ficco.ficco_query_stats(plan)
    finally:
        ficco.ficco_destroy(plan)
    torch.cuda.synchronize()
    own = C_dev[block * (M // G):(block + 1) * (M // G)].cpu().numpy().view(np.uint16)
    ref_own = og.gemm_rs_blocks(A, W, G)[block]
    assert og.rel_err(fi.bf16_bits_to_f32(own).astype(np.float64), ref_own) <= 8e-3
    blocks = [own if j == block else x[j] for j in range(G)]
    assert np.array_equal(out.cpu().numpy().view(np.uint16), orr.rs_reduce(blocks))


def test_reduce_gives_up_when_pieces_never_arrive(gpu):
    x = fi.make_partials(34, 4, 64, 256)
    _, st = reduce_once(gpu, x, 0, ficco.FICCO_FINE_FUSED, 4, allow_timeout=True,
                        opts=[(ficco.FICCO_OPT_HOLD_FLAGS, 1), (ficco.FICCO_OPT_SPIN_LIMIT_US, 5000)])
    assert st.timed_out == 1
    got, st2 = reduce_once(gpu, x, 0, ficco.FICCO_FINE_FUSED, 4)
    assert st2.timed_out == 0 and np.array_equal(got, orr.rs_reduce(list(x)))


def test_reduce_rejects_bad_arguments(gpu):
    dev = gpu["dev"]
    t = torch.zeros((4, 64, 64), dtype=torch.int16, device=dev)
    o = torch.zeros((64, 64), dtype=torch.int16, device=dev)
    plan = ficco.ficco_plan(256, 64, 64, 4, 2, ficco.FICCO_FINE_FUSED)
    try:
        for args in [(4, t, t, o, o), (-1, t, t, o, o), (0, None, t, o, o), (0, t, t, None, o), (0, t, t, o, o.cpu())]:
            with pytest.raises((ficco.FiccoError, TypeError)):
                ficco.ficco_rs_reduce(plan, *args, gpu["cs"])
    finally:
        ficco.ficco_destroy(plan)
    plan = ficco.ficco_plan(256, 128, 64, 4, 2, ficco.FICCO_FINE_2D)
    try:
        with pytest.raises(ficco.FiccoError):
            ficco.ficco_rs_reduce(plan, 0, t, t, o, o, gpu["cs"])
    finally:
        ficco.ficco_destroy(plan)


def test_reduce_full_size_block(gpu):
    # the block bench.py times: 2048 x 8192, 8 GPUs, two pieces per block
    cfg = fi.CONFIGS["cfg4_gemm_rs"]
    G, rows, N = cfg["shards"], cfg["M"] // cfg["shards"], cfg["N"]
    x = fi.make_partials(cfg["seed"], G, rows, N)
    want = orr.rs_reduce(list(x))
    for sched, c in [(ficco.FICCO_SERIAL, 1), (ficco.FICCO_FINE_FUSED, 2)]:
        got, st = reduce_once(gpu, x, 0, sched, c)
        assert np.array_equal(got, want), (sched, c)
