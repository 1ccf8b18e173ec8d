"""ficco_gemm_static - the entry point for callers that cannot allocate device memory - against the
existing entry point it is a variant of: ficco_run() of a one-shard, one-piece resident plan with the
operands in place (FICCO_MODE_GEMM_ONLY). Same kernel, same tile, same tile order: the outputs must be
equal bit for bit, and within the oracle's tolerance. Two calls in a row share the library's static
device array; the second has a smaller input, so anything the first call left behind (ticket counters,
the larger packed weight) must not leak into it."""
import numpy as np
import pytest

import ficco_inputs as fi
import paper_2512_10236_amd as ficco
from oracle import gemm as og

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 8e-3


def as_i16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))


def by_plan(gpu, A_dev, W_dev, M, K, N):
    """The existing entry point: a resident plan of one piece, GEMM only."""
    C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=gpu["dev"])
    plan = ficco.ficco_plan(M, K, N, 1, 1, ficco.FICCO_FINE_PERSISTENT)
    try:
        ficco.ficco_plan_set(plan, ficco.FICCO_OPT_MODE, ficco.FICCO_MODE_GEMM_ONLY)
        ficco.ficco_run(plan, None, A_dev, W_dev, C_dev, None, gpu["cs"], gpu["xs"])
        ficco.ficco_query_stats(plan)
    finally:
        ficco.ficco_destroy(plan)
    return C_dev.cpu().numpy().view(np.uint16)


def test_static_entry_point_matches_the_plan_path_twice_in_a_row(gpu):
    dev = gpu["dev"]
    # first a shape that runs several rounds of tiles (ticket draws) with ragged edges, then a smaller one
    shapes = [(4200, 2048, 1032, 31), (520, 512, 264, 32)]
    inputs = []
    for M, K, N, seed in shapes:
        A = fi.make_shards(seed, M, K, 1)[0]
        W = fi.make_weight(seed, K, N)
        inputs.append((A, W, as_i16(A).to(dev), as_i16(W).to(dev)))
    torch.cuda.synchronize()
    outs = []
    for (M, K, N, _), (A, W, A_dev, W_dev) in zip(shapes, inputs):       # the two static calls back to back on one stream
        print(f"ficco_gemm_static {M}x{K}x{N}", flush=True)
        C_dev = torch.full((M, N), 0x7FFF, dtype=torch.int16, device=dev)
        ficco.ficco_gemm_static(M, K, N, A_dev, W_dev, C_dev, gpu["cs"])
        outs.append(C_dev)
    torch.cuda.synchronize()
    for (M, K, N, _), (A, W, A_dev, W_dev), C_dev in zip(shapes, inputs, outs):
        got = C_dev.cpu().numpy().view(np.uint16)
        want = by_plan(gpu, A_dev, W_dev, M, K, N)
        assert np.array_equal(got, want), f"static entry point differs bitwise from the plan path at {M}x{K}x{N}"
        ref = og.ag_gemm([A], W)
        out = fi.bf16_bits_to_f32(got).astype(np.float64)
        assert np.isfinite(out).all()
        assert og.rel_err(out, ref) <= TOL


def test_static_entry_point_rejects_what_it_cannot_hold(gpu):
    dev = gpu["dev"]
    t = torch.zeros(64 * 64, dtype=torch.int16, device=dev)
    K = 4096
    N_over = ficco.FICCO_STATIC_MAX_WEIGHT_BYTES // (2 * K) + 8           # one step past the limit
    for args in [(64, K, N_over), (64, 96, 64), (64, 64, 12), (0, 64, 64)]:
        with pytest.raises(ficco.FiccoError) as e:
            ficco.ficco_gemm_static(*args, t, t, t, gpu["cs"])
        assert e.value.status == ficco.FICCO_ERR_SHAPE
    with pytest.raises(ficco.FiccoError) as e:
        ficco.ficco_gemm_static(64, 64, 64, t, None, t, gpu["cs"])
    assert e.value.status == ficco.FICCO_ERR_ARG
