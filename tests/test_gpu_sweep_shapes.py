"""GPU parity at the corners of the heuristic sweep (Sec. V-C / Sec. VI-D shapes: 8 shards,
M in {4096, 16384, 65536}, K in {4096, 8192}, N in {512, 1024, 3584, 14336}).

The oracle cannot finish these products in seconds, so it computes sampled rows one by one: 64 random
rows plus the first and the last row of every piece of the plan the library's own rule builds, all N
columns. The serial schedule is checked against those rows at the usual tolerance; the schedule the
library picks, and the finest piece count of the sweep, must then equal the serial result bit for
bit everywhere (every output element is accumulated over k in the same order whatever the schedule).
Inputs are the sweep's seeded bits from ficco_inputs, staged in device memory."""
import numpy as np
import pytest

import ficco_inputs as fi
import paper_2512_10236_amd as ficco
from oracle import gemm as og

from test_gpu_parity import check, run_ag

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

G = fi.SWEEP["shards"]
CORNERS = [(65536, 8192, 14336), (65536, 4096, 512), (4096, 8192, 14336)]


@pytest.mark.parametrize("M,K,N", CORNERS)
def test_sweep_corner_matches_oracle_rows_and_serial_bits(gpu, M, K, N):
    assert M in fi.SWEEP["M"] and K in fi.SWEEP["K"] and N in fi.SWEEP["N"]
    print(f"sweep corner {M}x{K}x{N}: inputs", flush=True)
    shards = fi.make_shards(fi.SWEEP["seed"], M, K, G)
    W = fi.make_weight(fi.SWEEP["seed"], K, N)
    sched, c = ficco.ficco_pick_schedule(M, K, N, G)
    assert sched != ficco.FICCO_FINE_2D                    # row pieces: the caller's row-major layout
    m = M // (G * c)
    rng = np.random.default_rng(M + K + N)
    rows = np.unique(np.concatenate([rng.integers(0, M, 64), np.arange(0, M, m), np.arange(m - 1, M, m)]))
    print(f"sweep corner {M}x{K}x{N}: oracle on {rows.size} rows", flush=True)
    ref = og.ag_gemm_rows(shards, W, rows)
    print(f"sweep corner {M}x{K}x{N}: serial", flush=True)
    base, _, _ = run_ag(gpu, shards, W, ficco.FICCO_SERIAL, 1, src="device")
    check(base[rows], ref, f"serial {M}x{K}x{N}")
    print(f"sweep corner {M}x{K}x{N}: the library's pick ({ficco.SCHEDULE_NAMES[sched]}, {c} pieces per shard)", flush=True)
    bits, _, info = run_ag(gpu, shards, W, ficco.FICCO_AUTO, 1, src="device")
    assert (info.schedule, info.chunks) == (sched, c)
    assert np.array_equal(bits, base), f"the picked schedule differs bitwise from serial at {M}x{K}x{N}"
    c_fine = max(cc for cc in fi.SWEEP["chunks_per_shard"] if (M // G) % cc == 0)
    print(f"sweep corner {M}x{K}x{N}: {c_fine} pieces per shard, fused launches", flush=True)
    bits, _, _ = run_ag(gpu, shards, W, ficco.FICCO_FINE_FUSED, c_fine, src="device")
    assert np.array_equal(bits, base), f"fused c={c_fine} differs bitwise from serial at {M}x{K}x{N}"
