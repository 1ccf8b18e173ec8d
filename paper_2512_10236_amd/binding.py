"""Thin ctypes binding of libficco (include/ficco.h): same names, argument marshalling only.

Every step of the path (transfers, flags, GEMM kernels, statistics) runs inside the library.
There is no CPU fallback: if the HIP library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

from . import _build

# ---- enums (mirrors of include/ficco.h)
FICCO_OK, FICCO_ERR_ARG, FICCO_ERR_SHAPE, FICCO_ERR_ALLOC = 0, -1, -2, -3
FICCO_ERR_HIP, FICCO_ERR_TIMEOUT, FICCO_ERR_STATE = -4, -5, -6
FICCO_SERIAL, FICCO_SHARD, FICCO_FINE_UNFUSED, FICCO_FINE_FUSED, FICCO_FINE_PERSISTENT, FICCO_FINE_2D = 0, 1, 2, 3, 4, 5
FICCO_AUTO = 100
FICCO_AUTO_ANY = 101
FICCO_STATIC_MAX_WEIGHT_BYTES = 8 << 20
FICCO_DIR_AG_GEMM, FICCO_DIR_GEMM_RS = 0, 1
FICCO_ORDER_STEP_MAJOR, FICCO_ORDER_SHARD_MAJOR, FICCO_ORDER_CUSTOM = 0, 1, 2
FICCO_MODE_PAIR, FICCO_MODE_GEMM_ONLY, FICCO_MODE_COPY_ONLY, FICCO_MODE_INDEPENDENT = 0, 1, 2, 3
(FICCO_OPT_DIRECTION, FICCO_OPT_ORDER, FICCO_OPT_MODE, FICCO_OPT_TIMING, FICCO_OPT_TILE,
 FICCO_OPT_FLAG_WRITE, FICCO_OPT_SPIN_LIMIT_US, FICCO_OPT_LOCAL_SHARD, FICCO_OPT_HOLD_FLAGS,
 FICCO_OPT_COPY_BACKEND, FICCO_OPT_LINKS, FICCO_OPT_PACKING, FICCO_OPT_REPEAT,
 FICCO_OPT_TILE_GROUP, FICCO_OPT_TILE_COLUMN_LISTS, FICCO_OPT_SOURCE_LAYOUT) = range(16)
FICCO_LAYOUT_ROW_MAJOR, FICCO_LAYOUT_K_SLICED, FICCO_LAYOUT_ROW_MAJOR_HOST = 0, 1, 2
FICCO_COPY_AUTO, FICCO_COPY_STREAM, FICCO_COPY_ENGINES = 0, 1, 2
(FICCO_TILE_AUTO, FICCO_TILE_256x256, FICCO_TILE_128x128, FICCO_TILE_256x128, FICCO_TILE_128x256,
 FICCO_TILE_64x256, FICCO_TILE_32x256, FICCO_TILE_128x128_DEEP, FICCO_TILE_128x192,
 FICCO_TILE_256x192) = range(10)

SCHEDULE_NAMES = {FICCO_SERIAL: "serial", FICCO_SHARD: "shard", FICCO_FINE_UNFUSED: "fine_unfused",
                  FICCO_FINE_FUSED: "fine_fused", FICCO_FINE_PERSISTENT: "fine_persistent",
                  FICCO_FINE_2D: "fine_2d"}


class ficco_plan_info_t(C.Structure):
    _fields_ = [("M", C.c_int64), ("K", C.c_int64), ("N", C.c_int64),
                ("shards", C.c_int32), ("chunks", C.c_int32),
                ("schedule", C.c_int32), ("direction", C.c_int32), ("order", C.c_int32), ("mode", C.c_int32),
                ("n_chunks", C.c_int32), ("n_groups", C.c_int32), ("chunk_rows", C.c_int64),
                ("tile_m", C.c_int32), ("tile_n", C.c_int32), ("tile_k", C.c_int32),
                ("resident_grid", C.c_int32), ("copy_backend", C.c_int32), ("links", C.c_int32),
                ("otb", C.c_double), ("mt_bytes", C.c_double)]


class ficco_stats_t(C.Structure):
    _fields_ = [("wall_us", C.c_double), ("copy_span_us", C.c_double), ("gemm_span_us", C.c_double),
                ("gemm_busy_us", C.c_double), ("copy_busy_us", C.c_double), ("exposed_comm_us", C.c_double),
                ("eff_tflops", C.c_double), ("copy_gbps", C.c_double),
                ("flops", C.c_int64), ("copy_bytes", C.c_int64),
                ("n_copies", C.c_int32), ("n_launches", C.c_int32), ("timed_out", C.c_int32),
                ("run_index", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class ficco_losses_t(C.Structure):
    _fields_ = [("t_gemm_whole_us", C.c_double), ("t_gemm_pieces_us", C.c_double),
                ("t_gemm_pieces_cont_us", C.c_double), ("t_copy_whole_us", C.c_double),
                ("t_copy_pieces_us", C.c_double), ("t_copy_pieces_cont_us", C.c_double),
                ("gemm_dil", C.c_double), ("gemm_cil", C.c_double),
                ("comm_dil", C.c_double), ("comm_cil", C.c_double), ("ideal_us", C.c_double),
                ("t_gemm_pieces_single_us", C.c_double), ("t_gemm_pieces_busy_us", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


EXPORTS = ["ficco_plan", "ficco_plan_grouped", "ficco_plan_pieces", "ficco_plan_set_slice_widths", "ficco_plan_slices", "ficco_plan_chain", "ficco_plan_set", "ficco_plan_set_arrival", "ficco_plan_info", "ficco_plan_arrival",
           "ficco_pack_weight", "ficco_run", "ficco_gemm_static", "ficco_graph_capture", "ficco_graph_launch", "ficco_rs_reduce", "ficco_query_stats", "ficco_query_spans", "ficco_profile_losses",
           "ficco_pick_schedule", "ficco_pick_schedule_rs", "ficco_pick_schedule_any", "ficco_pick_schedule_layout", "ficco_pick_slice_widths", "ficco_static_descriptors", "ficco_ideal_overlap_us", "ficco_destroy",
           "ficco_strerror", "ficco_last_hip_error", "ficco_version"]

_lib = None


def library_path() -> str:
    """The in-tree library, or the one FICCO_LIBRARY names (a measuring build made by ``_build.build_variant``)."""
    return os.environ.get("FICCO_LIBRARY") or _build.LIB


def load():
    """Load libficco.so (building nothing: run ``__graft_entry__.build()`` first). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python __graft_entry__.py` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    vp, i64, i32p = C.c_void_p, C.c_int64, C.POINTER(C.c_int32)
    dp = C.POINTER(C.c_double)
    lib.ficco_plan.argtypes = [i64, i64, i64, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    lib.ficco_plan_grouped.argtypes = [i64, i64, C.c_int, C.c_int, C.POINTER(i64), C.c_int, C.c_int, C.POINTER(vp)]
    lib.ficco_plan_pieces.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.c_int]
    lib.ficco_plan_set_slice_widths.argtypes = [vp, C.POINTER(i64), C.c_int]
    lib.ficco_plan_slices.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.c_int]
    lib.ficco_plan_chain.argtypes = [vp, vp]
    lib.ficco_plan_set.argtypes = [vp, C.c_int, i64]
    lib.ficco_plan_set_arrival.argtypes = [vp, i32p, C.c_int]
    lib.ficco_plan_info.argtypes = [vp, C.POINTER(ficco_plan_info_t)]
    lib.ficco_plan_arrival.argtypes = [vp, i32p, i32p, C.c_int]
    lib.ficco_pack_weight.argtypes = [vp, vp, vp]
    lib.ficco_run.argtypes = [vp, vp, vp, vp, vp, C.POINTER(vp), vp, vp]
    lib.ficco_gemm_static.argtypes = [i64, i64, i64, vp, vp, vp, vp]
    lib.ficco_graph_capture.argtypes = [vp, vp, vp, vp, vp, C.POINTER(vp)]
    lib.ficco_graph_launch.argtypes = [vp, vp]
    lib.ficco_rs_reduce.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp]
    lib.ficco_query_stats.argtypes = [vp, C.POINTER(ficco_stats_t)]
    lib.ficco_query_spans.argtypes = [vp, dp, dp, C.c_int, dp, dp, C.c_int]
    lib.ficco_profile_losses.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_int, C.c_int, C.POINTER(ficco_losses_t)]
    lib.ficco_pick_schedule.argtypes = [i64, i64, i64, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.ficco_pick_schedule_any.argtypes = [i64, i64, i64, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.ficco_pick_schedule_rs.argtypes = [i64, i64, i64, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.ficco_pick_schedule_layout.argtypes = [i64, i64, i64, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.ficco_pick_slice_widths.argtypes = [i64, i64, i64, C.c_int, C.c_int, C.POINTER(i64)]
    lib.ficco_static_descriptors.argtypes = [i64, i64, i64, dp, dp]
    lib.ficco_ideal_overlap_us.argtypes = [C.c_double, C.c_double, C.c_int]
    lib.ficco_ideal_overlap_us.restype = C.c_double
    lib.ficco_destroy.argtypes = [vp]
    lib.ficco_destroy.restype = None
    lib.ficco_strerror.argtypes = [C.c_int]
    lib.ficco_strerror.restype = C.c_char_p
    lib.ficco_last_hip_error.restype = C.c_int
    lib.ficco_version.restype = C.c_char_p
    _lib = lib
    return lib


class FiccoError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load()
        msg = lib.ficco_strerror(status).decode()
        if status == FICCO_ERR_HIP:
            msg += f" (hipError {lib.ficco_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")
        self.status = status


def _ok(status: int, where: str) -> int:
    if status != FICCO_OK:
        raise FiccoError(status, where)
    return status


def _ptr(x):
    """Address of a buffer: an int, None, or anything with ``data_ptr()`` (a torch tensor)."""
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    if hasattr(x, "cuda_stream"):          # torch.cuda.Stream
        return C.c_void_p(x.cuda_stream)
    raise TypeError(type(x))


# ---- the entry points, one Python function per C function ------------------------------------
def ficco_plan(M, K, N, shards, chunks, schedule):
    out = C.c_void_p()
    _ok(load().ficco_plan(M, K, N, shards, chunks, schedule, C.byref(out)), "ficco_plan")
    return out


def ficco_plan_grouped(K, N, rows, chunks, schedule):
    """``rows``: nested sequence ``[peers][experts]`` of token counts."""
    peers, experts = len(rows), len(rows[0])
    flat = (C.c_int64 * (peers * experts))(*[int(rows[j][e]) for j in range(peers) for e in range(experts)])
    out = C.c_void_p()
    _ok(load().ficco_plan_grouped(K, N, peers, experts, flat, chunks, schedule, C.byref(out)), "ficco_plan_grouped")
    return out


def ficco_plan_pieces(plan):
    n = ficco_plan_info(plan).n_chunks
    r0, nr = (C.c_int64 * n)(), (C.c_int64 * n)()
    _ok(load().ficco_plan_pieces(plan, r0, nr, n), "ficco_plan_pieces")
    return list(r0), list(nr)


def ficco_plan_set_slice_widths(plan, widths):
    """``widths``: columns of every slice of a FICCO_FINE_2D plan, or ``None`` for equal slices."""
    if widths is None:
        return _ok(load().ficco_plan_set_slice_widths(plan, None, 0), "ficco_plan_set_slice_widths")
    arr = (C.c_int64 * len(widths))(*[int(w) for w in widths])
    return _ok(load().ficco_plan_set_slice_widths(plan, arr, len(widths)), "ficco_plan_set_slice_widths")


def ficco_plan_slices(plan):
    n = ficco_plan_info(plan).chunks
    k0, w = (C.c_int64 * n)(), (C.c_int64 * n)()
    _ok(load().ficco_plan_slices(plan, k0, w, n), "ficco_plan_slices")
    return list(k0), list(w)


def ficco_plan_chain(plan, after):
    """Transfers of ``plan``'s runs wait (on the device) for the latest run of ``after``; ``None`` unchains."""
    return _ok(load().ficco_plan_chain(plan, after), "ficco_plan_chain")


def ficco_plan_set(plan, option, value):
    return _ok(load().ficco_plan_set(plan, option, int(value)), "ficco_plan_set")


def ficco_plan_set_arrival(plan, chunk_ids):
    arr = (C.c_int32 * len(chunk_ids))(*[int(i) for i in chunk_ids])
    return _ok(load().ficco_plan_set_arrival(plan, arr, len(chunk_ids)), "ficco_plan_set_arrival")


def ficco_plan_info(plan) -> ficco_plan_info_t:
    out = ficco_plan_info_t()
    _ok(load().ficco_plan_info(plan, C.byref(out)), "ficco_plan_info")
    return out


def ficco_plan_arrival(plan):
    n = ficco_plan_info(plan).n_chunks
    a, g = (C.c_int32 * n)(), (C.c_int32 * n)()
    _ok(load().ficco_plan_arrival(plan, a, g, n), "ficco_plan_arrival")
    return list(a), list(g)


def ficco_pack_weight(plan, W_dev, stream):
    return _ok(load().ficco_pack_weight(plan, _ptr(W_dev), _ptr(stream)), "ficco_pack_weight")


def ficco_run(plan, A_src, A_dev, W_dev, C_dev, peer_out, compute_stream, copy_stream):
    peers = None
    if peer_out is not None:
        peers = (C.c_void_p * len(peer_out))(*[_ptr(p) for p in peer_out])
    return _ok(load().ficco_run(plan, _ptr(A_src), _ptr(A_dev), _ptr(W_dev), _ptr(C_dev), peers,
                                _ptr(compute_stream), _ptr(copy_stream)), "ficco_run")


def ficco_gemm_static(M, K, N, A_dev, W_dev, C_dev, stream):
    """The resident GEMM over operands in place, without any device allocation (see include/ficco.h)."""
    return _ok(load().ficco_gemm_static(M, K, N, _ptr(A_dev), _ptr(W_dev), _ptr(C_dev), _ptr(stream)), "ficco_gemm_static")


def ficco_graph_capture(plan, A_src, A_dev, W_dev, C_dev, peer_out):
    peers = None
    if peer_out is not None:
        peers = (C.c_void_p * len(peer_out))(*[_ptr(p) for p in peer_out])
    return _ok(load().ficco_graph_capture(plan, _ptr(A_src), _ptr(A_dev), _ptr(W_dev), _ptr(C_dev), peers),
               "ficco_graph_capture")


def ficco_rs_reduce(plan, block, P_src, P_dev, own, out, stream):
    return _ok(load().ficco_rs_reduce(plan, block, _ptr(P_src), _ptr(P_dev), _ptr(own), _ptr(out), _ptr(stream)),
               "ficco_rs_reduce")


def ficco_graph_launch(plan, stream):
    return _ok(load().ficco_graph_launch(plan, _ptr(stream)), "ficco_graph_launch")


def ficco_query_stats(plan, allow_timeout: bool = False) -> ficco_stats_t:
    out = ficco_stats_t()
    st = load().ficco_query_stats(plan, C.byref(out))
    if st == FICCO_ERR_TIMEOUT and allow_timeout:
        return out
    _ok(st, "ficco_query_stats")
    return out


def ficco_query_spans(plan):
    info = ficco_plan_info(plan)
    n, g = info.n_chunks, info.n_groups
    cb, ce, gb, ge = (C.c_double * n)(), (C.c_double * n)(), (C.c_double * g)(), (C.c_double * g)()
    _ok(load().ficco_query_spans(plan, cb, ce, n, gb, ge, g), "ficco_query_spans")
    return list(cb), list(ce), list(gb), list(ge)


def ficco_profile_losses(plan, A_src, A_dev, W_dev, C_dev, compute_stream, copy_stream,
                         warmup=10, iters=5) -> ficco_losses_t:
    out = ficco_losses_t()
    _ok(load().ficco_profile_losses(plan, _ptr(A_src), _ptr(A_dev), _ptr(W_dev), _ptr(C_dev),
                                    _ptr(compute_stream), _ptr(copy_stream), warmup, iters, C.byref(out)),
        "ficco_profile_losses")
    return out


def ficco_pick_schedule(M, K, N, shards):
    s, c = C.c_int(), C.c_int()
    _ok(load().ficco_pick_schedule(M, K, N, shards, C.byref(s), C.byref(c)), "ficco_pick_schedule")
    return s.value, c.value


def ficco_pick_schedule_rs(M, K, N, shards):
    """The piece-count rule for the GEMM -> reduce-scatter direction."""
    s, c = C.c_int(), C.c_int()
    _ok(load().ficco_pick_schedule_rs(M, K, N, shards, C.byref(s), C.byref(c)), "ficco_pick_schedule_rs")
    return s.value, c.value


def ficco_pick_slice_widths(M, K, N, shards, slices):
    w = (C.c_int64 * max(int(slices), 1))()
    _ok(load().ficco_pick_slice_widths(M, K, N, shards, slices, w), "ficco_pick_slice_widths")
    return list(w)[:slices]


def ficco_pick_schedule_layout(M, K, N, shards, source_layout):
    """As :func:`ficco_pick_schedule_any` for a given ficco_source_layout of A_src."""
    s, c = C.c_int(), C.c_int()
    _ok(load().ficco_pick_schedule_layout(M, K, N, shards, source_layout, C.byref(s), C.byref(c)), "ficco_pick_schedule_layout")
    return s.value, c.value


def ficco_pick_schedule_any(M, K, N, shards):
    """As :func:`ficco_pick_schedule` with column pieces allowed (may answer FICCO_FINE_2D); A_src row-major."""
    s, c = C.c_int(), C.c_int()
    _ok(load().ficco_pick_schedule_any(M, K, N, shards, C.byref(s), C.byref(c)), "ficco_pick_schedule_any")
    return s.value, c.value


def ficco_static_descriptors(m, N, K):
    otb, mt = C.c_double(), C.c_double()
    _ok(load().ficco_static_descriptors(m, N, K, C.byref(otb), C.byref(mt)), "ficco_static_descriptors")
    return otb.value, mt.value


def ficco_ideal_overlap_us(t_comm_us, t_gemm_us, n):
    return float(load().ficco_ideal_overlap_us(t_comm_us, t_gemm_us, n))


def ficco_destroy(plan):
    load().ficco_destroy(plan)


def ficco_strerror(status):
    return load().ficco_strerror(status).decode()


def ficco_version():
    return load().ficco_version().decode()
