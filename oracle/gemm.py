"""ctypes front end of ``ficco_oracle.c`` (TEST INFRASTRUCTURE ONLY; see the package docstring).

The oracle is the *definition* of the pair's result (paper Sec. II-B, Fig. 3(a)-(b)):
``ref = [I_0; ...; I_{G-1}] @ W`` with bf16 inputs widened exactly to fp64 and fp64 accumulation
in ascending k. Schedules and chunk counts (Sec. III, V-B) must not change it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ficco_oracle.c")
_LIB = os.path.join(_HERE, "libficco_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc + OpenMP (a few hundred ms). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        pp = ctypes.POINTER(ctypes.c_void_p)
        lib.oracle_ag_gemm_f64.restype = ctypes.c_int
        lib.oracle_ag_gemm_f64.argtypes = [pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        lib.oracle_ag_gemm_rows_f64.restype = ctypes.c_int
        lib.oracle_ag_gemm_rows_f64.argtypes = [pp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                                ctypes.c_int64, ctypes.c_void_p]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _check(shards, W):
    shards = [np.ascontiguousarray(s, dtype=np.uint16) for s in shards]
    W = np.ascontiguousarray(W, dtype=np.uint16)
    assert len(shards) >= 1 and W.ndim == 2
    ms, K = shards[0].shape
    for s in shards:
        assert s.shape == (ms, K), "every shard is [M/G, K]"
    assert W.shape[0] == K, "W is [K, N]"
    ptrs = (ctypes.c_void_p * len(shards))(*[s.ctypes.data for s in shards])
    return shards, W, ms, K, W.shape[1], ptrs


def ag_gemm(shards, W) -> np.ndarray:
    """fp64 ``[G*ms, N]`` result of gathering the shards (bf16 bits) and multiplying by W (bf16 bits)."""
    shards, W, ms, K, N, ptrs = _check(shards, W)
    ref = np.empty((len(shards) * ms, N), dtype=np.float64)
    rc = _load().oracle_ag_gemm_f64(ptrs, len(shards), ms, K, W.ctypes.data, N, ref.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_ag_gemm_f64 failed")
    return ref


def ag_gemm_rows(shards, W, rows) -> np.ndarray:
    """Rows ``rows`` of :func:`ag_gemm`'s result, computed one by one (for sampling big shapes)."""
    shards, W, ms, K, N, ptrs = _check(shards, W)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((rows.size, N), dtype=np.float64)
    rc = _load().oracle_ag_gemm_rows_f64(ptrs, len(shards), ms, K, W.ctypes.data, N,
                                         rows.ctypes.data, rows.size, out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_ag_gemm_rows_f64 failed (row out of range?)")
    return out


def gemm_rs_blocks(A, W, peers: int):
    """GEMM -> reduce-scatter, data-movement half: this GPU's partial product ``A @ W`` cut into
    ``peers`` equal row blocks, block p being what peer p receives (Sec. II-A: reduce-scatter of a
    row-sharded output). The element-wise sum over GPUs is outside what one GPU computes."""
    A = np.ascontiguousarray(A, dtype=np.uint16)
    ref = ag_gemm([A], W)
    assert ref.shape[0] % peers == 0
    rb = ref.shape[0] // peers
    return [ref[p * rb:(p + 1) * rb] for p in range(peers)]


def ag_gemm_2d(A_sliced, W, shards: int) -> np.ndarray:
    """The 2D decomposition carried out step by step (Sec. V-A/B): ``A_sliced`` is
    ``[c, M, K/c]`` (bf16 bits), or a list of c blocks ``[M, k_s]`` when the slices differ in width;
    step s gathers slice s of every shard and its partial product with the matching rows
    ``[k0_s, k0_s + k_s)`` of W is accumulated into the output. fp64 throughout."""
    blocks = [np.ascontiguousarray(b, dtype=np.uint16) for b in A_sliced]
    W = np.ascontiguousarray(W, dtype=np.uint16)
    M = blocks[0].shape[0]
    assert all(b.ndim == 2 and b.shape[0] == M for b in blocks)
    assert W.shape[0] == sum(b.shape[1] for b in blocks) and M % shards == 0
    ms = M // shards
    acc = np.zeros((M, W.shape[1]), dtype=np.float64)
    k0 = 0
    for blk in blocks:
        pieces = [blk[j * ms:(j + 1) * ms] for j in range(shards)]
        acc += ag_gemm(pieces, W[k0:k0 + blk.shape[1]])
        k0 += blk.shape[1]
    return acc


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def rel_err(gpu_f64: np.ndarray, ref: np.ndarray) -> float:
    """The acceptance metric: max |gpu - ref| / (|ref| + 1)."""
    return float(np.max(np.abs(gpu_f64 - ref) / (np.abs(ref) + 1.0))) if ref.size else 0.0
