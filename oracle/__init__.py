"""CPU oracle for structured activation pruning -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``oracle.c`` (plain C, binary64 arithmetic).  It
is the slow definition the GPU library is compared with and shares nothing with
it.  Only the test suite, the smoke check and the benchmark's CPU-baseline leg
may import this package; the product path never does.

Element types: ``numpy.float32`` arrays are IEEE binary32; ``numpy.uint16``
arrays are bfloat16 bit patterns.

Paper passages followed: Sec. IV (block l2 ranking, top-k pruning), Sec. II-A
(Block Sparse Row: crow / col / values), Sec. III and Fig. 2 (weight gradient
from the pruned activation).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "oracle.c"
_LIB = _HERE / "liboracle.so"

F32, BF16 = 0, 1


def build(force: bool = False) -> Path:
    """Compile oracle.c with gcc (no BLAS, no intrinsics)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".{os.getpid()}.tmp")
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
             "-ffp-contract=off", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(str(build()))
        i64, i32, dbl, vp = C.c_int64, C.c_int, C.c_double, C.c_void_p
        lib.oracle_keep_count.restype = i64
        lib.oracle_keep_count.argtypes = [i64, dbl]
        lib.oracle_block_scores.restype = None
        lib.oracle_block_scores.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp]
        lib.oracle_select.restype = i32
        lib.oracle_select.argtypes = [vp, i64, i64, vp]
        lib.oracle_select_grouped.argtypes = [vp, i64, i64, i64, dbl, vp]
        lib.oracle_select_grouped.restype = i64
        lib.oracle_affine_dscale.restype = None
        lib.oracle_affine_dscale.argtypes = [vp, vp, i32, i64, i64, i64, i64, vp]
        lib.oracle_mask_dense.restype = None
        lib.oracle_mask_dense.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, vp, i64]
        lib.oracle_bsr_from_mask.restype = None
        lib.oracle_bsr_from_mask.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, vp, vp, vp]
        lib.oracle_bsr_to_dense.restype = None
        lib.oracle_bsr_to_dense.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, i32, vp]
        lib.oracle_dw_entry.restype = dbl
        lib.oracle_dw_entry.argtypes = [vp, vp, i32, i64, i64, i64, i64, i64]
        lib.oracle_dw.restype = None
        lib.oracle_dw.argtypes = [vp, vp, i32, i64, i64, i64, i64, i64, vp]
        lib.oracle_bsr_bytes.restype = i64
        lib.oracle_bsr_bytes.argtypes = [i64, i64, i32, i32, i32]
        lib.oracle_num_threads.restype = i32
        lib.oracle_set_threads.argtypes = [i32]
        _lib = lib
    return _lib


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bfloat16 bits), got {a.dtype}")


def _mat(a: np.ndarray) -> np.ndarray:
    if a.ndim != 2:
        raise ValueError("expected a 2-D array")
    return np.ascontiguousarray(a)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def grid(M: int, K: int, br: int, bc: int):
    """(nbr, nbc) of an [M x K] matrix cut into br x bc blocks."""
    return -(-M // br), -(-K // bc)


def keep_count(nblocks: int, keep: float) -> int:
    n = int(_load().oracle_keep_count(int(nblocks), float(keep)))
    if n < 0:
        raise ValueError("keep must lie in [0, 1]")
    return n


def block_scores(X: np.ndarray, br: int, bc: int) -> np.ndarray:
    X = _mat(X)
    M, K = X.shape
    nbr, nbc = grid(M, K, br, bc)
    out = np.empty(nbr * nbc, dtype=np.float64)
    _load().oracle_block_scores(_p(X), _dtype_of(X), M, K, K, br, bc, _p(out))
    return out


def select(scores: np.ndarray, n_keep: int) -> np.ndarray:
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    mask = np.empty(scores.size, dtype=np.uint8)
    if _load().oracle_select(_p(scores), scores.size, int(n_keep), _p(mask)) != 0:
        raise MemoryError
    return mask


def select_grouped(scores: np.ndarray, nbr: int, nbc: int, group_rows: int, keep: float):
    """Per-group selection (groups of `group_rows` block-rows) -> (mask, total kept)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    if scores.size != nbr * nbc:
        raise ValueError("scores must have nbr * nbc entries")
    mask = np.empty(scores.size, dtype=np.uint8)
    total = int(_load().oracle_select_grouped(_p(scores), int(nbr), int(nbc), int(group_rows), float(keep), _p(mask)))
    if total == -1:
        raise MemoryError
    if total < 0:
        raise ValueError("bad group size or keep ratio")
    return mask, total


def mask_dense(X: np.ndarray, br: int, bc: int, mask: np.ndarray) -> np.ndarray:
    X = _mat(X)
    M, K = X.shape
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.empty_like(X)
    _load().oracle_mask_dense(_p(X), _dtype_of(X), M, K, K, br, bc, _p(mask), _p(out), K)
    return out


def bsr_from_mask(X: np.ndarray, br: int, bc: int, mask: np.ndarray):
    X = _mat(X)
    M, K = X.shape
    nbr, _ = grid(M, K, br, bc)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n_keep = int(mask.astype(np.int64).sum())
    row_ptr = np.empty(nbr + 1, dtype=np.int32)
    col_idx = np.empty(n_keep, dtype=np.int32)
    values = np.empty((n_keep, br, bc), dtype=X.dtype)
    _load().oracle_bsr_from_mask(_p(X), _dtype_of(X), M, K, K, br, bc, _p(mask),
                                 _p(row_ptr), _p(col_idx), _p(values))
    return row_ptr, col_idx, values


def bsr_to_dense(row_ptr, col_idx, values, M: int, K: int, br: int, bc: int) -> np.ndarray:
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    values = np.ascontiguousarray(values)
    out = np.empty((M, K), dtype=values.dtype)
    _load().oracle_bsr_to_dense(_p(row_ptr), _p(col_idx), _p(values), _dtype_of(values),
                                M, K, K, br, bc, _p(out))
    return out


def dw(Xhat: np.ndarray, dY: np.ndarray) -> np.ndarray:
    """dW [K x N] in float64 from the masked dense activation."""
    Xhat, dY = _mat(Xhat), _mat(dY)
    if Xhat.dtype != dY.dtype or Xhat.shape[0] != dY.shape[0]:
        raise ValueError("Xhat and dY must share dtype and row count")
    M, K = Xhat.shape
    N = dY.shape[1]
    out = np.empty((K, N), dtype=np.float64)
    _load().oracle_dw(_p(Xhat), _p(dY), _dtype_of(Xhat), M, K, K, N, N, _p(out))
    return out


def affine_dscale(Xhat: np.ndarray, dY: np.ndarray) -> np.ndarray:
    """Scale gradient of the affine layer y = alpha * x + beta from the masked dense input:
    dalpha [K] in float64, dalpha[k] = sum_m Xhat[m,k] * dY[m,k]  (dY has the shape of X)."""
    Xhat, dY = _mat(Xhat), _mat(dY)
    if Xhat.dtype != dY.dtype or Xhat.shape != dY.shape:
        raise ValueError("Xhat and dY must share dtype and shape")
    M, K = Xhat.shape
    out = np.empty(K, dtype=np.float64)
    _load().oracle_affine_dscale(_p(Xhat), _p(dY), _dtype_of(Xhat), M, K, K, K, _p(out))
    return out


def dw_entry(Xhat: np.ndarray, dY: np.ndarray, k: int, n: int) -> float:
    Xhat, dY = _mat(Xhat), _mat(dY)
    M, K = Xhat.shape
    N = dY.shape[1]
    return float(_load().oracle_dw_entry(_p(Xhat), _p(dY), _dtype_of(Xhat), M, K, N, int(k), int(n)))


def bsr_bytes(n_keep: int, nbr: int, br: int, bc: int, elem_bytes: int) -> int:
    return int(_load().oracle_bsr_bytes(n_keep, nbr, br, bc, elem_bytes))


def prune(X: np.ndarray, br: int, bc: int, keep: float):
    """Whole forward-side path: scores -> mask -> (row_ptr, col_idx, values)."""
    nbr, nbc = grid(X.shape[0], X.shape[1], br, bc)
    scores = block_scores(X, br, bc)
    mask = select(scores, keep_count(nbr * nbc, keep))
    return (scores, mask) + bsr_from_mask(X, br, bc, mask)
