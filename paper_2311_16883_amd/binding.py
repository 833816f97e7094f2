"""ctypes binding of libbsr_actprune.so -- argument marshalling only.

Every function here has the name of the C entry point it calls (see
``include/bsr_actprune.h``) and does nothing but turn torch tensors into device
pointers, sizes and the current HIP stream, allocate missing output buffers
with torch, and raise on a non-zero status.  No step of the pruning path is
computed in Python or by torch operators; if the HIP library cannot be loaded
the import fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Sequence, Optional, Tuple

import torch

BSR_F32, BSR_BF16 = 0, 1
BSR_OP_SCORE_SELECT, BSR_OP_COMPRESS, BSR_OP_DECOMPRESS, BSR_OP_T_DENSE_MATMUL = 0, 1, 2, 3
BSR_OP_AFFINE_SCALE_GRAD = 4

BSR_OK = 0
BSR_ERR_NULL, BSR_ERR_SHAPE, BSR_ERR_DTYPE, BSR_ERR_KEEP = -1, -2, -3, -4
BSR_ERR_WORKSPACE, BSR_ERR_ALIGN, BSR_ERR_HIP, BSR_ERR_LIMIT = -5, -6, -7, -8

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libbsr_actprune.so"

EXPORTS = (
    "bsr_version", "bsr_error_string", "bsr_last_hip_error", "bsr_keep_count",
    "bsr_storage_bytes", "bsr_workspace_bytes", "bsr_score_select", "bsr_compress",
    "bsr_decompress", "bsr_t_dense_matmul", "bsr_grouped_keep_count", "bsr_score_select_grouped",
    "bsr_affine_scale_grad", "bsr_score_select_batched", "bsr_score_select_batched_workspace_bytes",
    "bsr_t_dense_matmul_batched", "bsr_t_dense_matmul_batched_workspace_bytes",
    "bsr_compress_batched", "bsr_compress_batched_workspace_bytes", "bsr_decompress_batched",
    "bsr_score_select_static", "bsr_score_select_static_max_blocks", "bsr_static_scratch_init",
    "bsr_score_select_grouped_batched",
)


class BsrError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        name = lib().bsr_error_string(code).decode()
        extra = f" (hipError_t {lib().bsr_last_hip_error()})" if code == BSR_ERR_HIP else ""
        super().__init__(f"{where}: {name}{extra}")


_lib = None


def lib() -> C.CDLL:
    """The loaded C library (built on first use only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        from . import build as _build
        _build.build_library()
    l = C.CDLL(str(LIB_PATH))
    i64, i32, dbl, vp, sz = C.c_int64, C.c_int, C.c_double, C.c_void_p, C.c_size_t
    l.bsr_version.restype = C.c_char_p
    l.bsr_version.argtypes = []
    l.bsr_error_string.restype = C.c_char_p
    l.bsr_error_string.argtypes = [i32]
    l.bsr_last_hip_error.restype = i32
    l.bsr_last_hip_error.argtypes = []
    l.bsr_keep_count.restype = i64
    l.bsr_keep_count.argtypes = [i64, dbl]
    l.bsr_storage_bytes.restype = i64
    l.bsr_storage_bytes.argtypes = [i64, i64, i32, i32, i64, i32]
    l.bsr_workspace_bytes.restype = sz
    l.bsr_workspace_bytes.argtypes = [i32, i64, i64, i64, i32, i32, i32]
    l.bsr_grouped_keep_count.restype = i64
    l.bsr_grouped_keep_count.argtypes = [i64, i64, i64, dbl]
    l.bsr_score_select_grouped.restype = i32
    l.bsr_score_select_grouped.argtypes = [vp, i32, i64, i64, i64, i32, i32, i64, dbl, vp, vp, vp, sz, vp]
    l.bsr_score_select.restype = i32
    l.bsr_score_select.argtypes = [vp, i32, i64, i64, i64, i32, i32, dbl, vp, vp, vp, sz, vp]
    l.bsr_compress.restype = i32
    l.bsr_compress.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, i64, vp, vp, vp, vp, sz, vp]
    l.bsr_decompress.restype = i32
    l.bsr_decompress.argtypes = [vp, vp, vp, i32, i64, i64, i64, i32, i32, vp, vp]
    l.bsr_t_dense_matmul.restype = i32
    l.bsr_t_dense_matmul.argtypes = [vp, vp, vp, i32, i64, i64, i32, i32, vp, i64, i64, vp, i64, i32,
                                     vp, sz, vp]
    l.bsr_score_select_batched_workspace_bytes.restype = sz
    l.bsr_score_select_batched_workspace_bytes.argtypes = [vp, i32, i32]
    l.bsr_score_select_batched.restype = i32
    l.bsr_score_select_batched.argtypes = [vp, i32, i32, vp, sz, vp]
    l.bsr_score_select_grouped_batched.restype = i32
    l.bsr_score_select_grouped_batched.argtypes = [vp, vp, i32, i32, vp, sz, vp]
    l.bsr_t_dense_matmul_batched_workspace_bytes.restype = sz
    l.bsr_t_dense_matmul_batched_workspace_bytes.argtypes = [vp, i32, i32]
    l.bsr_t_dense_matmul_batched.restype = i32
    l.bsr_t_dense_matmul_batched.argtypes = [vp, i32, i32, vp, sz, vp]
    l.bsr_compress_batched_workspace_bytes.restype = sz
    l.bsr_compress_batched_workspace_bytes.argtypes = [vp, i32, i32]
    l.bsr_compress_batched.restype = i32
    l.bsr_compress_batched.argtypes = [vp, i32, i32, vp, sz, vp]
    l.bsr_decompress_batched.restype = i32
    l.bsr_decompress_batched.argtypes = [vp, i32, i32, vp]
    l.bsr_affine_scale_grad.restype = i32
    l.bsr_affine_scale_grad.argtypes = [vp, vp, vp, i32, i64, i64, i32, i32, vp, i64, vp, i32, vp, sz, vp]
    l.bsr_score_select_static.restype = i32
    l.bsr_score_select_static.argtypes = [vp, i32, i64, i64, i64, i32, i32, dbl, vp, vp, vp]
    l.bsr_score_select_static_max_blocks.restype = i64
    l.bsr_score_select_static_max_blocks.argtypes = []
    l.bsr_static_scratch_init.restype = i32
    l.bsr_static_scratch_init.argtypes = []
    _lib = l
    return l


# ---------------------------------------------------------------------------
# marshalling helpers
# ---------------------------------------------------------------------------

def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return BSR_F32
    if t == torch.bfloat16:
        return BSR_BF16
    raise BsrError(BSR_ERR_DTYPE, f"dtype {t}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None or t.numel() == 0:
        return None if t is None else (t.data_ptr() or None)
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return h or None


def _dense2d(x: torch.Tensor, what: str) -> Tuple[int, int, int]:
    if x.dim() != 2 or not x.is_cuda:
        raise ValueError(f"{what} must be a 2-D device tensor")
    if x.shape[1] > 1 and x.stride(1) != 1:
        raise ValueError(f"{what} must be row-major (unit stride along columns)")
    ld = x.stride(0) if x.shape[0] > 1 else x.shape[1]
    if ld < x.shape[1]:
        raise ValueError(f"{what} has overlapping rows")
    return x.shape[0], x.shape[1], ld


def _workspace(nbytes: int, device, ws: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if ws is not None:
        return ws
    return torch.empty(max(nbytes, 1), dtype=torch.uint8, device=device) if nbytes > 0 else None


def _check(code: int, where: str) -> None:
    if code != BSR_OK:
        raise BsrError(code, where)


# ---------------------------------------------------------------------------
# host-side pure functions
# ---------------------------------------------------------------------------

def bsr_version() -> str:
    return lib().bsr_version().decode()


def bsr_keep_count(nblocks: int, keep: float) -> int:
    n = lib().bsr_keep_count(int(nblocks), float(keep))
    if n < 0:
        raise BsrError(BSR_ERR_KEEP, "bsr_keep_count")
    return int(n)


def bsr_storage_bytes(M: int, K: int, br: int, bc: int, n_keep: int, dtype) -> int:
    code = dtype if isinstance(dtype, int) else dtype_code(dtype)
    n = lib().bsr_storage_bytes(M, K, br, bc, n_keep, code)
    if n < 0:
        raise BsrError(BSR_ERR_SHAPE, "bsr_storage_bytes")
    return int(n)


def bsr_workspace_bytes(op: int, M: int, K: int, N: int, br: int, bc: int, dtype) -> int:
    code = dtype if isinstance(dtype, int) else dtype_code(dtype)
    return int(lib().bsr_workspace_bytes(op, M, K, N, br, bc, code))


# ---------------------------------------------------------------------------
# device entry points
# ---------------------------------------------------------------------------

def bsr_score_select(X: torch.Tensor, br: int, bc: int, keep: float, *,
                     scores: Optional[torch.Tensor] = None, want_scores: bool = False,
                     keep_mask: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                     stream=None):
    """-> keep_mask (uint8 [nblocks]) or (keep_mask, scores) when scores are requested."""
    M, K, ldx = _dense2d(X, "X")
    nblocks = (-(-M // br)) * (-(-K // bc)) if br > 0 and bc > 0 else 0
    if scores is None and want_scores:
        scores = torch.empty(nblocks, dtype=torch.float64, device=X.device)
    if keep_mask is None:
        keep_mask = torch.empty(nblocks, dtype=torch.uint8, device=X.device)
    code = dtype_code(X.dtype)
    if ws is None:
        ws = _workspace(bsr_workspace_bytes(BSR_OP_SCORE_SELECT, M, K, 0, br, bc, code), X.device, None)
    rc = lib().bsr_score_select(_ptr(X), code, M, K, ldx, br, bc, float(keep), _ptr(scores),
                                _ptr(keep_mask), _ptr(ws), ws.numel() if ws is not None else 0,
                                _stream(stream))
    _check(rc, "bsr_score_select")
    return (keep_mask, scores) if scores is not None else keep_mask


def bsr_score_select_static(X: torch.Tensor, br: int, bc: int, keep: float, keep_mask: torch.Tensor, *,
                            scores: Optional[torch.Tensor] = None, stream=None):
    """bsr_score_select without a workspace argument; the outputs are the caller's, nothing is allocated."""
    M, K, ldx = _dense2d(X, "X")
    rc = lib().bsr_score_select_static(_ptr(X), dtype_code(X.dtype), M, K, ldx, br, bc, float(keep),
                                       _ptr(scores), _ptr(keep_mask), _stream(stream))
    _check(rc, "bsr_score_select_static")
    return (keep_mask, scores) if scores is not None else keep_mask


def bsr_score_select_static_max_blocks() -> int:
    return int(lib().bsr_score_select_static_max_blocks())


def bsr_static_scratch_init() -> None:
    _check(lib().bsr_static_scratch_init(), "bsr_static_scratch_init")


def bsr_grouped_keep_count(nbr: int, nbc: int, group_rows: int, keep: float) -> int:
    n = int(lib().bsr_grouped_keep_count(int(nbr), int(nbc), int(group_rows), float(keep)))
    if n < 0:
        raise BsrError(BSR_ERR_KEEP, "bsr_grouped_keep_count")
    return n


def bsr_score_select_grouped(X: torch.Tensor, br: int, bc: int, group_rows: int, keep: float, *,
                             scores: Optional[torch.Tensor] = None, want_scores: bool = False,
                             keep_mask: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                             stream=None):
    """-> keep_mask (uint8 [nblocks]) or (keep_mask, scores); ranking groups of group_rows block-rows."""
    M, K, ldx = _dense2d(X, "X")
    nblocks = (-(-M // br)) * (-(-K // bc)) if br > 0 and bc > 0 else 0
    if scores is None and want_scores:
        scores = torch.empty(nblocks, dtype=torch.float64, device=X.device)
    if keep_mask is None:
        keep_mask = torch.empty(nblocks, dtype=torch.uint8, device=X.device)
    code = dtype_code(X.dtype)
    if ws is None:
        ws = _workspace(bsr_workspace_bytes(BSR_OP_SCORE_SELECT, M, K, 0, br, bc, code), X.device, None)
    rc = lib().bsr_score_select_grouped(_ptr(X), code, M, K, ldx, br, bc, int(group_rows), float(keep),
                                        _ptr(scores), _ptr(keep_mask), _ptr(ws),
                                        ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_score_select_grouped")
    return (keep_mask, scores) if scores is not None else keep_mask


def bsr_compress(X: torch.Tensor, br: int, bc: int, keep_mask: torch.Tensor, n_keep: int, *,
                 row_ptr: Optional[torch.Tensor] = None, col_idx: Optional[torch.Tensor] = None,
                 values: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                 stream=None):
    """-> (row_ptr int32 [nbr+1], col_idx int32 [n_keep], values [n_keep, br, bc])."""
    M, K, ldx = _dense2d(X, "X")
    nbr = -(-M // br) if br > 0 else 0
    dev = X.device
    if row_ptr is None:
        row_ptr = torch.empty(nbr + 1, dtype=torch.int32, device=dev)
    if col_idx is None:
        col_idx = torch.empty(max(n_keep, 0), dtype=torch.int32, device=dev)
    if values is None:
        values = torch.empty((max(n_keep, 0), br, bc), dtype=X.dtype, device=dev)
    code = dtype_code(X.dtype)
    if ws is None:
        ws = _workspace(bsr_workspace_bytes(BSR_OP_COMPRESS, M, K, 0, br, bc, code), dev, None)
    rc = lib().bsr_compress(_ptr(X), code, M, K, ldx, br, bc, _ptr(keep_mask), int(n_keep),
                            _ptr(row_ptr), _ptr(col_idx), _ptr(values), _ptr(ws),
                            ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_compress")
    return row_ptr, col_idx, values


def bsr_decompress(row_ptr: torch.Tensor, col_idx: torch.Tensor, values: torch.Tensor, M: int,
                   K: int, br: int, bc: int, *, out: Optional[torch.Tensor] = None, stream=None):
    """-> X_out [M x K]: kept blocks bit for bit, +0.0 elsewhere."""
    if out is None:
        out = torch.empty((M, K), dtype=values.dtype, device=values.device)
    _, _, ldx = _dense2d(out, "out")
    rc = lib().bsr_decompress(_ptr(row_ptr), _ptr(col_idx), _ptr(values), dtype_code(values.dtype),
                              M, K, ldx, br, bc, _ptr(out), _stream(stream))
    _check(rc, "bsr_decompress")
    return out


def bsr_t_dense_matmul(row_ptr: torch.Tensor, col_idx: torch.Tensor, values: torch.Tensor, M: int,
                       K: int, br: int, bc: int, dY: torch.Tensor, *,
                       dW: Optional[torch.Tensor] = None, accumulate: bool = False,
                       ws: Optional[torch.Tensor] = None, stream=None):
    """-> dW [K x N] float32 = Xhat^T dY (added to dW when accumulate)."""
    Md, N, lddy = _dense2d(dY, "dY")
    if Md != M:
        raise ValueError("dY must have M rows")
    if dW is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dW")
        dW = torch.empty((K, N), dtype=torch.float32, device=dY.device)
    _, _, lddw = _dense2d(dW, "dW")
    code = dtype_code(dY.dtype)
    if values.dtype != dY.dtype:
        raise BsrError(BSR_ERR_DTYPE, "values and dY differ in dtype")
    if ws is None:
        ws = _workspace(bsr_workspace_bytes(BSR_OP_T_DENSE_MATMUL, M, K, N, br, bc, code), dY.device, None)
    rc = lib().bsr_t_dense_matmul(_ptr(row_ptr), _ptr(col_idx), _ptr(values), code, M, K, br, bc,
                                  _ptr(dY), N, lddy, _ptr(dW), lddw, 1 if accumulate else 0,
                                  _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_t_dense_matmul")
    return dW


def bsr_affine_scale_grad(row_ptr: torch.Tensor, col_idx: torch.Tensor, values: torch.Tensor, M: int,
                          K: int, br: int, bc: int, dY: torch.Tensor, *,
                          dalpha: Optional[torch.Tensor] = None, accumulate: bool = False,
                          ws: Optional[torch.Tensor] = None, stream=None):
    """-> dalpha [K] float32: scale gradient of the affine layer from its pruned input (dY is [M x K])."""
    Md, Kd, lddy = _dense2d(dY, "dY")
    if Md != M or Kd != K:
        raise ValueError("dY must be [M x K]")
    if dalpha is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dalpha")
        dalpha = torch.empty(K, dtype=torch.float32, device=dY.device)
    code = dtype_code(dY.dtype)
    if values.dtype != dY.dtype:
        raise BsrError(BSR_ERR_DTYPE, "values and dY differ in dtype")
    if ws is None:
        ws = _workspace(bsr_workspace_bytes(BSR_OP_AFFINE_SCALE_GRAD, M, K, 0, br, bc, code), dY.device, None)
    rc = lib().bsr_affine_scale_grad(_ptr(row_ptr), _ptr(col_idx), _ptr(values), code, M, K, br, bc,
                                     _ptr(dY), lddy, _ptr(dalpha), 1 if accumulate else 0,
                                     _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_affine_scale_grad")
    return dalpha


class _SelectItem(C.Structure):
    """Mirror of bsr_select_item."""
    _fields_ = [("X", C.c_void_p), ("M", C.c_int64), ("K", C.c_int64), ("ldx", C.c_int64),
                ("br", C.c_int32), ("bc", C.c_int32), ("keep", C.c_double),
                ("scores", C.c_void_p), ("keep_mask", C.c_void_p)]


class SelectBatch:
    """The marshalled item array of one bsr_score_select_batched call; build it once for tensors
    that stay where they are and pass it again every step.  Holds references to the tensors."""

    def __init__(self, Xs: Sequence[torch.Tensor], blocks: Sequence[Tuple[int, int]], keeps: Sequence[float],
                 keep_masks: Optional[Sequence[torch.Tensor]] = None,
                 scores: Optional[Sequence[Optional[torch.Tensor]]] = None):
        n = len(Xs)
        if not (len(blocks) == len(keeps) == n) or n == 0:
            raise ValueError("one block shape and one keep ratio per tensor")
        self.dtype = dtype_code(Xs[0].dtype)
        self.device = Xs[0].device
        if keep_masks is None:
            keep_masks = []
            for X, (br, bc) in zip(Xs, blocks):
                M, K, _ = _dense2d(X, "X")
                keep_masks.append(torch.empty((-(-M // br)) * (-(-K // bc)), dtype=torch.uint8, device=X.device))
        self.Xs, self.keep_masks, self.scores = list(Xs), list(keep_masks), list(scores) if scores else [None] * n
        self.items = (_SelectItem * n)()
        for i, (X, (br, bc), keep) in enumerate(zip(Xs, blocks, keeps)):
            if dtype_code(X.dtype) != self.dtype:
                raise BsrError(BSR_ERR_DTYPE, "all tensors of a batch share one dtype")
            M, K, ldx = _dense2d(X, "X")
            self.items[i] = _SelectItem(_ptr(X), M, K, ldx, br, bc, float(keep), _ptr(self.scores[i]),
                                        _ptr(self.keep_masks[i]))
        self.n = n
        self.ws_bytes = int(lib().bsr_score_select_batched_workspace_bytes(self.items, n, self.dtype))


def bsr_score_select_batched(batch: SelectBatch, *, ws: Optional[torch.Tensor] = None, stream=None):
    """-> list of keep masks (uint8 [nblocks] each), the same as bsr_score_select tensor by tensor."""
    if ws is None:
        ws = _workspace(batch.ws_bytes, batch.device, None)
    rc = lib().bsr_score_select_batched(batch.items, batch.n, batch.dtype, _ptr(ws),
                                        ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_score_select_batched")
    return batch.keep_masks


def bsr_score_select_grouped_batched(batch: SelectBatch, group_rows: Sequence[int], *,
                                     ws: Optional[torch.Tensor] = None, stream=None):
    """-> list of keep masks, the same as bsr_score_select_grouped tensor by tensor with group_rows[i]."""
    if len(group_rows) != batch.n:
        raise ValueError("one group size per tensor")
    if ws is None:
        ws = _workspace(batch.ws_bytes, batch.device, None)
    rows = (C.c_int64 * batch.n)(*[int(r) for r in group_rows])
    rc = lib().bsr_score_select_grouped_batched(batch.items, rows, batch.n, batch.dtype, _ptr(ws),
                                                ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_score_select_grouped_batched")
    return batch.keep_masks


class _MatmulItem(C.Structure):
    """Mirror of bsr_matmul_item."""
    _fields_ = [("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("values", C.c_void_p),
                ("M", C.c_int64), ("K", C.c_int64), ("br", C.c_int32), ("bc", C.c_int32),
                ("dY", C.c_void_p), ("N", C.c_int64), ("lddy", C.c_int64),
                ("dW", C.c_void_p), ("lddw", C.c_int64), ("accumulate", C.c_int32)]


class MatmulBatch:
    """The marshalled item array of one bsr_t_dense_matmul_batched call (see SelectBatch).  Every entry of
    `problems` is (row_ptr, col_idx, values, M, K, br, bc, dY) or that plus a dW tensor to write into."""

    def __init__(self, problems: Sequence[tuple], accumulate: bool = False):
        n = len(problems)
        if n == 0:
            raise ValueError("empty batch")
        self.dtype = dtype_code(problems[0][7].dtype)
        self.device = problems[0][7].device
        self.items = (_MatmulItem * n)()
        self.keep, self.dWs = [], []
        for i, pr in enumerate(problems):
            row_ptr, col_idx, values, M, K, br, bc, dY = pr[:8]
            Md, N, lddy = _dense2d(dY, "dY")
            if Md != M or dtype_code(dY.dtype) != self.dtype or values.dtype != dY.dtype:
                raise ValueError("dY must have M rows and the batch one dtype")
            dW = pr[8] if len(pr) > 8 and pr[8] is not None else None
            if dW is None:
                if accumulate:
                    raise ValueError("accumulate needs existing dW tensors")
                dW = torch.empty((K, N), dtype=torch.float32, device=dY.device)
            _, _, lddw = _dense2d(dW, "dW")
            self.items[i] = _MatmulItem(_ptr(row_ptr), _ptr(col_idx), _ptr(values), M, K, br, bc, _ptr(dY), N, lddy,
                                        _ptr(dW), lddw, 1 if accumulate else 0)
            self.keep.append(pr)
            self.dWs.append(dW)
        self.n = n
        self.ws_bytes = int(lib().bsr_t_dense_matmul_batched_workspace_bytes(self.items, n, self.dtype))


def bsr_t_dense_matmul_batched(batch: MatmulBatch, *, ws: Optional[torch.Tensor] = None, stream=None):
    """-> list of dW tensors, each what bsr_t_dense_matmul gives for its item."""
    if ws is None:
        ws = _workspace(batch.ws_bytes, batch.device, None)
    rc = lib().bsr_t_dense_matmul_batched(batch.items, batch.n, batch.dtype, _ptr(ws),
                                          ws.numel() if ws is not None else 0, _stream(stream))
    _check(rc, "bsr_t_dense_matmul_batched")
    return batch.dWs


class _CompressItem(C.Structure):
    """Mirror of bsr_compress_item."""
    _fields_ = [("X", C.c_void_p), ("M", C.c_int64), ("K", C.c_int64), ("ldx", C.c_int64),
                ("br", C.c_int32), ("bc", C.c_int32), ("keep_mask", C.c_void_p), ("n_keep", C.c_int64),
                ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("values", C.c_void_p)]


class CompressBatch:
    """The marshalled item array of one bsr_compress_batched call (see SelectBatch).  Every entry of `problems` is
    (X, br, bc, keep_mask, n_keep) or that plus (row_ptr, col_idx, values) tensors to write into."""

    def __init__(self, problems: Sequence[tuple]):
        n = len(problems)
        if n == 0:
            raise ValueError("empty batch")
        self.dtype = dtype_code(problems[0][0].dtype)
        self.device = problems[0][0].device
        self.items = (_CompressItem * n)()
        self.keep, self.outputs = [], []
        for i, pr in enumerate(problems):
            X, br, bc, keep_mask, n_keep = pr[:5]
            if dtype_code(X.dtype) != self.dtype:
                raise ValueError("all tensors of a batch must have one dtype")
            M, K, ldx = _dense2d(X, "X")
            nbr = -(-M // br) if br > 0 else 0
            if len(pr) > 5:
                row_ptr, col_idx, values = pr[5:8]
            else:
                row_ptr = torch.empty(nbr + 1, dtype=torch.int32, device=X.device)
                col_idx = torch.empty(max(n_keep, 0), dtype=torch.int32, device=X.device)
                values = torch.empty((max(n_keep, 0), br, bc), dtype=X.dtype, device=X.device)
            self.items[i] = _CompressItem(_ptr(X), M, K, ldx, br, bc, _ptr(keep_mask), int(n_keep), _ptr(row_ptr),
                                          _ptr(col_idx), _ptr(values))
            self.keep.append((X, keep_mask))
            self.outputs.append((row_ptr, col_idx, values))
        self.n = n
        self.ws_bytes = int(lib().bsr_compress_batched_workspace_bytes(self.items, n, self.dtype))


def bsr_compress_batched(batch: CompressBatch, *, ws: Optional[torch.Tensor] = None, stream=None):
    """-> list of (row_ptr, col_idx, values), each what bsr_compress gives for its item."""
    if ws is None:
        ws = _workspace(batch.ws_bytes, batch.device, None)
    rc = lib().bsr_compress_batched(batch.items, batch.n, batch.dtype, _ptr(ws), ws.numel() if ws is not None else 0,
                                    _stream(stream))
    _check(rc, "bsr_compress_batched")
    return batch.outputs


class _DecompressItem(C.Structure):
    """Mirror of bsr_decompress_item."""
    _fields_ = [("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("values", C.c_void_p),
                ("M", C.c_int64), ("K", C.c_int64), ("ldx", C.c_int64), ("br", C.c_int32), ("bc", C.c_int32),
                ("X_out", C.c_void_p)]


class DecompressBatch:
    """The marshalled item array of one bsr_decompress_batched call (see SelectBatch).  Every entry of `problems` is
    (row_ptr, col_idx, values, M, K, br, bc) or that plus an output tensor to write into."""

    def __init__(self, problems: Sequence[tuple]):
        n = len(problems)
        if n == 0:
            raise ValueError("empty batch")
        self.dtype = dtype_code(problems[0][2].dtype)
        self.items = (_DecompressItem * n)()
        self.keep, self.outputs = [], []
        for i, pr in enumerate(problems):
            row_ptr, col_idx, values, M, K, br, bc = pr[:7]
            if dtype_code(values.dtype) != self.dtype:
                raise ValueError("all tensors of a batch must have one dtype")
            out = pr[7] if len(pr) > 7 and pr[7] is not None else \
                torch.empty((M, K), dtype=values.dtype, device=values.device)
            _, _, ldx = _dense2d(out, "out")
            self.items[i] = _DecompressItem(_ptr(row_ptr), _ptr(col_idx), _ptr(values), M, K, ldx, br, bc, _ptr(out))
            self.keep.append(pr)
            self.outputs.append(out)
        self.n = n


def bsr_decompress_batched(batch: DecompressBatch, *, stream=None):
    """-> list of dense tensors, each what bsr_decompress gives for its item."""
    rc = lib().bsr_decompress_batched(batch.items, batch.n, batch.dtype, _stream(stream))
    _check(rc, "bsr_decompress_batched")
    return batch.outputs
