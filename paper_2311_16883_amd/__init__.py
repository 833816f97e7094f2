"""Structured activation pruning hot path for AMD MI355X (gfx950).

Forward side: block l2 scoring, exact top-k block selection, Block Sparse Row
packing.  Backward side: weight gradient dW = Xhat^T dY straight from the BSR
tensor.  All compute lives in ``libbsr_actprune.so`` (hand-written HIP); this
package is the thin ctypes binding (``binding``), the in-tree build (``build``)
and the seeded synthetic workloads (``synth``).
"""
from .binding import (  # noqa: F401
    BSR_BF16, BSR_F32, BSR_OP_COMPRESS, BSR_OP_DECOMPRESS, BSR_OP_SCORE_SELECT,
    BSR_OP_T_DENSE_MATMUL, BsrError, bsr_compress, bsr_decompress, bsr_keep_count,
    bsr_score_select, bsr_storage_bytes, bsr_t_dense_matmul, bsr_version, bsr_workspace_bytes,
)
