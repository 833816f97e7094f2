"""Host side of the C ABI (CPU only): the library loads, exports every symbol
the header declares, its pure host functions agree with the oracle and the
paper's tables, and invalid arguments are rejected before anything is launched."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2311_16883_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent
GOLDEN = Path(__file__).resolve().parent / "golden"


def declared_symbols():
    text = (ROOT / "include" / "bsr_actprune.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bsr_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert set(syms) == set(B.EXPORTS) and len(syms) == 24
    lib = B.lib()
    for s in syms:
        assert getattr(lib, s) is not None
    assert "gfx950" in B.bsr_version()


def test_keep_count_agrees_with_oracle():
    for keep in (0.0, 0.1, 0.25, 1 / 3, 0.5, 0.7, 0.75, 0.9, 1.0):
        for n in list(range(0, 300)) + [4704, 9408, 37632, 49154, 75264, 301056]:
            assert B.bsr_keep_count(n, keep) == oracle.keep_count(n, keep)
    for bad in (-1e-9, 1.0000001, float("nan"), float("inf")):
        assert B.lib().bsr_keep_count(10, bad) == -1
    assert B.lib().bsr_keep_count(-1, 0.5) == -1


def test_grouped_keep_count_agrees_with_oracle():
    rng = np.random.default_rng(0)
    for nbr, nbc, g in [(7, 5, 3), (784, 12, 49), (3511, 14, 14), (784, 48, 7), (1, 1, 1), (10, 3, 100)]:
        for keep in (0.0, 0.1, 0.25, 1 / 3, 0.5, 0.9, 1.0):
            _, total = oracle.select_grouped(rng.random(nbr * nbc), nbr, nbc, g, keep)
            assert B.bsr_grouped_keep_count(nbr, nbc, g, keep) == total
    lib = B.lib()
    assert lib.bsr_grouped_keep_count(10, 10, 0, 0.5) == -1
    assert lib.bsr_grouped_keep_count(-1, 10, 2, 0.5) == -1
    assert lib.bsr_grouped_keep_count(10, 10, 2, 1.5) == -1
    assert lib.bsr_grouped_keep_count(0, 10, 2, 0.5) == 0


def test_storage_bytes_agree_with_oracle_and_table_2():
    for (M, K, br, bc, dt, e) in [(6272, 384, 1, 16, B.BSR_F32, 4), (25088, 1536, 32, 32, B.BSR_BF16, 2),
                                  (49152, 196, 14, 14, B.BSR_BF16, 2)]:
        nbr, nbc = oracle.grid(M, K, br, bc)
        for n_keep in (0, 1, nbr * nbc // 2, nbr * nbc):
            assert B.bsr_storage_bytes(M, K, br, bc, n_keep, dt) == oracle.bsr_bytes(n_keep, nbr, br, bc, e)
    # paper Table II, the b = 16 column (384-wide binary32 rows, 1 x b blocks)
    rows = [l.split() for l in (GOLDEN / "table2_bsr_overhead.txt").read_text().splitlines()
            if l and not l.startswith("#")]
    col = rows[0].index("16")
    R, D = 6272, 384
    for row in rows[1:]:
        s = int(row[0]) / 100
        n_keep = round((1 - s) * R * (D // 16))
        got = B.bsr_storage_bytes(R, D, 1, 16, n_keep, B.BSR_F32)
        overhead = 100.0 * (got - (1 - s) * R * D * 4) / (R * D * 4)
        assert abs(overhead - float(row[col])) <= 0.025
    assert B.lib().bsr_storage_bytes(10, 10, 0, 4, 1, 0) == -1
    assert B.lib().bsr_storage_bytes(10, 10, 2, 2, 26, 0) == -1


def test_workspace_bytes_are_sane():
    assert B.bsr_workspace_bytes(B.BSR_OP_SCORE_SELECT, 25088, 384, 0, 32, 32, B.BSR_BF16) >= 8 * 9408
    assert B.bsr_workspace_bytes(B.BSR_OP_SCORE_SELECT, 25088, 384, 0, 32, 32, 9) == 0
    assert B.bsr_workspace_bytes(99, 25088, 384, 0, 32, 32, B.BSR_BF16) == 0
    assert B.bsr_workspace_bytes(B.BSR_OP_T_DENSE_MATMUL, 25088, 384, 1536, 32, 32, B.BSR_BF16) % 256 == 0
    # mask -> BSR needs none at the benchmark's shapes, a counter per workgroup for millions of row segments
    assert B.bsr_workspace_bytes(B.BSR_OP_COMPRESS, 25088, 384, 0, 32, 32, B.BSR_BF16) == 0
    assert B.bsr_workspace_bytes(B.BSR_OP_COMPRESS, 49152, 196, 0, 14, 14, B.BSR_BF16) == 0
    assert 0 < B.bsr_workspace_bytes(B.BSR_OP_COMPRESS, 25088, 384, 0, 1, 4, B.BSR_BF16) <= 4 * 25088 + 256
    # block shapes that are re-tiled for the matrix cores: room for the 32x32 copy of the operand
    tiled = B.bsr_workspace_bytes(B.BSR_OP_T_DENSE_MATMUL, 25088, 384, 1536, 1, 32, B.BSR_BF16)
    assert tiled >= 25088 * 384 * 2 + 4 * 384 * 1536


def test_invalid_arguments_are_rejected_on_the_host():
    """None of these reaches a kernel launch: they are safe without a GPU."""
    lib = B.lib()
    fake = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = C.c_void_p(0x1001)
    ss = lambda **k: lib.bsr_score_select(
        k.get("X", fake), k.get("dtype", 0), k.get("M", 64), k.get("K", 64), k.get("ldx", 64),
        k.get("br", 16), k.get("bc", 16), k.get("keep", 0.5), None, k.get("mask", fake),
        k.get("ws", fake), k.get("ws_bytes", 1 << 20), None)
    assert ss(dtype=2) == B.BSR_ERR_DTYPE
    assert ss(M=-1) == B.BSR_ERR_SHAPE
    assert ss(br=0) == B.BSR_ERR_SHAPE
    assert ss(ldx=63) == B.BSR_ERR_SHAPE
    assert ss(keep=1.5) == B.BSR_ERR_KEEP
    assert ss(keep=float("nan")) == B.BSR_ERR_KEEP
    assert ss(X=None) == B.BSR_ERR_NULL
    assert ss(mask=None) == B.BSR_ERR_NULL
    assert ss(X=odd) == B.BSR_ERR_ALIGN
    assert ss(ws=None) == B.BSR_ERR_WORKSPACE
    assert ss(ws_bytes=8) == B.BSR_ERR_WORKSPACE
    assert ss(M=1 << 41) == B.BSR_ERR_SHAPE
    assert ss(M=1 << 30, K=1 << 30, ldx=1 << 30, br=1, bc=1) == B.BSR_ERR_SHAPE   # nblocks >= 2^31
    assert ss(M=0) == B.BSR_OK and ss(K=0, ldx=0) == B.BSR_OK                    # empty: nothing to do

    sg = lambda **k: lib.bsr_score_select_grouped(
        k.get("X", fake), k.get("dtype", 0), k.get("M", 64), 64, 64, 16, 16, k.get("group_rows", 2),
        k.get("keep", 0.5), None, k.get("mask", fake), k.get("ws", fake), k.get("ws_bytes", 1 << 20), None)
    assert sg(group_rows=0) == B.BSR_ERR_SHAPE
    assert sg(group_rows=-3) == B.BSR_ERR_SHAPE
    assert sg(keep=-0.5) == B.BSR_ERR_KEEP
    assert sg(dtype=7) == B.BSR_ERR_DTYPE
    assert sg(X=None) == B.BSR_ERR_NULL
    assert sg(ws_bytes=8) == B.BSR_ERR_WORKSPACE
    assert sg(M=0) == B.BSR_OK

    cp = lambda **k: lib.bsr_compress(
        k.get("X", fake), k.get("dtype", 1), 64, 64, 64, 16, 16, k.get("mask", fake),
        k.get("n_keep", 8), k.get("row_ptr", fake), k.get("col_idx", fake), k.get("values", fake),
        None, 0, None)
    assert cp(dtype=-1) == B.BSR_ERR_DTYPE
    assert cp(n_keep=17) == B.BSR_ERR_KEEP
    assert cp(n_keep=-1) == B.BSR_ERR_KEEP
    assert cp(row_ptr=None) == B.BSR_ERR_NULL
    assert cp(values=None) == B.BSR_ERR_NULL
    assert cp(values=odd) == B.BSR_ERR_ALIGN
    assert cp(col_idx=C.c_void_p(0x1002)) == B.BSR_ERR_ALIGN
    # 2.4 M row segments: the call wants its workspace
    assert lib.bsr_compress(fake, 1, 25088, 384, 384, 1, 4, fake, 100, fake, fake, fake, None, 0, None) \
        == B.BSR_ERR_WORKSPACE
    assert lib.bsr_compress(fake, 1, 25088, 384, 384, 1, 4, fake, 100, fake, fake, fake, fake, 64, None) \
        == B.BSR_ERR_WORKSPACE

    assert lib.bsr_decompress(fake, fake, fake, 1, 64, 64, 64, 16, 16, None, None) == B.BSR_ERR_NULL
    assert lib.bsr_decompress(fake, fake, fake, 5, 64, 64, 64, 16, 16, fake, None) == B.BSR_ERR_DTYPE
    assert lib.bsr_decompress(fake, fake, fake, 1, 64, 64, 32, 16, 16, fake, None) == B.BSR_ERR_SHAPE

    mm = lambda **k: lib.bsr_t_dense_matmul(
        fake, fake, fake, k.get("dtype", 1), 64, 64, 16, 16, k.get("dY", fake), k.get("N", 32),
        k.get("lddy", 32), k.get("dW", fake), k.get("lddw", 32), 0, k.get("ws", fake),
        k.get("ws_bytes", 1 << 30), None)
    assert mm(dtype=3) == B.BSR_ERR_DTYPE
    assert mm(N=-1) == B.BSR_ERR_SHAPE
    assert mm(lddy=31) == B.BSR_ERR_SHAPE
    assert mm(lddw=8) == B.BSR_ERR_SHAPE
    assert mm(dW=None) == B.BSR_ERR_NULL
    assert mm(dY=None) == B.BSR_ERR_NULL
    assert mm(dW=C.c_void_p(0x1002)) == B.BSR_ERR_ALIGN
    assert mm(N=0, lddy=0, lddw=0) == B.BSR_OK
    af = lambda **k: lib.bsr_affine_scale_grad(
        fake, fake, fake, k.get("dtype", 1), 64, 64, 16, 16, k.get("dY", fake), k.get("lddy", 64),
        k.get("dalpha", fake), 0, k.get("ws", fake), k.get("ws_bytes", 1 << 20), None)
    assert af(dtype=3) == B.BSR_ERR_DTYPE
    assert af(lddy=63) == B.BSR_ERR_SHAPE
    assert af(dalpha=None) == B.BSR_ERR_NULL
    assert af(dY=None) == B.BSR_ERR_NULL
    assert af(dalpha=C.c_void_p(0x1002)) == B.BSR_ERR_ALIGN
    assert af(ws_bytes=16) == B.BSR_ERR_WORKSPACE
    # several tensors per call: the first offending item decides, nothing is launched
    def items(**k):
        arr = (B._SelectItem * 2)()
        arr[0] = B._SelectItem(0x1000, 64, 64, 64, 16, 16, 0.5, None, 0x1000)
        arr[1] = B._SelectItem(k.get("X", 0x1000), k.get("M", 128), 64, k.get("ldx", 64), k.get("br", 16), 16,
                               k.get("keep", 0.25), None, k.get("mask", 0x1000))
        return arr
    bt = lambda arr, n=2, dtype=1, ws=fake, ws_bytes=1 << 20: lib.bsr_score_select_batched(arr, n, dtype, ws,
                                                                                          ws_bytes, None)
    assert bt(items(), n=-1) == B.BSR_ERR_SHAPE
    assert bt(None) == B.BSR_ERR_NULL
    assert bt(items(), n=0) == B.BSR_OK
    assert bt(items(), dtype=4) == B.BSR_ERR_DTYPE
    assert bt(items(br=0)) == B.BSR_ERR_SHAPE
    assert bt(items(ldx=32)) == B.BSR_ERR_SHAPE
    assert bt(items(keep=2.0)) == B.BSR_ERR_KEEP
    assert bt(items(X=None)) == B.BSR_ERR_NULL
    assert bt(items(mask=None)) == B.BSR_ERR_NULL
    assert bt(items(), ws=None) == B.BSR_ERR_WORKSPACE
    need = lib.bsr_score_select_batched_workspace_bytes(items(), 2, 1)
    assert need == sum(-(-B.bsr_workspace_bytes(B.BSR_OP_SCORE_SELECT, M, 64, 0, 16, 16, 1) // 256) * 256
                       for M in (64, 128))
    assert bt(items(), ws_bytes=need - 1) == B.BSR_ERR_WORKSPACE
    assert lib.bsr_score_select_batched_workspace_bytes(items(br=0), 2, 1) == 0
    # ... and the per-group ranking of several tensors: the same checks plus the group sizes
    rows = lambda a, b: (C.c_int64 * 2)(a, b)
    gb = lambda arr, gr=None, n=2, dtype=1, ws=fake, ws_bytes=1 << 20: lib.bsr_score_select_grouped_batched(
        arr, rows(2, 4) if gr is None else gr, n, dtype, ws, ws_bytes, None)
    assert gb(items(), n=-1) == B.BSR_ERR_SHAPE
    assert gb(items(), n=0) == B.BSR_OK
    assert gb(None) == B.BSR_ERR_NULL
    assert lib.bsr_score_select_grouped_batched(items(), None, 2, 1, fake, 1 << 20, None) == B.BSR_ERR_NULL
    assert gb(items(), gr=rows(2, 0)) == B.BSR_ERR_SHAPE
    assert gb(items(), gr=rows(-1, 4)) == B.BSR_ERR_SHAPE
    assert gb(items(), dtype=4) == B.BSR_ERR_DTYPE
    assert gb(items(br=0)) == B.BSR_ERR_SHAPE
    assert gb(items(keep=-0.1)) == B.BSR_ERR_KEEP
    assert gb(items(X=None)) == B.BSR_ERR_NULL
    assert gb(items(mask=None)) == B.BSR_ERR_NULL
    assert gb(items(), ws=None) == B.BSR_ERR_WORKSPACE
    assert gb(items(), ws_bytes=need - 1) == B.BSR_ERR_WORKSPACE
    assert gb(items(), ws=odd) == B.BSR_ERR_ALIGN
    def mm_items(**k):
        arr = (B._MatmulItem * 2)()
        arr[0] = B._MatmulItem(0x1000, 0x1000, 0x1000, 64, 64, 16, 16, 0x1000, 32, 32, 0x1000, 32, 0)
        arr[1] = B._MatmulItem(0x1000, 0x1000, 0x1000, k.get("M", 128), 64, k.get("br", 32), 32, k.get("dY", 0x1000),
                               k.get("N", 48), k.get("lddy", 48), k.get("dW", 0x1000), k.get("lddw", 48), 0)
        return arr
    bm = lambda arr, n=2, dtype=1, ws=fake, ws_bytes=1 << 24: lib.bsr_t_dense_matmul_batched(arr, n, dtype, ws,
                                                                                            ws_bytes, None)
    assert bm(mm_items(), n=-2) == B.BSR_ERR_SHAPE
    assert bm(None) == B.BSR_ERR_NULL
    assert bm(mm_items(), n=0) == B.BSR_OK
    assert bm(mm_items(), dtype=9) == B.BSR_ERR_DTYPE
    assert bm(mm_items(br=0)) == B.BSR_ERR_SHAPE
    assert bm(mm_items(lddy=40)) == B.BSR_ERR_SHAPE
    assert bm(mm_items(lddw=8)) == B.BSR_ERR_SHAPE
    assert bm(mm_items(dW=None)) == B.BSR_ERR_NULL
    assert bm(mm_items(dY=None)) == B.BSR_ERR_NULL
    assert bm(mm_items(dW=0x1002)) == B.BSR_ERR_ALIGN
    big = mm_items(M=25088, N=1536, lddy=1536, lddw=1536)           # a product that is split: needs its workspace
    need = lib.bsr_t_dense_matmul_batched_workspace_bytes(big, 2, 1)
    assert need >= 4 * 64 * 1536
    assert bm(big, ws=None) == B.BSR_ERR_WORKSPACE
    assert bm(big, ws_bytes=need - 1) == B.BSR_ERR_WORKSPACE
    assert lib.bsr_t_dense_matmul_batched_workspace_bytes(mm_items(br=0), 2, 1) == 0
    def cp_items(**k):
        arr = (B._CompressItem * 2)()
        arr[0] = B._CompressItem(0x1000, 64, 64, 64, 16, 16, 0x1000, 8, 0x1000, 0x1000, 0x1000)
        arr[1] = B._CompressItem(k.get("X", 0x1000), k.get("M", 128), k.get("K", 64), k.get("ldx", 64), k.get("br", 16),
                                 k.get("bc", 16), k.get("mask", 0x1000), k.get("n_keep", 16), k.get("row_ptr", 0x1000),
                                 k.get("col_idx", 0x1000), k.get("values", 0x1000))
        return arr
    bc_ = lambda arr, n=2, dtype=1, ws=None, ws_bytes=0: lib.bsr_compress_batched(arr, n, dtype, ws, ws_bytes, None)
    assert bc_(cp_items(), n=-1) == B.BSR_ERR_SHAPE
    assert bc_(None) == B.BSR_ERR_NULL
    assert bc_(cp_items(), n=0) == B.BSR_OK
    assert bc_(cp_items(), dtype=5) == B.BSR_ERR_DTYPE
    assert bc_(cp_items(br=0)) == B.BSR_ERR_SHAPE
    assert bc_(cp_items(ldx=8)) == B.BSR_ERR_SHAPE
    assert bc_(cp_items(n_keep=33)) == B.BSR_ERR_KEEP
    assert bc_(cp_items(X=None)) == B.BSR_ERR_NULL
    assert bc_(cp_items(mask=None)) == B.BSR_ERR_NULL
    assert bc_(cp_items(row_ptr=None)) == B.BSR_ERR_NULL
    assert bc_(cp_items(values=None)) == B.BSR_ERR_NULL
    assert bc_(cp_items(col_idx=0x1002)) == B.BSR_ERR_ALIGN
    assert lib.bsr_compress_batched_workspace_bytes(cp_items(), 2, 1) == 0
    tall = cp_items(M=1 << 21, K=8, ldx=8, br=1, bc=4, n_keep=100)          # per-workgroup counts in the workspace
    need = lib.bsr_compress_batched_workspace_bytes(tall, 2, 1)
    assert need == -(-B.bsr_workspace_bytes(B.BSR_OP_COMPRESS, 1 << 21, 8, 0, 1, 4, 1) // 256) * 256 > 0
    assert bc_(tall) == B.BSR_ERR_WORKSPACE
    assert bc_(tall, ws=fake, ws_bytes=need - 1) == B.BSR_ERR_WORKSPACE
    assert lib.bsr_compress_batched_workspace_bytes(cp_items(br=0), 2, 1) == 0
    def dc_items(**k):
        arr = (B._DecompressItem * 2)()
        arr[0] = B._DecompressItem(0x1000, 0x1000, 0x1000, 64, 64, 64, 16, 16, 0x1000)
        arr[1] = B._DecompressItem(k.get("row_ptr", 0x1000), 0x1000, k.get("values", 0x1000), 128, 64, k.get("ldx", 64),
                                   k.get("br", 16), 16, k.get("out", 0x1000))
        return arr
    bd = lambda arr, n=2, dtype=1: lib.bsr_decompress_batched(arr, n, dtype, None)
    assert bd(dc_items(), n=-1) == B.BSR_ERR_SHAPE
    assert bd(None) == B.BSR_ERR_NULL
    assert bd(dc_items(), n=0) == B.BSR_OK
    assert bd(dc_items(), dtype=7) == B.BSR_ERR_DTYPE
    assert bd(dc_items(br=-1)) == B.BSR_ERR_SHAPE
    assert bd(dc_items(ldx=63)) == B.BSR_ERR_SHAPE
    assert bd(dc_items(row_ptr=None)) == B.BSR_ERR_NULL
    assert bd(dc_items(out=None)) == B.BSR_ERR_NULL
    assert bd(dc_items(out=0x1001)) == B.BSR_ERR_ALIGN
    assert B.lib().bsr_error_string(B.BSR_ERR_WORKSPACE) == b"BSR_ERR_WORKSPACE"


def test_product_path_does_not_touch_the_oracle():
    """The binding and the kernels never import or link the CPU oracle."""
    pkg = ROOT / "paper_2311_16883_amd"
    for f in list(pkg.glob("*.py")) + list((pkg / "csrc").glob("*")):
        text = f.read_text()
        assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f


def test_static_entry_point_refuses_oversized_problems_on_the_host():
    lib = B.lib()
    limit = lib.bsr_score_select_static_max_blocks()
    assert limit == 524288
    fake = C.c_void_p(4096)      # never dereferenced: every call below is refused before any HIP call
    # 1025 * 512 blocks > limit
    assert lib.bsr_score_select_static(fake, B.BSR_BF16, 1025, 2048, 2048, 1, 4, 0.5, None, fake, None) == B.BSR_ERR_LIMIT
    assert lib.bsr_score_select_static(fake, B.BSR_F32, 1 << 30, 1 << 20, 1 << 20, 1, 1, 0.5, None, fake, None) == B.BSR_ERR_LIMIT
    assert lib.bsr_score_select_static(fake, 7, 64, 64, 64, 16, 16, 0.5, None, fake, None) == B.BSR_ERR_DTYPE
    assert lib.bsr_score_select_static(fake, B.BSR_F32, 64, 64, 64, 0, 16, 0.5, None, fake, None) == B.BSR_ERR_SHAPE
    assert lib.bsr_error_string(B.BSR_ERR_LIMIT) == b"BSR_ERR_LIMIT"
