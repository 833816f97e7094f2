"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.

Bars: block indices, row_ptr, col_idx and BSR values bit-exact; scores to a few
binary64 roundings (the reduction order differs, the precision does not);
dW to max|dW - ref| / max|ref| <= 1e-5 for binary32 inputs and <= 2e-2 for
bfloat16 inputs (both accumulate in binary32; exact bfloat16 products keep the
bfloat16 path far inside its bar, which a second, tighter assertion records).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_16883_amd import binding as B
from paper_2311_16883_amd import synth

pytestmark = pytest.mark.gpu

DW_TOL = {"f32": 1e-5, "bf16": 2e-2}
DW_TOL_DERIVED = 2e-5       # binary32 accumulation of exact products, either dtype


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def rand_pair(M, K, N, dtype, seed, dist="normal"):
    spec = synth.TensorSpec("t", M, K, N, 1, 1, dtype, dist)
    return synth.make_pair(spec, seed)


def gpu_prune(Xd, br, bc, keep):
    M, K = Xd.shape
    nbr, nbc = oracle.grid(M, K, br, bc)
    mask, scores = B.bsr_score_select(Xd, br, bc, keep, want_scores=True)
    n_keep = B.bsr_keep_count(nbr * nbc, keep)
    row_ptr, col_idx, values = B.bsr_compress(Xd, br, bc, mask, n_keep)
    return scores, mask, row_ptr, col_idx, values


def check_forward(X, br, bc, keep, label=""):
    """score/select/compress/decompress of X against the oracle; returns device BSR."""
    print(f"[case] forward {label} shape={X.shape} dtype={X.dtype} block={br}x{bc} keep={keep}", flush=True)
    M, K = X.shape
    Xd = to_dev(X)
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, br, bc, keep)
    scores, mask, row_ptr, col_idx, values = gpu_prune(Xd, br, bc, keep)
    torch.cuda.synchronize()
    g_scores = scores.cpu().numpy()
    finite = np.isfinite(o_scores)
    assert np.array_equal(np.isnan(g_scores), np.isnan(o_scores))
    n_el = br * bc
    assert np.all(np.abs(g_scores[finite] - o_scores[finite]) <= 2.0 ** -52 * n_el * np.abs(o_scores[finite]))
    g_mask = mask.cpu().numpy()
    if not np.array_equal(g_mask, o_mask):
        diff = np.flatnonzero(g_mask != o_mask)
        raise AssertionError(f"selection differs at blocks {diff[:8]}, oracle scores {o_scores[diff[:8]]}")
    assert np.array_equal(row_ptr.cpu().numpy(), o_rp)
    assert np.array_equal(col_idx.cpu().numpy(), o_ci)
    assert to_host(values).tobytes() == o_val.tobytes()
    back = B.bsr_decompress(row_ptr, col_idx, values, M, K, br, bc)
    torch.cuda.synchronize()
    assert to_host(back).tobytes() == oracle.mask_dense(X, br, bc, o_mask).tobytes()
    return (row_ptr, col_idx, values), o_mask


def dw_error(got: np.ndarray, ref: np.ndarray) -> float:
    scale = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(got.astype(np.float64) - ref))) / (scale if scale > 0 else 1.0)


FORWARD_CASES = [
    # M, K, br, bc, dtype, keep
    (256, 128, 16, 16, "f32", 0.5),
    (1000, 200, 32, 32, "f32", 0.25),        # ragged rows and columns
    (777, 196, 14, 14, "bf16", 0.5),         # the cross-patch block shape, ragged rows
    (1024, 384, 32, 32, "bf16", 0.5),
    (1024, 384, 32, 32, "bf16", 0.75),
    (130, 1000, 1, 8, "bf16", 0.1),          # row segments (1 x b)
    (300, 70, 7, 5, "f32", 0.9),             # nothing divides: scalar loads
    (2048, 1536, 64, 64, "bf16", 0.5),
    (96, 8192, 8, 4096, "bf16", 0.5),        # a block row wider than one workgroup pass
    (50, 3, 64, 64, "f32", 0.5),             # a single ragged block
    (4096, 384, 16, 16, "bf16", 0.9),        # > 4096 blocks: several radix levels
    (48, 40008, 8, 8, "bf16", 0.3),          # 5001 block-columns: index build and pack as two launches
    (2100, 264, 2, 8, "f32", 0.6),           # 1050 block-rows of 33 blocks: fused conversion, 2-row blocks
    (640, 1024, 64, 64, "f32", 0.4),         # 1024 vectors per block: several per thread in the fused copy
    # block rows narrower than 16 bytes on contiguous rows: block-rows staged through LDS
    (1001, 196, 14, 14, "f32", 0.5),         # 56-byte segments, ragged rows, 3 block-rows per workgroup
    (333, 60, 3, 6, "bf16", 0.7),            # 8 block-rows per workgroup, the last workgroup has 7
    (64, 2046, 4, 6, "bf16", 0.5),           # 341 block-columns: one block-row fills the LDS span
    (1030, 130, 8, 8, "bf16", 0.35),         # 16-byte segments on rows that are not 16-byte aligned; ragged columns
    # row segments (1 x b), the block shape Table II's overheads imply: many block-rows per workgroup
    (3000, 384, 1, 32, "bf16", 0.5),
    (2048, 384, 1, 384, "bf16", 0.5),        # b = K: whole rows pruned
    (4096, 96, 1, 4, "bf16", 0.5),           # 32 block-rows per workgroup
    (20000, 384, 1, 4, "bf16", 0.5),         # 1.9 M blocks: index build and LDS-staged pack as two launches
    (5000, 200, 2, 50, "f32", 0.25),         # segments of several 32-element pieces, ragged last piece
]


@pytest.mark.parametrize("M,K,br,bc,dtype,keep", FORWARD_CASES)
def test_forward_parity(M, K, br, bc, dtype, keep):
    X, _ = rand_pair(M, K, 8, dtype, seed=M + K, dist="gelu" if bc == 16 else "normal")
    check_forward(X, br, bc, keep)


def test_config1_tiny_end_to_end():
    spec = synth.tiny()[0]
    X, dY = synth.make_pair(spec, 0)
    (row_ptr, col_idx, values), o_mask = check_forward(X, spec.br, spec.bc, spec.keep, "config1")
    assert int(o_mask.sum()) == 64
    dW = B.bsr_t_dense_matmul(row_ptr, col_idx, values, spec.M, spec.K, spec.br, spec.bc, to_dev(dY))
    torch.cuda.synchronize()
    ref = oracle.dw(oracle.mask_dense(X, spec.br, spec.bc, o_mask), dY)
    assert dw_error(dW.cpu().numpy(), ref) <= DW_TOL["f32"]


@pytest.mark.parametrize("keep", [0.0, 1.0 / 128, 0.3, 1.0])
def test_degenerate_keeps(keep):
    spec = synth.tiny()[0]
    X, dY = synth.make_pair(spec, 1)
    (row_ptr, col_idx, values), o_mask = check_forward(X, spec.br, spec.bc, keep, "degenerate")
    dW = B.bsr_t_dense_matmul(row_ptr, col_idx, values, spec.M, spec.K, spec.br, spec.bc, to_dev(dY))
    torch.cuda.synchronize()
    ref = oracle.dw(oracle.mask_dense(X, spec.br, spec.bc, o_mask), dY)
    if keep == 0.0:
        assert not dW.cpu().numpy().any()
    else:
        assert dw_error(dW.cpu().numpy(), ref) <= DW_TOL["f32"]
    if keep == 1.0:   # keep-ratio 1 reproduces the dense gradient
        dense = X.astype(np.float64).T @ dY.astype(np.float64)
        assert dw_error(dW.cpu().numpy(), dense) <= DW_TOL["f32"]


@pytest.mark.parametrize("M,K,br,bc,dtype", [(512, 256, 16, 16, "f32"), (2048, 256, 16, 16, "bf16"),
                                             (1030, 130, 8, 8, "bf16")])
def test_ties_go_to_the_lowest_index(M, K, br, bc, dtype):
    rng = np.random.default_rng(M)
    # constant matrix: all full blocks tie; the first n_keep linear indices survive
    X = np.full((M, K), 1.5, dtype=np.float32)
    X = X if dtype == "f32" else synth.f32_to_bf16_bits(X)
    for keep in (0.5, 0.37):
        check_forward(X, br, bc, keep, "constant")
    # small integers: exact sums in any order, many ties at every level
    Xi = rng.integers(-2, 3, size=(M, K)).astype(np.float32)
    Xi = Xi if dtype == "f32" else synth.f32_to_bf16_bits(Xi)
    for keep in (0.5, 0.11, 0.93):
        check_forward(Xi, br, bc, keep, "integers")


def selection_stress(M, K, br, bc, keep, seed):
    """Distributions that stress the selection: continuous, heavy tails with dead blocks and
    NaN / huge outliers, thousands of exact ties around the threshold, every block equal."""
    rng = np.random.default_rng(seed)
    X = synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32))
    check_forward(X, br, bc, keep, "normal")
    # heavy tails and dead blocks: a third of the blocks are exactly zero, a few are huge / NaN
    Xo = rng.standard_normal((M, K), dtype=np.float32)
    dead = rng.random((M // br, K // bc)) < 0.33
    Xo *= ~np.kron(dead, np.ones((br, bc), dtype=bool))
    Xo[17, 5] = 1e30
    Xo[M // 2, 100] = np.nan
    check_forward(Xo, br, bc, keep, "outliers f32")
    # small integers: thousands of exact ties at the threshold
    Xi = synth.f32_to_bf16_bits(rng.integers(-1, 2, size=(M, K)).astype(np.float32))
    check_forward(Xi, br, bc, keep, "integer ties")
    # every block ties
    Xc = synth.f32_to_bf16_bits(np.full((M, K), 0.5, dtype=np.float32))
    check_forward(Xc, br, bc, keep, "all equal")


@pytest.mark.parametrize("keep", [0.5, 0.1, 0.9, 0.999])
@pytest.mark.parametrize("M,K,br,bc", [(8192, 512, 16, 16),      # 16384 blocks
                                       (2048, 1536, 8, 8),       # 49152 blocks
                                       (2040, 2048, 8, 8)])      # 65280 blocks, ragged per-thread counts
def test_grid_wide_selection_sizes(M, K, br, bc, keep):
    """More than 12288 blocks: sampled bracket, bucket histogram, candidates selected by the last
    workgroup (linear 32-bit codes, lane-read ranking, general radix select when too many tie)."""
    selection_stress(M, K, br, bc, keep, seed=5)


@pytest.mark.parametrize("keep", [0.5, 0.1, 0.9, 0.999])
def test_single_workgroup_selection_twelve_keys_per_thread(keep):
    """8193 ... 12288 blocks: one workgroup of 1024 threads with up to twelve keys per thread."""
    selection_stress(5120, 512, 16, 16, keep, seed=8)           # 10240 blocks
    selection_stress(3064, 512, 8, 16, keep, seed=9)            # 12256 blocks, ragged per-thread counts


@pytest.mark.parametrize("keep", [0.5, 0.1, 0.9, 0.999])
def test_grid_wide_selection_large(keep):
    """Slices longer than the keys a thread preloads, and (second case) the 256-key sample."""
    selection_stress(4096, 1536, 8, 8, keep, seed=6)            # 98304 blocks
    rng = np.random.default_rng(7)
    X = synth.f32_to_bf16_bits(rng.standard_normal((8192, 1024), dtype=np.float32))
    check_forward(X, 4, 4, keep, "524288 blocks")


@pytest.mark.parametrize("M,K,br,bc,group_rows,keep", [
    (2744, 196, 14, 14, 14, 0.5),        # 14 samples of 196 patches, one group per sample (196 blocks each)
    (6272, 384, 32, 32, 49, 0.5),        # groups of 8 samples (1568 rows = 49 block-rows, 588 blocks)
    (6272, 1536, 32, 32, 49, 0.25),      # 2352 blocks per group: the 1024-thread workgroups
    (1000, 200, 8, 8, 7, 0.3),           # ragged rows / columns, ragged last group
    (8192, 512, 16, 16, 300, 0.5),       # 9600 blocks per group: twelve keys per thread
    (8192, 512, 16, 16, 400, 0.5),       # 12800 blocks per group: grid-wide selection group after group
    (512, 128, 16, 16, 64, 0.6),         # one group: the ungrouped selection
])
def test_grouped_selection_parity(M, K, br, bc, group_rows, keep):
    """Sec. IV, local ranking: groups of block-rows select on their own; mask, counts and the BSR
    built from the mask against the oracle, plus constant and small-integer inputs for the ties."""
    rng = np.random.default_rng(M + K + group_rows)
    nbr, nbc = oracle.grid(M, K, br, bc)
    inputs = [synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32)),
              synth.f32_to_bf16_bits(rng.integers(-1, 2, size=(M, K)).astype(np.float32)),
              synth.f32_to_bf16_bits(np.full((M, K), 0.75, dtype=np.float32))]
    for X in inputs:
        o_scores = oracle.block_scores(X, br, bc)
        o_mask, total = oracle.select_grouped(o_scores, nbr, nbc, group_rows, keep)
        assert B.bsr_grouped_keep_count(nbr, nbc, group_rows, keep) == total
        Xd = to_dev(X)
        mask = B.bsr_score_select_grouped(Xd, br, bc, group_rows, keep)
        row_ptr, col_idx, values = B.bsr_compress(Xd, br, bc, mask, total)
        torch.cuda.synchronize()
        g_mask = mask.cpu().numpy()
        if not np.array_equal(g_mask, o_mask):
            d = np.flatnonzero(g_mask != o_mask)
            raise AssertionError(f"grouped selection differs at blocks {d[:6]}; oracle scores {o_scores[d[:6]]}")
        o_rp, o_ci, o_val = oracle.bsr_from_mask(X, br, bc, o_mask)
        assert np.array_equal(row_ptr.cpu().numpy(), o_rp)
        assert np.array_equal(col_idx.cpu().numpy(), o_ci)
        assert to_host(values).tobytes() == o_val.tobytes()


GROUPED_BATCH = [
    # M, K, br, bc, group_rows, keep
    (2744, 196, 14, 14, 14, 0.5),        # 196 blocks per group
    (6272, 384, 32, 32, 49, 0.5),        # 588 blocks per group: shares the launch of the first
    (6272, 1536, 32, 32, 49, 0.25),      # 2352 blocks per group: the 1024-thread workgroups
    (1000, 200, 8, 8, 7, 0.3),           # ragged rows / columns, ragged last group
    (8192, 512, 16, 16, 300, 0.5),       # 9600 blocks per group: twelve keys per thread
    (8192, 512, 16, 16, 400, 0.5),       # 12800 blocks per group: on its own, group after group
    (512, 128, 16, 16, 64, 0.6),         # one group: the ungrouped selection
    (640, 128, 16, 16, 8, 0.0),          # nothing kept
    (640, 128, 16, 16, 8, 1.0),          # everything kept
]


def test_batched_grouped_selection_equals_single_calls_and_oracle():
    """Sec. IV, local ranking, several tensors per call: the masks of bsr_score_select_grouped tensor by
    tensor, and of the oracle's per-group selection."""
    rng = np.random.default_rng(41)
    Xs, hosts = [], []
    for (M, K, br, bc, rows, keep) in GROUPED_BATCH:
        X = synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32))
        hosts.append(X)
        Xs.append(to_dev(X))
    batch = B.SelectBatch(Xs, [(c[2], c[3]) for c in GROUPED_BATCH], [c[5] for c in GROUPED_BATCH])
    masks = B.bsr_score_select_grouped_batched(batch, [c[4] for c in GROUPED_BATCH])
    torch.cuda.synchronize()
    for (M, K, br, bc, rows, keep), X, Xd, mask in zip(GROUPED_BATCH, hosts, Xs, masks):
        nbr, nbc = oracle.grid(M, K, br, bc)
        if nbr * nbc == 0:
            continue
        o_mask, total = oracle.select_grouped(oracle.block_scores(X, br, bc), nbr, nbc, rows, keep)
        single = B.bsr_score_select_grouped(Xd, br, bc, rows, keep)
        torch.cuda.synchronize()
        assert np.array_equal(mask.cpu().numpy(), single.cpu().numpy()), (M, K, br, bc, rows, keep)
        assert np.array_equal(mask.cpu().numpy(), o_mask), (M, K, br, bc, rows, keep)
        assert int(mask.sum()) == total
    with pytest.raises(B.BsrError):
        B.bsr_score_select_grouped_batched(batch, [0] * len(GROUPED_BATCH))


def test_nan_inf_and_signed_zero_blocks():
    X, _ = rand_pair(128, 128, 8, "f32", seed=3)
    X[5, 5] = np.nan
    X[40, 100] = np.inf
    X[70, 3] = -0.0
    X[100:116, 16:32] = 0.0
    check_forward(X, 16, 16, 0.5, "nan/inf")
    Xb = synth.f32_to_bf16_bits(X)
    check_forward(Xb, 16, 16, 0.25, "nan/inf bf16")


def test_strided_input_and_output_views():
    X, dY = rand_pair(200, 96, 40, "bf16", seed=9)
    big = torch.zeros((200, 160), dtype=torch.bfloat16, device="cuda")
    big[:, 32:128] = to_dev(X)
    view = big[:, 32:128]                       # ldx = 160, base offset 64 bytes
    mask, scores = B.bsr_score_select(view, 8, 8, 0.5, want_scores=True)
    n_keep = B.bsr_keep_count(mask.numel(), 0.5)
    row_ptr, col_idx, values = B.bsr_compress(view, 8, 8, mask, n_keep)
    torch.cuda.synchronize()
    _, o_mask, o_rp, o_ci, o_val = oracle.prune(X, 8, 8, 0.5)
    assert np.array_equal(mask.cpu().numpy(), o_mask)
    assert np.array_equal(col_idx.cpu().numpy(), o_ci) and np.array_equal(row_ptr.cpu().numpy(), o_rp)
    assert to_host(values).tobytes() == o_val.tobytes()
    out = torch.full((200, 100), 7.0, dtype=torch.bfloat16, device="cuda")
    B.bsr_decompress(row_ptr, col_idx, values, 200, 96, 8, 8, out=out[:, 2:98])
    torch.cuda.synchronize()
    host = to_host(out)
    assert host[:, 2:98].tobytes() == oracle.mask_dense(X, 8, 8, o_mask).tobytes()
    assert np.all(host[:, :2] == host[0, 0]) and np.all(host[:, 98:] == host[0, 0])   # untouched


DW_CASES = [
    # M, K, N, br, bc, dtype, keep
    (512, 128, 96, 16, 16, "f32", 0.5),
    (1000, 200, 130, 32, 32, "f32", 0.25),
    (777, 196, 196, 14, 14, "bf16", 0.5),
    (2048, 384, 1536, 32, 32, "bf16", 0.5),
    (2048, 1536, 384, 32, 32, "bf16", 0.5),
    (1024, 256, 64, 64, 64, "bf16", 0.75),
    (640, 384, 100, 16, 16, "bf16", 0.1),
    (260, 72, 40, 1, 8, "f32", 0.5),
    (1100, 196, 150, 14, 14, "f32", 0.5),    # binary32 on the matrix cores: zero-filled tiles, ragged everything
    (4100, 384, 260, 64, 64, "f32", 0.4),    # binary32, 64x64 blocks, several splits
    (2048, 256, 192, 16, 16, "f32", 0.9),
    (300, 70, 33, 7, 5, "bf16", 0.6),
    # shapes without a matrix-core variant of their own: re-tiled into 32x32 blocks first
    (2000, 384, 200, 1, 32, "bf16", 0.5),    # row segments (the block shape Table II's overheads imply)
    (1024, 128, 64, 1, 4, "bf16", 0.5),      # the smallest segments of Table II
    (1500, 200, 130, 1, 8, "f32", 0.3),      # K not a multiple of 32
    (1000, 384, 96, 1, 384, "bf16", 0.5),    # b = K: whole rows pruned
    (777, 300, 100, 7, 5, "bf16", 0.6),      # blocks that straddle the 32-row tiles
    (640, 512, 64, 128, 128, "bf16", 0.3),   # blocks larger than a tile
    (900, 1200, 40, 3, 100, "bf16", 0.5),    # several column chunks, blocks across their borders
]


@pytest.mark.parametrize("M,K,N,br,bc,dtype,keep", DW_CASES)
def test_dw_parity(M, K, N, br, bc, dtype, keep):
    print(f"[case] dW M={M} K={K} N={N} block={br}x{bc} {dtype} keep={keep}", flush=True)
    X, dY = rand_pair(M, K, N, dtype, seed=M + N, dist="gelu" if K > 1000 else "normal")
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, br, bc, keep)
    ref = oracle.dw(oracle.mask_dense(X, br, bc, o_mask), dY)
    dYd = to_dev(dY)
    # BSR operands come from the oracle here so that this test isolates the operator
    rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
    val = to_dev(o_val.reshape(-1, bc)).reshape(o_val.shape)
    dW = B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, dYd)
    torch.cuda.synchronize()
    err = dw_error(dW.cpu().numpy(), ref)
    assert err <= DW_TOL[dtype] and err <= DW_TOL_DERIVED, err
    # accumulate on top of an existing gradient
    base = torch.full((K, N), 0.25, dtype=torch.float32, device="cuda")
    B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, dYd, dW=base, accumulate=True)
    torch.cuda.synchronize()
    assert dw_error(base.cpu().numpy() - 0.25, ref) <= 1e-4 * max(1.0, 0.25 / np.max(np.abs(ref)))
    # strided dY and dW views
    wide = torch.zeros((M, N + 24), dtype=dYd.dtype, device="cuda")
    wide[:, 8:8 + N] = dYd
    outw = torch.zeros((K, N + 8), dtype=torch.float32, device="cuda")
    B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, wide[:, 8:8 + N], dW=outw[:, 4:4 + N])
    torch.cuda.synchronize()
    # (a strided dY may take another kernel than the contiguous one: the same sums in another order)
    assert dw_error(outw[:, 4:4 + N].cpu().numpy(), dW.cpu().numpy().astype(np.float64)) <= 2e-6
    assert not outw[:, :4].any() and not outw[:, 4 + N:].any()


def test_results_are_reproducible_run_to_run():
    X, dY = rand_pair(2048, 384, 256, "bf16", seed=77)
    Xd, dYd = to_dev(X), to_dev(dY)
    outs = []
    for _ in range(2):
        scores, mask, rp, ci, val = gpu_prune(Xd, 32, 32, 0.5)
        dW = B.bsr_t_dense_matmul(rp, ci, val, 2048, 384, 32, 32, dYd)
        torch.cuda.synchronize()
        outs.append([scores.cpu().numpy().tobytes(), mask.cpu().numpy().tobytes(), rp.cpu().numpy().tobytes(),
                     ci.cpu().numpy().tobytes(), to_host(val).tobytes(), dW.cpu().numpy().tobytes()])
    assert outs[0] == outs[1]


def test_empty_inputs():
    for (M, K) in [(0, 64), (64, 0)]:
        X = torch.empty((M, K), dtype=torch.float32, device="cuda")
        mask = B.bsr_score_select(X, 16, 16, 0.5)
        assert mask.numel() == 0
        rp, ci, val = B.bsr_compress(X, 16, 16, mask, 0)
        torch.cuda.synchronize()
        assert rp.cpu().numpy().tolist() == [0] * (-(-M // 16) + 1)
        dY = torch.ones((M, 8), dtype=torch.float32, device="cuda")
        dW = B.bsr_t_dense_matmul(rp, ci, val, M, K, 16, 16, dY)
        torch.cuda.synchronize()
        assert dW.shape == (K, 8) and not dW.cpu().numpy().any()


# ----------------------------------------------------------------------------
# scale gradient of the block-sparse affine layer
# ----------------------------------------------------------------------------

AFFINE_CASES = [
    # M, K, br, bc, dtype, keep
    (2048, 384, 32, 32, "bf16", 0.5),
    (1000, 200, 32, 32, "f32", 0.25),        # ragged rows and columns
    (777, 196, 14, 14, "bf16", 0.5),         # 4-byte vectors
    (3000, 384, 1, 32, "bf16", 0.5),         # row segments
    (300, 70, 7, 5, "f32", 0.9),             # scalar columns
    (1024, 4096, 16, 16, "bf16", 0.3),       # several column chunks per row
    (96, 8192, 8, 4096, "bf16", 0.5),        # a block row wider than one workgroup's columns
    (40, 64, 64, 64, "f32", 1.0),            # one ragged block-row, everything kept
]


@pytest.mark.parametrize("M,K,br,bc,dtype,keep", AFFINE_CASES)
def test_affine_scale_grad_parity(M, K, br, bc, dtype, keep):
    print(f"[case] affine M={M} K={K} block={br}x{bc} {dtype} keep={keep}", flush=True)
    X, dY = rand_pair(M, K, K, dtype, seed=M + K + 5)
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, br, bc, keep)
    ref = oracle.affine_dscale(oracle.mask_dense(X, br, bc, o_mask), dY)
    dYd = to_dev(dY)
    rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
    val = to_dev(o_val.reshape(-1, bc)).reshape(o_val.shape)
    got = B.bsr_affine_scale_grad(rp, ci, val, M, K, br, bc, dYd)
    again = B.bsr_affine_scale_grad(rp, ci, val, M, K, br, bc, dYd)
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    assert g.tobytes() == again.cpu().numpy().tobytes()                       # reproducible
    # products are exact in binary32 for bfloat16; sums of at most M terms in binary32
    xh, dy = synth.to_f64(oracle.mask_dense(X, br, bc, o_mask)), synth.to_f64(dY)
    bound = 2.0 ** -23 * (np.log2(max(M, 2)) + 4) * np.sum(np.abs(xh * dy), axis=0)
    assert np.all(np.abs(g - ref) <= bound + 1e-30), float(np.max(np.abs(g - ref) / (bound + 1e-30)))
    # block-columns without a kept block give exactly zero
    nbr, nbc = oracle.grid(M, K, br, bc)
    dead = np.flatnonzero(o_mask.reshape(nbr, nbc).sum(axis=0) == 0)
    for j in dead:
        assert not g[j * bc:(j + 1) * bc].any()
    # accumulate, and a strided dY view
    base = torch.full((K,), 0.5, dtype=torch.float32, device="cuda")
    B.bsr_affine_scale_grad(rp, ci, val, M, K, br, bc, dYd, dalpha=base, accumulate=True)
    wide = torch.zeros((M, K + 16), dtype=dYd.dtype, device="cuda")
    wide[:, 8:8 + K] = dYd
    viewed = B.bsr_affine_scale_grad(rp, ci, val, M, K, br, bc, wide[:, 8:8 + K])
    torch.cuda.synchronize()
    assert np.all(np.abs(base.cpu().numpy() - 0.5 - ref) <= bound + 1e-6 * 0.5 + 1e-30)
    assert np.all(np.abs(viewed.cpu().numpy() - ref) <= bound + 1e-30)


@pytest.mark.parametrize("M,K,br,bc,dtype", [(777, 196, 14, 14, "bf16"), (3000, 384, 1, 32, "bf16"),
                                             (1500, 200, 1, 8, "f32"), (20000, 384, 1, 4, "bf16")])
@pytest.mark.parametrize("keep", [0.0, 1.0])
def test_degenerate_keeps_on_the_lds_staged_and_retiled_paths(M, K, br, bc, dtype, keep):
    """Nothing kept / everything kept for the narrow and few-row block shapes: forward side, dW through the
    re-tiled operand and the affine scale gradient."""
    X, dY = rand_pair(M, K, 40, dtype, seed=M + bc)
    (row_ptr, col_idx, values), o_mask = check_forward(X, br, bc, keep, "degenerate")
    dYd = to_dev(dY)
    dW = B.bsr_t_dense_matmul(row_ptr, col_idx, values, M, K, br, bc, dYd)
    G = to_dev(rand_pair(M, K, K, dtype, seed=M + bc + 1)[1])
    da = B.bsr_affine_scale_grad(row_ptr, col_idx, values, M, K, br, bc, G)
    torch.cuda.synchronize()
    if keep == 0.0:
        assert not dW.cpu().numpy().any() and not da.cpu().numpy().any()
    else:
        dense = synth.to_f64(X).T @ synth.to_f64(dY)
        assert dw_error(dW.cpu().numpy(), dense) <= DW_TOL[dtype]
        ref = np.einsum("mk,mk->k", synth.to_f64(X), synth.to_f64(to_host(G)))
        assert np.max(np.abs(da.cpu().numpy() - ref)) <= 1e-4 * np.max(np.abs(ref))


def test_affine_scale_grad_empty_inputs():
    rp = torch.zeros(1, dtype=torch.int32, device="cuda")
    ci = torch.zeros(0, dtype=torch.int32, device="cuda")
    val = torch.zeros((0, 16, 16), dtype=torch.float32, device="cuda")
    G = torch.ones((0, 64), dtype=torch.float32, device="cuda")
    out = torch.full((64,), 3.0, dtype=torch.float32, device="cuda")
    B.bsr_affine_scale_grad(rp, ci, val, 0, 64, 16, 16, G, dalpha=out, accumulate=True)      # no rows: unchanged
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 3.0)
    B.bsr_affine_scale_grad(rp, ci, val, 0, 64, 16, 16, G, dalpha=out)                       # no rows: zero
    torch.cuda.synchronize()
    assert not out.cpu().numpy().any()


# ----------------------------------------------------------------------------
# several tensors per call
# ----------------------------------------------------------------------------

BATCH_BF16 = [
    # M, K, br, bc, keep
    (2744, 196, 14, 14, 0.5),       # LDS-staged scoring, one workgroup selects (2744 blocks)
    (6272, 384, 32, 32, 0.5),       # 2352 blocks
    (25088, 384, 32, 32, 0.5),      # 9408 blocks: twelve keys per thread
    (6272, 1536, 32, 32, 0.25),     # 9408 blocks again, another keep ratio
    (8192, 1536, 32, 32, 0.5),      # 12288 blocks: the last single-workgroup size
    (4480, 1024, 32, 32, 0.4),      # 4480 blocks: the smallest that ride along with the grid-wide passes of a batch
    (12544, 1536, 32, 32, 0.5),     # 18816 blocks: grid-wide passes
    (4096, 1536, 8, 8, 0.9),        # 98304 blocks: grid-wide, long slices
    (3000, 384, 1, 32, 0.5),        # row segments: scored one by one inside the call
    (512, 128, 16, 16, 1.0),        # everything kept
    (512, 128, 16, 16, 0.0),        # nothing kept
    (640, 256, 16, 16, 0.3),        # 640 blocks: the 256-thread selection
    (1030, 130, 8, 8, 0.35),        # ragged, LDS-staged with 8-byte accesses
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_batched_score_select_equals_single_calls(dtype):
    cases = BATCH_BF16 if dtype == "bf16" else [c for c in BATCH_BF16 if c[0] * c[1] <= 4_000_000]
    Xs_host = [rand_pair(M, K, 8, dtype, seed=100 + i)[0] for i, (M, K, br, bc, keep) in enumerate(cases)]
    Xs = [to_dev(X) for X in Xs_host]
    want_scores = [torch.empty(oracle.grid(M, K, br, bc)[0] * oracle.grid(M, K, br, bc)[1], dtype=torch.float64,
                               device="cuda") if i % 2 == 0 else None
                   for i, (M, K, br, bc, keep) in enumerate(cases)]
    batch = B.SelectBatch(Xs, [(c[2], c[3]) for c in cases], [c[4] for c in cases], scores=want_scores)
    masks = B.bsr_score_select_batched(batch)
    torch.cuda.synchronize()
    first = [m.cpu().numpy().copy() for m in masks]
    for m in masks:
        m.fill_(7)
    masks = B.bsr_score_select_batched(batch)                       # again: the workspace carries nothing over
    torch.cuda.synchronize()
    for i, ((M, K, br, bc, keep), X, Xd) in enumerate(zip(cases, Xs_host, Xs)):
        single, sc = B.bsr_score_select(Xd, br, bc, keep, want_scores=True)
        torch.cuda.synchronize()
        got = masks[i].cpu().numpy()
        assert np.array_equal(got, single.cpu().numpy()), f"item {i} differs from the single call"
        assert np.array_equal(got, first[i]), f"item {i} differs between two batched calls"
        o_scores = oracle.block_scores(X, br, bc)
        nbr, nbc = oracle.grid(M, K, br, bc)
        o_mask = oracle.select(o_scores, oracle.keep_count(nbr * nbc, keep))
        assert np.array_equal(got, o_mask), f"item {i} differs from the oracle"
        if want_scores[i] is not None:
            assert want_scores[i].cpu().numpy().tobytes() == sc.cpu().numpy().tobytes()


def test_batched_score_select_more_items_than_one_launch_holds():
    rng = np.random.default_rng(77)
    shapes = [(256 + 32 * (i % 5), 128 + 64 * (i % 3), 16, 16, 0.1 + 0.025 * i) for i in range(30)]
    shapes += [(12544, 1536, 32, 32, 0.5)] * 26                      # 26 grid-wide selections: two launches of each pass
    Xs_host = [synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32)) for M, K, *_ in shapes[:30]]
    big = synth.f32_to_bf16_bits(rng.standard_normal((12544, 1536), dtype=np.float32))
    Xs = [to_dev(X) for X in Xs_host] + [to_dev(np.roll(big, i, axis=0)) for i in range(26)]
    batch = B.SelectBatch(Xs, [(s[2], s[3]) for s in shapes], [s[4] for s in shapes])
    masks = B.bsr_score_select_batched(batch)
    torch.cuda.synchronize()
    for i, (M, K, br, bc, keep) in enumerate(shapes):
        single = B.bsr_score_select(Xs[i], br, bc, keep)
        torch.cuda.synchronize()
        assert np.array_equal(masks[i].cpu().numpy(), single.cpu().numpy()), f"item {i}"
    for i in (0, 7, 29):
        M, K, br, bc, keep = shapes[i]
        o_scores = oracle.block_scores(Xs_host[i], br, bc)
        assert np.array_equal(masks[i].cpu().numpy(), oracle.select(o_scores, oracle.keep_count(o_scores.size, keep)))


DW_BATCH = [
    # M, K, N, br, bc, keep
    (2048, 384, 1536, 32, 32, 0.5),
    (2048, 1536, 384, 32, 32, 0.5),
    (4100, 384, 260, 32, 32, 0.25),       # several splits, ragged rows, N not a multiple of 8
    (777, 196, 196, 14, 14, 0.5),
    (1024, 256, 64, 64, 64, 0.75),
    (640, 384, 100, 16, 16, 0.1),
    (2000, 384, 200, 1, 32, 0.5),         # re-tiled inside the call, on its own
    (300, 70, 33, 7, 5, 0.6),             # small: the general kernel, on its own
    (512, 128, 96, 32, 32, 0.0),          # nothing kept
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_batched_dw_equals_single_calls(dtype):
    problems, refs, singles = [], [], []
    for i, (M, K, N, br, bc, keep) in enumerate(DW_BATCH):
        X, dY = rand_pair(M, K, N, dtype, seed=300 + i)
        o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, br, bc, keep)
        rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
        val = to_dev(o_val.reshape(-1, bc)).reshape(o_val.shape)
        dYd = to_dev(dY)
        problems.append((rp, ci, val, M, K, br, bc, dYd))
        singles.append(B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, dYd))
        refs.append(oracle.dw(oracle.mask_dense(X, br, bc, o_mask), dY) if M * K * N <= 2.5e8 else None)
    batch = B.MatmulBatch(problems)
    outs = B.bsr_t_dense_matmul_batched(batch)
    torch.cuda.synchronize()
    for i, (got, single, ref) in enumerate(zip(outs, singles, refs)):
        # products that share a launch may split their contraction less often than on their own: equal to rounding
        assert dw_error(got.cpu().numpy(), single.cpu().numpy().astype(np.float64)) <= 2e-6, f"item {i}"
        if ref is not None:
            assert dw_error(got.cpu().numpy(), ref) <= DW_TOL[dtype], f"item {i}"
    # a batch of one is the single call, bit for bit
    for i in (0, 3, 6, 7):
        alone = B.bsr_t_dense_matmul_batched(B.MatmulBatch([problems[i]]))
        torch.cuda.synchronize()
        assert alone[0].cpu().numpy().tobytes() == singles[i].cpu().numpy().tobytes(), f"item {i} alone"
    # accumulate on top of existing gradients, twice the same batch
    acc = [(p + (torch.full_like(o, 0.5),)) for p, o in zip(problems, outs)]
    batch2 = B.MatmulBatch(acc, accumulate=True)
    outs2 = B.bsr_t_dense_matmul_batched(batch2)
    torch.cuda.synchronize()
    for i, (a, o) in enumerate(zip(outs2, outs)):
        want = o.cpu().numpy().astype(np.float64) + 0.5
        assert np.max(np.abs(a.cpu().numpy() - want)) <= 1e-6 * max(1.0, float(np.max(np.abs(want)))), f"item {i}"


def test_batched_dw_more_items_than_one_launch_holds():
    rng = np.random.default_rng(5)
    M, K, N = 1568, 384, 192
    X = synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32))
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, 32, 32, 0.5)
    rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
    val = to_dev(o_val.reshape(-1, 32)).reshape(o_val.shape)
    dYs = [to_dev(synth.f32_to_bf16_bits(rng.standard_normal((M, N), dtype=np.float32))) for _ in range(37)]
    batch = B.MatmulBatch([(rp, ci, val, M, K, 32, 32, dY) for dY in dYs])
    outs = B.bsr_t_dense_matmul_batched(batch)
    torch.cuda.synchronize()
    first = [o.cpu().numpy().copy() for o in outs]
    B.bsr_t_dense_matmul_batched(batch)
    torch.cuda.synchronize()
    xhat = synth.to_f64(oracle.mask_dense(X, 32, 32, o_mask))
    for i, dY in enumerate(dYs):
        # products that share a launch split their contraction less often than a product on its own:
        # same sums in another order, so equal to rounding, and the same from run to run
        single = B.bsr_t_dense_matmul(rp, ci, val, M, K, 32, 32, dY)
        torch.cuda.synchronize()
        assert outs[i].cpu().numpy().tobytes() == first[i].tobytes(), f"item {i} not reproducible"
        assert dw_error(first[i], single.cpu().numpy().astype(np.float64)) <= 2e-6, f"item {i}"
        if i % 9 == 0:
            ref = xhat.T @ synth.to_f64(to_host(dY))
            assert dw_error(first[i], ref) <= DW_TOL_DERIVED, f"item {i}"


@pytest.mark.parametrize("bs", [32, 64])
def test_dw_wide_tiles_ragged_everything(bs):
    """bfloat16 products with 32 or more tiles of 384 x 128 go to the kernel with workgroup-wide
    tiles: rows, columns and output columns that end inside a block, a tile, a 16-byte chunk."""
    M, K, N = 2000, 1500, 1000
    print(f"[case] wide-tile dW M={M} K={K} N={N} block={bs}", flush=True)
    X, dY = rand_pair(M, K, N, "bf16", seed=bs, dist="gelu")
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, bs, bs, 0.5)
    ref = oracle.dw(oracle.mask_dense(X, bs, bs, o_mask), dY)
    rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
    val = to_dev(o_val.reshape(-1, bs)).reshape(o_val.shape)
    dYd = to_dev(dY)
    dW = B.bsr_t_dense_matmul(rp, ci, val, M, K, bs, bs, dYd)
    torch.cuda.synchronize()
    assert dw_error(dW.cpu().numpy(), ref) <= DW_TOL_DERIVED
    base = torch.full((K, N), 0.25, dtype=torch.float32, device="cuda")
    B.bsr_t_dense_matmul(rp, ci, val, M, K, bs, bs, dYd, dW=base, accumulate=True)
    torch.cuda.synchronize()
    assert dw_error(base.cpu().numpy() - 0.25, ref) <= 1e-4 * max(1.0, 0.25 / np.max(np.abs(ref)))


def test_dw_wide_tiles_random_shapes():
    """Seeded random shapes through the wide-tile kernel, single calls and a batched call: block size 32 or
    64, rows / columns / output columns that end anywhere (N a multiple of 8, as the kernel needs), keep
    ratios from nearly nothing to everything, dY as a view of a wider matrix, dW with a pitch of its own."""
    rng = np.random.default_rng(16883)
    problems, refs, shapes = [], [], []
    for i in range(8):
        bs = int(rng.choice([32, 64]))
        M = int(rng.integers(40 * bs, 90 * bs)) + int(rng.integers(0, bs))
        K = int(rng.integers(500, 1300))
        N = 8 * int(rng.integers(40, 80))
        keep = float(rng.choice([0.02, 0.25, 0.5, 0.75, 1.0]))
        print(f"[case] wide-tile dW, random shape {i}: M={M} K={K} N={N} block={bs} keep={keep}", flush=True)
        X, dY = rand_pair(M, K, N, "bf16", seed=7000 + i, dist="gelu" if i % 2 else "normal")
        _, o_mask, o_rp, o_ci, o_val = oracle.prune(X, bs, bs, keep)
        ref = oracle.dw(oracle.mask_dense(X, bs, bs, o_mask), dY)
        rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
        val = to_dev(o_val.reshape(-1, bs)).reshape(o_val.shape)
        wide = torch.zeros((M, N + 8 * (i % 3)), dtype=torch.bfloat16, device="cuda")
        wide[:, :N] = to_dev(dY)
        dYd = wide[:, :N]                                    # leading dimension N, N + 8 or N + 16
        out = torch.full((K, N + 4 * (i % 2)), -1.0, dtype=torch.float32, device="cuda")
        dW = out[:, :N]
        B.bsr_t_dense_matmul(rp, ci, val, M, K, bs, bs, dYd, dW=dW)
        torch.cuda.synchronize()
        assert dw_error(dW.cpu().numpy(), ref) <= DW_TOL_DERIVED, f"single call, shape {i}"
        if out.shape[1] > N:
            assert bool((out[:, N:] == -1.0).all()), f"columns beyond dW were written, shape {i}"
        problems.append((rp, ci, val, M, K, bs, bs, dYd))
        refs.append(ref)
        shapes.append((M, K, N, bs, keep))
    outs = B.bsr_t_dense_matmul_batched(B.MatmulBatch(problems))
    torch.cuda.synchronize()
    for i, (o, ref) in enumerate(zip(outs, refs)):
        assert dw_error(o.cpu().numpy(), ref) <= DW_TOL_DERIVED, f"batched call, item {i}: {shapes[i]}"


def test_batched_dw_with_more_tiles_than_compute_units():
    """24 products of 16 tiles each: the first sixteen products are run tile by tile, each tile
    by one workgroup over all 500 block-rows (more than one table's worth: two chunks), the
    last eight are split along the contraction and summed by the reduction."""
    M, K, N = 16000, 1536, 512
    pairs = []
    for i in range(3):
        print(f"[case] batched wide-tile dW, inputs {i}", flush=True)
        X, dY = rand_pair(M, K, N, "bf16", seed=900 + i, dist="gelu")
        o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, 32, 32, 0.5)
        rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
        val = to_dev(o_val.reshape(-1, 32)).reshape(o_val.shape)
        pairs.append((X, dY, o_mask, (rp, ci, val, M, K, 32, 32, to_dev(dY))))
    problems = [pairs[i % 3][3] for i in range(24)]
    outs = B.bsr_t_dense_matmul_batched(B.MatmulBatch(problems))
    torch.cuda.synchronize()
    got = [o.cpu().numpy() for o in outs]
    for i in (0, 23):                 # one product of either kind against the oracle, whole
        X, dY, o_mask, _ = pairs[i % 3]
        ref = oracle.dw(oracle.mask_dense(X, 32, 32, o_mask), dY)
        assert dw_error(got[i], ref) <= DW_TOL_DERIVED, f"item {i}"
    for i in range(3, 24):            # the same inputs give the same sums, in the same or another order
        assert dw_error(got[i], got[i % 3].astype(np.float64)) <= 2e-6, f"item {i}"


@pytest.mark.parametrize("br,bc,dtype,skips,big", [
    (32, 32, "bf16", True, False), (64, 64, "bf16", True, False), (32, 32, "f32", True, False),
    (64, 64, "f32", True, False), (32, 32, "bf16", True, True), (64, 64, "bf16", True, True),
    (16, 16, "bf16", False, False), (14, 14, "bf16", False, False), (1, 32, "bf16", False, False),
    (7, 5, "bf16", False, False),
])
def test_non_finite_dy_per_block_shape_family(br, bc, dtype, skips, big):
    """One +inf in dY.  The oracle multiplies the zeros of pruned blocks with it (0 * inf = NaN in a
    whole column of dW).  The library guarantees less and more: columns of dW other than the one of
    the inf are untouched by it; rows of dW that belong to a kept block of the inf's block-row get
    +-inf; rows that belong to a pruned block of that block-row are finite for 32x32 and 64x64 blocks
    (pruned blocks are never multiplied), and for the other block shapes either finite or NaN (their
    kept blocks are multiplied inside zero-filled tiles, and a zero of the tile times inf is NaN)."""
    M, N = 448, 48
    K = 210 if bc == 14 else (245 if bc == 5 else 256)
    if big:                                # enough tiles for the kernel with workgroup-wide tiles
        M, K, N = 2048, 1536, 1024
    X, dY = rand_pair(M, K, N, dtype, seed=br * 100 + bc)
    o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, br, bc, 0.5)
    nbr, nbc = -(-M // br), -(-K // bc)
    mask2 = o_mask.reshape(nbr, nbc)
    i0 = next(i for i in range(nbr) if 0 < mask2[i].sum() < nbc)          # a block-row with kept and pruned blocks
    m0, n0 = i0 * br + (br // 2), 7
    clean = oracle.dw(oracle.mask_dense(X, br, bc, o_mask), dY)           # the reference without the inf
    dYf = synth.to_f64(dY) if dtype == "bf16" else dY.astype(np.float64)
    xhat = synth.to_f64(oracle.mask_dense(X, br, bc, o_mask)) if dtype == "bf16" else oracle.mask_dense(X, br, bc, o_mask).astype(np.float64)
    without_row = clean[:, n0] - xhat[m0, :] * dYf[m0, n0]                # column n0 without row m0's term
    bad = dY.copy()
    if dtype == "bf16":
        bad[m0, n0] = 0x7F80                                              # +inf in bfloat16
    else:
        bad[m0, n0] = np.inf
    rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
    val = to_dev(o_val.reshape(-1, bc)).reshape(o_val.shape)
    got = B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, to_dev(bad)).cpu().numpy().astype(np.float64)
    scale = float(np.max(np.abs(clean)))
    other = np.delete(np.arange(N), n0)
    assert np.all(np.isfinite(got[:, other]))
    assert np.max(np.abs(got[:, other] - clean[:, other])) <= DW_TOL_DERIVED * scale
    nan_rows = 0
    for k in range(K):
        j = k // bc
        x = xhat[m0, k]
        if mask2[i0, j] and x != 0.0:
            assert got[k, n0] == np.sign(x) * np.inf, (k, got[k, n0])
        elif not mask2[i0, j]:
            if np.isnan(got[k, n0]):
                nan_rows += 1
                assert not skips, f"row {k} of a pruned {br}x{bc} block is NaN"
            else:
                assert abs(got[k, n0] - without_row[k]) <= DW_TOL_DERIVED * scale, (k, got[k, n0], without_row[k])
    print(f"[case] {br}x{bc} {dtype}: {nan_rows} rows of pruned blocks are NaN", flush=True)


def test_selection_of_near_ties_and_permuted_blocks():
    """What the library guarantees for scores that are equal or nearly equal.  Blocks that hold the
    same values in another order have the same sum of squares in exact arithmetic; with small
    integers every partial sum is exact in binary64 whatever the order, so both sides see an exact
    tie and the lower index wins.  A block that is larger by one unit in the last place of the score
    (2^-52 relative) wins over its twin on both sides as long as the sums themselves are exact, which
    they are for values whose squares need few bits."""
    rng = np.random.default_rng(11)
    br = bc = 16
    nbr, nbc = 32, 16
    base = rng.integers(-7, 8, size=(br, bc)).astype(np.float32)
    X = np.zeros((nbr * br, nbc * bc), dtype=np.float32)
    for i in range(nbr):
        for j in range(nbc):
            blk = base.copy().reshape(-1)
            rng.shuffle(blk)                                             # same multiset, another order
            X[i * br:(i + 1) * br, j * bc:(j + 1) * bc] = blk.reshape(br, bc)
    # a few blocks get one element nudged so that the sum of squares grows by a part in 2^40: exact in
    # binary64 (the squares are small integers plus a tiny power of two), invisible in binary32 sums
    favoured = [(3, 5), (17, 2), (30, 15)]
    for (i, j) in favoured:
        blk = X[i * br:(i + 1) * br, j * bc:(j + 1) * bc]
        r, c = np.argwhere(blk == 0)[0]
        blk[r, c] = np.float32(2.0 ** -12)                               # the sum of squares grows by 2^-24
    for keep in (3 / 512, 0.25, 0.5):
        o_scores, o_mask, _, _, _ = oracle.prune(X, br, bc, keep)
        assert len(np.unique(o_scores)) == 2
        if keep == 3 / 512:                                              # exactly the three nudged blocks
            assert sorted(np.flatnonzero(o_mask)) == sorted(i * nbc + j for i, j in favoured)
        mask = B.bsr_score_select(torch.from_numpy(X).cuda(), br, bc, keep).cpu().numpy()
        assert np.array_equal(mask, o_mask), np.flatnonzero(mask != o_mask)[:8]


SMALL_SQUARE = [
    # M, K, N, b, keep: small square blocks, a weight matrix of at most 224 x 224 (cross-patch layers)
    (777, 196, 196, 14, 0.5),       # the ResMLP patch axis; the last block-row has 7 rows
    (1000, 96, 64, 8, 0.3),
    (1234, 224, 224, 16, 0.6),      # the largest weight matrix, full 16-row groups, ragged last block-row
    (900, 120, 100, 12, 0.5),
    (640, 50, 36, 10, 0.4),         # one tile of rows, two of columns
    (500, 160, 160, 16, 1.0),       # everything kept
    (448, 196, 196, 14, 0.0),       # nothing kept
    (3500, 196, 196, 14, 0.5),      # 250 block-rows
    (700, 56, 40, 4, 0.5),          # 14 block-columns of 4: a block row is half a 16-byte copy
    (512, 28, 12, 2, 0.5),          # the smallest blocks
    (600, 128, 64, 8, 0.5),         # 16 block-columns: more than the tile has slots, another kernel's product
]


def test_batched_dw_small_square_blocks():
    """In a batched call bfloat16 products with small square blocks and a small weight matrix take the kernel
    whose workgroups own all of dW: every shape against the oracle's whole matrix, and twice the same."""
    problems, refs = [], []
    for i, (M, K, N, b, keep) in enumerate(SMALL_SQUARE):
        X, dY = rand_pair(M, K, N, "bf16", seed=700 + i)
        o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, b, b, keep)
        rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
        val = to_dev(o_val.reshape(-1, b)).reshape(o_val.shape) if o_val.size else torch.empty((0, b, b), dtype=torch.bfloat16, device="cuda")
        problems.append((rp, ci, val, M, K, b, b, to_dev(dY)))
        refs.append(oracle.dw(oracle.mask_dense(X, b, b, o_mask), dY))
    batch = B.MatmulBatch(problems)
    outs = B.bsr_t_dense_matmul_batched(batch)
    torch.cuda.synchronize()
    first = [o.cpu().numpy().copy() for o in outs]
    for o in outs:
        o.fill_(3.0)
    outs = B.bsr_t_dense_matmul_batched(batch)
    torch.cuda.synchronize()
    for i, (got, ref) in enumerate(zip(outs, refs)):
        assert got.cpu().numpy().tobytes() == first[i].tobytes(), f"item {i} not reproducible"
        assert dw_error(first[i], ref) <= DW_TOL_DERIVED, f"item {i}: {SMALL_SQUARE[i]}"
    # accumulate on top of existing gradients
    acc = [(p + (torch.full_like(o, 0.5),)) for p, o in zip(problems, outs)]
    outs2 = B.bsr_t_dense_matmul_batched(B.MatmulBatch(acc, accumulate=True))
    torch.cuda.synchronize()
    for i, (a, ref) in enumerate(zip(outs2, refs)):
        want = ref + 0.5
        assert np.max(np.abs(a.cpu().numpy() - want)) <= 1e-5 * max(1.0, float(np.max(np.abs(want)))), f"item {i}"


PACK_BATCH = [
    # M, K, br, bc, keep
    (2048, 384, 32, 32, 0.5),           # direct kernels, 16-byte vectors
    (2048, 1536, 32, 32, 0.5),
    (1000, 200, 16, 16, 0.25),          # ragged rows and columns
    (777, 196, 14, 14, 0.5),            # narrow blocks: LDS-staged kernels
    (1568, 196, 14, 14, 0.5),
    (300, 384, 1, 8, 0.5),              # row segments: LDS-staged kernels
    (64, 20000, 1, 4, 0.3),             # more block-columns than a block-row list holds: index build + pack
    (20000, 384, 1, 4, 0.5),            # LDS-staged with a counting pass first (needs its workspace)
    (512, 128, 32, 32, 0.0),            # nothing kept
    (512, 128, 32, 32, 1.0),            # everything kept
    (0, 64, 16, 16, 0.5),               # no rows
    (100, 70, 7, 5, 0.6),               # odd sizes: 2-byte / 4-byte vectors
]


def test_batched_dw_small_square_blocks_random_shapes():
    """Seeded random block sizes, block-column counts, output widths, row counts and keep ratios inside what
    the small-square-block kernel takes (even b <= 16, at most 14 block-columns, N a multiple of 4 up to 224,
    block-rows of dY on 16-byte boundaries), several batched calls, the whole dW against the oracle."""
    rng = np.random.default_rng(2311)
    for call in range(6):
        problems, refs, shapes = [], [], []
        for i in range(5):
            b = int(rng.choice([2, 4, 6, 8, 10, 12, 14, 16]))
            nbc = int(rng.integers(1, 15))
            K = nbc * b - int(rng.integers(0, b))                    # a ragged last block-column now and then
            K = max(K, 1)
            N = 4 * int(rng.integers(1, 57))
            while (b * N * 2) % 16 != 0:
                N += 4
            N = min(N, 224)
            M = b * int(rng.integers(16, 120)) + int(rng.integers(0, b))
            keep = float(rng.choice([0.1, 0.3, 0.5, 0.8, 1.0]))
            X, dY = rand_pair(M, K, N, "bf16", seed=9000 + 10 * call + i)
            _, o_mask, o_rp, o_ci, o_val = oracle.prune(X, b, b, keep)
            rp, ci = torch.from_numpy(o_rp).cuda(), torch.from_numpy(o_ci).cuda()
            val = to_dev(o_val.reshape(-1, b)).reshape(o_val.shape) if o_val.size else \
                torch.empty((0, b, b), dtype=torch.bfloat16, device="cuda")
            problems.append((rp, ci, val, M, K, b, b, to_dev(dY)))
            refs.append(oracle.dw(oracle.mask_dense(X, b, b, o_mask), dY))
            shapes.append((M, K, N, b, keep))
        outs = B.bsr_t_dense_matmul_batched(B.MatmulBatch(problems))
        torch.cuda.synchronize()
        for o, ref, shape in zip(outs, refs, shapes):
            assert dw_error(o.cpu().numpy(), ref) <= DW_TOL_DERIVED, f"call {call}: (M, K, N, b, keep) = {shape}"


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_batched_compress_and_decompress_equal_single_calls(dtype):
    problems, singles, masks, Xs = [], [], [], []
    for i, (M, K, br, bc, keep) in enumerate(PACK_BATCH):
        if M > 0:
            X, _ = rand_pair(M, K, 1, dtype, seed=500 + i)
            Xd = to_dev(X)
        else:
            X = np.zeros((0, K), dtype=np.uint16 if dtype == "bf16" else np.float32)
            Xd = torch.empty((0, K), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
        nbr, nbc = oracle.grid(M, K, br, bc)
        n_keep = B.bsr_keep_count(nbr * nbc, keep)
        mask = B.bsr_score_select(Xd, br, bc, keep) if M > 0 else torch.empty(0, dtype=torch.uint8, device="cuda")
        singles.append(B.bsr_compress(Xd, br, bc, mask, n_keep))
        problems.append((Xd, br, bc, mask, n_keep))
        masks.append(mask)
        Xs.append(X)
    batch = B.CompressBatch(problems)
    assert batch.ws_bytes > 0                                   # the counting-pass item
    for rp, ci, val in batch.outputs:                           # stale contents must be overwritten
        rp.fill_(-7)
        ci.fill_(-7)
        val.view(torch.uint8).fill_(0xA5)
    outs = B.bsr_compress_batched(batch)
    torch.cuda.synchronize()
    for i, ((rp, ci, val), (srp, sci, sval)) in enumerate(zip(outs, singles)):
        assert np.array_equal(rp.cpu().numpy(), srp.cpu().numpy()), f"item {i} row_ptr"
        assert np.array_equal(ci.cpu().numpy(), sci.cpu().numpy()), f"item {i} col_idx"
        assert to_host(val).tobytes() == to_host(sval).tobytes(), f"item {i} values"
    # ... and against the oracle for the items it finishes quickly
    for i in (0, 2, 3, 5, 11):
        M, K, br, bc, keep = PACK_BATCH[i]
        o_rp, o_ci, o_val = oracle.bsr_from_mask(Xs[i], br, bc, masks[i].cpu().numpy())
        assert np.array_equal(outs[i][0].cpu().numpy(), o_rp) and np.array_equal(outs[i][1].cpu().numpy(), o_ci)
        assert to_host(outs[i][2]).tobytes() == o_val.tobytes(), f"item {i}"
    dbatch = B.DecompressBatch([(rp, ci, val, M, K, br, bc) for (rp, ci, val), (M, K, br, bc, _) in
                                zip(outs, PACK_BATCH)])
    for o in dbatch.outputs:
        if o.numel():
            o.view(torch.uint8).fill_(0x5A)
    backs = B.bsr_decompress_batched(dbatch)
    torch.cuda.synchronize()
    for i, (back, (M, K, br, bc, _)) in enumerate(zip(backs, PACK_BATCH)):
        single = B.bsr_decompress(*outs[i], M, K, br, bc)
        torch.cuda.synchronize()
        assert to_host(back).tobytes() == to_host(single).tobytes(), f"item {i}"
        if M > 0 and M * K <= 1 << 21:
            assert to_host(back).tobytes() == oracle.mask_dense(Xs[i], br, bc, masks[i].cpu().numpy()).tobytes()


def test_batched_compress_more_items_than_one_launch_holds():
    rng = np.random.default_rng(9)
    problems, Xs = [], []
    for i in range(53):
        M, K = 96 + 32 * (i % 5), 128
        br, bc = (32, 32) if i % 2 == 0 else (14, 14)
        X = synth.f32_to_bf16_bits(rng.standard_normal((M, K), dtype=np.float32))
        Xd = to_dev(X)
        nbr, nbc = oracle.grid(M, K, br, bc)
        mask = B.bsr_score_select(Xd, br, bc, 0.5)
        problems.append((Xd, br, bc, mask, B.bsr_keep_count(nbr * nbc, 0.5)))
        Xs.append(X)
    outs = B.bsr_compress_batched(B.CompressBatch(problems))
    backs = B.bsr_decompress_batched(B.DecompressBatch(
        [(rp, ci, val, pr[0].shape[0], 128, pr[1], pr[2]) for (rp, ci, val), pr in zip(outs, problems)]))
    torch.cuda.synchronize()
    for i, (pr, (rp, ci, val), back) in enumerate(zip(problems, outs, backs)):
        m = pr[3].cpu().numpy()
        o_rp, o_ci, o_val = oracle.bsr_from_mask(Xs[i], pr[1], pr[2], m)
        assert np.array_equal(rp.cpu().numpy(), o_rp) and np.array_equal(ci.cpu().numpy(), o_ci), f"item {i}"
        assert to_host(val).tobytes() == o_val.tobytes(), f"item {i}"
        assert to_host(back).tobytes() == oracle.mask_dense(Xs[i], pr[1], pr[2], m).tobytes(), f"item {i}"


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_small_shapes_through_every_call(dtype):
    """Seeded sweep: ragged edges, ties, keep ratios from 0 to 1 and every block shape family, through the
    single calls and once more through the calls that take several tensors."""
    rng = np.random.default_rng(2024 if dtype == "bf16" else 2025)
    blocks = [(32, 32), (64, 64), (16, 16), (14, 14), (1, 4), (1, 8), (1, 32), (7, 5), (3, 20), (2, 50), (128, 16)]
    cases = []
    for _ in range(28):
        br, bc = blocks[int(rng.integers(len(blocks)))]
        M = int(rng.integers(1, 6 * br + 40))
        K = int(rng.integers(1, 5 * bc + 70))
        N = int(rng.integers(1, 150))
        nb = -(-M // br) * -(-K // bc)
        keep = float(rng.choice([0.0, 1.0 / nb, 0.25, 0.5, 1.0 - 1.0 / nb, 1.0, float(rng.random())]))
        cases.append((M, K, N, br, bc, min(max(keep, 0.0), 1.0)))
    singles = []
    for i, (M, K, N, br, bc, keep) in enumerate(cases):
        print(f"[case] random {i}: M={M} K={K} N={N} block={br}x{bc} keep={keep:.4f} {dtype}", flush=True)
        if i % 3 == 0:                                   # small integers: many exactly equal scores
            Xi = rng.integers(-2, 3, size=(M, K)).astype(np.float32)
            X = synth.f32_to_bf16_bits(Xi) if dtype == "bf16" else Xi
            dY = rand_pair(M, K, N, dtype, seed=900 + i)[1]
        else:
            X, dY = rand_pair(M, K, N, dtype, seed=900 + i)
        (rp, ci, val), o_mask = check_forward(X, br, bc, keep, label=f"random {i}")
        dYd = to_dev(dY)
        dW = B.bsr_t_dense_matmul(rp, ci, val, M, K, br, bc, dYd)
        torch.cuda.synchronize()
        ref = oracle.dw(oracle.mask_dense(X, br, bc, o_mask), dY)
        assert dw_error(dW.cpu().numpy(), ref) <= DW_TOL_DERIVED, f"case {i}"
        singles.append((to_dev(X), o_mask, rp, ci, val, dYd, dW))
    # the same tensors through the calls for several tensors
    sel = B.SelectBatch([s[0] for s in singles], [(c[3], c[4]) for c in cases], [c[5] for c in cases])
    B.bsr_score_select_batched(sel)
    nks = [B.bsr_keep_count(-(-c[0] // c[3]) * -(-c[1] // c[4]), c[5]) for c in cases]
    cb = B.CompressBatch([(s[0], c[3], c[4], m, nk) for s, c, m, nk in zip(singles, cases, sel.keep_masks, nks)])
    outs = B.bsr_compress_batched(cb)
    db = B.DecompressBatch([(rp, ci, val, c[0], c[1], c[3], c[4]) for (rp, ci, val), c in zip(outs, cases)])
    backs = B.bsr_decompress_batched(db)
    mm = B.MatmulBatch([(rp, ci, val, c[0], c[1], c[3], c[4], s[5]) for (rp, ci, val), c, s in
                        zip(outs, cases, singles)])
    dWs = B.bsr_t_dense_matmul_batched(mm)
    torch.cuda.synchronize()
    for i, (s, c) in enumerate(zip(singles, cases)):
        assert np.array_equal(sel.keep_masks[i].cpu().numpy(), s[1]), f"case {i} mask"
        assert np.array_equal(outs[i][0].cpu().numpy(), s[2].cpu().numpy()), f"case {i} row_ptr"
        assert np.array_equal(outs[i][1].cpu().numpy(), s[3].cpu().numpy()), f"case {i} col_idx"
        assert to_host(outs[i][2]).tobytes() == to_host(s[4]).tobytes(), f"case {i} values"
        want = B.bsr_decompress(s[2], s[3], s[4], c[0], c[1], c[3], c[4])
        torch.cuda.synchronize()
        assert to_host(backs[i]).tobytes() == to_host(want).tobytes(), f"case {i} dense"
        assert dw_error(dWs[i].cpu().numpy(), s[6].cpu().numpy().astype(np.float64)) <= 2e-6, f"case {i} dW"
