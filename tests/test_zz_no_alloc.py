"""bsr_score_select_static (the entry point that allocates nothing) against
bsr_score_select, through the C ABI: masks and scores bit for bit, on calls in a
row that share the library's static scratch array, each smaller than the one
before, with and without caller-provided scores; then the size limit.

This file is collected last on purpose: a failure here must not hide others.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2311_16883_amd import binding as B
from paper_2311_16883_amd import synth

pytestmark = pytest.mark.gpu


def _x(M, K, dtype, seed):
    spec = synth.TensorSpec("t", M, K, 8, 1, 1, dtype, "normal")
    X, _ = synth.make_pair(spec, seed)
    if X.dtype == np.uint16:
        return torch.from_numpy(X.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(X).cuda()


def _raw_static(X, br, bc, keep, scores, mask):
    """The raw C symbol, no helper in between."""
    l = B.lib()
    M, K = X.shape
    return l.bsr_score_select_static(C.c_void_p(X.data_ptr()), B.dtype_code(X.dtype), M, K, X.stride(0), br, bc,
                                     C.c_double(keep), C.c_void_p(scores.data_ptr()) if scores is not None else None,
                                     C.c_void_p(mask.data_ptr()), None)


# (M, K, br, bc, keep, dtype): grid-wide selection (65536 and 16384 blocks), the one-workgroup
# selection (4096 blocks), a ragged 14x14 case; every call smaller than the one before
CASES = [
    (4096, 4096, 16, 16, 0.5, "bf16"),
    (2048, 2048, 16, 16, 0.25, "f32"),
    (2048, 512, 16, 16, 0.5, "bf16"),
    (1000, 196, 14, 14, 0.5, "bf16"),
]


def test_static_scratch_matches_workspace_call_on_calls_in_a_row():
    B.bsr_static_scratch_init()
    torch.cuda.synchronize()
    for rep in range(2):                      # the second sweep starts from the scratch the first one left
        for ci, (M, K, br, bc, keep, dtype) in enumerate(CASES):
            for want_scores in (False, True):
                print(f"[case] static rep={rep} {M}x{K} {br}x{bc} keep={keep} {dtype} scores={want_scores}", flush=True)
                X = _x(M, K, dtype, 100 + ci)
                nblocks = (-(-M // br)) * (-(-K // bc))
                assert nblocks <= B.bsr_score_select_static_max_blocks()
                ref = B.bsr_score_select(X, br, bc, keep, want_scores=True)
                ref_mask, ref_scores = ref
                mask = torch.full((nblocks,), 7, dtype=torch.uint8, device="cuda")
                scores = torch.full((nblocks,), -1.0, dtype=torch.float64, device="cuda") if want_scores else None
                rc = _raw_static(X, br, bc, keep, scores, mask)
                assert rc == B.BSR_OK, B.lib().bsr_error_string(rc)
                torch.cuda.synchronize()
                assert torch.equal(mask, ref_mask)
                assert int(mask.sum()) == B.bsr_keep_count(nblocks, keep)
                if want_scores:
                    assert scores.cpu().numpy().tobytes() == ref_scores.cpu().numpy().tobytes()


def test_static_scratch_rejects_sizes_beyond_its_capacity():
    limit = B.bsr_score_select_static_max_blocks()
    assert limit == 524288
    # 1 x 4 blocks of a [1025 x 2048] matrix: 1025 * 512 = 524800 blocks > limit; refused on the host
    X = torch.zeros((1025, 2048), dtype=torch.bfloat16, device="cuda")
    mask = torch.full((1025 * 512,), 7, dtype=torch.uint8, device="cuda")
    rc = _raw_static(X, 1, 4, 0.5, None, mask)
    assert rc == B.BSR_ERR_LIMIT
    assert B.lib().bsr_error_string(rc) == b"BSR_ERR_LIMIT"
    torch.cuda.synchronize()
    assert int(mask.min()) == 7 and int(mask.max()) == 7        # nothing was written
    # exactly at the limit it runs
    X = _x(1024, 2048, "bf16", 7)
    mask = torch.empty((limit,), dtype=torch.uint8, device="cuda")
    assert _raw_static(X, 1, 4, 0.5, None, mask) == B.BSR_OK
    ref = B.bsr_score_select(X, 1, 4, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(mask, ref)
