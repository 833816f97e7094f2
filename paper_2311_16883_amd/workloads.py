"""Per-call times of the four entry points at every workload family of ``synth.py``.

``python -m paper_2311_16883_amd.workloads`` runs, for one tensor of each family, the
calls of the path one after the other on the current stream (score + select, mask -> BSR,
BSR -> dense, dW) and prints a Markdown table: microseconds per call (HIP events around the
call, minimum / median of 50 after 10 warm-up calls), the dW rate on kept blocks and the forward
rate ``(1 + 2 keep) |X| / (score + select + mask -> BSR)``, both from the minima.  Single calls with nothing else on the
GPU: launch latency is part of every figure.  Inputs are the seeded synthetic tensors.

By default a call is repeated on the same buffers, so operands of up to a few hundred MB may
still sit in the memory-side cache from the previous repetition ("warm").  ``--cold`` rewrites
a 1 GiB scratch buffer before every timed call, which leaves nothing of the operands in any cache.
"""
from __future__ import annotations

import sys

import numpy as np
import torch

from . import binding as B
from . import synth


def _event():
    return torch.cuda.Event(enable_timing=True)


_scratch = None


def _time_us(f, reps: int = 50, warmup: int = 10, cold: bool = False):
    """(minimum, median) over `reps` timed calls after `warmup` untimed ones, in microseconds."""
    global _scratch
    if cold and _scratch is None:
        _scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    for _ in range(warmup):
        f()
    torch.cuda.synchronize()
    ts = []
    for rep in range(reps):
        if cold:
            _scratch.fill_(rep)
        a, b = _event(), _event()
        a.record()
        f()
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b) * 1e3)
    return min(ts), float(np.median(ts))


def _to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def specs():
    sweep = {s.name: s for s in synth.s24_sweep()}
    picked = ["s24_fc1_b16_k50", "s24_fc2_b16_k50", "s24_fc1_b32_k50", "s24_fc2_b32_k50", "s24_fc1_b64_k50",
              "s24_fc2_b64_k10", "s24_fc2_b64_k50", "s24_fc2_b64_k90"]
    return (list(synth.tiny()) + list(synth.s12_fc1_f32()) + list(synth.s12_layer(128)) +
            [sweep[n] for n in picked] + list(synth.b24_fc2()) + list(synth.b24_fc2(hot_first=True)))


def main() -> None:
    assert torch.cuda.is_available(), "needs a GPU"
    cold = "--cold" in sys.argv[1:]
    print("# cold: a 1 GiB buffer is rewritten before every timed call" if cold
          else "# warm: repeated calls on the same buffers")
    print("| workload | X, dY, block, keep | score+select | mask->BSR | BSR->dense | dW | dW TFLOP/s (kept) "
          "| forward GB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for sp in specs():
        X, dY = synth.make_pair(sp, 3)
        Xd, dYd = _to_dev(X), _to_dev(dY)
        code = B.dtype_code(Xd.dtype)
        n_keep = B.bsr_keep_count(sp.nblocks, sp.keep)
        ops = (B.BSR_OP_SCORE_SELECT, B.BSR_OP_COMPRESS, B.BSR_OP_T_DENSE_MATMUL)
        nbytes = max(B.bsr_workspace_bytes(op, sp.M, sp.K, sp.N, sp.br, sp.bc, code) for op in ops)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        mask = torch.empty(sp.nblocks, dtype=torch.uint8, device="cuda")
        rp = torch.empty(sp.nbr + 1, dtype=torch.int32, device="cuda")
        ci = torch.empty(n_keep, dtype=torch.int32, device="cuda")
        val = torch.empty((n_keep, sp.br, sp.bc), dtype=Xd.dtype, device="cuda")
        Xh = torch.empty_like(Xd)
        dW = torch.empty((sp.K, sp.N), dtype=torch.float32, device="cuda")
        t1 = _time_us(lambda: B.bsr_score_select(Xd, sp.br, sp.bc, sp.keep, keep_mask=mask, ws=ws), cold=cold)
        t2 = _time_us(lambda: B.bsr_compress(Xd, sp.br, sp.bc, mask, n_keep, row_ptr=rp, col_idx=ci, values=val,
                                             ws=ws), cold=cold)
        t3 = _time_us(lambda: B.bsr_decompress(rp, ci, val, sp.M, sp.K, sp.br, sp.bc, out=Xh), cold=cold)
        t4 = _time_us(lambda: B.bsr_t_dense_matmul(rp, ci, val, sp.M, sp.K, sp.br, sp.bc, dYd, dW=dW, ws=ws),
                      cold=cold)
        flops = 2.0 * n_keep * sp.br * sp.bc * sp.N
        fwd_bytes = (1 + 2 * sp.keep) * sp.M * sp.K * Xd.element_size()
        name = sp.name + ("_first_columns_hot" if sp.hot_first else "")
        cells = " | ".join(f"{t[0]:.1f} / {t[1]:.1f}" for t in (t1, t2, t3, t4))
        print(f"| {name} | [{sp.M}x{sp.K}], [{sp.M}x{sp.N}], {sp.br}x{sp.bc} {sp.dtype}, {sp.keep} | {cells} | "
              f"{flops / t4[0] / 1e6:.1f} | {fwd_bytes / (t1[0] + t2[0]) / 1e3:.0f} |", flush=True)
        del Xd, dYd, val, Xh, dW, ws


if __name__ == "__main__":
    main()
