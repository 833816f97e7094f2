#!/usr/bin/env python3
"""Benchmark of the structured-activation-pruning hot path on one MI355X.

Default workload (``config.workload``): the full pruned-activation set of
ResMLP-S12 at batch 128, bfloat16 storage, binary32 accumulation, 50 % of the
blocks kept: for each of the 12 residual blocks the cross-patch linear input
[49152 x 196] (14 x 14 blocks), the fc1 input [25088 x 384] and the fc2 input
[25088 x 1536] (32 x 32 blocks), each with its output gradient.  Inputs are
seeded synthetic stand-ins (``paper_2311_16883_amd/synth.py``) and are resident
in HBM before the clock starts.

One step = one pass of the whole path over all 36 tensors, every call through
the C ABI: score+select -> compress -> decompress (the forward side; one
batched call per stage over all 36 tensors, or with ``--order layer`` residual
block by residual block), then the 36 weight gradients in one batched call (the
backward side).

Prints ONE JSON line.  ``value`` is the whole-step rate: block-sparse dW flops
on the kept blocks per step divided by the wall time of the whole step (so the
compressor's time counts against it).  ``phases`` gives the parts on clocks of
their own (HIP events around every call, 10 warm-up + 50 timed by default,
minimum and median).  After the clocks the buffers that were timed are compared
with the oracle (``parity``); a mismatch ends the run with a non-zero status and
no JSON line.

``--workload`` selects the other workload families (single calls, one tensor at
a time, warm and cold caches) and the bandwidth-against-size curve; they print
one JSON line of their own and, with ``--table FILE``, a Markdown table.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "compress GB/s + block-sparse dW TFLOP/s (nonzero blocks) at ResMLP-S12, 50% keep"
DW_TOL = {"f32": 1e-5, "bf16": 2e-2}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--workload", default="s12",
                   choices=("s12", "tiny", "s12_fc1_f32", "s12_layer", "s24_sweep", "b24_fc2", "sizes", "all"),
                   help="s12: the benchmark step (default).  The others time single calls, one tensor at a time: "
                        "the configurations of the other workload families, the bandwidth-against-size curve "
                        "(sizes), or all of them")
    p.add_argument("--table", default=None, help="with a --workload other than s12: also write a Markdown table there")
    p.add_argument("--layers", type=int, default=12, help="residual blocks of the workload (12 = ResMLP-S12)")
    p.add_argument("--batch", type=int, default=128)
    p.add_argument("--order", choices=("layer", "stage"), default="stage",
                   help="stage: every stage over all 36 tensors before the next stage (one batched call per stage); "
                        "layer: score+select -> compress -> decompress of one residual block's inputs before the next "
                        "block's, so that the conversion finds its tensor in the memory-side cache -- measured slower: "
                        "twelve times the short dependent kernels of the selection")
    p.add_argument("--launch", choices=("graph", "eager"), default="graph",
                   help="graph: capture the step once into a HIP graph and replay it in the timed region (same "
                        "kernels, same work, no host time per launch); eager: enqueue every step from the host")
    p.add_argument("--phase-warmup", type=int, default=10)
    p.add_argument("--phase-reps", type=int, default=50)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-parity-check", action="store_true",
                   help="skip the comparison of the timed buffers with the oracle (for profiler runs)")
    p.add_argument("--no-next-rows", action="store_true",
                   help="skip the measurements outside the timed step (per-sample ranking, row segments, affine "
                        "scale gradient), so that a profile of the run holds the step's kernels only")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run a plain 256 MiB device copy (known traffic) for scaling rocprofv3 byte counters")
    return p.parse_args()


def sources_sha16() -> str:
    """Fingerprint of the kernel sources: counter summaries under profiles/ carry the one they were taken at."""
    h = hashlib.sha256()
    for f in sorted((ROOT / "paper_2311_16883_amd" / "csrc").glob("*")):
        if f.suffix in (".hip", ".h"):
            h.update(f.name.encode())
            h.update(f.read_bytes())
    return h.hexdigest()[:16]


class Clock:
    """HIP events around every call on the current stream: `warmup` untimed calls, then `reps` timed ones."""

    def __init__(self, torch, warmup, reps):
        self.torch, self.warmup, self.reps = torch, warmup, reps
        self.scratch = None

    def __call__(self, fn, cold=False, reps=None):
        torch = self.torch
        reps = reps or self.reps
        if cold and self.scratch is None:
            self.scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        for _ in range(self.warmup):
            fn()
        torch.cuda.synchronize()
        pairs = []
        for rep in range(reps):
            if cold:
                self.scratch.fill_(rep & 1)           # 1 GiB rewritten: nothing of the operands stays in a cache
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in pairs)
        return {"min": ms[0], "median": ms[len(ms) // 2]}


def to_dev(torch, np, a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_host(torch, np, t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


# ---------------------------------------------------------------------------------------
# the other workload families: single calls, one tensor at a time
# ---------------------------------------------------------------------------------------

def family_specs(synth, which):
    sweep = list(synth.s24_sweep())
    fam = {
        "tiny": list(synth.tiny()),
        "s12_fc1_f32": list(synth.s12_fc1_f32()),
        "s12_layer": list(synth.s12_layer(128)),
        "s24_sweep": sweep,
        "b24_fc2": list(synth.b24_fc2()) + list(synth.b24_fc2(hot_first=True)),
    }
    if which == "all":
        return [s for k in ("tiny", "s12_fc1_f32", "s12_layer", "s24_sweep", "b24_fc2") for s in fam[k]]
    return fam[which]


def size_specs(synth):
    """fc1- and fc2-shaped inputs from 1 to 512 samples: the bandwidth-against-size curve."""
    from dataclasses import replace
    base = {s.name: s for s in synth.s12_layer(128)}
    out = []
    for batch in (1, 4, 16, 64, 128, 256, 512):
        for kind in ("fc1", "fc2"):
            out.append(replace(base[kind], name=f"{kind}_batch{batch}", M=batch * 196))
    return out


def run_single_calls(args, torch, np, B, synth, specs, clock, forward_only=False):
    rows = []
    for sp in specs:
        X, dY = synth.make_pair(sp, 3)
        Xd, dYd = to_dev(torch, np, X), to_dev(torch, np, dY)
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
        calls = {
            "score_select": lambda: B.bsr_score_select(Xd, sp.br, sp.bc, sp.keep, keep_mask=mask, ws=ws),
            "compress": lambda: B.bsr_compress(Xd, sp.br, sp.bc, mask, n_keep, row_ptr=rp, col_idx=ci, values=val, ws=ws),
            "decompress": lambda: B.bsr_decompress(rp, ci, val, sp.M, sp.K, sp.br, sp.bc, out=Xh),
            "dw": lambda: B.bsr_t_dense_matmul(rp, ci, val, sp.M, sp.K, sp.br, sp.bc, dYd, dW=dW, ws=ws),
        }
        if forward_only:
            del calls["dw"]
        flops = 2.0 * n_keep * sp.br * sp.bc * sp.N
        x_bytes = sp.M * sp.K * Xd.element_size()
        fwd_bytes = (1 + 2 * sp.keep) * x_bytes
        row = {"name": sp.name + ("_first_columns_hot" if sp.hot_first else ""),
               "X": [sp.M, sp.K], "N": sp.N, "block": [sp.br, sp.bc], "dtype": sp.dtype, "keep": sp.keep,
               "x_MB": round(x_bytes / 1e6, 2)}
        for cache in ("warm", "cold"):
            us = {}
            for name, f in calls.items():
                f()
                t = clock(f, cold=(cache == "cold"))
                us[name] = {"min": round(t["min"] * 1e3, 1), "median": round(t["median"] * 1e3, 1)}
            entry = {"us": us,
                     "forward_GBps": round(fwd_bytes / ((us["score_select"]["median"] + us["compress"]["median"]) * 1e3), 1),
                     "decompress_GBps": round((1 + sp.keep) * x_bytes / (us["decompress"]["median"] * 1e3), 1)}
            if "dw" in us:
                entry["dw_TFLOPs"] = round(flops / us["dw"]["median"] / 1e6, 1)
            row[cache] = entry
        rows.append(row)
        print(f"[bench] {row['name']}: done", file=sys.stderr, flush=True)
        del Xd, dYd, val, Xh, dW, ws
    return rows


def write_table(path, rows, command):
    lines = [f"Single calls, one tensor at a time, nothing else on the GPU: `{command}`.",
             "Microseconds per call, HIP events around the call, minimum / median of the timed calls after the warm-up calls.",
             "warm = repeated calls on the same buffers (operands of up to a few hundred MB may still sit in the",
             "memory-side cache); cold = a 1 GiB buffer is rewritten before every timed call.",
             "forward GB/s = (1 + 2 keep) |X| / (score+select + mask->BSR); dW TFLOP/s counts the kept blocks only; both from the medians.",
             "",
             "| workload | X, N, block, dtype, keep | cache | score+select | mask->BSR | BSR->dense | dW | dW TFLOP/s | forward GB/s |",
             "|---|---|---|---|---|---|---|---|---|"]
    for r in rows:
        for cache in ("warm", "cold"):
            e = r[cache]
            cells = " | ".join(f"{e['us'][k]['min']:.1f} / {e['us'][k]['median']:.1f}" if k in e["us"] else "-"
                               for k in ("score_select", "compress", "decompress", "dw"))
            lines.append(f"| {r['name']} | [{r['X'][0]}x{r['X'][1]}], {r['N']}, {r['block'][0]}x{r['block'][1]}, "
                         f"{r['dtype']}, {r['keep']} | {cache} | {cells} | {e.get('dw_TFLOPs', '-')} | {e['forward_GBps']} |")
    Path(path).write_text("\n".join(lines) + "\n")


def other_workloads(args, torch, np, B, synth):
    clock = Clock(torch, args.phase_warmup, args.phase_reps)
    rows, curve = [], []
    if args.workload in ("sizes", "all"):
        curve = run_single_calls(args, torch, np, B, synth, size_specs(synth), clock, forward_only=True)
    if args.workload != "sizes":
        rows = run_single_calls(args, torch, np, B, synth, family_specs(synth, args.workload), clock)
    if args.table:
        cmd = "python bench.py " + " ".join(sys.argv[1:])
        write_table(args.table, curve + rows, cmd)
    print(json.dumps({
        "metric": METRIC, "workload": args.workload, "unit": "us per call", "n_gpus": 1, "data": "synthetic",
        "timing": {"warmup_calls": args.phase_warmup, "timed_calls": args.phase_reps, "clock": "HIP events around every call"},
        "workloads": rows, "bandwidth_vs_size": curve}))


# ---------------------------------------------------------------------------------------
# the benchmark step
# ---------------------------------------------------------------------------------------

def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path is a single-GPU kernel pipeline "
              "(rows shard over GPUs with no exchange but the usual gradient all-reduce); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2311_16883_amd import binding as B
    from paper_2311_16883_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload != "s12":
        other_workloads(args, torch, np, B, synth)
        return

    specs = synth.s12_full(batch=args.batch, layers=args.layers)
    tensors, host0 = [], {}
    t_gen = time.time()
    for idx, spec in enumerate(specs):
        X, dY = synth.make_pair(spec, seed=idx)
        if spec.name.startswith("L0."):
            host0[spec.name] = (spec, X, dY)                     # layer 0 stays on the host for the parity check
        tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        n_keep = B.bsr_keep_count(spec.nblocks, spec.keep)
        tensors.append(dict(
            spec=spec, n_keep=n_keep, layer=int(spec.name[1:spec.name.index(".")]),
            X=to_dev(torch, np, X), dY=to_dev(torch, np, dY),
            mask=torch.empty(spec.nblocks, dtype=torch.uint8, device=dev),
            row_ptr=torch.empty(spec.nbr + 1, dtype=torch.int32, device=dev),
            col_idx=torch.empty(n_keep, dtype=torch.int32, device=dev),
            values=torch.empty((n_keep, spec.br, spec.bc), dtype=tdt, device=dev),
            dW=torch.empty((spec.K, spec.N), dtype=torch.float32, device=dev),
        ))
    # every tensor has its own dense output for the decompress row (a buffer shared by the tensors of one
    # shape would be rewritten while still in the memory-side cache, and its writes would never reach HBM)
    for t in tensors:
        s = t["spec"]
        t["Xhat"] = torch.empty((s.M, s.K), dtype=t["X"].dtype, device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    # ---- the calls of a step.  Forward side: one batched call per stage and group of tensors. ----
    if args.order == "layer":
        groups = [[t for t in tensors if t["layer"] == l] for l in range(args.layers)]
    else:
        groups = [tensors]
    fwd = []
    for grp in groups:
        sel = B.SelectBatch([t["X"] for t in grp], [(t["spec"].br, t["spec"].bc) for t in grp],
                            [t["spec"].keep for t in grp], keep_masks=[t["mask"] for t in grp])
        cpb = B.CompressBatch([(t["X"], t["spec"].br, t["spec"].bc, t["mask"], t["n_keep"], t["row_ptr"], t["col_idx"],
                                t["values"]) for t in grp])
        dcb = B.DecompressBatch([(t["row_ptr"], t["col_idx"], t["values"], t["spec"].M, t["spec"].K, t["spec"].br,
                                  t["spec"].bc, t["Xhat"]) for t in grp])
        fwd.append((sel, cpb, dcb))
    # the calls of a stage run one after the other on one stream: they share a workspace
    sel_ws = torch.empty(max(max(f[0].ws_bytes for f in fwd), 256), dtype=torch.uint8, device=dev)
    cpb_ws = torch.empty(max(max(f[1].ws_bytes for f in fwd), 256), dtype=torch.uint8, device=dev)

    def product(t):
        s = t["spec"]
        return (t["row_ptr"], t["col_idx"], t["values"], s.M, s.K, s.br, s.bc, t["dY"], t["dW"])

    # backward side: every weight gradient of the step in one call
    mm = B.MatmulBatch([product(t) for t in tensors])
    mm_ws = torch.empty(max(mm.ws_bytes, 256), dtype=torch.uint8, device=dev)
    # ... and, for the clock of the dominant launch, the 24 products with 32 x 32 blocks on their own
    gemm = [t for t in tensors if t["spec"].br == 32]
    mm_gemm = B.MatmulBatch([product(t) for t in gemm])
    mm_gemm_ws = torch.empty(max(mm_gemm.ws_bytes, 256), dtype=torch.uint8, device=dev)

    def select_all():
        for sel, _, _ in fwd:
            B.bsr_score_select_batched(sel, ws=sel_ws)

    def compress_all():
        for _, cpb, _ in fwd:
            B.bsr_compress_batched(cpb, ws=cpb_ws)

    def decompress_all():
        for _, _, dcb in fwd:
            B.bsr_decompress_batched(dcb)

    def forward_all(with_decompress=False):
        for sel, cpb, dcb in fwd:
            B.bsr_score_select_batched(sel, ws=sel_ws)
            B.bsr_compress_batched(cpb, ws=cpb_ws)
            if with_decompress:
                B.bsr_decompress_batched(dcb)

    def dw_all():
        B.bsr_t_dense_matmul_batched(mm, ws=mm_ws)

    def step():
        forward_all(with_decompress=True)
        dw_all()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # A step is a few dozen calls through ctypes and about a hundred kernel launches.  By default it is
    # captured once into a HIP graph and replayed (the library only launches kernels on the stream it is
    # given, so every call is capturable); if the capture fails the steps are issued eagerly.
    step()                                       # eager once: library loaded, workspaces touched
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    step()
    host_enqueue_ms = (time.perf_counter() - h0) * 1e3     # host side of one eager step (enqueue only)
    torch.cuda.synchronize()
    run_step = step
    launch = args.launch
    if launch == "graph":
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            run_step = graph.replay
        except Exception as e:                                   # noqa: BLE001 - any capture failure
            print(f"bench.py: graph capture failed ({e}); issuing the steps eagerly", file=sys.stderr)
            torch.cuda.synchronize()
            launch = "eager (graph capture failed)"
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- clocks of the parts (HIP events on the launch stream, after the timed region) ----
    clock = Clock(torch, args.phase_warmup, args.phase_reps)
    phase = {
        "forward": clock(forward_all),              # score+select and mask -> BSR in the step's order
        "score_select": clock(select_all),
        "compress": clock(compress_all),
        "decompress": clock(decompress_all),
        "dw": clock(dw_all),
    }
    gemm_launch = clock(lambda: B.bsr_t_dense_matmul_batched(mm_gemm, ws=mm_gemm_ws))
    forward_all()                                   # (the stage-by-stage clocks leave the same buffers behind)

    def flops(t):
        s = t["spec"]
        return 2.0 * t["n_keep"] * s.br * s.bc * s.N

    def x_bytes(t):
        s = t["spec"]
        return s.M * s.K * s.elem_bytes

    def dw_bytes(t):                               # kept values and dY read once, dW written once
        s = t["spec"]
        return (t["n_keep"] * s.br * s.bc * t["X"].element_size() + s.M * s.N * t["dY"].element_size() + 4 * s.K * s.N)

    by_kind = {}
    for kind in ("xpatch", "fc1", "fc2"):
        t = next(t for t in tensors if t["spec"].name.endswith(kind))
        s = t["spec"]
        ws = torch.empty(max(B.bsr_workspace_bytes(B.BSR_OP_T_DENSE_MATMUL, s.M, s.K, s.N, s.br, s.bc,
                                                   B.dtype_code(t["X"].dtype)), 256), dtype=torch.uint8, device=dev)
        c = clock(lambda: B.bsr_t_dense_matmul(t["row_ptr"], t["col_idx"], t["values"], s.M, s.K, s.br, s.bc, t["dY"],
                                               dW=t["dW"], ws=ws))
        by_kind[kind] = {"ms_per_call": {k: round(v, 5) for k, v in c.items()},
                         "TFLOPs": round(flops(t) / (c["median"] * 1e-3) / 1e12, 2)}
        del ws

    # ---- next row: the paper's local ranking (groups of block-rows select on their own) ----
    # One sample has 196 rows: 14 block-rows of 14 for the cross-patch input; 32 does not divide
    # 196, so fc1 / fc2 use groups of 8 samples = 49 block-rows.  Not part of the timed step.
    next_rows = None
    if not args.no_next_rows:
        # (masks of their own: the step's masks stay what the parity check expects)
        grp_sel = B.SelectBatch([t["X"] for t in tensors], [(t["spec"].br, t["spec"].bc) for t in tensors],
                                [t["spec"].keep for t in tensors])
        grp_rows = [14 if t["spec"].br == 14 else 49 for t in tensors]
        grp_ws = torch.empty(max(grp_sel.ws_bytes, 256), dtype=torch.uint8, device=dev)

        def grouped_all():
            B.bsr_score_select_grouped_batched(grp_sel, grp_rows, ws=grp_ws)

        grouped = clock(grouped_all)

        # 1 x b row segments (the block shape Table II's overheads imply) and b = K, at the fc1 shape
        def row_segments(bc):
            t = next(t for t in tensors if t["spec"].name.endswith("fc1"))
            s = t["spec"]
            nbr, nbc = s.M, -(-s.K // bc)
            n_keep = B.bsr_keep_count(nbr * nbc, s.keep)
            code = B.dtype_code(t["X"].dtype)
            nbytes = max(B.bsr_workspace_bytes(op, s.M, s.K, s.N, 1, bc, code)
                         for op in (B.BSR_OP_SCORE_SELECT, B.BSR_OP_COMPRESS, B.BSR_OP_T_DENSE_MATMUL))
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
            mask = torch.empty(nbr * nbc, dtype=torch.uint8, device=dev)
            rp = torch.empty(nbr + 1, dtype=torch.int32, device=dev)
            ci = torch.empty(n_keep, dtype=torch.int32, device=dev)
            val = torch.empty((n_keep, 1, bc), dtype=t["X"].dtype, device=dev)
            scratch_dense = torch.empty_like(t["Xhat"])
            scratch_dw = torch.empty_like(t["dW"])
            calls = {
                "score_select": lambda: B.bsr_score_select(t["X"], 1, bc, s.keep, keep_mask=mask, ws=ws),
                "compress": lambda: B.bsr_compress(t["X"], 1, bc, mask, n_keep, row_ptr=rp, col_idx=ci, values=val, ws=ws),
                "decompress": lambda: B.bsr_decompress(rp, ci, val, s.M, s.K, 1, bc, out=scratch_dense),
                "dw": lambda: B.bsr_t_dense_matmul(rp, ci, val, s.M, s.K, 1, bc, t["dY"], dW=scratch_dw, ws=ws),
            }
            out = {}
            for name, f in calls.items():
                f()
                out[name] = round(clock(f, reps=max(args.phase_reps // 5, 3))["median"] * 1e3, 1)
            return out

        fc1 = next(t for t in tensors if t["spec"].name.endswith("fc1"))
        row_seg_us = {f"1x{bc}": row_segments(bc) for bc in (32, fc1["spec"].K)}

        # scale gradient of the block-sparse affine layer, from the fc1 input's BSR form and a gradient of
        # the input's shape (the fc2 output gradient of the same layer is [25088 x 384])
        g = next(u for u in tensors if u["spec"].name.endswith("fc2"))["dY"]
        s = fc1["spec"]
        aff_ws = torch.empty(max(B.bsr_workspace_bytes(B.BSR_OP_AFFINE_SCALE_GRAD, s.M, s.K, 0, s.br, s.bc,
                                                       B.dtype_code(g.dtype)), 256), dtype=torch.uint8, device=dev)
        aff_out = torch.empty(s.K, dtype=torch.float32, device=dev)
        aff = clock(lambda: B.bsr_affine_scale_grad(fc1["row_ptr"], fc1["col_idx"], fc1["values"], s.M, s.K, s.br, s.bc,
                                                    g, dalpha=aff_out, ws=aff_ws))
        aff_bytes = 2 * fc1["n_keep"] * s.br * s.bc * g.element_size()   # kept values + the matching part of the gradient
        next_rows = {
            "per_sample_score_select": {"ms_per_step": {k: round(v, 4) for k, v in grouped.items()},
                                        "group_block_rows": {"xpatch": 14, "fc1": 49, "fc2": 49},
                                        "vs_whole_matrix_ms": round(phase["score_select"]["median"], 4)},
            "row_segments_fc1_us_per_call": row_seg_us,
            "affine_scale_grad_fc1": {"us_per_call": round(aff["median"] * 1e3, 1),
                                      "GBps": round(aff_bytes / (aff["median"] * 1e-3) / 1e9, 1), "bytes": aff_bytes},
        }

    # ---- parity of the buffers that were timed: layer 0 against the oracle ----
    parity = None
    if not args.no_parity_check:
        import oracle
        run_step()
        torch.cuda.synchronize()
        parity = {"tensors": [], "dw_samples": 0, "dw_max_err": 0.0}
        rng = np.random.default_rng(2311)
        for t in tensors:
            s = t["spec"]
            if s.name not in host0:
                continue
            _, X, dY = host0[s.name]
            o_scores, o_mask, o_rp, o_ci, o_val = oracle.prune(X, s.br, s.bc, s.keep)
            ok = (np.array_equal(t["mask"].cpu().numpy(), o_mask) and np.array_equal(t["row_ptr"].cpu().numpy(), o_rp)
                  and np.array_equal(t["col_idx"].cpu().numpy(), o_ci)
                  and to_host(torch, np, t["values"]).tobytes() == o_val.tobytes())
            xhat = oracle.mask_dense(X, s.br, s.bc, o_mask)
            ok = ok and to_host(torch, np, t["Xhat"]).tobytes() == xhat.tobytes()
            ks, ns = rng.integers(0, s.K, 256), rng.integers(0, s.N, 256)
            ref = np.array([oracle.dw_entry(xhat, dY, int(k), int(n)) for k, n in zip(ks, ns)])
            got = t["dW"].cpu().numpy()[ks, ns].astype(np.float64)
            scale = float(np.max(np.abs(ref)))
            err = float(np.max(np.abs(got - ref))) / (scale if scale > 0 else 1.0)
            parity["tensors"].append(s.name)
            parity["dw_samples"] += len(ks)
            parity["dw_max_err"] = max(parity["dw_max_err"], err)
            if not ok or not (err <= DW_TOL[s.dtype]):
                print(f"bench.py: the timed buffers of {s.name} differ from the oracle "
                      f"(forward side equal: {ok}, dW error {err:.3e})", file=sys.stderr)
                sys.exit(1)
        parity["dw_max_err"] = float(f"{parity['dw_max_err']:.3e}")
        parity["compared"] = "mask, row_ptr, col_idx, values, decompressed X bytewise; dW on sampled entries, max|d|/max|ref|"

    # ---- the line ----
    total_flops = sum(flops(t) for t in tensors)
    keep = specs[0].keep
    comp_alg_bytes = sum((1.0 + 2.0 * keep) * x_bytes(t) for t in tensors)
    comp_ms = phase["forward"]["median"]
    dense_bytes = sum(x_bytes(t) for t in tensors)
    bsr_bytes = sum(B.bsr_storage_bytes(t["spec"].M, t["spec"].K, t["spec"].br, t["spec"].bc, t["n_keep"],
                                        B.dtype_code(t["X"].dtype)) for t in tensors)

    # The dominant launch: the 24 fc1 / fc2 products of the step in one call = one launch of the wide-tile
    # kernel plus the reduction of the partial tiles it leaves.  Flops on kept blocks and algorithmic bytes of
    # that call over its own duration; the bound is whichever roof is lower at its arithmetic intensity.
    gemm_flops = sum(flops(t) for t in gemm)
    gemm_bytes = sum(dw_bytes(t) for t in gemm)
    gemm_ms = gemm_launch["median"]
    ai = gemm_flops / gemm_bytes
    hbm_roof_tflops = ai * HBM_PEAK_GBPS / 1e3
    tflops = gemm_flops / (gemm_ms * 1e-3) / 1e12
    gbps = gemm_bytes / (gemm_ms * 1e-3) / 1e9
    bound = "hbm" if hbm_roof_tflops < MFMA_BF16_PEAK_TFLOPS else "mfma"
    # HBM bytes of that call as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy of
    # known size): from the committed summary, and only while the kernels are the ones it was measured on
    traffic, traffic_note = None, "no counter summary"
    tfile = ROOT / "profiles" / "dw_hbm_traffic.json"
    if tfile.exists():
        try:
            rec = json.loads(tfile.read_text())
            if rec.get("sources_sha16") == sources_sha16():
                traffic, traffic_note = rec.get("bytes_per_launch"), "rocprofv3 counters, profiles/dw_hbm_traffic.json"
            else:
                traffic_note = "profiles/dw_hbm_traffic.json was measured on other kernel sources: not reported"
        except Exception:                                            # noqa: BLE001
            pass
    roofline = {
        "bound": bound,
        "achieved": round(gbps, 1) if bound == "hbm" else round(tflops, 2),
        "peak": HBM_PEAK_GBPS if bound == "hbm" else MFMA_BF16_PEAK_TFLOPS,
        "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
        "frac": round(gbps / HBM_PEAK_GBPS if bound == "hbm" else tflops / MFMA_BF16_PEAK_TFLOPS, 5),
        "traffic": traffic, "traffic_note": traffic_note,
        "kernel": "dw_wide_batched_kernel<32> and the reduction of its partial tiles: the 24 fc1/fc2 products "
                  "of the step through one bsr_t_dense_matmul_batched call",
        "ms_per_launch": {k: round(v, 5) for k, v in gemm_launch.items()},
        "flops_per_launch": gemm_flops, "algorithmic_bytes_per_launch": gemm_bytes,
        "arithmetic_intensity": round(ai, 1), "roof_at_this_intensity_TFLOPs": round(min(hbm_roof_tflops, MFMA_BF16_PEAK_TFLOPS), 1),
        "hbm_side": {"achieved_GBps": round(gbps, 1), "peak_GBps": HBM_PEAK_GBPS, "frac": round(gbps / HBM_PEAK_GBPS, 5)},
        "mfma_side": {"achieved_TFLOPs": round(tflops, 2), "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                      "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 5)},
    }
    result = {
        "metric": METRIC,
        "value": round(total_flops / (ms_per_step * 1e-3) / 1e12, 4),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResMLP-S12 full activation set, batch {args.batch}, {args.layers} layers x "
                               "(xpatch 14x14, fc1 32x32, fc2 32x32), bf16, keep 0.5",
                   "tensors_per_step": len(tensors), "keep": keep,
                   "launch": "hip graph replay" if launch == "graph" else launch,
                   "order": ("per residual block: score+select -> compress -> decompress of its three inputs (one "
                             "batched call each); then all 36 dW in one batched call") if args.order == "layer" else
                            "stage by stage over all 36 tensors (one batched call per stage)"},
        "phases": {
            "timing": {"warmup_calls": args.phase_warmup, "timed_calls": args.phase_reps,
                       "clock": "HIP events around every repetition; rates from the medians"},
            "compress_GBps": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9, 2),
            "compress_input_GBps": round(dense_bytes / (comp_ms * 1e-3) / 1e9, 2),
            "dw_TFLOPs": round(total_flops / (phase["dw"]["median"] * 1e-3) / 1e12, 3),
            "ms": {k: {m: round(v, 4) for m, v in c.items()} for k, c in phase.items()},
            "dw_single_calls": by_kind,
        },
        "roofline": roofline,
        "roofline_compress": {"bound": "hbm", "achieved": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9, 2),
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 5),
                              "bytes_per_step": comp_alg_bytes,
                              "what": "(1 + 2 keep) |X| of all 36 tensors over the median of phases.ms.forward "
                                      "(score+select and mask -> BSR, in the step's order)"},
        "parity_checked": parity is not None,
        "parity": parity,
        "next_rows": next_rows,
        "activation_memory": {"dense_MiB": round(dense_bytes / 2 ** 20, 2), "bsr_MiB": round(bsr_bytes / 2 ** 20, 2),
                              "saved_frac": round(1.0 - bsr_bytes / dense_bytes, 4)},
        "host_enqueue_ms": round(host_enqueue_ms, 3),
        "input_generation_s": round(t_gen, 1),
    }

    if not args.no_cpu_baseline and "L0.fc1" in host0:
        import oracle
        spec, X, dY = host0["L0.fc1"]
        cores = oracle.num_threads()
        c0 = time.perf_counter()
        scores = oracle.block_scores(X, spec.br, spec.bc)
        mask = oracle.select(scores, oracle.keep_count(spec.nblocks, spec.keep))
        oracle.bsr_from_mask(X, spec.br, spec.bc, mask)
        c1 = time.perf_counter()
        xhat = oracle.mask_dense(X, spec.br, spec.bc, mask)
        ncols = 1024                                          # bounded sample of the output columns
        sub = np.ascontiguousarray(dY[:, :ncols])
        c2 = time.perf_counter()
        oracle.dw(xhat, sub)
        c3 = time.perf_counter()
        nk = int(mask.sum())
        f = 2.0 * nk * spec.br * spec.bc * ncols
        whole = (c1 - c0) + (c3 - c2)
        result["cpu_baseline"] = {
            "value": round(f / whole / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"layer 0 fc1 [{spec.M}x{spec.K}] bf16: score+select+BSR on the whole tensor, "
                      f"dW on the first {ncols} of {spec.N} output columns.  The rate counts the flops of the kept "
                      "blocks only (the metric's unit) while the oracle's loop runs over the whole masked dense "
                      "matrix, zeros included: twice that many multiply-adds at this keep ratio",
            "compress_GBps": round((1.0 + 2.0 * spec.keep) * X.nbytes / (c1 - c0) / 1e9, 3),
            "dw_TFLOPs": round(f / (c3 - c2) / 1e12, 6),
            "seconds": round(whole, 2),
        }

    print(json.dumps(result))


if __name__ == "__main__":
    main()
