#!/usr/bin/env python3
"""Benchmark of the structured-activation-pruning hot path on one MI355X.

Workload (``config.workload``): the full pruned-activation set of ResMLP-S12 at
batch 128, bfloat16 storage, binary32 accumulation, 50 % of the blocks kept:
for each of the 12 residual blocks the cross-patch linear input [49152 x 196]
(14 x 14 blocks), the fc1 input [25088 x 384] and the fc2 input [25088 x 1536]
(32 x 32 blocks), each with its output gradient.  Inputs are seeded synthetic
stand-ins (``paper_2311_16883_amd/synth.py``) and are resident in HBM before
the clock starts.

One step = one pass of the whole path over all 36 tensors:
score+select -> compress -> decompress -> dW, every call through the C ABI.

Prints ONE JSON line.  ``value`` is the whole-step rate: block-sparse dW flops
on the kept blocks per step divided by the wall time of the whole step (so the
compressor's time counts against it).  ``phases`` gives the two halves of the
metric on their own clocks: compress GB/s and dW TFLOP/s.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--layers", type=int, default=12, help="residual blocks of the workload (12 = ResMLP-S12)")
    p.add_argument("--batch", type=int, default=128)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--phase-reps", type=int, default=5)
    p.add_argument("--launch", choices=("graph", "eager"), default="graph",
                   help="graph: capture the step once into a HIP graph and replay it in the timed region (same "
                        "kernels, same work, no host time per launch); eager: enqueue every step from the host")
    p.add_argument("--graph", action="store_true", help="same as --launch graph")
    p.add_argument("--streams", type=int, default=4,
                   help="HIP streams (default priority) the independent tensors of a step are spread over")
    p.add_argument("--select", choices=("batched", "single"), default="batched",
                   help="batched: one bsr_score_select_batched call for all tensors of the step (a handful of "
                        "launches); single: one bsr_score_select call per tensor on its stream")
    p.add_argument("--dw", choices=("batched", "single"), default="batched",
                   help="batched: one bsr_t_dense_matmul_batched call for all tensors of the step after their BSR "
                        "forms exist; single: one bsr_t_dense_matmul call per tensor on its stream")
    p.add_argument("--pack", choices=("batched", "single"), default="batched",
                   help="batched: one bsr_compress_batched and one bsr_decompress_batched call for all tensors of the "
                        "step; single: one bsr_compress and one bsr_decompress call per tensor on its stream")
    p.add_argument("--no-next-rows", action="store_true",
                   help="skip the measurements outside the timed step (per-sample ranking, row segments), "
                        "so that a profile of the run holds the step's kernels only")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run a plain 256 MiB device copy (known traffic) for scaling rocprofv3 byte counters")
    return p.parse_args()


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

    def to_dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    specs = synth.s12_full(batch=args.batch, layers=args.layers)
    tensors = []
    host_sample = None
    t_gen = time.time()
    for idx, spec in enumerate(specs):
        X, dY = synth.make_pair(spec, seed=idx)
        if host_sample is None and spec.name.endswith("fc1"):
            host_sample = (spec, X, dY)
        tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        n_keep = B.bsr_keep_count(spec.nblocks, spec.keep)
        code = B.dtype_code(tdt)
        ws_bytes = max(B.bsr_workspace_bytes(op, spec.M, spec.K, spec.N, spec.br, spec.bc, code)
                       for op in range(4))
        tensors.append(dict(
            spec=spec, n_keep=n_keep, X=to_dev(X), dY=to_dev(dY),
            mask=torch.empty(spec.nblocks, dtype=torch.uint8, device=dev),
            row_ptr=torch.empty(spec.nbr + 1, dtype=torch.int32, device=dev),
            col_idx=torch.empty(n_keep, dtype=torch.int32, device=dev),
            values=torch.empty((n_keep, spec.br, spec.bc), dtype=tdt, device=dev),
            dW=torch.empty((spec.K, spec.N), dtype=torch.float32, device=dev),
            ws=torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev),
        ))
        del X, dY
    # every tensor has its own dense output for the decompress row (a buffer shared by the tensors of one
    # shape would be rewritten while still in the memory-side cache, and its writes would never reach HBM)
    for t in tensors:
        s = t["spec"]
        t["Xhat"] = torch.empty((s.M, s.K), dtype=t["X"].dtype, device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    def score_select(t):
        s = t["spec"]
        B.bsr_score_select(t["X"], s.br, s.bc, s.keep, keep_mask=t["mask"], ws=t["ws"])

    def compress(t):
        s = t["spec"]
        B.bsr_compress(t["X"], s.br, s.bc, t["mask"], t["n_keep"], row_ptr=t["row_ptr"],
                       col_idx=t["col_idx"], values=t["values"], ws=t["ws"])

    def decompress(t):
        s = t["spec"]
        B.bsr_decompress(t["row_ptr"], t["col_idx"], t["values"], s.M, s.K, s.br, s.bc, out=t["Xhat"])

    def dw(t):
        s = t["spec"]
        B.bsr_t_dense_matmul(t["row_ptr"], t["col_idx"], t["values"], s.M, s.K, s.br, s.bc, t["dY"],
                             dW=t["dW"], ws=t["ws"])

    phases = [("score_select", score_select), ("compress", compress), ("decompress", decompress), ("dw", dw)]
    batched = args.select == "batched"
    dw_batched = args.dw == "batched"
    pack_batched = args.pack == "batched"
    per_tensor = [p for p in phases if not (batched and p[0] == "score_select") and not (dw_batched and p[0] == "dw")
                  and not (pack_batched and p[0] in ("compress", "decompress"))]
    if pack_batched:
        # mask -> BSR and BSR -> dense of every tensor of the step in one call each
        cpb = B.CompressBatch([(t["X"], t["spec"].br, t["spec"].bc, t["mask"], t["n_keep"], t["row_ptr"], t["col_idx"],
                                t["values"]) for t in tensors])
        cpb_ws = torch.empty(max(cpb.ws_bytes, 256), dtype=torch.uint8, device=dev)
        dcb = B.DecompressBatch([(t["row_ptr"], t["col_idx"], t["values"], t["spec"].M, t["spec"].K, t["spec"].br,
                                  t["spec"].bc, t["Xhat"]) for t in tensors])
    if dw_batched:
        # every weight gradient of the step in one call, once all BSR forms exist: same results, the kernels of
        # one block shape share launches
        mm = B.MatmulBatch([(t["row_ptr"], t["col_idx"], t["values"], t["spec"].M, t["spec"].K, t["spec"].br,
                             t["spec"].bc, t["dY"], t["dW"]) for t in tensors])
        mm_ws = torch.empty(max(mm.ws_bytes, 256), dtype=torch.uint8, device=dev)

    def dw_all():
        if dw_batched:
            B.bsr_t_dense_matmul_batched(mm, ws=mm_ws)
        else:
            for t in tensors:
                dw(t)
    if batched:
        # scores and selection of all tensors of the step in one call: same masks, a handful of launches
        sel = B.SelectBatch([t["X"] for t in tensors], [(t["spec"].br, t["spec"].bc) for t in tensors],
                            [t["spec"].keep for t in tensors], keep_masks=[t["mask"] for t in tensors])
        sel_ws = torch.empty(max(sel.ws_bytes, 256), dtype=torch.uint8, device=dev)

    def score_select_all():
        if batched:
            B.bsr_score_select_batched(sel, ws=sel_ws)
        else:
            for t in tensors:
                score_select(t)

    # The tensors of a step are independent: spread them over a few streams so that the
    # short dependent kernels of one tensor overlap with the others'.  Stream i waits for
    # the main stream at the start of a step and the main stream waits for every stream
    # at its end, so the step is still one unit of work on the main stream.
    side = [torch.cuda.Stream() for _ in range(max(args.streams, 1))] if args.streams > 1 else []
    # Tensors are dealt to the streams largest first, each to the stream with the least bytes so
    # far (the three tensor shapes of a layer differ 4x in size; a plain stride would put all
    # the large ones on the same two streams).
    per_stream = [[] for _ in side]
    if side:
        weight = lambda t: t["spec"].M * (2 * t["spec"].K + t["spec"].N)
        load = [0] * len(side)
        for t in sorted(tensors, key=weight, reverse=True):
            i = load.index(min(load))
            per_stream[i].append(t)
            load[i] += weight(t)

    def step():
        main_stream = torch.cuda.current_stream()
        if batched:
            score_select_all()
        if pack_batched:
            B.bsr_compress_batched(cpb, ws=cpb_ws)
            B.bsr_decompress_batched(dcb)
        if not side or not per_tensor:
            for t in tensors:
                for _, f in per_tensor:
                    f(t)
            if dw_batched:
                dw_all()
            return
        fork = torch.cuda.Event()
        fork.record(main_stream)
        for st in side:
            st.wait_event(fork)
        # enqueue round-robin, one tensor per stream at a time, so that every stream has work early
        for k in range(max(len(l) for l in per_stream)):
            for st, l in zip(side, per_stream):
                if k < len(l):
                    with torch.cuda.stream(st):
                        for _, f in per_tensor:
                            f(l[k])
        for st in side:
            done = torch.cuda.Event()
            done.record(st)
            main_stream.wait_event(done)
        if dw_batched:
            dw_all()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # With every stage batched a step is four calls through ctypes and about sixteen kernel launches; with
    # per-tensor calls (--select / --pack / --dw single) it is up to 144 calls and 190 launches, and the host
    # needs about as long to enqueue them as the GPU to run them.  By default the step is captured once into
    # a HIP graph and replayed (the library only launches kernels on the stream it is given, so every call
    # is capturable); if the capture fails the steps are issued eagerly.
    step()                                       # eager once: library loaded, workspaces touched
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    step()
    host_enqueue_ms = (time.perf_counter() - h0) * 1e3     # host side of one eager step (enqueue only)
    torch.cuda.synchronize()
    run_step = step
    launch = "graph" if args.graph else args.launch
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

    # ---- per-phase clocks (HIP events on the launch stream, after the timed region) ----
    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps      # ms

    phase_ms = {}
    for name, f in phases:
        if name == "score_select":
            phase_ms[name] = timed(score_select_all, args.phase_reps)
        elif name == "dw":
            phase_ms[name] = timed(dw_all, args.phase_reps)
        elif pack_batched and name == "compress":
            phase_ms[name] = timed(lambda: B.bsr_compress_batched(cpb, ws=cpb_ws), args.phase_reps)
        elif pack_batched and name == "decompress":
            phase_ms[name] = timed(lambda: B.bsr_decompress_batched(dcb), args.phase_reps)
        else:
            phase_ms[name] = timed(lambda: [f(t) for t in tensors], args.phase_reps)

    # ---- next row: the paper's local ranking (groups of block-rows select on their own) ----
    # One sample has 196 rows: 14 block-rows of 14 for the cross-patch input; 32 does not divide
    # 196, so fc1 / fc2 use groups of 8 samples = 49 block-rows.  Not part of the timed step.
    mask_g = torch.empty(max(t["spec"].nblocks for t in tensors), dtype=torch.uint8, device=dev)

    def group_rows(s):
        return 14 if s.br == 14 else 49

    def score_select_grouped(t):
        s = t["spec"]
        B.bsr_score_select_grouped(t["X"], s.br, s.bc, group_rows(s), s.keep, keep_mask=mask_g[:s.nblocks],
                                   ws=t["ws"])

    grouped_ms = None if args.no_next_rows else timed(lambda: [score_select_grouped(t) for t in tensors],
                                                      args.phase_reps)

    # ---- next row: 1 x b row segments (the block shape Table II's overheads imply) and b = K,
    # at the fc1 shape, one tensor, every call of the path.  Not part of the timed step.
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
        calls = {
            "score_select": lambda: B.bsr_score_select(t["X"], 1, bc, s.keep, keep_mask=mask, ws=ws),
            "compress": lambda: B.bsr_compress(t["X"], 1, bc, mask, n_keep, row_ptr=rp, col_idx=ci, values=val, ws=ws),
            "decompress": lambda: B.bsr_decompress(rp, ci, val, s.M, s.K, 1, bc, out=t["Xhat"]),
            "dw": lambda: B.bsr_t_dense_matmul(rp, ci, val, s.M, s.K, 1, bc, t["dY"], dW=t["dW"], ws=ws),
        }
        out = {}
        for name, f in calls.items():
            f()
            out[name] = round(timed(f, max(args.phase_reps, 3)) * 1e3, 1)
        return out

    fc1_K = next(t["spec"].K for t in tensors if t["spec"].name.endswith("fc1"))
    row_seg_us = None if args.no_next_rows else {f"1x{bc}": row_segments(bc) for bc in (32, fc1_K)}

    # ---- next row: scale gradient of the block-sparse affine layer, from the fc1 input's BSR form and a
    # gradient of the input's shape (the fc2 output gradient of the same layer is [25088 x 384]).
    def affine_us():
        t = next(t for t in tensors if t["spec"].name.endswith("fc1"))
        g = next(u for u in tensors if u["spec"].name.endswith("fc2"))["dY"]
        s = t["spec"]
        assert tuple(g.shape) == (s.M, s.K)
        code = B.dtype_code(g.dtype)
        ws = torch.empty(max(B.bsr_workspace_bytes(B.BSR_OP_AFFINE_SCALE_GRAD, s.M, s.K, 0, s.br, s.bc, code), 256),
                         dtype=torch.uint8, device=dev)
        out = torch.empty(s.K, dtype=torch.float32, device=dev)
        f = lambda: B.bsr_affine_scale_grad(t["row_ptr"], t["col_idx"], t["values"], s.M, s.K, s.br, s.bc, g,
                                            dalpha=out, ws=ws)
        f()
        us = timed(f, max(args.phase_reps, 5)) * 1e3
        n_keep = B.bsr_keep_count(s.nblocks, s.keep)
        alg = 2 * n_keep * s.br * s.bc * g.element_size()       # kept values + the matching part of the gradient
        return {"us_per_call": round(us, 1), "GBps": round(alg / (us * 1e-6) / 1e9, 1), "bytes": alg}

    affine = None if args.no_next_rows else affine_us()

    # ---- the dominant kernel: one event pair around every dW launch ----
    def per_launch_ms(fn, group):
        pairs = []
        for _ in range(args.phase_reps):
            for t in group:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn(t)
                e1.record()
                pairs.append((e0, e1))
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)

    def flops(t):
        s = t["spec"]
        return 2.0 * t["n_keep"] * s.br * s.bc * s.N

    def x_bytes(t):
        s = t["spec"]
        return s.M * s.K * s.elem_bytes

    # (with the batched call the 36 products share a few launches: their mean is the call's time / 36)
    dw_launch_ms = phase_ms["dw"] / len(tensors) if dw_batched else per_launch_ms(dw, tensors)
    total_flops = sum(flops(t) for t in tensors)
    flops_per_launch = total_flops / len(tensors)
    by_kind = {}
    for kind in ("xpatch", "fc1", "fc2"):
        grp = [t for t in tensors if t["spec"].name.endswith(kind)]
        ms = per_launch_ms(dw, grp)
        by_kind[kind] = {"ms_per_launch": round(ms, 5),
                         "TFLOPs": round(flops(grp[0]) / (ms * 1e-3) / 1e12, 3)}

    keep = specs[0].keep
    comp_alg_bytes = sum((1.0 + 2.0 * keep) * x_bytes(t) for t in tensors)
    comp_ms = phase_ms["score_select"] + phase_ms["compress"]
    dense_bytes = sum(x_bytes(t) for t in tensors)
    bsr_bytes = sum(B.bsr_storage_bytes(t["spec"].M, t["spec"].K, t["spec"].br, t["spec"].bc, t["n_keep"],
                                        B.dtype_code(t["X"].dtype)) for t in tensors)

    # HBM bytes per dW launch as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a
    # plain copy of known size); taken from the committed summary, not measured in this run
    traffic = None
    tfile = ROOT / "profiles" / "dw_hbm_traffic.json"
    if tfile.exists():
        try:
            traffic = json.loads(tfile.read_text()).get("bytes_per_launch")
        except Exception:
            traffic = None

    achieved_tflops = flops_per_launch / (dw_launch_ms * 1e-3) / 1e12
    # the same launches against the memory side: kept values + dY read once, dW written once
    dw_alg_bytes = sum(t["n_keep"] * t["spec"].br * t["spec"].bc * t["X"].element_size()
                       + t["spec"].M * t["spec"].N * t["dY"].element_size() + 4 * t["spec"].K * t["spec"].N
                       for t in tensors) / len(tensors)
    dw_alg_GBps = dw_alg_bytes / (dw_launch_ms * 1e-3) / 1e9
    result = {
        "metric": "compress GB/s + block-sparse dW TFLOP/s (nonzero blocks) at ResMLP-S12, 50% keep",
        "value": round(total_flops / (ms_per_step * 1e-3) / 1e12, 4),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResMLP-S12 full activation set, batch {args.batch}, {args.layers} layers x "
                               "(xpatch 14x14, fc1 32x32, fc2 32x32), bf16, keep 0.5",
                   "tensors_per_step": len(tensors), "keep": keep,
                   "streams": max(args.streams, 1) if per_tensor else 1,
                   "launch": "hip graph replay" if launch == "graph" else launch,
                   "score_select": "one batched call per step" if batched else "one call per tensor",
                   "dw": "one batched call per step" if dw_batched else "one call per tensor",
                   "pack": "one batched call per step each" if pack_batched else "one call per tensor each",
                   "step": "score+select -> compress -> decompress -> dW for every tensor"},
        "phases": {
            "compress_GBps": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9, 2),
            "compress_input_GBps": round(dense_bytes / (comp_ms * 1e-3) / 1e9, 2),
            "dw_TFLOPs": round(total_flops / (phase_ms["dw"] * 1e-3) / 1e12, 3),
            "ms": {k: round(v, 4) for k, v in phase_ms.items()},
            "dw_by_tensor": by_kind,
        },
        "roofline": {"bound": "mfma", "achieved": round(achieved_tflops, 3), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 5),
                     "traffic": traffic, "kernel": "bsr_t_dense_matmul (dW)",
                     "flops_per_launch": flops_per_launch, "ms_per_launch": round(dw_launch_ms, 5),
                     "hbm_side": {"algorithmic_bytes_per_launch": round(dw_alg_bytes), "achieved_GBps": round(dw_alg_GBps, 1),
                                  "peak_GBps": HBM_PEAK_GBPS, "frac": round(dw_alg_GBps / HBM_PEAK_GBPS, 5)}},
        "roofline_compress": {"bound": "hbm", "achieved": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9, 2),
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": round(comp_alg_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 5),
                              "bytes_per_step": comp_alg_bytes},
        "next_rows": None if args.no_next_rows else {
            "per_sample_score_select": {"ms_per_step": round(grouped_ms, 4),
                                        "group_block_rows": {"xpatch": 14, "fc1": 49, "fc2": 49},
                                        "vs_whole_matrix_ms": round(phase_ms["score_select"], 4)},
            "row_segments_fc1_us_per_call": row_seg_us,
            "affine_scale_grad_fc1": affine},
        "activation_memory": {"dense_MiB": round(dense_bytes / 2 ** 20, 2), "bsr_MiB": round(bsr_bytes / 2 ** 20, 2),
                              "saved_frac": round(1.0 - bsr_bytes / dense_bytes, 4)},
        "host_enqueue_ms": round(host_enqueue_ms, 3),
        "input_generation_s": round(t_gen, 1),
    }

    if not args.no_cpu_baseline and host_sample is not None:
        import oracle
        spec, X, dY = host_sample
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
                      f"dW on the first {ncols} of {spec.N} output columns",
            "compress_GBps": round((1.0 + 2.0 * spec.keep) * X.nbytes / (c1 - c0) / 1e9, 3),
            "dw_TFLOPs": round(f / (c3 - c2) / 1e12, 6),
            "seconds": round(whole, 2),
        }

    print(json.dumps(result))


if __name__ == "__main__":
    main()
