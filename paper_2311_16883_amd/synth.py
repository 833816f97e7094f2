"""Seeded synthetic ResMLP-shaped activations and output gradients.

Input generation only: nothing of the pruning method (no block scores, no
selection, no BSR, no matrix product) lives here, so the CPU oracle's callers
and the GPU path's callers can both draw their inputs from this module.

The tensors stand in for the activations of ResMLP on ImageNet / CIFAR that the
paper measures on (Sec. III, Fig. 4 and 5; Sec. V): same shapes, and value
statistics of a normalised linear-layer input (standard normal) or of a GELU
output (exact erf form of a standard normal).  Output gradients are normal with
standard deviation 1e-3.  Everything is drawn on the host with
``numpy.random.default_rng`` so that a (seed, spec) pair names the data.

bfloat16 tensors are returned as ``numpy.uint16`` bit patterns (round to
nearest even from binary32).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import List, Optional

import numpy as np
from scipy.special import erf

DY_STD = 1e-3


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round binary32 to bfloat16 (nearest even); NaN stays a quiet NaN."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if nan.any():
        out[nan] = ((u[nan] >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact binary64 view of a float32 / bfloat16-bits array."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def gelu_erf(z: np.ndarray) -> np.ndarray:
    """GELU, exact erf form, evaluated in binary64."""
    z = z.astype(np.float64)
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


@dataclass(frozen=True)
class TensorSpec:
    """One linear layer's saved input X [M x K] and output gradient dY [M x N]."""
    name: str
    M: int
    K: int
    N: int
    br: int
    bc: int
    dtype: str = "bf16"          # "f32" | "bf16"
    x_dist: str = "normal"       # "normal" | "gelu"
    keep: float = 0.5
    hot_cols: float = 0.0        # fraction of columns of X scaled by hot_scale
    hot_scale: float = 5.0
    hot_first: bool = False      # True: the first columns are the hot ones

    @property
    def nbr(self) -> int:
        return -(-self.M // self.br)

    @property
    def nbc(self) -> int:
        return -(-self.K // self.bc)

    @property
    def nblocks(self) -> int:
        return self.nbr * self.nbc

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


def _store(a32: np.ndarray, dtype: str) -> np.ndarray:
    return a32 if dtype == "f32" else f32_to_bf16_bits(a32)


_CHUNK_ROWS = 2048          # rows per independently seeded chunk (fixes the data, not the thread count)
_THREADS = min(16, os.cpu_count() or 1)


def _chunked(M: int, ncols: int, out_dtype, fill) -> np.ndarray:
    """Fill an [M x ncols] array chunk by chunk; chunk c only depends on (seed, c)."""
    out = np.empty((M, ncols), dtype=out_dtype)
    chunks = [(c, r0, min(M, r0 + _CHUNK_ROWS)) for c, r0 in enumerate(range(0, M, _CHUNK_ROWS))]

    def work(item):
        c, r0, r1 = item
        out[r0:r1] = fill(c, r1 - r0)

    if len(chunks) > 1 and _THREADS > 1:
        with ThreadPoolExecutor(max_workers=_THREADS) as ex:
            list(ex.map(work, chunks))
    else:
        for item in chunks:
            work(item)
    return out


def make_x(spec: TensorSpec, seed: int) -> np.ndarray:
    hot = None
    if spec.hot_cols > 0.0:
        nhot = int(np.floor(spec.hot_cols * spec.K))
        hot = np.arange(nhot) if spec.hot_first else \
            np.random.default_rng([seed, 3]).permutation(spec.K)[:nhot]
    if spec.x_dist not in ("normal", "gelu"):
        raise ValueError(spec.x_dist)

    def fill(c, rows):
        z = np.random.default_rng([seed, 1, c]).standard_normal((rows, spec.K), dtype=np.float32)
        if spec.x_dist == "gelu" or hot is not None:
            x = gelu_erf(z) if spec.x_dist == "gelu" else z.astype(np.float64)
            if hot is not None:
                x[:, hot] *= spec.hot_scale
            z = x.astype(np.float32)
        return _store(z, spec.dtype)

    return _chunked(spec.M, spec.K, np.float32 if spec.dtype == "f32" else np.uint16, fill)


def make_dy(spec: TensorSpec, seed: int) -> np.ndarray:
    def fill(c, rows):
        g = np.random.default_rng([seed, 2, c]).standard_normal((rows, spec.N), dtype=np.float32)
        g *= np.float32(DY_STD)
        return _store(g, spec.dtype)

    return _chunked(spec.M, spec.N, np.float32 if spec.dtype == "f32" else np.uint16, fill)


def make_pair(spec: TensorSpec, seed: int):
    return make_x(spec, seed), make_dy(spec, seed)


# ---------------------------------------------------------------------------
# The five workloads (shapes of ResMLP-S12 / S24 / B24: 196 patches, hidden
# dimension D, MLP width 4D; Sec. III Fig. 4 uses the (64, 196, 384) input).
# ---------------------------------------------------------------------------

def tiny() -> List[TensorSpec]:
    return [TensorSpec("tiny", 256, 128, 64, 16, 16, "f32", "gelu", 0.5)]


def s12_fc1_f32(keeps=(0.25, 0.5, 0.75)) -> List[TensorSpec]:
    return [TensorSpec(f"s12_fc1_f32_k{int(k * 100)}", 64 * 196, 384, 1536, 32, 32, "f32", "normal", k)
            for k in keeps]


def s12_layer(batch: int = 128, D: int = 384, patches: int = 196, keep: float = 0.5,
              dtype: str = "bf16", b: int = 32, pb: int = 14) -> List[TensorSpec]:
    """The three pruned linear-layer inputs of one ResMLP block."""
    rows = batch * patches
    return [
        TensorSpec("xpatch", batch * D, patches, patches, pb, pb, dtype, "normal", keep),
        TensorSpec("fc1", rows, D, 4 * D, b, b, dtype, "normal", keep),
        TensorSpec("fc2", rows, 4 * D, D, b, b, dtype, "gelu", keep),
    ]


def s12_full(batch: int = 128, layers: int = 12) -> List[TensorSpec]:
    out = []
    for l in range(layers):
        out += [replace(s, name=f"L{l}.{s.name}") for s in s12_layer(batch)]
    return out


def s24_sweep(batch: int = 256, blocks=(16, 32, 64), keeps=(0.1, 0.25, 0.5, 0.9)) -> List[TensorSpec]:
    rows = batch * 196
    out = []
    for b in blocks:
        for k in keeps:
            out.append(TensorSpec(f"s24_fc1_b{b}_k{int(k * 100)}", rows, 384, 1536, b, b, "bf16", "normal", k))
            out.append(TensorSpec(f"s24_fc2_b{b}_k{int(k * 100)}", rows, 1536, 384, b, b, "bf16", "gelu", k))
    return out


def b24_fc2(batch: int = 256, hot_first: bool = False) -> List[TensorSpec]:
    return [TensorSpec("b24_fc2", batch * 196, 3072, 768, 64, 64, "bf16", "gelu", 0.5,
                       hot_cols=0.1, hot_scale=5.0, hot_first=hot_first)]


def scaled(spec: TensorSpec, M: Optional[int] = None, N: Optional[int] = None) -> TensorSpec:
    """Same layer with fewer rows / output columns (parity-test sizes)."""
    return replace(spec, M=M or spec.M, N=N or spec.N)
