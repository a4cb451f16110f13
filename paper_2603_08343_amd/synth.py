"""Seeded synthetic inputs for the Walsh-Hadamard output layer.

This module holds none of the layer's arithmetic: it only draws random tensors with the shapes and
value distributions of the paper's workloads (training / prefill / decode token batches feeding the
attention output layer, paper Sec. 5) and rounds them to the I/O dtype.  It is the one module that
both the GPU path's callers and the CPU oracle's callers use, so that both see identical bits.

Recipe (every workload): one numpy Generator(PCG64(seed)) stream, drawn in the fixed order
x, alpha, beta, dy, outlier mask;  x, dy ~ N(0,1);  alpha ~ U(0.5,1.5);  beta ~ N(0, 0.02^2);
optionally 1 % of x entries (i.i.d. Bernoulli) multiplied by 20 to mimic attention-output outliers.
alpha and beta are always float32.  For bf16 I/O, x and dy are rounded to nearest-even bfloat16 and
returned as uint16 bit patterns.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    d: int
    dtype: str            # "f32" or "bf16"
    backward: bool
    outliers: bool = False
    note: str = ""


# The benchmark configurations; the C4b row is the bandwidth-bound shape added so that
# d = 4096 has one (the decode rows at d = 4096 are latency-bound by construction).
WORKLOADS = {w.name: w for w in [
    Workload("C1_tiny", 64, 256, "f32", False, note="4 heads x 64, forward only"),
    Workload("C2_train", 16 * 2048, 1024, "bf16", True, note="B=16 S=2048, 16 heads x 64"),
    Workload("C3_prefill", 8 * 4096, 2048, "bf16", False, outliers=True,
             note="B=8 S=4096, 16 heads x 128, 1% entries x20"),
    Workload("C4_decode_n1", 1, 4096, "bf16", False, note="32 heads x 128, one token per sequence"),
    Workload("C4_decode_n16", 16, 4096, "bf16", False),
    Workload("C4_decode_n64", 64, 4096, "bf16", False),
    Workload("C4_decode_n256", 256, 4096, "bf16", False),
    Workload("C4b_roofline", 32768, 4096, "bf16", True, note="added bandwidth-bound shape at d=4096"),
    Workload("C5_large", 4 * 8192, 8192, "bf16", True, note="B=4 S=8192, 64 heads x 128"),
    # widths d = 12 * 2^m: the paper's own Tiny and Base models (Table 2) at a training-sized token
    # batch, and a wide one next to C5
    Workload("W_tiny_768", 32 * 1024, 768, "bf16", True, note="Table 2 Tiny: 12 heads x 64, B=32 S=1024"),
    Workload("W_base_1536", 32 * 1024, 1536, "bf16", True, note="Table 2 Base: 16 heads x 96, B=32 S=1024"),
    Workload("W_wide_6144", 4 * 8192, 6144, "bf16", True, note="48 heads x 128, B=4 S=8192"),
    # float32 I/O at a bandwidth-bound size: the butterfly schedule's kernels
    Workload("F32_4096", 16384, 4096, "f32", True, note="float32 tensors, 32 heads x 128, B=4 S=4096"),
]}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs here are finite, so NaN payloads need no care."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    N: int
    d: int
    dtype: str
    x: np.ndarray                 # [N,d] float32, or uint16 bf16 bits
    alpha: np.ndarray             # [d] float32
    beta: np.ndarray              # [d] float32
    dy: Optional[np.ndarray]      # like x, or None for forward-only


def make_inputs(N: int, d: int, dtype: str, seed: int = 0, backward: bool = True,
                outliers: bool = False) -> Inputs:
    if dtype not in ("f32", "bf16"):
        raise ValueError("dtype must be 'f32' or 'bf16'")
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((N, d), dtype=np.float32)
    alpha = rng.uniform(0.5, 1.5, size=d).astype(np.float32)
    beta = (0.02 * rng.standard_normal(d)).astype(np.float32)
    dy = rng.standard_normal((N, d), dtype=np.float32) if backward else None
    if outliers:
        mask = rng.random((N, d), dtype=np.float32) < np.float32(0.01)
        x = np.where(mask, x * np.float32(20.0), x)
    if dtype == "bf16":
        x = f32_to_bf16_bits(x)
        dy = f32_to_bf16_bits(dy) if dy is not None else None
    return Inputs(N, d, dtype, x, alpha, beta, dy)


def make_workload(name: str, seed: int = 0, N: Optional[int] = None) -> Inputs:
    """Inputs of a named workload; `N` overrides the token count (same recipe, fewer tokens)."""
    w = WORKLOADS[name]
    return make_inputs(N if N is not None else w.N, w.d, w.dtype, seed, w.backward, w.outliers)
