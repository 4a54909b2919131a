"""Seeded synthetic inputs shaped like the paper's LLM linear layers.

This module is the only code shared by the tests of the CPU oracle and of the HIP
library.  It holds none of the method's arithmetic (no LiquidQuant, no activation
quantization, no dequantization, no matmul): it draws FP16 weights and FP16 activations
and nothing else.  The INT8-plus-per-token-scale form in which activations reach the W4A8
GEMM (Sec. 6 of the paper: dynamic per-token quantization upstream of the kernel) is
produced by each side for itself: the tests take it from the oracle, the benchmark from
the library's own activation-quantization kernel.

Recipe: numpy.random.Generator(PCG64(seed)); draw order W, then X, then the outlier
channel indices.  W ~ N(0, sigma) in FP32 rounded to FP16; X ~ N(0, 1) rounded to FP16;
`outlier_frac` of the K channels (at least one when the fraction is non-zero) are
multiplied by 20 (and rounded to FP16 again).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class GemmShape:
    name: str
    M: int
    N: int
    K: int
    group: int = 64
    sigma_w: float = 0.02
    outlier_frac: float = 0.0
    seed: int = 0


def _mk(prefix, Ms, N, K, **kw):
    return [GemmShape(f"{prefix}_M{M}_N{N}_K{K}", M, N, K, **kw) for M in Ms]


# The five workload families (tiny / decode / 7B MLP / 70B layers / prefill sweep).
TINY = [GemmShape("tiny_M8_N256_K512", 8, 256, 512, seed=0)]
DECODE = _mk("decode", (1, 4, 16), 4096, 4096, seed=1)
MLP_7B = (_mk("mlp7b_up", (32, 128, 512), 11008, 4096, outlier_frac=0.001, seed=2)
          + _mk("mlp7b_down", (32, 128, 512), 4096, 11008, outlier_frac=0.001, seed=2))
LAYERS_70B = (_mk("l70b_up", (16, 256, 2048), 28672, 8192, group=128, sigma_w=0.015, seed=3)
              + _mk("l70b_down", (16, 256, 2048), 8192, 28672, group=128, sigma_w=0.015, seed=3)
              + _mk("l70b_qkv", (16, 256, 2048), 10240, 8192, group=128, sigma_w=0.015, seed=3))
PREFILL = _mk("prefill", (1024, 2048, 4096, 8192), 8192, 8192, seed=4)

ALL_SHAPES = TINY + DECODE + MLP_7B + LAYERS_70B + PREFILL


def by_name(name: str) -> GemmShape:
    """A shape of ALL_SHAPES, or any other one spelled `<label>_M<M>_N<N>_K<K>[_g<group>]`
    (group 64 unless given; the recipe of the prefill sweep)."""
    for s in ALL_SHAPES:
        if s.name == name:
            return s
    import re

    m = re.fullmatch(r"[A-Za-z0-9]+_M(\d+)_N(\d+)_K(\d+)(?:_g(64|128))?", name)
    if not m:
        raise KeyError(name)
    return GemmShape(name, int(m.group(1)), int(m.group(2)), int(m.group(3)), group=int(m.group(4) or 64), seed=4)


def make_weights(N, K, sigma=0.02, seed=0, rng=None):
    """FP16-valued weights W [N,K] returned as float32 (exactly representable in FP16)."""
    rng = rng or np.random.Generator(np.random.PCG64(seed))
    W = rng.standard_normal((N, K), dtype=np.float32)
    W *= np.float32(sigma)
    return W.astype(np.float16).astype(np.float32)


def make_activations_f16(M, K, outlier_frac=0.0, seed=0, rng=None):
    """FP16 activations X [M,K] before quantization (outlier channels multiplied by 20)."""
    rng = rng or np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((M, K), dtype=np.float32).astype(np.float16).astype(np.float32)
    if outlier_frac > 0:
        n_out = max(1, int(round(outlier_frac * K)))
        idx = rng.choice(K, size=n_out, replace=False)
        X[:, idx] *= np.float32(20.0)
    return X.astype(np.float16)


def make_smooth(K, seed=0):
    """Positive FP32 smooth scales [K], log-normal around 1 (stand-in for SmoothQuant's)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.exp(rng.standard_normal(K, dtype=np.float32) * np.float32(0.5)).astype(np.float32)


def make_problem_f16(shape: GemmShape):
    """Returns (W float32 [N,K] with FP16 values, X float16 [M,K]) for one shape."""
    rng = np.random.Generator(np.random.PCG64(shape.seed))
    W = make_weights(shape.N, shape.K, shape.sigma_w, rng=rng)
    X = make_activations_f16(shape.M, shape.K, shape.outlier_frac, rng=rng)
    return W, X


def make_q_i8(N, K, seed=0, lo=-119, hi=119, style="uniform"):
    """Level-1 INT8 weights drawn directly (for packer / kernel edge cases).

    styles: "uniform" over [lo, hi]; "extreme" puts both ends of the protective range in
    every group of 64; "constant" makes every row constant; "narrow" keeps each row
    within a span of 10 codes.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if style == "uniform":
        Q = rng.integers(lo, hi + 1, size=(N, K), dtype=np.int16)
    elif style == "extreme":
        Q = rng.integers(lo, hi + 1, size=(N, K), dtype=np.int16)
        Q[:, 0::64] = lo
        Q[:, 1::64] = hi
    elif style == "constant":
        Q = np.repeat(rng.integers(lo, hi + 1, size=(N, 1), dtype=np.int16), K, axis=1)
    elif style == "narrow":
        base = rng.integers(lo, hi - 9, size=(N, 1), dtype=np.int16)
        Q = base + rng.integers(0, 10, size=(N, K), dtype=np.int16)
    else:
        raise ValueError(style)
    return Q.astype(np.int8)
