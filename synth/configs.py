"""The five synthetic workloads and a few adversarial symbol streams.

Recipe (all draws from numpy.random.Generator(PCG64(seed)), float32):
  student_t(df)  = N(0,1) / sqrt(Gamma(df/2, 1) * 2/df), then * scale
  laplace(b)     = b * (Exp(1) - Exp(1))
  uniform(a, b)  = a + (b-a) * U[0,1)
  outliers       = after the base draw, k ~ Binomial(n, p) distinct uniformly
                   chosen elements (the same law as an independent coin of
                   probability p per element) are replaced by +-10*sigma
                   (fair sign), sigma being the population standard deviation
                   of the base draw (float64 accumulation).
seed(cfg, layer, tensor_index) = 1_000_000*cfg + 100*layer + tensor_index;
config 1 uses seed 0 as its text says; activation vectors use
5_000_000 + 100*layer + tensor_index.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

ASYMMETRIC = 1
UNSIGNED = 0


@dataclass(frozen=True)
class TensorSpec:
    cfg: int
    layer: int
    index: int          # position in the layer's tensor list
    name: str
    rows: int           # out features (1 for a norm-gain vector)
    cols: int           # in features
    dist: str           # "student_t" | "laplace" | "uniform"
    df: float
    scale: float        # multiplier (student_t), b (laplace); unused for uniform
    outlier_p: float
    bits: int
    scheme: int         # ASYMMETRIC | UNSIGNED
    seed: int

    @property
    def n(self) -> int:
        return self.rows * self.cols


def tensor_seed(cfg: int, layer: int, index: int) -> int:
    return 1_000_000 * cfg + 100 * layer + index


def x_seed(layer: int, index: int) -> int:
    return 5_000_000 + 100 * layer + index


def config_chunk_symbols(cfg: int) -> int:
    return 8192 if cfg == 3 else 4096


def config_bits(cfg: int) -> int:
    return 4 if cfg == 3 else 8


_SHAPES = {
    2: [("q", 2048, 2048), ("k", 2048, 2048), ("v", 2048, 2048), ("o", 2048, 2048),
        ("gate", 8192, 2048), ("up", 8192, 2048), ("down", 2048, 8192)],
    3: [("qkv", 9216, 3072), ("o", 3072, 3072), ("gate_up", 16384, 3072), ("down", 3072, 8192)],
    4: [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
        ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)],
}
_LAYERS = {2: 24, 3: 32, 4: 32}


def config_tensors(cfg: int, layers: int | None = None) -> List[TensorSpec]:
    """Tensor list of workload `cfg` (1..5); `layers` truncates the layer count.

    Config 5 runs on config 4's tensors, so it returns the same list."""
    if cfg == 1:
        return [TensorSpec(1, 0, 0, "w", 2048, 2048, "student_t", 4.0, 0.02, 0.0, 8, ASYMMETRIC, 0)]
    if cfg == 5:
        cfg = 4
    if cfg not in _SHAPES:
        raise ValueError(f"unknown config {cfg}")
    nl = _LAYERS[cfg] if layers is None else min(layers, _LAYERS[cfg])
    out: List[TensorSpec] = []
    for layer in range(nl):
        for i, (name, r, c) in enumerate(_SHAPES[cfg]):
            if cfg == 2:
                out.append(TensorSpec(2, layer, i, name, r, c, "student_t", 4.0, 0.02, 0.001, 8,
                                      ASYMMETRIC, tensor_seed(2, layer, i)))
            elif cfg == 3:
                out.append(TensorSpec(3, layer, i, name, r, c, "laplace", 0.0, 0.015, 0.0, 4,
                                      ASYMMETRIC, tensor_seed(3, layer, i)))
            else:
                out.append(TensorSpec(4, layer, i, name, r, c, "student_t", 5.0, 0.02, 0.0, 8,
                                      ASYMMETRIC, tensor_seed(4, layer, i)))
        if cfg == 2:  # two norm-gain vectors per layer, unsigned 8-bit
            for j, name in enumerate(("norm_attn", "norm_mlp")):
                out.append(TensorSpec(2, layer, 50 + j, name, 1, 2048, "uniform", 0.0, 0.0, 0.0, 8,
                                      UNSIGNED, tensor_seed(2, layer, 50 + j)))
    if cfg == 2 and nl == _LAYERS[2]:  # final norm
        out.append(TensorSpec(2, nl, 50, "norm_final", 1, 2048, "uniform", 0.0, 0.0, 0.0, 8,
                              UNSIGNED, tensor_seed(2, nl, 50)))
    return out


_BLOCK = 1 << 20   # draws are made block by block into preallocated memory


def make_tensor(spec: TensorSpec) -> np.ndarray:
    """Flat float32 weights of `spec`, row-major [rows, cols].

    Draws are taken in blocks of 2**20 elements (for each block: the first
    variate array, then the second), which is part of the recipe."""
    rng = np.random.Generator(np.random.PCG64(spec.seed))
    n = spec.n
    w = np.empty(n, dtype=np.float32)
    tmp = np.empty(min(n, _BLOCK), dtype=np.float32)
    for lo in range(0, n, _BLOCK):
        hi = min(n, lo + _BLOCK)
        a = w[lo:hi]
        b = tmp[: hi - lo]
        if spec.dist == "student_t":
            rng.standard_normal(out=a, dtype=np.float32)
            rng.standard_gamma(spec.df / 2.0, out=b, dtype=np.float32)
            np.multiply(b, np.float32(2.0 / spec.df), out=b)
            np.sqrt(b, out=b)
            np.divide(a, b, out=a)
            np.multiply(a, np.float32(spec.scale), out=a)
        elif spec.dist == "laplace":
            rng.standard_exponential(out=a, dtype=np.float32)
            rng.standard_exponential(out=b, dtype=np.float32)
            np.subtract(a, b, out=a)
            np.multiply(a, np.float32(spec.scale), out=a)
        elif spec.dist == "uniform":
            rng.random(out=a, dtype=np.float32)
            np.multiply(a, np.float32(0.4), out=a)
            np.add(a, np.float32(0.8), out=a)
        else:
            raise ValueError(spec.dist)
    del tmp
    if spec.outlier_p > 0.0:
        mean = float(np.mean(w, dtype=np.float64))
        sigma = float(np.sqrt(max(np.mean(np.square(w, dtype=np.float64)) - mean * mean, 0.0)))
        k = int(rng.binomial(n, spec.outlier_p))
        pos = rng.choice(n, size=k, replace=False)
        sign = np.where(rng.random(k, dtype=np.float32) < np.float32(0.5), -1.0, 1.0)
        w[pos] = (sign * (10.0 * sigma)).astype(np.float32)
    return w


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns.

    Used only to prepare activation inputs; finite inputs assumed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def make_x_bf16(layer: int, index: int, length: int) -> np.ndarray:
    """Activation vector N(0,1), rounded to bf16; returns uint16 bit patterns."""
    rng = np.random.Generator(np.random.PCG64(x_seed(layer, index)))
    return f32_to_bf16_bits(rng.standard_normal(length, dtype=np.float32))


def adversarial_symbol_cases(bits: int = 8):
    """Small symbol streams (uint8, one symbol per byte) that stress the coder.

    Yields (name, symbols, chunk_symbols)."""
    A = 1 << bits
    rng = np.random.Generator(np.random.PCG64(777 + bits))
    yield "single_symbol", np.full(1000, 3, np.uint8), 256
    yield "two_symbols", (rng.random(5000) < 0.9).astype(np.uint8), 512
    yield "n_equals_1", np.array([A - 1], np.uint8), 4096
    yield "all_symbols_uniform", np.tile(np.arange(A, dtype=np.uint8), 64), 1024
    geo = np.minimum(rng.geometric(0.5, 70000) - 1, A - 1).astype(np.uint8)
    yield "geometric", geo, 4096
    yield "chunk_minus_1", geo[:4095], 4096
    yield "chunk_plus_1", geo[:4097], 4096
    yield "ragged_tail", geo[:3 * 4096 + 17], 4096
    yield "odd_n", geo[:10001], 2048
    # Fibonacci-weighted counts give the deepest possible Huffman tree (m symbols: the
    # longest code has m - 1 bits).  The counts are capped at 200000 below to keep the case
    # small, which flattens the top of the tree: with 8-bit symbols the longest code comes
    # out at 28 bits, not 32 (codes of exactly 32 bits are exercised through
    # codebooks given by their lengths instead); with 4-bit symbols, 15 bits.
    m = min(A, 33)
    fib = [1, 1]
    while len(fib) < m:
        fib.append(fib[-1] + fib[-2])
    reps = np.array(fib[:m], dtype=np.int64)
    # scale down the total while keeping every count >= 1 and the ordering strict
    sym = np.repeat(np.arange(m, dtype=np.uint8), np.minimum(reps, 200000))
    rng.shuffle(sym)
    yield "fibonacci_deep", sym, 4096
