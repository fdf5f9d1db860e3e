"""Seeded synthetic inputs for the HLQ bit-serial LUT GEMV/GEMM path.

This module only draws random arrays; it contains none of the method's arithmetic
(no bit-plane split, no dequantisation, no table, no matmul).  Both the HIP library
and the CPU oracle consume the arrays it returns; neither is imported here.

The paper's workloads are LLaMA checkpoints; only their *layer shapes* and the
bell-shaped value distribution of weights (Motivation, "Bell-Shaped Distribution of
Weights") are kept.  Everything is drawn from a counter-based generator (Philox) keyed
by (base seed, free-form string key), so any tensor can be regenerated in isolation.

Conventions (HLQ format, Eq. 3 of the paper):
  codes  uint8  [K, N]       bit j of codes[k, n] is bit-plane j of weight (k, n)
  scales fp16   [q, K//G, N] one scale per (plane, quant group along K, column)
  zeros  fp16   [K//G, N]    one offset per (quant group, column)
  x      fp16   [M, K]
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np

BASE_SEED = 251019482


def _rng(*key) -> np.random.Generator:
    """Philox stream keyed by BASE_SEED and an arbitrary tuple of ints / strings."""
    words = [BASE_SEED]
    for k in key:
        if isinstance(k, (int, np.integer)):
            words.append(int(k) & 0xFFFFFFFF)
        else:
            words.append(zlib.crc32(str(k).encode()))
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(words)))


@dataclass(frozen=True)
class Shape:
    name: str
    K: int
    N: int


# LLaMA-3.1-8B decoder layer (hidden 4096, kv 1024, ffn 14336), as K x N.
LLAMA31_8B_LAYER = (
    Shape("q_proj", 4096, 4096),
    Shape("k_proj", 4096, 1024),
    Shape("v_proj", 4096, 1024),
    Shape("o_proj", 4096, 4096),
    Shape("gate_proj", 4096, 14336),
    Shape("up_proj", 4096, 14336),
    Shape("down_proj", 14336, 4096),
)

# LLaMA-3.1-70B decoder layer (hidden 8192, kv 1024, ffn 28672) and its LM head.
LLAMA31_70B_LAYER = (
    Shape("q_proj", 8192, 8192),
    Shape("k_proj", 8192, 1024),
    Shape("v_proj", 8192, 1024),
    Shape("o_proj", 8192, 8192),
    Shape("gate_proj", 8192, 28672),
    Shape("up_proj", 8192, 28672),
    Shape("down_proj", 28672, 8192),
)
LLAMA31_70B_LM_HEAD = Shape("lm_head", 8192, 128256)


def make_codes(K: int, N: int, q: int, *key) -> np.ndarray:
    """codes[k, n] uniform in {0 .. 2^q - 1}: every bit-plane is i.i.d. fair bits."""
    rng = _rng("codes", K, N, q, *key)
    return rng.integers(0, 1 << q, size=(K, N), dtype=np.uint8)


def make_scales(K: int, N: int, q: int, G: int, *key) -> np.ndarray:
    """|N(0, 0.02)| (std), sorted descending across planes, then cast to fp16 (RNE)."""
    rng = _rng("scales", K, N, q, G, *key)
    s = np.abs(rng.normal(0.0, 0.02, size=(q, K // G, N)))
    s = -np.sort(-s, axis=0)
    return s.astype(np.float16)


def make_zeros(K: int, N: int, G: int, *key) -> np.ndarray:
    """N(0, 0.005) (std), cast to fp16 (RNE)."""
    rng = _rng("zeros", K, N, G, *key)
    return rng.normal(0.0, 0.005, size=(K // G, N)).astype(np.float16)


def make_weight(K: int, N: int, q: int, G: int, *key):
    """(codes, scales, zeros) for one HLQ weight matrix."""
    return (
        make_codes(K, N, q, *key),
        make_scales(K, N, q, G, *key),
        make_zeros(K, N, G, *key),
    )


def make_x(M: int, K: int, *key, outliers: bool = False) -> np.ndarray:
    """X ~ N(0, 1) fp16.  With outliers, round(0.01*K) seeded channels (the same K
    indices for every row) are scaled by 20 before the fp16 cast."""
    rng = _rng("x", M, K, *key)
    x = rng.normal(0.0, 1.0, size=(M, K))
    if outliers:
        n_out = max(1, int(round(0.01 * K)))
        ch = _rng("x_outlier_channels", K, *key).permutation(K)[:n_out]
        x[:, ch] *= 20.0
    return x.astype(np.float16)


def make_dense_weight(K: int, N: int, *key, std: float = 0.02) -> np.ndarray:
    """Unquantised weights W[K, N] fp32 ~ N(0, std): the bell shape the quantizer is designed for
    (Sec. 3 "Motivation", Bell-Shaped Distribution of Weights; the weight-distribution figure there)."""
    rng = _rng("dense_weight", K, N, *key)
    return rng.normal(0.0, std, size=(K, N)).astype(np.float32)


def sample_columns(N: int, count: int, *key) -> np.ndarray:
    """Sorted sample of distinct column indices that always holds 0 and N-1."""
    count = min(count, N)
    rng = _rng("cols", N, count, *key)
    cols = set(rng.permutation(N)[:count].tolist())
    cols.update((0, N - 1))
    return np.array(sorted(cols), dtype=np.int64)
