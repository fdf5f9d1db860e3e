"""CPU oracle for the HLQ bit-serial LUT GEMV/GEMM path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares no code with the HIP library and never sees the packed GPU layout:
it consumes the unpacked HLQ tensors

    codes  uint8 [K, N]        bit j of codes[k, n] = bit-plane j   (App. B example)
    scales fp16  [q, K/G, N]   s_j per (plane, group along K, column)   (Eq. 3, Alg. 1)
    zeros  fp16  [K/G, N]      z   per (group, column)
    X      fp16  [M, K]

and works in fp64 throughout.

Because the LUT method is an exact re-association of dequantise-then-multiply
(Sec. 2 "Bit-Serial LUT-Based GEMM"; App. D calls the mirror form lossless), the
reference result has a plain definition and `gemm_dequant` is that definition written
out: reconstruct W^ by Eq. 3 / Eq. 6, then an ordinary matrix product.

`gemm_lut` and `gemm_lut_mirror` follow the algorithm's steps as App. B and App. D
describe them (16-entry tables over groups of four activations, nibble lookups per
bit-plane, per-plane scales; the +-1 re-parametrisation with 8 stored entries).  They
exist to pin the identity "LUT accumulation == dequantise-then-multiply"; they are
not used as the parity reference.

Pins (tests/test_oracle_*.py): the bit-plane worked example of App. B; the
bits-per-weight figures of Table 1 and the model sizes of Table 3; exact rational
brute force on tiny inputs; the uniform special case s_j = 2^j * Delta (Alg. 1 init)
against textbook integer dequantisation; one-hot activations; all-zero / all-one
planes; linearity; LUT == dequant; mirror == plain; the lossy-table variant (App. D, Table
Quantization: fp16 or int8 entries) equals the plain lookup path on entries the storage type
holds exactly.  No function here is unpinned.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

LUT_GROUP = 4  # activations per lookup table (App. B / App. D: groups of four)


# --------------------------------------------------------------------------- format
def bit_planes(codes: np.ndarray, q: int) -> np.ndarray:
    """Split integer codes into q single-bit matrices; plane j holds bit j (LSB = 0).

    App. B: (9, 7, 6, 3) -> lowest plane (1, 1, 0, 1), highest plane (1, 0, 0, 0)."""
    codes = np.asarray(codes)
    return np.stack([(codes >> j) & 1 for j in range(q)]).astype(np.uint8)


def codes_from_planes(planes: np.ndarray) -> np.ndarray:
    """Inverse of bit_planes."""
    out = np.zeros(planes.shape[1:], dtype=np.uint8)
    for j in range(planes.shape[0]):
        out |= (planes[j].astype(np.uint8) & 1) << j
    return out


def bits_per_weight(q: int, G: int, uniform: bool = False) -> float:
    """Average bits per weight with fp16 scales and zero (Table 1 caption).

    HLQ stores q one-bit planes plus q scales and one zero per group of G weights;
    uniform quantisation stores one scale and one zero."""
    n_meta = 2 if uniform else q + 1
    return q + 16.0 * n_meta / G


def packed_bytes(K: int, N: int, q: int, G: int) -> int:
    """Bytes of an HLQ weight: K*N*q/8 for the planes + 2*(q+1)*(K/G)*N for fp16 s, z."""
    assert K % G == 0 and (K * N * q) % 8 == 0
    return K * N * q // 8 + 2 * (q + 1) * (K // G) * N


def dequantize(codes, scales, zeros, q: int, G: int) -> np.ndarray:
    """W^[k, n] = sum_j s_j[k//G, n] * b_j[k, n] + z[k//G, n]  in fp64 (Eq. 3 / Eq. 6)."""
    K, N = codes.shape
    assert scales.shape == (q, K // G, N) and zeros.shape == (K // G, N)
    planes = bit_planes(codes, q)
    W = np.repeat(zeros.astype(np.float64), G, axis=0)
    for j in range(q):
        W += np.repeat(scales[j].astype(np.float64), G, axis=0) * planes[j]
    return W


# ------------------------------------------------------------------------ reference
def gemm_dequant(X, codes, scales, zeros, q: int, G: int, cols=None) -> np.ndarray:
    """Y = X @ W^ in fp64: the definition the LUT method must reproduce.

    `cols` restricts the result to the listed output columns."""
    if cols is not None:
        cols = np.asarray(cols)
        codes, scales, zeros = codes[:, cols], scales[:, :, cols], zeros[:, cols]
    W = dequantize(codes, scales, zeros, q, G)
    return np.asarray(X).astype(np.float64) @ W


def gemm_naive(X, codes, scales, zeros, q: int, G: int) -> np.ndarray:
    """Same definition as an explicit triple loop, k ascending (small inputs only)."""
    M, K = X.shape
    N = codes.shape[1]
    Y = np.zeros((M, N), dtype=np.float64)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                g = k // G
                w = float(zeros[g, n])
                for j in range(q):
                    if (int(codes[k, n]) >> j) & 1:
                        w += float(scales[j, g, n])
                acc += float(X[m, k]) * w
            Y[m, n] = acc
    return Y


def gemm_exact(X, codes, scales, zeros, q: int, G: int):
    """Exact rational evaluation of sum_k x_k (sum_j s_j b_j + z); tiny inputs only.

    fp16 values are dyadic rationals, so Fraction arithmetic carries no rounding."""
    M, K = X.shape
    N = codes.shape[1]
    Y = [[Fraction(0)] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                g = k // G
                w = Fraction(float(zeros[g, n]))
                for j in range(q):
                    if (int(codes[k, n]) >> j) & 1:
                        w += Fraction(float(scales[j, g, n]))
                acc += Fraction(float(X[m, k])) * w
            Y[m][n] = acc
    return Y


# ------------------------------------------------------------------ the LUT algorithm
def build_tables(x_row: np.ndarray) -> np.ndarray:
    """T[t, i] = sum_{r<4} bit_r(i) * x[4t + r]: all 16 dot products of four
    activations with a 4-vector of single-bit weights (App. B)."""
    K = x_row.shape[0]
    assert K % LUT_GROUP == 0
    xg = x_row.astype(np.float64).reshape(K // LUT_GROUP, LUT_GROUP)
    T = np.zeros((K // LUT_GROUP, 1 << LUT_GROUP), dtype=np.float64)
    for i in range(1 << LUT_GROUP):
        for r in range(LUT_GROUP):
            if (i >> r) & 1:
                T[:, i] += xg[:, r]
    return T


def nibbles(plane: np.ndarray) -> np.ndarray:
    """idx[t, n] = sum_r plane[4t + r, n] << r : the table index of each weight nibble."""
    K, N = plane.shape
    p = plane.reshape(K // LUT_GROUP, LUT_GROUP, N).astype(np.int64)
    return p[:, 0] | (p[:, 1] << 1) | (p[:, 2] << 2) | (p[:, 3] << 3)


def gemm_lut(X, codes, scales, zeros, q: int, G: int) -> np.ndarray:
    """Bit-serial LUT GEMM in the paper's order (Sec. 2, App. B):
    split planes offline -> per row build tables -> per plane, per quant group sum the
    looked-up entries -> scale by s_j -> add z * (sum of the group's activations)."""
    M, K = X.shape
    N = codes.shape[1]
    assert G % LUT_GROUP == 0 and K % G == 0
    planes = bit_planes(codes, q)
    idx = [nibbles(planes[j]) for j in range(q)]          # offline step
    tpg = G // LUT_GROUP                                   # tables per quant group
    Y = np.zeros((M, N), dtype=np.float64)
    for m in range(M):
        T = build_tables(X[m])
        xsum = X[m].astype(np.float64).reshape(K // G, G).sum(axis=1)
        for g in range(K // G):
            for j in range(q):
                p = np.zeros(N, dtype=np.float64)
                for t in range(g * tpg, (g + 1) * tpg):
                    p += T[t, idx[j][t]]                   # lookup + add, no multiply
                Y[m] += scales[j, g].astype(np.float64) * p
            Y[m] += zeros[g].astype(np.float64) * xsum[g]
    return Y


def mirror_params(scales, zeros):
    """+-1 re-parametrisation (App. D, Mirror Storage): s^_j = s_j / 2,
    z^ = z + (1/2) sum_j s_j, with b^_j = 2 b_j - 1.  fp64, never rounded back."""
    s_hat = scales.astype(np.float64) / 2.0
    z_hat = zeros.astype(np.float64) + s_hat.sum(axis=0)
    return s_hat, z_hat


def build_tables_mirror(x_row: np.ndarray) -> np.ndarray:
    """Half table of the +-1 form: entry i < 8 is sum_r (+-)x[4t + r] with sign + where
    bit r of i is set, and the fourth activation always taken with sign -.  The entry for
    index i >= 8 is minus the entry for 15 - i (antisymmetry), so it is not stored."""
    K = x_row.shape[0]
    xg = x_row.astype(np.float64).reshape(K // LUT_GROUP, LUT_GROUP)
    T = np.zeros((K // LUT_GROUP, 8), dtype=np.float64)
    for i in range(8):
        for r in range(LUT_GROUP):
            sign = 1.0 if (i >> r) & 1 else -1.0
            T[:, i] += sign * xg[:, r]
    return T


def gemm_lut_mirror(X, codes, scales, zeros, q: int, G: int) -> np.ndarray:
    """Bit-serial LUT GEMM in the +-1 form with 8 stored entries per table (App. D)."""
    M, K = X.shape
    N = codes.shape[1]
    planes = bit_planes(codes, q)
    idx = [nibbles(planes[j]) for j in range(q)]
    s_hat, z_hat = mirror_params(scales, zeros)
    tpg = G // LUT_GROUP
    Y = np.zeros((M, N), dtype=np.float64)
    for m in range(M):
        T = build_tables_mirror(X[m])
        xsum = X[m].astype(np.float64).reshape(K // G, G).sum(axis=1)
        for g in range(K // G):
            for j in range(q):
                p = np.zeros(N, dtype=np.float64)
                for t in range(g * tpg, (g + 1) * tpg):
                    i = idx[j][t]
                    hi = i >= 8
                    v = T[t, np.where(hi, 15 - i, i)]      # stored half
                    p += np.where(hi, -v, v)               # other half by negation
                Y[m] += s_hat[j, g] * p
            Y[m] += z_hat[g] * xsum[g]
    return Y


def quantise_tables(T: np.ndarray, entry: str) -> np.ndarray:
    """Lossy table storage (App. D, Table Quantization).  T [tables, 16] fp64 -> the values a lookup
    returns when entries are stored as
      "fp16": IEEE binary16, round to nearest even (the paper's NEON tables);
      "int8": one scale per table, max|entry| / 127, entries rounded to the nearest integer in
              [-127, 127] (the paper only says "mapping FP16 table values to int8"; a scale per
              16-entry table is the finest choice, so this is the smallest error the option can have)."""
    if entry == "fp16":
        return T.astype(np.float16).astype(np.float64)
    if entry == "int8":
        scale = np.abs(T).max(axis=1, keepdims=True) / 127.0
        safe = np.where(scale > 0, scale, 1.0)
        return np.clip(np.rint(T / safe), -127, 127) * scale
    raise ValueError(entry)


def gemm_lut_lossy_tables(X, codes, scales, zeros, q: int, G: int, entry: str) -> np.ndarray:
    """gemm_lut with quantised table entries; everything else (accumulation, scales, zero term with the
    exact activation sums) as in gemm_lut, so the difference to it is the table precision alone."""
    M, K = X.shape
    N = codes.shape[1]
    planes = bit_planes(codes, q)
    idx = [nibbles(planes[j]) for j in range(q)]
    tpg = G // LUT_GROUP
    Y = np.zeros((M, N), dtype=np.float64)
    for m in range(M):
        T = quantise_tables(build_tables(X[m]), entry)
        xsum = X[m].astype(np.float64).reshape(K // G, G).sum(axis=1)
        for g in range(K // G):
            for j in range(q):
                p = np.zeros(N, dtype=np.float64)
                for t in range(g * tpg, (g + 1) * tpg):
                    p += T[t, idx[j][t]]
                Y[m] += scales[j, g].astype(np.float64) * p
            Y[m] += zeros[g].astype(np.float64) * xsum[g]
    return Y


# ------------------------------------------------------------------------- criterion
def row_rel_err(Y, Y_ref) -> np.ndarray:
    """Per row m: max_n |Y - Y_ref| / max_n |Y_ref|  (the parity criterion)."""
    Y = np.asarray(Y, dtype=np.float64)
    Y_ref = np.asarray(Y_ref, dtype=np.float64)
    num = np.abs(Y - Y_ref).max(axis=1)
    den = np.abs(Y_ref).max(axis=1)
    den = np.where(den == 0.0, 1.0, den)
    return num / den
