"""CPU oracle for the HLQ quantizer (Alg. 1 in Sec. 4.1; Sec. 4.2 "Weight Error Reduction via Hierarchical Linear
Quantization").  TEST INFRASTRUCTURE ONLY: only tests and the smoke check may import this module;
it shares no code with the HIP library.

The method is a heuristic iteration, so the oracle takes the algorithm's steps in the paper's
order and notation, in fp64:

    reshape W[K, N] into groups of G consecutive k per column           (Alg. 1 step 1)
    Delta = (max - min) / (2^q - 1); s = [Delta, 2 Delta, ...]; z = min  (steps 2-3)
    C = all 2^q binary combinations, C[c, j] = bit j of c                (step 4)
    repeat T_max times:
        W^ = W~ - z;  V = s C^T;  c* = argmin_c |W^ - V_c|;  B = C[c*]   (steps 6-9, Bit-Pattern Selection)
        (s, z) = LSE(W~, B)                                              (step 10, Linear Reconstruction / LSE)

Plane j of the result is bit j of the code and belongs to s_j (initially 2^j Delta), the same
convention hlq_pack uses.  Readings where the paper is silent:
  - ties in the argmin go to the smallest code (numpy's argmin, first minimum);
  - the least-squares system [B 1] can be rank deficient (a plane constant over the group, two
    planes equal or complementary, all weights equal).  Columns are taken in the order
    1, b_0, b_1, ...; a column that is linearly dependent on the ones before it (decided exactly, on
    the integer Gram matrix) keeps its previous parameter, whose contribution is moved to the
    right-hand side; the remaining columns are solved by ordinary least squares;
  - the result is (B^(T), s^(T), z^(T)) exactly as the loop leaves them (the codes were chosen
    against s^(T-1), z^(T-1)); scales and zeros are rounded to fp16 only when stored.

Pins (tests/test_oracle_quantize.py): the first bit-pattern selection equals textbook uniform
round-to-nearest; the objective never increases (each half-step is a minimisation); the LSE step
equals numpy.linalg.lstsq on full-rank groups and the two-cluster means for q = 1; brute force
over all bit assignments on tiny groups bounds it from below; on Gaussian weights the final error
is well below round-to-nearest (the qualitative claim of the weight-distribution / MSE figure of Sec. 3); degenerate groups.
"""
from __future__ import annotations

import numpy as np


def combinations(q: int) -> np.ndarray:
    """C[c, j] = bit j of c (Alg. 1 step 4)."""
    c = np.arange(1 << q)
    return np.stack([(c >> j) & 1 for j in range(q)], axis=1).astype(np.float64)


def to_groups(W: np.ndarray, G: int) -> np.ndarray:
    """W[K, N] -> W~[(K/G) * N, G]: group (g, n) holds W[g*G : (g+1)*G, n]; row index g * N + n."""
    K, N = W.shape
    assert K % G == 0
    return np.ascontiguousarray(W.reshape(K // G, G, N).transpose(0, 2, 1).reshape(-1, G)).astype(np.float64)


def from_groups_codes(codes_g: np.ndarray, K: int, N: int, G: int) -> np.ndarray:
    return np.ascontiguousarray(codes_g.reshape(K // G, N, G).transpose(0, 2, 1).reshape(K, N)).astype(np.uint8)


def init_params(Wg: np.ndarray, q: int):
    """Alg. 1 steps 2-3: uniform grid over [min, max] of each group."""
    lo, hi = Wg.min(axis=1), Wg.max(axis=1)
    delta = (hi - lo) / float((1 << q) - 1)
    s = delta[:, None] * (2.0 ** np.arange(q))[None, :]
    return s, lo.copy()


def select_bits(Wg: np.ndarray, s: np.ndarray, z: np.ndarray, q: int) -> np.ndarray:
    """Bit-pattern selection (Sec. 4.2, Bit-Pattern Selection; Eq. 5): per weight the combination whose value is nearest."""
    C = combinations(q)
    V = s @ C.T                                          # [groups, 2^q]
    What = Wg - z[:, None]
    dist = np.abs(What[:, :, None] - V[:, None, :])      # [groups, G, 2^q]
    return np.argmin(dist, axis=2).astype(np.int64)      # first minimum on ties


def _det_int(M):
    """Exact determinant of a small integer matrix (fraction-free elimination)."""
    M = [[int(v) for v in row] for row in M]
    n = len(M)
    if n == 0:
        return 1
    prev, sign = 1, 1
    for k in range(n - 1):
        if M[k][k] == 0:
            swap = next((i for i in range(k + 1, n) if M[i][k] != 0), None)
            if swap is None:
                return 0
            M[k], M[swap] = M[swap], M[k]
            sign = -sign
        for i in range(k + 1, n):
            for j in range(k + 1, n):
                M[i][j] = (M[i][j] * M[k][k] - M[i][k] * M[k][j]) // prev
        prev = M[k][k]
    return sign * M[n - 1][n - 1]


def independent_columns(A_int: np.ndarray):
    """Greedy maximal independent subset of the columns of the 0/1 matrix A, in column order,
    decided exactly on the integer Gram matrix."""
    gram = A_int.T.astype(np.int64) @ A_int.astype(np.int64)
    active = []
    for col in range(A_int.shape[1]):
        idx = active + [col]
        if _det_int(gram[np.ix_(idx, idx)]) != 0:
            active.append(col)
    return active


def lse(Wg: np.ndarray, codes_g: np.ndarray, s_prev: np.ndarray, z_prev: np.ndarray, q: int):
    """Linear reconstruction (Sec. 4.2, Linear Reconstruction: the LSE step): least squares for (z, s_0, ..., s_{q-1}) given the bits, group by
    group.  Unknowns of dependent columns keep their previous values (see the module header)."""
    ng, G = Wg.shape
    s, z = s_prev.copy(), z_prev.copy()
    for g in range(ng):
        bits = np.stack([(codes_g[g] >> j) & 1 for j in range(q)], axis=1)
        A = np.concatenate([np.ones((G, 1), dtype=np.int64), bits.astype(np.int64)], axis=1)   # columns 1, b_0..
        theta_prev = np.concatenate([[z_prev[g]], s_prev[g]])
        active = independent_columns(A)
        fixed = [c for c in range(q + 1) if c not in active]
        rhs = Wg[g] - A[:, fixed].astype(np.float64) @ theta_prev[fixed]
        sol, *_ = np.linalg.lstsq(A[:, active].astype(np.float64), rhs, rcond=None)
        theta = theta_prev.copy()
        theta[active] = sol
        z[g], s[g] = theta[0], theta[1:]
    return s, z


def objective(Wg: np.ndarray, codes_g: np.ndarray, s: np.ndarray, z: np.ndarray, q: int) -> np.ndarray:
    """Squared reconstruction error per group (Eq. 7)."""
    bits = np.stack([(codes_g >> j) & 1 for j in range(q)], axis=2).astype(np.float64)   # [groups, G, q]
    What = np.einsum("ngj,nj->ng", bits, s) + z[:, None]
    return ((Wg - What) ** 2).sum(axis=1)


def quantize(W: np.ndarray, q: int, G: int, t_max: int = 10, history: bool = False):
    """Alg. 1 on W[K, N].  Returns codes u8 [K, N], scales f64 [q, K/G, N], zeros f64 [K/G, N]
    (and, with history=True, the objective after every half-step: [2 * t_max, groups])."""
    K, N = W.shape
    Wg = to_groups(np.asarray(W, dtype=np.float64), G)
    s, z = init_params(Wg, q)
    codes_g = np.zeros(Wg.shape, dtype=np.int64)
    hist = []
    for _ in range(t_max):
        codes_g = select_bits(Wg, s, z, q)
        if history:
            hist.append(objective(Wg, codes_g, s, z, q))
        s, z = lse(Wg, codes_g, s, z, q)
        if history:
            hist.append(objective(Wg, codes_g, s, z, q))
    codes = from_groups_codes(codes_g, K, N, G)
    S = np.ascontiguousarray(s.reshape(K // G, N, q).transpose(2, 0, 1))
    Z = z.reshape(K // G, N)
    if history:
        return codes, S, Z, np.array(hist)
    return codes, S, Z


def rtn_uniform(W: np.ndarray, q: int, G: int):
    """Textbook asymmetric round-to-nearest on a uniform grid (the comparison quantizer of the MSE figure of Sec. 3):
    code = clip(round((w - min) / Delta)), W^ = Delta * code + min.  Independent of the functions above."""
    K, N = W.shape
    Wg = np.asarray(W, dtype=np.float64).reshape(K // G, G, N)
    lo, hi = Wg.min(axis=1, keepdims=True), Wg.max(axis=1, keepdims=True)
    delta = (hi - lo) / float((1 << q) - 1)
    safe = np.where(delta > 0, delta, 1.0)
    codes = np.clip(np.floor((Wg - lo) / safe + 0.5), 0, (1 << q) - 1)
    What = codes * delta + lo
    return codes.reshape(K, N).astype(np.uint8), What.reshape(K, N)


def reconstruct(codes: np.ndarray, S: np.ndarray, Z: np.ndarray, q: int, G: int) -> np.ndarray:
    """W^[k, n] = sum_j S[j, k/G, n] * bit_j(codes[k, n]) + Z[k/G, n]   (Eq. 3)."""
    K, N = codes.shape
    g = np.arange(K) // G
    out = np.asarray(Z, dtype=np.float64)[g, :].copy()
    for j in range(q):
        out += np.asarray(S[j], dtype=np.float64)[g, :] * ((codes >> j) & 1)
    return out
