"""Pins for the plain-C fp64 oracle: exact rationals, the numpy oracle, special cases."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import synth


def test_half_conversion_through_one_hot():
    # one-hot x with unit scale reads back each fp16 scale exactly, incl. subnormals / extremes
    vals = np.array([0.0, 6e-8, 6.1e-5, 1.0, 0.333, 65504.0, -2.5, 1e-3], dtype=np.float16)
    K, N, G = 8, 1, 8
    for v in vals:
        S = np.full((1, 1, 1), v, dtype=np.float16)
        Z = np.zeros((1, 1), dtype=np.float16)
        codes = np.ones((K, N), dtype=np.uint8)
        X = np.zeros((1, K), dtype=np.float16)
        X[0, 3] = 1.0
        assert c_oracle.gemm_f64(X, codes, S, Z, 1, G)[0, 0] == float(v)
        X[0, 3] = v                                  # and the activation side
        S[...] = 1.0
        assert c_oracle.gemm_f64(X, codes, S, Z, 1, G)[0, 0] == float(v)


@pytest.mark.parametrize("K,N,q,G,M", [(16, 4, 2, 8, 2), (16, 3, 3, 4, 1), (8, 2, 4, 8, 2)])
def test_c_vs_exact(K, N, q, G, M):
    codes, S, Z = synth.make_weight(K, N, q, G, "c-exact")
    X = synth.make_x(M, K, "c-exact")
    exact = O.gemm_exact(X, codes, S, Z, q, G)
    Y = c_oracle.gemm_f64(X, codes, S, Z, q, G)
    for m in range(M):
        for n in range(N):
            e = exact[m][n]
            assert abs(Fraction(float(Y[m, n])) - e) <= abs(e) * Fraction(1, 10**13) + Fraction(1, 10**15)


@pytest.mark.parametrize("q,G", [(2, 128), (3, 64), (4, 32), (1, 256)])
def test_c_vs_numpy(q, G):
    K, N, M = 512, 200, 3
    codes, S, Z = synth.make_weight(K, N, q, G, "c-np")
    X = synth.make_x(M, K, "c-np", outliers=True)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    Y = c_oracle.gemm_f64(X, codes, S, Z, q, G)
    assert np.abs(Y - ref).max() <= 1e-12 * np.abs(ref).max()
    cols = synth.sample_columns(N, 17, "c-np")
    Yc = c_oracle.gemm_f64(X, codes, S, Z, q, G, cols=cols)
    assert np.array_equal(Yc, Y[:, cols])
    np.testing.assert_allclose(O.gemm_dequant(X, codes, S, Z, q, G, cols=cols), ref[:, cols], rtol=1e-13)


def test_c_uniform_special_case():
    K, N, q, G, M = 256, 24, 3, 64, 2
    codes = synth.make_codes(K, N, q, "c-uni")
    Z = synth.make_zeros(K, N, G, "c-uni")
    X = synth.make_x(M, K, "c-uni")
    delta = synth.make_scales(K, N, 1, G, "c-uni")[0].astype(np.float64)
    S = np.stack([delta * (1 << j) for j in range(q)]).astype(np.float16)
    W = np.repeat(delta, G, axis=0) * codes + np.repeat(Z.astype(np.float64), G, axis=0)
    np.testing.assert_allclose(c_oracle.gemm_f64(X, codes, S, Z, q, G), X.astype(np.float64) @ W,
                               rtol=1e-12, atol=1e-12)
