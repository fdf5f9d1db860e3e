"""Pins for the quantizer oracle (Alg. 1): things the paper and the mathematics fix, none of which
come from the oracle itself or from the GPU."""
import itertools

import numpy as np
import pytest

from oracle import hlq_quantize_oracle as Q
from paper_2510_19482_amd import synth


def gaussian(K, N, *key):
    return synth.make_dense_weight(K, N, *key).astype(np.float64)


@pytest.mark.parametrize("q,G", [(2, 128), (3, 64), (4, 32), (1, 128)])
def test_first_selection_is_uniform_round_to_nearest(q, G):
    # with s = [Delta, 2 Delta, ...] the candidate values are Delta * c: choosing the nearest is
    # textbook asymmetric RTN (Alg. 1 steps 2-3 and 6-9 at t = 1)
    W = gaussian(256, 24, "rtn", q, G)
    Wg = Q.to_groups(W, G)
    s, z = Q.init_params(Wg, q)
    codes = Q.from_groups_codes(Q.select_bits(Wg, s, z, q), 256, 24, G)
    ref_codes, _ = Q.rtn_uniform(W, q, G)
    assert np.array_equal(codes, ref_codes)
    # t_max = 0 leaves the uniform grid: reconstruct with it and compare values too
    _, What = Q.rtn_uniform(W, q, G)
    S0 = s.reshape(256 // G, 24, q).transpose(2, 0, 1)
    assert np.allclose(Q.reconstruct(codes, S0, z.reshape(256 // G, 24), q, G), What, rtol=0, atol=1e-15)


@pytest.mark.parametrize("q,G", [(2, 128), (3, 128), (4, 64), (1, 32)])
def test_objective_never_increases(q, G):
    # selection minimises over B with (s, z) fixed, LSE over (s, z) with B fixed (Sec. 4.2: Bit-Pattern Selection, Linear Reconstruction)
    W = gaussian(256, 16, "mono", q, G)
    _, _, _, hist = Q.quantize(W, q, G, t_max=6, history=True)
    assert hist.shape[0] == 12
    assert np.all(hist[1:] <= hist[:-1] * (1 + 1e-12) + 1e-24)


@pytest.mark.parametrize("q", [2, 3, 4])
def test_lse_equals_library_least_squares_on_full_rank_groups(q):
    G = 64
    W = gaussian(128, 8, "lse", q)
    Wg = Q.to_groups(W, G)
    s0, z0 = Q.init_params(Wg, q)
    codes_g = Q.select_bits(Wg, s0, z0, q)
    s1, z1 = Q.lse(Wg, codes_g, s0, z0, q)
    for g in range(Wg.shape[0]):
        B = np.stack([(codes_g[g] >> j) & 1 for j in range(q)], axis=1).astype(np.float64)
        A = np.concatenate([B, np.ones((G, 1))], axis=1)          # Linear Reconstruction: [B 1] [s; z]
        if np.linalg.matrix_rank(A) < q + 1:
            continue
        sol = np.linalg.lstsq(A, Wg[g], rcond=None)[0]
        assert np.allclose(s1[g], sol[:q], rtol=1e-9, atol=1e-12)
        assert np.isclose(z1[g], sol[q], rtol=1e-9, atol=1e-12)


def test_one_bit_lse_is_the_two_cluster_means():
    # q = 1: the least-squares fit of {z, z + s} to two clusters is their means
    G = 128
    W = gaussian(256, 6, "onebit")
    Wg = Q.to_groups(W, G)
    s0, z0 = Q.init_params(Wg, 1)
    codes_g = Q.select_bits(Wg, s0, z0, 1)
    s1, z1 = Q.lse(Wg, codes_g, s0, z0, 1)
    for g in range(Wg.shape[0]):
        m0 = Wg[g][codes_g[g] == 0].mean()
        m1 = Wg[g][codes_g[g] == 1].mean()
        assert np.isclose(z1[g], m0) and np.isclose(s1[g, 0], m1 - m0)


@pytest.mark.parametrize("q,G", [(1, 6), (2, 5)])
def test_brute_force_lower_bound_and_fixed_point_on_tiny_groups(q, G):
    # exhaustive search over every bit assignment of a tiny group (each followed by its exact least-squares
    # fit) gives the global optimum of Eq. 7: the alternating heuristic can only be worse or equal, and its
    # result must be a fixed point of both half-steps
    rng = np.random.default_rng(11)
    for trial in range(6):
        w = rng.normal(0, 0.02, size=G)
        best = np.inf
        for assign in itertools.product(range(1 << q), repeat=G):
            B = np.array([[(c >> j) & 1 for j in range(q)] for c in assign], dtype=np.float64)
            A = np.concatenate([B, np.ones((G, 1))], axis=1)
            sol, *_ = np.linalg.lstsq(A, w, rcond=None)
            best = min(best, float(((A @ sol - w) ** 2).sum()))
        W = w.reshape(G, 1)
        codes, S, Z, hist = Q.quantize(W, q, G, t_max=20, history=True)
        final = float(hist[-1][0])
        assert final >= best - 1e-18
        assert final <= float(hist[0][0]) + 1e-24
        Wg = Q.to_groups(W, G)
        s = S.transpose(1, 2, 0).reshape(-1, q)
        z = Z.reshape(-1)
        codes_g = Q.select_bits(Wg, s, z, q)
        s2, z2 = Q.lse(Wg, codes_g, s, z, q)
        assert float(Q.objective(Wg, codes_g, s2, z2, q)[0]) <= final + 1e-24


@pytest.mark.parametrize("q", [2, 3])
def test_beats_round_to_nearest_on_gaussian_weights(q):
    # MSE figure of Sec. 3 / Sec. 4.2: on bell-shaped weights the fitted grid has clearly lower error than the uniform one
    G = 128
    W = gaussian(512, 32, "fig3", q)
    codes, S, Z = Q.quantize(W, q, G, t_max=10)
    mse_hlq = ((Q.reconstruct(codes, S, Z, q, G) - W) ** 2).mean()
    _, What = Q.rtn_uniform(W, q, G)
    mse_rtn = ((What - W) ** 2).mean()
    assert mse_hlq < 0.75 * mse_rtn
    # and group by group it is never worse than where it started
    err_h = ((Q.reconstruct(codes, S, Z, q, G) - W) ** 2).reshape(512 // G, G, 32).sum(axis=1)
    err_r = ((What - W) ** 2).reshape(512 // G, G, 32).sum(axis=1)
    assert np.all(err_h <= err_r * (1 + 1e-12))


def test_degenerate_groups():
    q, G = 2, 32
    W = np.zeros((64, 3))
    W[:32, 0] = 0.5                                  # constant group: Delta = 0, every code 0
    W[32:, 0] = np.where(np.arange(32) % 2 == 0, -1.0, 1.0)   # two values only: planes equal / constant
    W[:, 1] = np.linspace(-1, 1, 64)                 # exactly uniform data
    W[:, 2] = gaussian(64, 1, "deg")[:, 0]
    codes, S, Z = Q.quantize(W, q, G, t_max=10)
    assert np.all(np.isfinite(S)) and np.all(np.isfinite(Z))
    rec = Q.reconstruct(codes, S, Z, q, G)
    assert np.allclose(rec[:32, 0], 0.5) and np.allclose(rec[32:, 0], W[32:, 0])
    _, What = Q.rtn_uniform(W, q, G)
    assert ((rec - W) ** 2).sum() <= ((What - W) ** 2).sum() + 1e-20


def test_independent_columns_is_exact():
    ones = np.ones(8, dtype=np.int64)
    b0 = np.array([0, 1, 0, 1, 0, 1, 0, 1])
    assert Q.independent_columns(np.stack([ones, b0, 1 - b0], axis=1)) == [0, 1]       # complementary planes
    assert Q.independent_columns(np.stack([ones, b0, b0], axis=1)) == [0, 1]           # equal planes
    assert Q.independent_columns(np.stack([ones, ones, b0], axis=1)) == [0, 2]         # constant plane
    assert Q.independent_columns(np.stack([ones, 0 * ones, b0], axis=1)) == [0, 2]
    b1 = np.array([0, 0, 1, 1, 0, 0, 1, 1])
    assert Q.independent_columns(np.stack([ones, b0, b1], axis=1)) == [0, 1, 2]
