"""hlq_quantize (Alg. 1 on the GPU) against the fp64 oracle: codes bit for bit, parameters to fp16
rounding, and the chain quantize -> pack -> GEMV."""
import numpy as np
import pytest
import torch

from oracle import hlq_oracle as O
from oracle import hlq_quantize_oracle as QO
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, gemv_gpu

pytestmark = pytest.mark.gpu


def half_ulps(a16: np.ndarray, b16: np.ndarray) -> np.ndarray:
    """distance in fp16 units in the last place between two fp16 arrays (sign-magnitude order)"""
    def key(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a16) - key(b16))


def run_gpu(W, q, G, t_max, with_err=False):
    d = B.make_desc(W.shape[0], W.shape[1], q, G)
    out = B.hlq_quantize(d, dev(W), t_max, with_err=with_err)
    torch.cuda.synchronize()
    return d, [t.cpu().numpy() for t in out]


@pytest.mark.parametrize("q,G", [(1, 128), (2, 128), (3, 128), (4, 128), (2, 32), (3, 64), (2, 256), (4, 32)])
def test_quantize_equals_oracle(q, G):
    K, N, T = 512, 72, 10           # N is not a multiple of the 64-lane wavefront
    print("quantize", q, G, flush=True)
    W = synth.make_dense_weight(K, N, "quant", q, G)
    codes_ref, S_ref, Z_ref = QO.quantize(W.astype(np.float64), q, G, t_max=T)
    d, (codes, S, Z, err) = run_gpu(W, q, G, T, with_err=True)
    # the argmin is taken in fp64 on both sides: the codes agree except at exact ties, which random
    # data does not produce
    assert np.array_equal(codes, codes_ref)
    # parameters: the same least-squares problem solved by elimination here and by lstsq there, then
    # rounded to fp16: equal up to one unit in the last place in rare boundary cases
    for got, ref in ((S, S_ref), (Z, Z_ref)):
        u = half_ulps(got.view(np.float16) if got.dtype != np.float16 else got, ref.astype(np.float16))
        assert u.max() <= 1
        assert (u != 0).mean() <= 1e-3
    # per-group error (Eq. 7) with the unrounded parameters
    err_ref = ((QO.reconstruct(codes_ref, S_ref, Z_ref, q, G) - W.astype(np.float64)) ** 2).reshape(K // G, G, N).sum(axis=1)
    assert np.allclose(err, err_ref, rtol=1e-5, atol=1e-12)


@pytest.mark.parametrize("t_max", [1, 2, 3])
def test_iteration_count_is_honoured(t_max):
    q, G = 2, 128
    W = synth.make_dense_weight(256, 64, "tmax")
    codes_ref, S_ref, Z_ref = QO.quantize(W.astype(np.float64), q, G, t_max=t_max)
    _, (codes, S, Z) = run_gpu(W, q, G, t_max)
    assert np.array_equal(codes, codes_ref)
    assert half_ulps(S, S_ref.astype(np.float16)).max() <= 1 and half_ulps(Z, Z_ref.astype(np.float16)).max() <= 1
    if t_max == 1:   # the first selection is uniform round-to-nearest (Alg. 1 steps 2-3, 6-9)
        assert np.array_equal(codes, QO.rtn_uniform(W.astype(np.float64), q, G)[0])


def test_degenerate_groups_follow_the_rank_rule():
    q, G = 2, 32
    W = np.zeros((128, 8), dtype=np.float32)
    W[:32, 0] = 0.5                                                  # constant group
    W[32:64, 0] = np.where(np.arange(32) % 2 == 0, -1.0, 1.0)        # two values
    W[64:, 0] = np.linspace(-1, 1, 64)
    W[:, 1] = np.linspace(-1, 1, 128)                                # exactly uniform data
    W[:, 2:] = synth.make_dense_weight(128, 6, "deg")
    W[:32, 3] = np.repeat(np.array([0.1, 0.2, 0.3], dtype=np.float32), [10, 10, 12])   # three values
    codes_ref, S_ref, Z_ref = QO.quantize(W.astype(np.float64), q, G, t_max=10)
    _, (codes, S, Z) = run_gpu(W, q, G, 10)
    assert np.array_equal(codes, codes_ref)
    assert np.all(np.isfinite(S.astype(np.float32))) and np.all(np.isfinite(Z.astype(np.float32)))
    assert half_ulps(S, S_ref.astype(np.float16)).max() <= 1 and half_ulps(Z, Z_ref.astype(np.float16)).max() <= 1


@pytest.mark.parametrize("q,G", [(1, 32), (3, 32), (4, 32), (3, 128), (4, 128), (4, 256)])
def test_groups_with_few_distinct_values(q, G):
    # groups holding only 1..6 distinct values leave most codes unused, so the least-squares system
    # is rank deficient in many different ways (constant planes, equal planes, complementary planes)
    K, N = max(2 * G, 128), 48
    rng = np.random.default_rng(1000 * q + G)
    W = np.empty((K, N), dtype=np.float32)
    for n in range(N):
        for g in range(K // G):
            nd = 1 + (n + g) % 6
            vals = (rng.standard_normal(nd) * 0.02).astype(np.float32)
            W[g * G:(g + 1) * G, n] = vals[rng.integers(0, nd, G)]
    codes_ref, S_ref, Z_ref = QO.quantize(W.astype(np.float64), q, G, t_max=10)
    _, (codes, S, Z, err) = run_gpu(W, q, G, 10, with_err=True)
    assert np.all(np.isfinite(S.astype(np.float32))) and np.all(np.isfinite(Z.astype(np.float32)))
    assert np.array_equal(codes, codes_ref)
    assert half_ulps(S, S_ref.astype(np.float16)).max() <= 1 and half_ulps(Z, Z_ref.astype(np.float16)).max() <= 1
    err_ref = ((QO.reconstruct(codes_ref, S_ref, Z_ref, q, G) - W.astype(np.float64)) ** 2).reshape(K // G, G, N).sum(axis=1)
    assert np.allclose(err, err_ref, rtol=1e-5, atol=1e-12)


def test_beats_round_to_nearest_at_size():
    # a whole 8B-shaped projection matrix: properties that hold at any size (the claim of the MSE figure of Sec. 3; never
    # worse than the uniform grid it starts from), plus sampled groups against the oracle
    q, G, K, N = 2, 128, 4096, 1024
    W = synth.make_dense_weight(K, N, "big")
    d, (codes, S, Z, err) = run_gpu(W, q, G, 10, with_err=True)
    Wd = W.astype(np.float64)
    rec = QO.reconstruct(codes, S.astype(np.float64), Z.astype(np.float64), q, G)
    _, rtn = QO.rtn_uniform(Wd, q, G)
    e_rtn = ((rtn - Wd) ** 2).reshape(K // G, G, N).sum(axis=1)
    assert np.all(err <= e_rtn * (1 + 1e-5) + 1e-12)
    assert ((rec - Wd) ** 2).mean() < 0.75 * ((rtn - Wd) ** 2).mean()
    cols = synth.sample_columns(N, 12, "big")
    codes_ref, S_ref, Z_ref = QO.quantize(Wd[:, cols], q, G, t_max=10)
    assert np.array_equal(codes[:, cols], codes_ref)
    assert half_ulps(S[:, :, cols], S_ref.astype(np.float16)).max() <= 1


def test_quantize_pack_gemv_chain():
    # the loop W -> HLQ -> packed -> y closes: y from the GPU-quantized, GPU-packed weights equals
    # x @ W^ computed by the oracle from the oracle-quantized tensors
    q, G, K, N = 3, 128, 1024, 264
    W = synth.make_dense_weight(K, N, "chain")
    x = synth.make_x(1, K, "chain")
    d = B.make_desc(K, N, q, G)
    codes, S, Z = B.hlq_quantize(d, dev(W), 10)
    packed = B.hlq_pack(d, codes, S, Z)
    y = gemv_gpu(d, packed, x[0], out_f32=False)
    c_ref, S_ref, Z_ref = QO.quantize(W.astype(np.float64), q, G, t_max=10)
    ref = O.gemm_dequant(x, c_ref, S_ref.astype(np.float16), Z_ref.astype(np.float16), q, G)
    assert O.row_rel_err(y, ref).max() <= TOL
    # and the quantized product is close to the unquantized one (3 bits; the largest single deviation, normalised by the largest output)
    exact = x.astype(np.float64) @ W.astype(np.float64)
    assert O.row_rel_err(ref, exact).max() < 0.4


def test_argument_errors():
    import ctypes
    d = B.make_desc(256, 64, 2, 128)
    f = B.lib.hlq_quantize
    assert f(ctypes.byref(d), None, 10, 0x1000, 0x1000, 0x1000, None, None) == 1
    assert f(ctypes.byref(d), 0x1000, 0, 0x1000, 0x1000, 0x1000, None, None) == 3
    assert f(ctypes.byref(d), 0x1002, 10, 0x1000, 0x1000, 0x1000, None, None) == 5
