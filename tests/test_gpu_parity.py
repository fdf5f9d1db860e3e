"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI."""
import sys

import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, gemm_gpu, gemv_gpu, pack_on_gpu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


# -------------------------------------------------------------------------- pack / unpack
@pytest.mark.parametrize("K,N,q,G", [(128, 8, 1, 32), (256, 264, 2, 128), (384, 1000, 3, 64),
                                     (512, 520, 4, 256), (1024, 4096, 2, 128), (128, 72, 4, 32)])
def test_pack_unpack_bit_exact(K, N, q, G):
    say("pack/unpack", K, N, q, G)
    codes, S, Z = synth.make_weight(K, N, q, G, "roundtrip")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    assert packed.numel() == O.packed_bytes(K, N, q, G)
    c2, s2, z2 = B.hlq_unpack(d, packed)
    torch.cuda.synchronize()
    assert np.array_equal(c2.cpu().numpy(), codes)
    assert np.array_equal(s2.cpu().numpy().view(np.uint16), S.view(np.uint16))
    assert np.array_equal(z2.cpu().numpy().view(np.uint16), Z.view(np.uint16))


def test_pack_is_injective_on_single_bit_flips():
    K, N, q, G = 256, 16, 3, 64
    codes, S, Z = synth.make_weight(K, N, q, G, "flip")
    d, base = pack_on_gpu(codes, S, Z, q, G)
    base = base.cpu().numpy()
    rng = np.random.default_rng(5)
    for _ in range(8):
        k, n, j = rng.integers(K), rng.integers(N), rng.integers(q)
        c2 = codes.copy()
        c2[k, n] ^= (1 << j)
        _, p2 = pack_on_gpu(c2, S, Z, q, G)
        diff = np.unpackbits(base ^ p2.cpu().numpy()).sum()
        assert diff == 1, (k, n, j, diff)


# ------------------------------------------------------------------------------- GEMV
@pytest.mark.parametrize("q", [1, 2, 3, 4])
@pytest.mark.parametrize("G", [32, 64, 128, 256])
@pytest.mark.parametrize("K,N", [(256, 8), (768, 520), (1536, 4104)])
def test_gemv_vs_oracle(K, N, q, G, gemv_path):
    say("gemv", K, N, q, G)
    codes, S, Z = synth.make_weight(K, N, q, G, "gemv")
    x = synth.make_x(1, K, "gemv", outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(x, codes, S, Z, q, G)
    for out_f32 in (True, False):
        y = gemv_gpu(d, packed, x[0], out_f32=out_f32)
        err = O.row_rel_err(y, ref)
        assert err.max() <= (gemv_path if out_f32 else TOL), (out_f32, err)


def test_gemv_one_hot_reads_back_weights(gemv_path):
    K, N, q, G = 256, 264, 3, 64
    codes, S, Z = synth.make_weight(K, N, q, G, "onehot")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    W = O.dequantize(codes, S, Z, q, G)
    for k in (0, 1, 2, 3, 4, 31, 32, 63, 64, 127, 128, 200, 255):
        x = np.zeros(K, dtype=np.float16)
        x[k] = 1.0
        y = gemv_gpu(d, packed, x, out_f32=True)[0]
        np.testing.assert_allclose(y, W[k], rtol=1e-6, atol=1e-9, err_msg=f"k={k}")


def test_gemv_degenerate_planes_and_zero_x(gemv_path):
    K, N, q, G = 512, 512, 2, 128
    _, S, Z = synth.make_weight(K, N, q, G, "degen")
    x = synth.make_x(1, K, "degen")
    for fill in (0, (1 << q) - 1):
        codes = np.full((K, N), fill, dtype=np.uint8)
        d, packed = pack_on_gpu(codes, S, Z, q, G)
        ref = O.gemm_dequant(x, codes, S, Z, q, G)
        y = gemv_gpu(d, packed, x[0], out_f32=True)
        assert O.row_rel_err(y, ref).max() <= gemv_path
    y0 = gemv_gpu(d, packed, np.zeros(K, dtype=np.float16), out_f32=True)
    assert np.all(y0 == 0.0)


def test_gemv_output_is_overwritten_and_tail_untouched(gemv_path):
    K, N, q, G = 256, 264, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "canary")
    x = synth.make_x(1, K, "canary")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    buf = torch.full((N + 64,), 777.0, dtype=torch.float16, device="cuda")
    B.hlq_lut_gemv(d, packed, dev(x[0]), y=buf[:N])
    torch.cuda.synchronize()
    out = buf.float().cpu().numpy()
    assert np.all(out[N:] == 777.0)
    ref = O.gemm_dequant(x, codes, S, Z, q, G)
    assert O.row_rel_err(out[None, :N], ref).max() <= TOL


@pytest.mark.parametrize("scale", [2.0 ** -20, 2.0 ** -12, 2.0 ** -6, 1.0, 64.0, 2048.0])
def test_gemv_any_activation_magnitude(scale, gemv_path):
    # the result must keep its relative accuracy whatever the magnitude of x (down to fp16
    # subnormals and up to values near the fp16 maximum), and when one slice of K is tiny and
    # another large
    K, N, q, G = 2048, 200, 2, 64
    codes, S, Z = synth.make_weight(K, N, q, G, "mag")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    x = (synth.make_x(1, K, "mag").astype(np.float64) * scale).astype(np.float16)
    xs = [x, x.copy()]
    xs[1][0, : K // 2] = (xs[1][0, : K // 2].astype(np.float64) * 2.0 ** -10).astype(np.float16)
    if scale == 2048.0:
        xs[0][0, 5] = np.float16(65504.0)
        xs[0][0, 6] = np.float16(-65504.0)
    for xv in xs:
        ref = O.gemm_dequant(xv, codes, S, Z, q, G)
        y = gemv_gpu(d, packed, xv[0], out_f32=True)
        assert O.row_rel_err(y, ref).max() <= max(gemv_path, 1e-4 if scale < 1e-4 else 0.0), scale


# ------------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M", [2, 3, 4, 5, 8, 16, 37])
@pytest.mark.parametrize("q,G", [(2, 128), (4, 128), (3, 64), (1, 32), (2, 256)])
def test_gemm_vs_oracle(M, q, G):
    K, N = 768, 520
    say("gemm", M, K, N, q, G)
    codes, S, Z = synth.make_weight(K, N, q, G, "gemm")
    X = synth.make_x(M, K, "gemm", outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    try:
        B.set_gemm_path(B.GEMM_LUT)           # table lookups: fp32 tables and sums
        Y = gemm_gpu(d, packed, X, out_f32=True)
        assert O.row_rel_err(Y, ref).max() <= 2e-5
        B.set_gemm_path(B.GEMM_MFMA)          # matrix cores: W^ rounded to fp16
        Y = gemm_gpu(d, packed, X, out_f32=True)
        assert O.row_rel_err(Y, ref).max() <= 1e-3
    finally:
        B.set_gemm_path(B.GEMM_AUTO)
    Y = gemm_gpu(d, packed, X, out_f32=False)
    assert O.row_rel_err(Y, ref).max() <= TOL


def test_gemm_leading_dimensions():
    M, K, N, q, G = 5, 512, 264, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "ld")
    X = synth.make_x(M, K, "ld")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    Xbig = torch.zeros((M, K + 64), dtype=torch.float16, device="cuda")
    Xbig[:, :K] = dev(X)
    Ybig = torch.full((M, N + 24), -5.0, dtype=torch.float32, device="cuda")
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    try:
        for path, tol in ((B.GEMM_LUT, 2e-5), (B.GEMM_MFMA, 1e-3)):
            B.set_gemm_path(path)
            Ybig.fill_(-5.0)
            B.hlq_lut_gemm(d, packed, Xbig[:, :K], Y=Ybig[:, :N], out_f32=True)
            torch.cuda.synchronize()
            out = Ybig.cpu().numpy().astype(np.float64)
            assert np.all(out[:, N:] == -5.0)
            assert O.row_rel_err(out[:, :N], ref).max() <= tol, path
    finally:
        B.set_gemm_path(B.GEMM_AUTO)


def test_gemm_m1_equals_gemv():
    K, N, q, G = 512, 264, 3, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "m1")
    X = synth.make_x(1, K, "m1")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    a = gemm_gpu(d, packed, X, out_f32=True)
    b = gemv_gpu(d, packed, X[0], out_f32=True)
    assert np.array_equal(a, b)


def test_gemv_is_deterministic():
    K, N, q, G = 4096, 4096, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "det")
    x = synth.make_x(1, K, "det")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    a = gemv_gpu(d, packed, x[0], out_f32=True)
    for _ in range(3):
        assert np.array_equal(a, gemv_gpu(d, packed, x[0], out_f32=True))
