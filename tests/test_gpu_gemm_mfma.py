"""The matrix-core formulation of hlq_lut_gemm against the oracle: row-block sizes, ragged M, N and
K slices, every (q, G), and agreement with the table-lookup formulation."""
import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, gemm_gpu, pack_on_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["matrix-core", "fp16-rebuild-only"])
def mfma_path(request):
    # "matrix-core" sends a few rows to the GEMV kernel with several activation rows per operand,
    # "fp16-rebuild-only" keeps them on the tiled fp16 kernel; larger M is the same in both
    B.set_gemm_path(B.GEMM_MFMA if request.param == "matrix-core" else B.GEMM_MFMA_FP16)
    yield
    B.set_gemm_path(B.GEMM_AUTO)


@pytest.mark.parametrize("M", [2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 64, 65, 100, 128, 200])
@pytest.mark.parametrize("q,G", [(2, 128), (3, 128), (4, 64), (1, 32), (2, 256)])
def test_mfma_vs_oracle(M, q, G):
    K, N = 1280, 584          # 10 chunks; 9 full tiles + a 8-column tail; 3 column groups
    print("mfma", M, q, G, flush=True)
    codes, S, Z = synth.make_weight(K, N, q, G, "mfma")
    X = synth.make_x(M, K, "mfma", outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = c_oracle.gemm_f64(X, codes, S, Z, q, G)
    Y = gemm_gpu(d, packed, X, out_f32=True)
    err = O.row_rel_err(Y, ref)
    assert err.max() <= 1e-3, err.max()
    Y16 = gemm_gpu(d, packed, X, out_f32=False)
    assert O.row_rel_err(Y16, ref).max() <= TOL


@pytest.mark.parametrize("M,q,G", [(4, 4, 128), (7, 2, 128), (16, 4, 128), (3, 3, 64), (8, 2, 64), (2, 2, 32), (4, 1, 32)])
def test_few_rows_strides_long_k_and_repeatability(M, q, G):
    # K long enough that it is cut across workgroups; X and Y with leading dimensions; rows of very
    # different magnitude (one common power-of-two scale serves all rows of a pass)
    K, N = 8192, 200
    codes, S, Z = synth.make_weight(K, N, q, G, "fewrows")
    X = synth.make_x(M, K, "fewrows", outliers=True).astype(np.float64)
    X[0] *= 2.0 ** -9
    if M > 2:
        X[M - 1] *= 2.0 ** 6
    X = X.astype(np.float16)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = c_oracle.gemm_f64(X, codes, S, Z, q, G)
    Xd = torch.zeros(M, K + 24, dtype=torch.float16, device="cuda")
    Xd[:, :K] = dev(X)
    Yd = torch.full((M, N + 8), 5.0, dtype=torch.float32, device="cuda")
    outs = []
    for rep in range(2):
        B.hlq_lut_gemm(d, packed, Xd[:, :K], Y=Yd[:, :N], out_f32=True)
        torch.cuda.synchronize()
        outs.append(Yd.cpu().numpy().astype(np.float64))
    assert np.array_equal(outs[0], outs[1])
    assert np.all(outs[0][:, N:] == 5.0)
    assert O.row_rel_err(outs[0][:, :N], ref).max() <= 1e-3


def test_mfma_identity_rows_read_back_weights():
    # X = rows of the identity: Y[m, :] = W^[k_m, :] rounded to fp16 -- checks the contraction order,
    # the lane exchange and the output layout entry by entry
    K, N, q, G = 256, 128, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "mfma-id")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    W = O.dequantize(codes, S, Z, q, G)
    X = np.eye(K, dtype=np.float16)
    Y = gemm_gpu(d, packed, X, out_f32=True)
    np.testing.assert_allclose(Y, W, rtol=2e-3, atol=1e-6)


@pytest.mark.parametrize("M", [3, 16, 29])
def test_few_rows_one_hot_read_back_weights(M):
    # one-hot rows, fewer than one 32-row tile: checks the lane exchange, the A-fragment addressing
    # (swizzled LDS rows, rows past M) and the output layout entry by entry
    K, N, q, G = 512, 200, 3, 64
    codes, S, Z = synth.make_weight(K, N, q, G, "one-hot-rows")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    W = O.dequantize(codes, S, Z, q, G)
    ks = (np.arange(M) * 37 + 5) % K
    X = np.zeros((M, K), dtype=np.float16)
    X[np.arange(M), ks] = 1.0
    Y = gemm_gpu(d, packed, X, out_f32=True)
    np.testing.assert_allclose(Y, W[ks], rtol=2e-3, atol=1e-6)


def test_mfma_equals_lut_path_within_tolerance():
    M, K, N, q, G = 48, 2048, 1032, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "mfma-lut")
    X = synth.make_x(M, K, "mfma-lut", outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    a = gemm_gpu(d, packed, X, out_f32=True)
    B.set_gemm_path(B.GEMM_LUT)
    b = gemm_gpu(d, packed, X, out_f32=True)
    assert O.row_rel_err(a, b).max() <= 1e-3


# ---------------------------------------------------------------------------------------------------
# Scales outside what the fp16 weight rebuild of the tiled kernel can represent (|s| >= 512: s * 2^7 is
# not finite in fp16).  Any finite fp16 scale is a valid HLQ parameter (Eq. 3); the tiled kernel notices
# such values and the fp32 kernel launched behind it computes the call again.
@pytest.mark.parametrize("M", [40, 200])
@pytest.mark.parametrize("big", [600.0, 30000.0])
def test_large_scales_take_the_fp32_fallback(M, big):
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    K, N, q, G = 1024, 328, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "bigscale")
    S = S.copy()
    S[0, 3, 17] = np.float16(big)           # one scale of one group of one column
    S[1, 5, 200] = np.float16(-big)
    X = synth.make_x(M, K, "bigscale", M)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    ws = B.alloc_workspace(d, M)
    Y = B.hlq_lut_gemm(d, packed, dev(X), out_f32=True, ws=ws)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy().astype(np.float64)
    assert np.isfinite(Y).all()
    assert O.row_rel_err(Y, ref).max() <= 2e-5          # fp32 throughout
    # the flag is down again: the same workspace serves an ordinary call on the matrix cores next
    assert int(ws[:131072].view(torch.int32).abs().sum().item()) == 0
    codes2, S2, Z2 = synth.make_weight(K, N, q, G, "bigscale-after")
    d2, packed2 = pack_on_gpu(codes2, S2, Z2, q, G)
    Y2 = B.hlq_lut_gemm(d2, packed2, dev(X), out_f32=True, ws=ws)
    torch.cuda.synchronize()
    assert O.row_rel_err(Y2.cpu().numpy().astype(np.float64), O.gemm_dequant(X, codes2, S2, Z2, q, G)).max() <= 1e-3
    assert int(ws[:131072].view(torch.int32).abs().sum().item()) == 0


def test_large_scales_in_a_grouped_launch():
    # one problem of three has an out-of-range scale: the whole grouped call is recomputed, every problem right
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    M, q, G = 70, 3, 64
    shapes = [synth.Shape("a", 512, 200), synth.Shape("b", 1024, 72), synth.Shape("c", 256, 520)]
    descs, packs, Xs, Ys, refs = [], [], [], [], []
    for i, s in enumerate(shapes):
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "bigscale-group", s.name)
        if i == 1:
            S = S.copy()
            S[2, 0, 5] = np.float16(65504.0)
            Z = Z.copy()
            Z[1, 9] = np.float16(-20000.0)
        X = synth.make_x(M, s.K, "bigscale-group", s.name)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d); packs.append(p); Xs.append(dev(X))
        Ys.append(torch.full((M, s.N), 7.0, dtype=torch.float32, device="cuda"))
        refs.append(O.gemm_dequant(X, codes, S, Z, q, G))
    batch = B.GemmBatch(descs, packs, Xs, Ys, out_f32=True)
    for rep in range(2):
        batch.launch()
        torch.cuda.synchronize()
        for s, Y, ref in zip(shapes, Ys, refs):
            assert O.row_rel_err(Y.cpu().numpy().astype(np.float64), ref).max() <= 2e-5, s.name
        assert int(batch.ws[:131072].view(torch.int32).abs().sum().item()) == 0
