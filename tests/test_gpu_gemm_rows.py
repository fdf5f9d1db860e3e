"""The many-rows kernel (3 <= M <= 16 rows at quant groups of 128 / 256, reached through
hlq_lut_gemm_batch): every row count, every plane count, ragged tiles, surplus wavefronts, K split
across workgroups, strided X / Y, rows of very different magnitude, one-hot rows -- against the oracle."""
import numpy as np
import pytest
import torch

from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, pack_on_gpu

pytestmark = pytest.mark.gpu

F32_TOL = 2e-4     # exact bf8 x fp4 products, matrix-core accumulation keeps 13 bits below the largest product of a run


def say(*a):
    print(*a, flush=True)


@pytest.fixture(autouse=True)
def rows_kernel_for_all_row_counts():
    # by default the many-rows kernel takes 5..16 rows of large launches only; here it gets everything from 3 rows up
    B.set_gemm_path(B.GEMM_ROWS16)
    yield
    B.set_gemm_path(B.GEMM_AUTO)
    B.set_gemv_plan(0, 0, 0)


def run_batch(d, packed, X, out_f32=True, ldx=None, ldy=None):
    M, K = X.shape
    Xd = dev(X)
    if ldx is not None:
        buf = torch.zeros((M, ldx), dtype=torch.float16, device="cuda")
        buf[:, :K] = Xd
        Xd = buf[:, :K]
    dt = torch.float32 if out_f32 else torch.float16
    if ldy is not None:
        ybuf = torch.full((M, ldy), 7.0, dtype=dt, device="cuda")
        Y = ybuf[:, :d.N]
    else:
        ybuf = None
        Y = torch.full((M, d.N), 7.0, dtype=dt, device="cuda")
    B.GemmBatch([d], [packed], [Xd], [Y], out_f32=out_f32).launch()
    torch.cuda.synchronize()
    if ybuf is not None:
        assert bool((ybuf[:, d.N:] == 7.0).all()), "wrote past the row's N columns"
    return Y.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("M", list(range(3, 17)))
@pytest.mark.parametrize("q,G", [(4, 128), (2, 128), (3, 256), (1, 128)])
def test_every_row_count(M, q, G):
    K, N = 2304, 1096            # 18 chunks (several K slices), 17 full tiles + an 8-column tail: three tile groups,
    say("rows", M, "q", q, "G", G)   # the last one with surplus wavefronts
    codes, S, Z = synth.make_weight(K, N, q, G, "rows")
    X = synth.make_x(M, K, "rows", M, outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    info = B.gemv_plan_query([d], M)[0]
    Y = run_batch(d, packed, X)
    err = O.row_rel_err(Y, ref)
    say("   max row err", float(err.max()), "slices", info.slices)
    assert err.max() <= F32_TOL
    Y2 = run_batch(d, packed, X)
    assert np.array_equal(Y, Y2)          # split-K order is fixed
    Y16 = run_batch(d, packed, X, out_f32=False)
    assert O.row_rel_err(Y16, ref).max() <= TOL


@pytest.mark.parametrize("w,cpw", [(4, 1), (4, 2), (2, 3), (8, 1), (4, 6), (8, 18), (2, 64)])
@pytest.mark.parametrize("M", [4, 7, 13])
def test_forced_work_splits(M, w, cpw):
    # wavefronts per workgroup and run lengths that cut K inside the workgroup, across workgroups, or both
    K, N, q, G = 2304, 520, 3, 128
    B.set_gemv_plan(0, w, cpw)
    codes, S, Z = synth.make_weight(K, N, q, G, "rows-plan")
    X = synth.make_x(M, K, "rows-plan", M)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    info = B.gemv_plan_query([d], M)[0]
    say("rows", M, "plan", w, cpw, "slices", info.slices, "chunks/slice", info.chunks_per_slice, "waves/tile", info.waves_per_tile)
    assert O.row_rel_err(run_batch(d, packed, X), O.gemm_dequant(X, codes, S, Z, q, G)).max() <= F32_TOL


@pytest.mark.parametrize("M", [3, 6, 16])
def test_strided_rows(M):
    K, N, q, G = 1024, 200, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "rows-ld")
    X = synth.make_x(M, K, "rows-ld", M, outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    Y = run_batch(d, packed, X, ldx=K + 64, ldy=N + 24)
    assert O.row_rel_err(Y, O.gemm_dequant(X, codes, S, Z, q, G)).max() <= F32_TOL


@pytest.mark.parametrize("M", [4, 8, 12])
def test_rows_of_very_different_magnitude(M):
    # each row has a power-of-two scale of its own: a row 2^15 times smaller than its neighbour keeps its precision
    K, N, q, G = 2048, 264, 4, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "rows-mag")
    X = synth.make_x(M, K, "rows-mag", M, outliers=True).astype(np.float64)
    for m in range(M):
        X[m] *= 2.0 ** (-15 + (30 * m) // (M - 1) - 7)      # 2^-22 ... 2^8
    X = X.astype(np.float16)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    err = O.row_rel_err(run_batch(d, packed, X), O.gemm_dequant(X, codes, S, Z, q, G))
    say("   per-row errors", [float(f"{e:.2e}") for e in err])
    assert err.max() <= F32_TOL


def test_zero_rows_and_zero_chunks():
    # an all-zero row (scale taken from a zero maximum) and a row that is zero on whole chunks
    K, N, q, G, M = 1024, 136, 2, 128, 9
    codes, S, Z = synth.make_weight(K, N, q, G, "rows-zero")
    X = synth.make_x(M, K, "rows-zero")
    X[3] = 0
    X[5, 128:640] = 0
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    Y = run_batch(d, packed, X)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    assert np.all(Y[3] == 0)
    keep = [m for m in range(M) if m != 3]
    assert O.row_rel_err(Y[keep], ref[keep]).max() <= F32_TOL


@pytest.mark.parametrize("M", [3, 5, 16])
def test_one_hot_rows_read_back_weights(M):
    # X[m] = e_k(m): Y[m] = W^[k(m), :]; catches any mix-up of rows, terms, k order or scales
    K, N, q, G = 1024, 200, 3, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "rows-onehot")
    ks = [(97 * m + 5) % K for m in range(M)]
    X = np.zeros((M, K), dtype=np.float16)
    for m, k in enumerate(ks):
        X[m, k] = 1.0
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    Y = run_batch(d, packed, X)
    W = O.dequantize(codes, S, Z, q, G)
    np.testing.assert_allclose(Y, W[ks], rtol=0, atol=2e-7)


def test_grouped_launch_of_several_problems():
    q, G, M = 4, 128, 11
    shapes = [synth.Shape("a", 1024, 520), synth.Shape("b", 512, 64), synth.Shape("c", 4096, 200), synth.Shape("d", 1024, 8)]
    descs, packs, Xs, Ys, refs = [], [], [], [], []
    for s in shapes:
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "rows-group", s.name)
        X = synth.make_x(M, s.K, "rows-group", s.name, outliers=True)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d); packs.append(p); Xs.append(dev(X))
        Ys.append(torch.full((M, s.N), 7.0, dtype=torch.float32, device="cuda"))
        refs.append(O.gemm_dequant(X, codes, S, Z, q, G))
    batch = B.GemmBatch(descs, packs, Xs, Ys, out_f32=True)
    for rep in range(3):
        batch.launch()
        torch.cuda.synchronize()
        for s, Y, ref in zip(shapes, Ys, refs):
            assert O.row_rel_err(Y.cpu().numpy().astype(np.float64), ref).max() <= F32_TOL, s.name
    assert int(batch.ws[:131072].view(torch.int32).abs().sum().item()) == 0     # arrival counters are back at zero
