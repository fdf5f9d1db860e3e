"""Grouped launches and every launch shape of the GEMV kernel against the oracle."""
import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, gemv_gpu, pack_on_gpu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture(autouse=True)
def auto_plan():
    yield
    B.set_gemv_plan(0, 0, 0)


@pytest.mark.parametrize("tn,w,cpw", [(1, 1, 1), (1, 2, 3), (1, 4, 1), (1, 8, 2), (1, 16, 1), (2, 4, 2),
                                      (2, 8, 1), (2, 16, 3), (2, 1, 64), (1, 4, 64)])
@pytest.mark.parametrize("q,G", [(2, 128), (3, 128), (1, 64), (2, 256), (4, 32)])
def test_gemv_every_launch_shape(tn, w, cpw, q, G, gemv_path):
    K, N = 2304, 1096            # 18 chunks, 17 full tiles + a 8-column tail
    say("plan", tn, w, cpw, "q", q, "G", G)
    B.set_gemv_plan(tn, w, cpw)
    codes, S, Z = synth.make_weight(K, N, q, G, "plans")
    x = synth.make_x(1, K, "plans", outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(x, codes, S, Z, q, G)
    y = gemv_gpu(d, packed, x[0], out_f32=True)
    assert O.row_rel_err(y, ref).max() <= gemv_path
    y2 = gemv_gpu(d, packed, x[0], out_f32=True)
    assert np.array_equal(y, y2)          # split-K order is fixed


def test_bad_plan_rejected():
    for args in [(3, 0, 0), (0, 17, 0), (-1, 0, 0), (0, 0, -2)]:
        with pytest.raises(B.HlqError):
            B.set_gemv_plan(*args)


@pytest.mark.parametrize("q", [2, 3])
def test_batch_equals_single_calls_and_oracle(q, gemv_path):
    G = 128
    shapes = [synth.Shape("a", 1024, 520), synth.Shape("b", 512, 64), synth.Shape("c", 2048, 1032),
              synth.Shape("d", 1024, 8)]
    descs, packs, xs, ys, refs = [], [], [], [], []
    for s in shapes:
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "batch", s.name)
        x = synth.make_x(1, s.K, "batch", s.name)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d); packs.append(p); xs.append(dev(x[0]))
        ys.append(torch.full((s.N,), 7.0, dtype=torch.float32, device="cuda"))
        refs.append(O.gemm_dequant(x, codes, S, Z, q, G))
    batch = B.GemvBatch(descs, packs, xs, ys, out_f32=True)
    for rep in range(2):                     # the workspace is reusable as is
        batch.launch()
        torch.cuda.synchronize()
        for s, y, ref in zip(shapes, ys, refs):
            got = y.cpu().numpy().astype(np.float64)[None, :]
            assert O.row_rel_err(got, ref).max() <= gemv_path, s.name


def test_batch_argument_errors():
    import ctypes
    d = B.make_desc(256, 64, 2, 128)
    d3 = B.make_desc(256, 64, 3, 128)
    arr = (B.HlqDesc * 2)(d, d3)
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    assert B.lib.hlq_lut_gemv_batch(2, arr, ptrs, ptrs, ptrs, 0, 0x1000, 1 << 30, None) == 3   # mixed q
    assert B.lib.hlq_lut_gemv_batch(0, arr, ptrs, ptrs, ptrs, 0, 0x1000, 1 << 30, None) == 3
    assert B.lib.hlq_lut_gemv_batch(9, arr, ptrs, ptrs, ptrs, 0, 0x1000, 1 << 30, None) == 3
    arr2 = (B.HlqDesc * 2)(d, d)
    assert B.lib.hlq_lut_gemv_batch(2, arr2, ptrs, ptrs, ptrs, 0, 0x1000, 16, None) == 4
    assert B.lib.hlq_lut_gemv_batch(2, arr2, None, ptrs, ptrs, 0, 0x1000, 1 << 30, None) == 1


def test_one_workspace_serves_different_shapes():
    q, G = 2, 128
    big = B.make_desc(4096, 4096, q, G)
    ws = B.alloc_workspace(big, 1)
    for (K, N) in [(4096, 4096), (512, 72), (2048, 1032), (4096, 4096)]:
        codes, S, Z = synth.make_weight(K, N, q, G, "ws", K, N)
        x = synth.make_x(1, K, "ws", K, N)
        d, packed = pack_on_gpu(codes, S, Z, q, G)
        y = B.hlq_lut_gemv(d, packed, dev(x[0]), out_f32=True, ws=ws)
        torch.cuda.synchronize()
        ref = c_oracle.gemm_f64(x, codes, S, Z, q, G)
        assert O.row_rel_err(y.cpu().numpy().astype(np.float64)[None, :], ref).max() <= 2e-4   # default path


@pytest.mark.parametrize("M,q,G", [(2, 4, 128), (4, 2, 128), (8, 4, 128), (3, 3, 64), (2, 2, 32), (16, 2, 128), (5, 2, 64),
                                   (3, 2, 128), (5, 3, 128), (6, 1, 256), (7, 4, 128), (4, 2, 64),   # every row count of the few-rows kernel
                                   (40, 3, 128), (130, 2, 128), (200, 4, 64), (257, 1, 32), (70, 2, 256)])
def test_gemm_batch_equals_single_calls_and_oracle(M, q, G):
    # M within one pass of the few-rows kernel -> one grouped launch of the GEMV kernel; beyond it one
    # grouped launch of the tiled kernel (all three row-tile heights, a ragged last row block): the
    # results must be the same as with single calls
    # the narrowest problem is 8 columns wide for the few-rows kernel (exact products); for the tiled kernel
    # (weights rounded to fp16) it is 72 wide: the row-wise bar divides by the largest of a row's
    # outputs, and with 8 outputs and outlier activations that maximum is too small a yardstick
    shapes = [synth.Shape("a", 1024, 520), synth.Shape("b", 512, 64), synth.Shape("c", 4096, 200),
              synth.Shape("d", 1024, 8 if M <= 16 else 72)]
    descs, packs, Xs, Ys, refs, singles = [], [], [], [], [], []
    for s in shapes:
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "gbatch", s.name)
        X = synth.make_x(M, s.K, "gbatch", s.name, outliers=True)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d); packs.append(p); Xs.append(dev(X))
        Ys.append(torch.full((M, s.N), 7.0, dtype=torch.float32, device="cuda"))
        refs.append(c_oracle.gemm_f64(X, codes, S, Z, q, G))
        singles.append(B.hlq_lut_gemm(d, p, Xs[-1], out_f32=True))
    batch = B.GemmBatch(descs, packs, Xs, Ys, out_f32=True)
    for rep in range(2):                     # the workspace is reusable as is
        batch.launch()
        torch.cuda.synchronize()
        for s, Y, ref, one in zip(shapes, Ys, refs, singles):
            got = Y.cpu().numpy().astype(np.float64)
            # the bar of the fp16-rebuild kernels that serve M > 8 (weights rounded to fp16; the
            # 8-column problem normalises by the maximum over only 8 outputs)
            assert O.row_rel_err(got, ref).max() <= TOL, s.name
            assert O.row_rel_err(got, one.cpu().numpy().astype(np.float64)).max() <= TOL, s.name


def test_gemm_batch_argument_errors():
    import ctypes
    d = B.make_desc(256, 64, 2, 128)
    d3 = B.make_desc(256, 64, 3, 128)
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    ld_ok = (ctypes.c_int64 * 2)(256, 256)
    ldy_ok = (ctypes.c_int64 * 2)(64, 64)
    ld_bad = (ctypes.c_int64 * 2)(256, 100)
    ld_odd = (ctypes.c_int64 * 2)(260, 260)
    mixed = (B.HlqDesc * 2)(d, d3)
    same = (B.HlqDesc * 2)(d, d)
    f = B.lib.hlq_lut_gemm_batch
    assert f(2, mixed, ptrs, ptrs, 2, ld_ok, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 3      # mixed q
    assert f(0, same, ptrs, ptrs, 2, ld_ok, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 3
    assert f(9, same, ptrs, ptrs, 2, ld_ok, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 3
    assert f(2, same, ptrs, ptrs, 2, ld_bad, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 5     # ldx < K
    assert f(2, same, ptrs, ptrs, 2, ld_odd, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 5     # ldx % 8
    assert f(2, same, ptrs, ptrs, 2, ld_ok, ptrs, ldy_ok, 0, 0x1000, 16, None) == 4           # workspace
    assert f(2, same, None, ptrs, 2, ld_ok, ptrs, ldy_ok, 0, 0x1000, 1 << 30, None) == 1
    assert f(2, same, ptrs, ptrs, 0, ld_ok, ptrs, ldy_ok, 0, 0x1000, 16, None) == 0           # M = 0: no-op
