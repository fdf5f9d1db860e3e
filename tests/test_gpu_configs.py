"""The five benchmark configurations at full size, HIP path vs the C oracle: every output at
M = 1 (also for the 128256-wide head); for the prefill sizes every row of whole column tiles
(first, middle, last) plus one column of EVERY 64-column tile, so that each (column group, row
block, wavefront) of a launch has outputs under test."""
import sys

import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import synth

from gpu_util import TOL, gemm_gpu, gemv_gpu, pack_on_gpu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def tile_columns(N):
    """Columns checked where the oracle cannot afford all of them: the whole first, middle and last
    64-column tile (every lane of a wavefront, the ragged tail if there is one) and one column of every
    tile, at a lane that moves with the tile (every wavefront of every workgroup of the launch)."""
    ntiles = (N + 63) // 64
    cols = set()
    for t in {0, ntiles // 2, ntiles - 1}:
        cols.update(range(64 * t, min(64 * t + 64, N)))
    for t in range(ntiles):
        w = min(64, N - 64 * t)
        cols.add(64 * t + (7 * t + 3) % w)
    return np.array(sorted(cols), dtype=np.int64)


def check(shape, q, G, M, cfg, outliers, ncols=None):
    say("config", cfg, shape.name, shape.K, shape.N, "q", q, "G", G, "M", M)
    codes, S, Z = synth.make_weight(shape.K, shape.N, q, G, cfg, shape.name)
    X = synth.make_x(M, shape.K, cfg, shape.name, outliers=outliers)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    if ncols == "tiles":
        cols = tile_columns(shape.N)
    else:
        cols = None if ncols is None else synth.sample_columns(shape.N, ncols, cfg, shape.name)
    ref = c_oracle.gemm_f64(X, codes, S, Z, q, G, cols=cols)
    Y = gemv_gpu(d, packed, X[0]) if M == 1 else gemm_gpu(d, packed, X)
    if cols is not None:
        Y = Y[:, cols]
    err = O.row_rel_err(Y, ref)
    say("   max row err", float(err.max()))
    assert err.max() <= TOL
    del packed
    torch.cuda.empty_cache()


def test_config1_single_layer_decode():
    check(synth.Shape("cfg1", 4096, 4096), 2, 128, 1, "cfg1", False)


@pytest.mark.parametrize("q", [2, 3])
@pytest.mark.parametrize("shape", synth.LLAMA31_8B_LAYER, ids=lambda s: s.name)
def test_config2_8b_layer_decode(shape, q):
    check(shape, q, 128, 1, "cfg2", False)


@pytest.mark.parametrize("M", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("shape", [synth.LLAMA31_8B_LAYER[1], synth.LLAMA31_8B_LAYER[0],
                                   synth.LLAMA31_8B_LAYER[6]], ids=lambda s: s.name)
def test_config3_small_batch(shape, M):
    check(shape, 4, 128, M, "cfg3", True)


@pytest.mark.parametrize("M", [512, 2048])
@pytest.mark.parametrize("shape", [synth.LLAMA31_8B_LAYER[0], synth.LLAMA31_8B_LAYER[1], synth.LLAMA31_8B_LAYER[4],
                                   synth.LLAMA31_8B_LAYER[6]], ids=lambda s: s.name)
def test_config4_prefill(shape, M):
    # every distinct shape of the layer as a single call, every row, whole tiles + a column of every tile
    check(shape, 2, 128, M, "cfg4", True, ncols="tiles")


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("shape", [synth.LLAMA31_70B_LAYER[0], synth.LLAMA31_70B_LAYER[1],
                                   synth.LLAMA31_70B_LAYER[4], synth.LLAMA31_70B_LAYER[6]], ids=lambda s: s.name)
def test_config5_70b_layer_decode(shape, G):
    check(shape, 2, G, 1, "cfg5", False)          # every output column


@pytest.mark.parametrize("G", [64, 128])
def test_config5_lm_head(G):
    check(synth.LLAMA31_70B_LM_HEAD, 2, G, 1, "cfg5", False)   # all 128256 outputs


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("path", ["matrix cores", "lookups"])
def test_config5_70b_whole_layer_one_grouped_launch(G, path):
    # the seven GEMVs of the 70B layer in one hlq_lut_gemv_batch call (the launch the benchmark times for
    # this configuration), both formulations, every output against the C oracle
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    q = 2
    shapes = synth.LLAMA31_70B_LAYER
    descs, packs, xs, ys, refs = [], [], [], [], []
    for s in shapes:
        say("config cfg5 grouped", path, s.name, s.K, s.N, "G", G)
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "cfg5g", s.name)
        X = synth.make_x(1, s.K, "cfg5g", s.name)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        refs.append(c_oracle.gemm_f64(X, codes, S, Z, q, G))
        descs.append(d); packs.append(p); xs.append(dev(X[0]))
        ys.append(torch.empty(s.N, dtype=torch.float16, device="cuda"))
        del codes, S, Z
    B.set_gemv_path(B.GEMV_LUT if path == "lookups" else B.GEMV_MX)
    try:
        B.GemvBatch(descs, packs, xs, ys).launch()
        torch.cuda.synchronize()
    finally:
        B.set_gemv_path(B.GEMV_AUTO)
    for s, y, ref in zip(shapes, ys, refs):
        err = O.row_rel_err(y.float().cpu().numpy().astype(np.float64)[None, :], ref)
        say("   ", s.name, "max row err", float(err.max()))
        assert err.max() <= TOL, s.name
    del packs, xs, ys
    torch.cuda.empty_cache()


@pytest.mark.parametrize("shape", [synth.Shape("qkv_fused", 4096, 6144), synth.Shape("gate_up_fused", 4096, 28672)],
                         ids=lambda s: s.name)
def test_fused_decode_shapes(shape):
    # the fused projections of the decode loop bench.py times (q|k|v as one N = 6144 GEMV, gate|up as
    # one N = 28672 GEMV); sampled columns for the wide one
    check(shape, 2, 128, 1, "fused", False, ncols=None if shape.N <= 8192 else 2048)


@pytest.mark.parametrize("M", [512, 2048])
def test_config4_prefill_whole_layer_one_grouped_launch(M):
    # the launches bench.py times for the M = 2048 and M = 512 figures: all seven matrices of the 8B layer
    # in one hlq_lut_gemm_batch call; every row, whole tiles + one column of every tile against the C oracle
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    q, G = 2, 128
    shapes = synth.LLAMA31_8B_LAYER
    descs, packs, Xs, Ys, refs, colsets = [], [], [], [], [], []
    for s in shapes:
        say("config cfg4 grouped", s.name, s.K, s.N)
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "cfg4g", s.name)
        X = synth.make_x(M, s.K, "cfg4g", s.name, outliers=True)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        cols = tile_columns(s.N)
        refs.append(c_oracle.gemm_f64(X, codes, S, Z, q, G, cols=cols))
        colsets.append(cols)
        descs.append(d); packs.append(p); Xs.append(dev(X))
        Ys.append(torch.empty((M, s.N), dtype=torch.float16, device="cuda"))
        del codes, S, Z, X
    B.GemmBatch(descs, packs, Xs, Ys).launch()
    torch.cuda.synchronize()
    for s, Y, ref, cols in zip(shapes, Ys, refs, colsets):
        err = O.row_rel_err(Y[:, torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64), ref)
        say("   ", s.name, "max row err", float(err.max()))
        assert err.max() <= TOL, s.name
    del packs, Xs, Ys
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M", [1, 2, 4, 5, 8, 16])
def test_config3_small_batch_whole_layer_one_grouped_launch(M):
    # configuration 3 in the launch the small-batch figures are quoted on: the seven matrices of the 8B layer,
    # q = 4, in one hlq_lut_gemm_batch call with the default dispatch (few-rows kernel up to M = 4, many-rows
    # kernel with two and four chained operands above), every output column against the C oracle
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    q, G = 4, 128
    shapes = synth.LLAMA31_8B_LAYER
    descs, packs, Xs, Ys, refs = [], [], [], [], []
    for s in shapes:
        say("config cfg3 grouped", s.name, s.K, s.N, "M", M)
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "cfg3g", s.name)
        X = synth.make_x(M, s.K, "cfg3g", s.name, M, outliers=True)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        refs.append(c_oracle.gemm_f64(X, codes, S, Z, q, G))
        descs.append(d); packs.append(p); Xs.append(dev(X))
        Ys.append(torch.empty((M, s.N), dtype=torch.float16, device="cuda"))
        del codes, S, Z, X
    B.GemmBatch(descs, packs, Xs, Ys).launch()
    torch.cuda.synchronize()
    for s, Y, ref in zip(shapes, Ys, refs):
        err = O.row_rel_err(Y.float().cpu().numpy().astype(np.float64), ref)
        say("   ", s.name, "max row err", float(err.max()))
        assert err.max() <= TOL, s.name
    del packs, Xs, Ys
    torch.cuda.empty_cache()


@pytest.mark.parametrize("q", [2, 3])
@pytest.mark.parametrize("path", ["matrix cores", "lookups"])
def test_config2_whole_layer_one_grouped_launch(q, path):
    # the launch bench.py times: the seven GEMVs of the 8B layer in one hlq_lut_gemv_batch call, both
    # formulations, every output against the C oracle
    from paper_2510_19482_amd import binding as B
    from gpu_util import dev
    G = 128
    shapes = synth.LLAMA31_8B_LAYER
    descs, packs, xs, ys, refs = [], [], [], [], []
    for s in shapes:
        say("config cfg2 grouped", path, s.name, s.K, s.N, "q", q)
        codes, S, Z = synth.make_weight(s.K, s.N, q, G, "cfg2g", s.name)
        X = synth.make_x(1, s.K, "cfg2g", s.name)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        refs.append(c_oracle.gemm_f64(X, codes, S, Z, q, G))
        descs.append(d); packs.append(p); xs.append(dev(X[0]))
        ys.append(torch.empty(s.N, dtype=torch.float16, device="cuda"))
        del codes, S, Z
    B.set_gemv_path(B.GEMV_LUT if path == "lookups" else B.GEMV_MX)
    try:
        B.GemvBatch(descs, packs, xs, ys).launch()
        torch.cuda.synchronize()
    finally:
        B.set_gemv_path(B.GEMV_AUTO)
    for s, y, ref in zip(shapes, ys, refs):
        err = O.row_rel_err(y.float().cpu().numpy().astype(np.float64)[None, :], ref)
        say("   ", s.name, "max row err", float(err.max()))
        assert err.max() <= TOL, s.name
    del packs, xs, ys
    torch.cuda.empty_cache()
