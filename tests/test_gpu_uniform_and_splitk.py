"""GPU parity: the uniform special case of HLQ on the shapes of the paper's kernel-latency table, the
hand-over of split-K partial sums under many back-to-back launches on one workspace, and K values whose
chunk count does not divide evenly into the planner's slices."""
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


# ---------------------------------------------------------------------------------------------------
# Alg. 1 starts from s_j = 2^j * Delta, z = min: with such scales HLQ is ordinary uniform quantisation,
# W^ = Delta * code + z.  The appendix's kernel-latency table compares exactly these two parameter
# sets ("uniform" against free per-plane scales) on 11008 x 4096 and 4096 x 32000 at two bits; the
# benchmark times both, this test checks both against the oracle, every output column.
@pytest.mark.parametrize("K,N", [(11008, 4096), (4096, 32000)])
def test_uniform_special_case_on_latency_table_shapes(K, N, gemv_path):
    q, G = 2, 128
    codes = synth.make_codes(K, N, q, "uniform")
    delta = synth.make_scales(K, N, 1, G, "uniform-delta")[0]            # fp16 [K/G, N]
    S = np.stack([(delta.astype(np.float32) * (1 << j)).astype(np.float16) for j in range(q)])
    assert np.array_equal(S[1].astype(np.float64), 2.0 * delta.astype(np.float64))   # 2^j * Delta is exact in fp16
    Z = synth.make_zeros(K, N, G, "uniform")
    x = synth.make_x(1, K, "uniform", K, N)
    say("uniform case", K, N)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    # the oracle's definition (per-plane scales) ...
    ref = c_oracle.gemm_f64(x, codes, S, Z, q, G)
    # ... and, on a slice of the columns, textbook integer dequantisation Delta * code + z in numpy
    cols = np.arange(0, N, 97)
    Wc = (np.repeat(delta[:, cols].astype(np.float64), G, axis=0) * codes[:, cols].astype(np.float64)
          + np.repeat(Z[:, cols].astype(np.float64), G, axis=0))
    np.testing.assert_allclose(ref[:, cols], x.astype(np.float64) @ Wc, rtol=1e-11, atol=1e-11)
    y16 = gemv_gpu(d, packed, x[0])
    y32 = gemv_gpu(d, packed, x[0], out_f32=True)
    e16, e32 = O.row_rel_err(y16, ref).max(), O.row_rel_err(y32, ref).max()
    say("   row err fp16 out", float(e16), "fp32 out", float(e32))
    assert e16 <= TOL and e32 <= gemv_path
    # the free-scale parameters the table's other column uses, same shape
    codes2, S2, Z2 = synth.make_weight(K, N, q, G, "uniform-vs-hlq")
    d2, packed2 = pack_on_gpu(codes2, S2, Z2, q, G)
    ref2 = c_oracle.gemm_f64(x, codes2, S2, Z2, q, G)
    e = O.row_rel_err(gemv_gpu(d2, packed2, x[0]), ref2).max()
    say("   free per-plane scales: row err", float(e))
    assert e <= TOL


# ---------------------------------------------------------------------------------------------------
# Split-K hand-over.  Partial sums are written through to device scope, the workgroup waits for the
# writes, bumps the tile's arrival counter, and the last arriver adds the partials in slice order and
# resets the counter.  Many launches of DIFFERENT shapes, back to back on ONE workspace with no host
# synchronisation in between, exercise every reuse of counters and partial areas; a stale partial, a
# counter left non-zero or an early reader shows as a changed bit in some output.  The expected
# output of each shape comes from one launch on a fresh workspace, itself checked against the oracle.
SPLITK_SHAPES = [(14336, 4096), (4096, 1024), (6400, 520), (8192, 2048), (28672, 512), (1024, 4096)]


@pytest.mark.parametrize("plan", [(0, 0), (4, 2), (8, 1), (2, 3)], ids=lambda p: f"W{p[0]}cpw{p[1]}")
def test_split_k_many_launches_one_workspace(gemv_path, plan):
    q, G = 2, 128
    B.set_gemv_plan(0, plan[0], plan[1])
    try:
        cases = []
        ws_bytes = 0
        for (K, N) in SPLITK_SHAPES:
            codes, S, Z = synth.make_weight(K, N, q, G, "splitk")
            x = synth.make_x(1, K, "splitk", K, N)
            d, packed = pack_on_gpu(codes, S, Z, q, G)
            ref = c_oracle.gemm_f64(x, codes, S, Z, q, G)
            xd = dev(x[0])
            y0 = B.hlq_lut_gemv(d, packed, xd, out_f32=True)        # fresh workspace
            torch.cuda.synchronize()
            e = O.row_rel_err(y0.cpu().numpy().astype(np.float64)[None, :], ref).max()
            info = B.gemv_plan_query([d], 1)[0]
            say("   ", K, N, "slices", info.slices, "chunks/slice", info.chunks_per_slice, "row err", float(e))
            assert e <= gemv_path
            cases.append((d, packed, xd, y0.clone()))
            ws_bytes = max(ws_bytes, B.workspace_bytes(d, 1))
        assert sum(B.gemv_plan_query([c[0]], 1)[0].slices > 1 for c in cases) >= 2, "no shape splits K"
        ws = B._new_workspace(ws_bytes, "cuda")
        rounds = 40
        order = [(3 * i + (i // len(cases))) % len(cases) for i in range(rounds * len(cases))]
        outs = [torch.empty(cases[c][0].N, dtype=torch.float32, device="cuda") for c in order]
        for c, y in zip(order, outs):
            d, packed, xd, _ = cases[c]
            B.hlq_lut_gemv(d, packed, xd, y=y, out_f32=True, ws=ws)
        torch.cuda.synchronize()
        for i, (c, y) in enumerate(zip(order, outs)):
            if not torch.equal(y.view(torch.int32), cases[c][3].view(torch.int32)):
                bad = (y.view(torch.int32) != cases[c][3].view(torch.int32)).nonzero().flatten()
                pytest.fail(f"launch {i} (shape {SPLITK_SHAPES[c]}): {bad.numel()} outputs differ from the same "
                            f"GEMV on a fresh workspace, first at column {int(bad[0])}")
        say("   ", len(order), "launches on one workspace: all bit-identical")
        # and the counters are back at zero
        assert int(ws[:131072].view(torch.int32).abs().sum().item()) == 0
    finally:
        B.set_gemv_plan(0, 0, 0)


# ---------------------------------------------------------------------------------------------------
# Chunk counts the planner's rounding once turned into trailing slices without a chunk (K = 6400 is
# 50 chunks: runs of two on four wavefronts give seven slices of eight, the seventh starts past K).
@pytest.mark.parametrize("K", [6272, 6400, 7296, 8448])
@pytest.mark.parametrize("M", [1, 2, 4])
def test_k_with_ragged_slices(K, M):
    N, q, G = 1160, 4, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "ragged-k")
    X = synth.make_x(M, K, "ragged-k", K, M, outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    info = B.gemv_plan_query([d], M)[0]
    say("ragged K", K, "M", M, "slices", info.slices, "chunks/slice", info.chunks_per_slice)
    assert (info.slices - 1) * info.chunks_per_slice < K // 128
    Y = gemv_gpu(d, packed, X[0]) if M == 1 else gemm_gpu(d, packed, X)
    assert O.row_rel_err(Y, ref).max() <= TOL


@pytest.mark.parametrize("plan", [(4, 2), (8, 1), (1, 1)], ids=lambda p: f"W{p[0]}cpw{p[1]}")
def test_k_with_ragged_slices_forced_plans(gemv_path, plan):
    K, N, q, G = 6400, 1160, 2, 64
    codes, S, Z = synth.make_weight(K, N, q, G, "ragged-k-forced")
    X = synth.make_x(1, K, "ragged-k-forced")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    B.set_gemv_plan(0, plan[0], plan[1])
    try:
        info = B.gemv_plan_query([d], 1)[0]
        say("ragged K, forced plan", plan, "slices", info.slices, "chunks/slice", info.chunks_per_slice)
        y = gemv_gpu(d, packed, X[0], out_f32=True)
    finally:
        B.set_gemv_plan(0, 0, 0)
    assert O.row_rel_err(y, ref).max() <= gemv_path
