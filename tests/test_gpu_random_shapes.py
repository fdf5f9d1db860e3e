"""Seeded random sweep over shapes, plane counts, group sizes and row counts, default dispatch: every call goes
wherever the library's own rules send it (GEMV kernels, few-rows, many-rows, tiled; single calls and grouped
launches), and every output element is compared with the oracle.  Complements the per-kernel files, which force
their kernel: this one catches a rule that routes an odd shape to a kernel that cannot take it."""
import numpy as np
import pytest
import torch

from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, pack_on_gpu

pytestmark = pytest.mark.gpu

# fp32 outputs, whichever kernel the rules pick.  The per-kernel files hold each kernel to its own, tighter bar (2e-5
# lookups, 2e-4 matrix-core GEMV, 1e-3 tiled kernel on layer-sized K); on a short K the fp16-rebuilt weights of the tiled
# kernel at four planes come to 1.0e-3 (K = 640), so this sweep uses 1.5e-3, still inside the 2e-3 of fp16 outputs.
BAR = 1.5e-3


def say(*a):
    print(*a, flush=True)


def cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        G = int(rng.choice([32, 64, 128, 256]))
        chunks = int(rng.choice([1, 2, 3, 5, 8, 13, 18, 33, 50]))
        if G == 256 and chunks % 2:
            chunks += 1
        K = 128 * chunks
        N = 8 * int(rng.choice([1, 2, 7, 8, 9, 17, 33, 64, 65, 130]))
        q = int(rng.integers(1, 5))
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 33, 70]))
        out.append((K, N, q, G, M))
    return out


@pytest.mark.parametrize("K,N,q,G,M", cases(40, 20251019))
def test_single_call_default_dispatch(K, N, q, G, M):
    say("single", K, N, q, G, M)
    codes, S, Z = synth.make_weight(K, N, q, G, "rnd")
    X = synth.make_x(M, K, "rnd", M, outliers=True)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    if M == 1:
        Y = B.hlq_lut_gemv(d, packed, dev(X[0]), out_f32=True)[None, :]
    else:
        Y = B.hlq_lut_gemm(d, packed, dev(X), out_f32=True)
    torch.cuda.synchronize()
    err = O.row_rel_err(Y.cpu().numpy().astype(np.float64), ref).max()
    say("   err", float(err))
    assert err <= BAR
    if M > 1:
        Y16 = B.hlq_lut_gemm(d, packed, dev(X), out_f32=False)
        torch.cuda.synchronize()
        assert O.row_rel_err(Y16.float().cpu().numpy().astype(np.float64), ref).max() <= TOL


@pytest.mark.parametrize("seed", range(12))
def test_grouped_launch_default_dispatch(seed):
    rng = np.random.default_rng(1000 + seed)
    G = int(rng.choice([64, 128, 128, 256]))
    q = int(rng.integers(1, 5))
    M = int(rng.choice([1, 2, 4, 5, 8, 9, 16, 24]))
    count = int(rng.integers(2, 6))
    descs, packs, Xs, Ys, refs = [], [], [], [], []
    for i in range(count):
        chunks = int(rng.choice([2, 4, 8, 18, 32]))
        K = 128 * chunks
        N = 8 * int(rng.choice([1, 8, 9, 33, 64, 130, 256]))
        codes, S, Z = synth.make_weight(K, N, q, G, "rnd-group", seed, i)
        X = synth.make_x(M, K, "rnd-group", seed, i, outliers=True)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d); packs.append(p)
        Xs.append(dev(X if M > 1 else X[0]))
        Ys.append(torch.full((M, N) if M > 1 else (N,), 7.0, dtype=torch.float32, device="cuda"))
        refs.append(O.gemm_dequant(X, codes, S, Z, q, G))
    say("group", seed, "q", q, "G", G, "M", M, [(d.K, d.N) for d in descs])
    batch = B.GemmBatch(descs, packs, Xs, Ys, out_f32=True) if M > 1 else B.GemvBatch(descs, packs, Xs, Ys, out_f32=True)
    for rep in range(2):
        batch.launch()
        torch.cuda.synchronize()
        for d, Y, ref in zip(descs, Ys, refs):
            got = Y.cpu().numpy().astype(np.float64).reshape(ref.shape)
            assert O.row_rel_err(got, ref).max() <= BAR, (d.K, d.N)
