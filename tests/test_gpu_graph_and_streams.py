"""Calls are asynchronous on the caller's stream and legal under stream capture.  A captured call,
replayed several times with new inputs and with eager work and synchronisations in between, gives
what the eager call gives (the split-K hand-over state in the workspace must return to its initial
state after every launch); a call on a side stream gives what the default stream gives.  The eager
results themselves are checked against the oracle in the parity tests; one oracle check per case
here ties the two together."""
import numpy as np
import pytest
import torch

from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, pack_on_gpu

pytestmark = pytest.mark.gpu


def close(a, b):
    a, b = a.float(), b.float()
    return (a - b).abs().max().item() <= 1e-3 * b.abs().max().item()


def oracle_ok(codes, S, Z, q, G, X, Y):
    ref = O.gemm_dequant(X, codes, S, Z, q, G)
    err = O.row_rel_err(Y.float().cpu().numpy().astype(np.float64), ref)
    return float(np.max(err)) <= TOL


# (name, K, N, q, G, M): shapes whose K is cut across workgroups, so every launch uses the workspace
CASES = [
    ("gemv, K split", 14336, 512, 2, 128, 1),
    ("gemv lookups, K split", 14336, 512, 2, 128, 1),
    ("few rows on the GEMV kernel", 8192, 264, 4, 128, 3),
    ("tiled kernel, K split + reduce kernel", 14336, 256, 2, 128, 16),
    ("tiled kernel, several row blocks", 2048, 520, 3, 64, 200),
]


@pytest.mark.parametrize("name,K,N,q,G,M", CASES)
def test_graph_replays_match_eager(name, K, N, q, G, M):
    print("graph", name, K, N, q, G, M, flush=True)
    lookups = "lookups" in name
    codes, S, Z = synth.make_weight(K, N, q, G, "graph", name)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    xs_host = [synth.make_x(M, K, "graph", name, i, outliers=True) for i in range(2)]
    xs = [dev(x) for x in xs_host]
    x_static = torch.empty_like(xs[0])
    y_static = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    ws_graph = B.alloc_workspace(d, M)
    ws_eager = B.alloc_workspace(d, M)
    if lookups:
        B.set_gemv_path(B.GEMV_LUT)
    try:
        def call(x, y, ws):
            if M == 1:
                B.hlq_lut_gemv(d, packed, x[0], y=y[0], ws=ws)
            else:
                B.hlq_lut_gemm(d, packed, x, Y=y, ws=ws)

        x_static.copy_(xs[0])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call(x_static, y_static, ws_graph)
        for rep, i in enumerate((0, 1, 1, 0)):
            x_static.copy_(xs[i])
            y_eager = torch.zeros_like(y_static)
            call(xs[i], y_eager, ws_eager)          # the program's own eager work between replays
            torch.cuda.synchronize()
            y_static.fill_(float("nan"))            # a replay that wrote nothing would be seen
            g.replay()
            torch.cuda.synchronize()
            assert close(y_static, y_eager), (name, rep)
            if rep == 1:
                assert oracle_ok(codes, S, Z, q, G, xs_host[i], y_static)
        # the eager workspace is as reusable as the captured one: same call, same result
        y2 = torch.zeros_like(y_static)
        call(xs[0], y2, ws_graph)
        torch.cuda.synchronize()
        assert close(y2, y_static)
    finally:
        B.set_gemv_path(B.GEMV_AUTO)


def test_grouped_launches_replay():
    print("graph grouped", flush=True)
    q, G = 2, 128
    shapes = [(14336, 256), (4096, 520), (4096, 72)]
    descs, packs, ws_ = [], [], []
    for i, (K, N) in enumerate(shapes):
        codes, S, Z = synth.make_weight(K, N, q, G, "graphgroup", i)
        d, p = pack_on_gpu(codes, S, Z, q, G)
        descs.append(d)
        packs.append(p)
    for M in (1, 40):
        xs = [[dev(synth.make_x(M, K, "graphgroup", i, v, outliers=True)) for i, (K, N) in enumerate(shapes)] for v in range(2)]
        x_static = [torch.empty_like(x) for x in xs[0]]
        y_static = [torch.zeros((M, N), dtype=torch.float16, device="cuda") for (K, N) in shapes]
        y_eager = [torch.zeros_like(y) for y in y_static]
        if M == 1:
            captured = B.GemvBatch(descs, packs, [x[0] for x in x_static], [y[0] for y in y_static])
            eager = [B.GemvBatch(descs, packs, [x[0] for x in xs[v]], [y[0] for y in y_eager]) for v in range(2)]
        else:
            captured = B.GemmBatch(descs, packs, x_static, y_static)
            eager = [B.GemmBatch(descs, packs, xs[v], y_eager) for v in range(2)]
        for a, b in zip(x_static, xs[0]):
            a.copy_(b)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            captured.launch()
        for rep, v in enumerate((0, 1, 0)):
            for a, b in zip(x_static, xs[v]):
                a.copy_(b)
            eager[v].launch()
            torch.cuda.synchronize()
            for y in y_static:
                y.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            for i in range(len(shapes)):
                assert close(y_static[i], y_eager[i]), (M, rep, i)


def test_side_stream_matches_default_stream():
    print("side stream", flush=True)
    K, N, q, G = 14336, 520, 2, 128
    codes, S, Z = synth.make_weight(K, N, q, G, "stream")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    for M in (1, 24):
        X = dev(synth.make_x(M, K, "stream", M, outliers=True))
        Y0 = B.hlq_lut_gemm(d, packed, X)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()                   # default priority
        side.wait_stream(torch.cuda.current_stream())
        Y1 = torch.zeros_like(Y0)
        ws = B.alloc_workspace(d, M, stream=side)
        for _ in range(3):                           # back-to-back on the same workspace
            B.hlq_lut_gemm(d, packed, X, Y=Y1, ws=ws, stream=side)
        side.synchronize()
        assert close(Y1, Y0), M
