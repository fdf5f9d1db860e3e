"""The documented size limits: K = 2^21 (16384 chunks per tile, the longest byte offsets inside a
tile, the deepest K split) and N = 2^20 (16384 column tiles) still agree with the oracle; one step
beyond either limit is refused on the host."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

from gpu_util import TOL, dev, pack_on_gpu

pytestmark = pytest.mark.gpu


def test_longest_K():
    K, N, q, G = 1 << 21, 72, 4, 32          # one full tile and a ragged one; most metadata per chunk
    print("limits: K", K, N, q, G, flush=True)
    codes, S, Z = synth.make_weight(K, N, q, G, "maxK")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    assert packed.numel() == O.packed_bytes(K, N, q, G)
    # round trip of the far end of the blob
    c2, s2, z2 = B.hlq_unpack(d, packed)
    torch.cuda.synchronize()
    assert np.array_equal(c2[-4096:].cpu().numpy(), codes[-4096:])
    assert np.array_equal(s2[:, -64:].cpu().numpy().view(np.uint16), S[:, -64:].view(np.uint16))
    del c2, s2, z2
    for M in (1, 3, 40):                      # GEMV kernel, its few-rows form, tiled kernel
        X = synth.make_x(M, K, "maxK", M, outliers=True)
        ref = c_oracle.gemm_f64(X, codes, S, Z, q, G)
        for path in ((B.GEMV_MX, B.GEMV_LUT) if M == 1 else (B.GEMV_AUTO,)):
            B.set_gemv_path(path)
            try:
                Y = B.hlq_lut_gemm(d, packed, dev(X), out_f32=True)
                torch.cuda.synchronize()
            finally:
                B.set_gemv_path(B.GEMV_AUTO)
            err = O.row_rel_err(Y.cpu().numpy().astype(np.float64), ref).max()
            print("  M", M, "path", path, "err", err, flush=True)
            assert err <= TOL


def test_widest_N():
    K, N, q, G = 128, 1 << 20, 1, 128
    print("limits: N", K, N, q, G, flush=True)
    codes, S, Z = synth.make_weight(K, N, q, G, "maxN")
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    for M in (1, 2, 33):
        X = synth.make_x(M, K, "maxN", M)
        ref = c_oracle.gemm_f64(X, codes, S, Z, q, G)
        Y = B.hlq_lut_gemm(d, packed, dev(X), out_f32=True)
        torch.cuda.synchronize()
        err = O.row_rel_err(Y.cpu().numpy().astype(np.float64), ref).max()
        print("  M", M, "err", err, flush=True)
        assert err <= TOL


def test_one_step_beyond_is_refused():
    t = ctypes.c_size_t()
    for K, N in (((1 << 21) + 128, 8), (128, (1 << 20) + 8)):
        d = B.make_desc(K, N, 2, 128)
        assert B.lib.hlq_packed_bytes(ctypes.byref(d), ctypes.byref(t), None, None) == 3
