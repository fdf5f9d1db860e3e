"""Helpers for the GPU parity tests: move seeded numpy inputs to the device, call the C ABI
through the binding, bring results back."""
import numpy as np
import torch

from paper_2510_19482_amd import binding as B
from paper_2510_19482_amd import synth

TOL = 2e-3   # max_n |y - y*| / max_n |y*| per row: the parity bar for fp16 in / fp32 accumulate


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pack_on_gpu(codes, S, Z, q, G):
    K, N = codes.shape
    d = B.make_desc(K, N, q, G)
    packed = B.hlq_pack(d, dev(codes), dev(S), dev(Z))
    return d, packed


def gemv_gpu(d, packed, x_row, out_f32=False):
    y = B.hlq_lut_gemv(d, packed, dev(x_row), out_f32=out_f32)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)[None, :]


def gemm_gpu(d, packed, X, out_f32=False):
    Y = B.hlq_lut_gemm(d, packed, dev(X), out_f32=out_f32)
    torch.cuda.synchronize()
    return Y.float().cpu().numpy().astype(np.float64)


def weight(shape_or_K, N=None, q=2, G=128, *key):
    if N is None:
        K, N = shape_or_K.K, shape_or_K.N
    else:
        K = shape_or_K
    return synth.make_weight(K, N, q, G, *key)
