"""Thin ctypes binding over libhlq.so: argument marshalling only.

Every step of the path (pack, tables, lookups, scaling, reduction) runs inside the HIP
library; torch is used for device memory and the current stream.  There is no fallback: if
the library has not been built, importing this module raises."""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HLQ_LIB", os.path.join(_PKG, "libhlq.so"))

HLQ_OK = 0
HLQ_OUT_F16 = 0
HLQ_OUT_F32 = 1


class HlqDesc(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("N", ctypes.c_int32), ("q", ctypes.c_int32),
                ("G", ctypes.c_int32), ("layout", ctypes.c_uint32)]


class GemvPlanInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("formulation", "waves_per_workgroup", "waves_per_tile", "chunks_per_slice",
                                              "slices", "tile_groups", "first_block", "blocks")]


class HlqError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn}: {status_string(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2510_19482_amd.build` "
            "(there is no CPU fallback)")
    # torch ships its own copy of the HIP runtime (same SONAME as the system one).  It has to be
    # loaded first: libhlq then binds to that copy, and both sides share one runtime, one device
    # context and the same stream handles.  Loaded the other way round the process ends up with
    # two runtimes and launches fail with "no ROCm-capable device".
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i64, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64, ctypes.c_uint32
    dp = ctypes.POINTER(HlqDesc)
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.hlq_status_string.restype = ctypes.c_char_p
    lib.hlq_status_string.argtypes = [ctypes.c_int]
    lib.hlq_layout_version.restype = u32
    lib.hlq_layout_version.argtypes = []
    lib.hlq_packed_bytes.restype = ctypes.c_int
    lib.hlq_packed_bytes.argtypes = [dp, szp, szp, szp]
    lib.hlq_workspace_bytes.restype = ctypes.c_int
    lib.hlq_workspace_bytes.argtypes = [dp, i64, szp]
    lib.hlq_pack.restype = ctypes.c_int
    lib.hlq_pack.argtypes = [dp, vp, vp, vp, vp, sz, vp]
    lib.hlq_unpack.restype = ctypes.c_int
    lib.hlq_unpack.argtypes = [dp, vp, vp, vp, vp, vp]
    lib.hlq_lut_gemv.restype = ctypes.c_int
    lib.hlq_lut_gemv.argtypes = [dp, vp, vp, vp, ctypes.c_int, vp, sz, vp]
    lib.hlq_lut_gemv_static.restype = ctypes.c_int
    lib.hlq_lut_gemv_static.argtypes = [dp, vp, vp, vp, ctypes.c_int, vp]
    lib.hlq_batch_workspace_bytes.restype = ctypes.c_int
    lib.hlq_batch_workspace_bytes.argtypes = [ctypes.c_int, dp, szp]
    lib.hlq_workspace_init.restype = ctypes.c_int
    lib.hlq_workspace_init.argtypes = [vp, sz, vp]
    lib.hlq_quantize.restype = ctypes.c_int
    lib.hlq_quantize.argtypes = [dp, vp, ctypes.c_int, vp, vp, vp, vp, vp]
    lib.hlq_gemm_batch_workspace_bytes.restype = ctypes.c_int
    lib.hlq_gemm_batch_workspace_bytes.argtypes = [ctypes.c_int, dp, ctypes.c_int64, szp]
    lib.hlq_lut_gemm_batch.restype = ctypes.c_int
    lib.hlq_lut_gemm_batch.argtypes = [ctypes.c_int, dp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int64,
                                       ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(vp),
                                       ctypes.POINTER(ctypes.c_int64), ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.hlq_lut_gemv_batch.restype = ctypes.c_int
    lib.hlq_lut_gemv_batch.argtypes = [ctypes.c_int, dp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       ctypes.POINTER(vp), ctypes.c_int, vp, sz, vp]
    lib.hlq_gemv_plan_query.restype = ctypes.c_int
    lib.hlq_gemv_plan_query.argtypes = [ctypes.c_int, dp, i64, ctypes.POINTER(GemvPlanInfo)]
    lib.hlq_set_gemv_plan.restype = ctypes.c_int
    lib.hlq_set_gemv_plan.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.hlq_set_gemm_path.restype = ctypes.c_int
    lib.hlq_set_gemm_path.argtypes = [ctypes.c_int]
    lib.hlq_set_gemv_path.restype = ctypes.c_int
    lib.hlq_set_gemv_path.argtypes = [ctypes.c_int]
    lib.hlq_stream_read.restype = ctypes.c_int
    lib.hlq_stream_read.argtypes = [vp, sz, ctypes.c_int, vp, sz, vp]
    lib.hlq_mfma_probe.restype = ctypes.c_int
    lib.hlq_mfma_probe.argtypes = [ctypes.c_int, vp, sz, ctypes.c_int, ctypes.c_int, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    lib.hlq_stream_read_shaped.restype = ctypes.c_int
    lib.hlq_stream_read_shaped.argtypes = [vp, sz, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, sz, vp]
    lib.hlq_lut_gemm.restype = ctypes.c_int
    lib.hlq_lut_gemm.argtypes = [dp, vp, vp, i64, i64, vp, i64, ctypes.c_int, vp, sz, vp]
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.hlq_status_string(int(status)).decode()


def layout_version() -> int:
    return int(lib.hlq_layout_version())


def make_desc(K: int, N: int, q: int, G: int, layout: int | None = None) -> HlqDesc:
    return HlqDesc(K, N, q, G, layout_version() if layout is None else layout)


def _check(fn: str, status: int) -> None:
    if status != HLQ_OK:
        raise HlqError(fn, status)


def set_gemv_plan(tiles_per_wave: int = 0, waves_per_workgroup: int = 0, chunks_per_wave: int = 0) -> None:
    _check("hlq_set_gemv_plan", lib.hlq_set_gemv_plan(tiles_per_wave, waves_per_workgroup, chunks_per_wave))


def gemv_plan_query(descs, M: int = 1):
    """Work split of a grouped GEMV / few-rows launch over `descs` (host arithmetic, no GPU needed)."""
    n = len(descs)
    arr = (HlqDesc * n)(*descs)
    out = (GemvPlanInfo * n)()
    _check("hlq_gemv_plan_query", lib.hlq_gemv_plan_query(n, arr, M, out))
    return list(out)


GEMM_AUTO, GEMM_LUT, GEMM_MFMA, GEMM_MFMA_FP16, GEMM_ROWS16 = 0, 1, 2, 3, 4


def set_gemm_path(path: int = 0) -> None:
    _check("hlq_set_gemm_path", lib.hlq_set_gemm_path(path))


GEMV_AUTO, GEMV_LUT, GEMV_MX = 0, 1, 2
GEMV_TABLE_F32, GEMV_TABLE_MIRROR, GEMV_TABLE_F16, GEMV_TABLE_I8 = 3, 4, 5, 6


def set_gemv_path(path: int = 0) -> None:
    _check("hlq_set_gemv_path", lib.hlq_set_gemv_path(path))


def packed_bytes(desc: HlqDesc):
    """(total, bits, meta) byte counts of the packed blob."""
    t, b, m = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check("hlq_packed_bytes", lib.hlq_packed_bytes(ctypes.byref(desc), ctypes.byref(t), ctypes.byref(b), ctypes.byref(m)))
    return t.value, b.value, m.value


def workspace_bytes(desc: HlqDesc, M: int) -> int:
    w = ctypes.c_size_t()
    _check("hlq_workspace_bytes", lib.hlq_workspace_bytes(ctypes.byref(desc), M, ctypes.byref(w)))
    return w.value


# ---- torch-facing helpers (device tensors in, device tensors out) -------------------------
def _stream_ptr(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def hlq_pack(desc: HlqDesc, codes, scales, zeros, packed=None, stream=None):
    """codes u8 [K,N], scales fp16 [q,K/G,N], zeros fp16 [K/G,N] (cuda tensors) -> packed u8 blob."""
    import torch
    total, _, _ = packed_bytes(desc)
    if packed is None:
        packed = torch.empty(total, dtype=torch.uint8, device=codes.device)
    _check("hlq_pack", lib.hlq_pack(ctypes.byref(desc), _ptr(codes), _ptr(scales), _ptr(zeros),
                                    _ptr(packed), packed.numel() * packed.element_size(), _stream_ptr(stream)))
    return packed


def hlq_unpack(desc: HlqDesc, packed, stream=None):
    import torch
    K, N, q, G = desc.K, desc.N, desc.q, desc.G
    codes = torch.empty((K, N), dtype=torch.uint8, device=packed.device)
    scales = torch.empty((q, K // G, N), dtype=torch.float16, device=packed.device)
    zeros = torch.empty((K // G, N), dtype=torch.float16, device=packed.device)
    _check("hlq_unpack", lib.hlq_unpack(ctypes.byref(desc), _ptr(packed), _ptr(codes), _ptr(scales),
                                        _ptr(zeros), _stream_ptr(stream)))
    return codes, scales, zeros


def batch_workspace_bytes(descs) -> int:
    arr = (HlqDesc * len(descs))(*descs)
    w = ctypes.c_size_t()
    _check("hlq_batch_workspace_bytes", lib.hlq_batch_workspace_bytes(len(descs), arr, ctypes.byref(w)))
    return w.value


def _new_workspace(nbytes: int, device, stream=None):
    import torch
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check("hlq_workspace_init", lib.hlq_workspace_init(_ptr(ws), ws.numel(), _stream_ptr(stream)))
    return ws


def alloc_workspace(desc: HlqDesc, M: int, device="cuda", stream=None):
    """Allocate and initialise a workspace for GEMV/GEMM calls on `desc` with up to M rows."""
    return _new_workspace(workspace_bytes(desc, M), device, stream)


def alloc_batch_workspace(descs, device="cuda", stream=None):
    return _new_workspace(batch_workspace_bytes(descs), device, stream)


def hlq_quantize(desc: HlqDesc, W, t_max: int = 10, with_err: bool = False, stream=None):
    """Alg. 1 on W fp32 cuda [K, N] -> codes u8 [K, N], scales fp16 [q, K/G, N], zeros fp16 [K/G, N]
    (and the per-group squared error fp32 [K/G, N] with with_err=True)."""
    import torch
    assert W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (desc.K, desc.N)
    dev = W.device
    codes = torch.empty((desc.K, desc.N), dtype=torch.uint8, device=dev)
    scales = torch.empty((desc.q, desc.K // desc.G, desc.N), dtype=torch.float16, device=dev)
    zeros = torch.empty((desc.K // desc.G, desc.N), dtype=torch.float16, device=dev)
    err = torch.empty((desc.K // desc.G, desc.N), dtype=torch.float32, device=dev) if with_err else None
    _check("hlq_quantize", lib.hlq_quantize(ctypes.byref(desc), _ptr(W), t_max, _ptr(codes), _ptr(scales), _ptr(zeros),
                                            _ptr(err) if with_err else None, _stream_ptr(stream)))
    return (codes, scales, zeros, err) if with_err else (codes, scales, zeros)


def hlq_stream_read(src, nbytes: int, sink, blocks: int = 0, offset: int = 0, stream=None):
    """Measurement helper: read nbytes of `src` (a cuda tensor) from byte `offset` on, once."""
    _check("hlq_stream_read", lib.hlq_stream_read(_ptr(src) + offset, nbytes, blocks, _ptr(sink),
                                                  sink.numel() * sink.element_size(), _stream_ptr(stream)))


def hlq_stream_read_shaped(src, nbytes: int, sink, blocks: int = 0, unroll: int = 4, temporal: bool = False,
                           offset: int = 0, stream=None):
    """hlq_stream_read with its loop shape and cache policy as arguments (for sweeps)."""
    _check("hlq_stream_read_shaped", lib.hlq_stream_read_shaped(_ptr(src) + offset, nbytes, blocks, unroll, int(temporal),
                                                                _ptr(sink), sink.numel() * sink.element_size(),
                                                                _stream_ptr(stream)))


def hlq_mfma_probe(operands, iters: int, blocks: int, sink, kind: int = 0, stream=None) -> float:
    """Launch the matrix-core-only measurement loop (kind 0: fp16 32x32x16, 1: bf8 x fp4 16x16x128); returns the
    floating-point operations of the launch."""
    flop = ctypes.c_double(0.0)
    _check("hlq_mfma_probe", lib.hlq_mfma_probe(kind, _ptr(operands), operands.numel() * operands.element_size(), iters, blocks,
                                                _ptr(sink), sink.numel() * sink.element_size(), ctypes.byref(flop),
                                                _stream_ptr(stream)))
    return flop.value


class GemvBatch:
    """Pre-marshalled arguments of one hlq_lut_gemv_batch call (host arrays built once)."""

    def __init__(self, descs, packed, xs, ys, out_f32=False, ws=None):
        n = len(descs)
        self.n = n
        self.descs = (HlqDesc * n)(*descs)
        self.packed = (ctypes.c_void_p * n)(*[_ptr(p) for p in packed])
        self.xs = (ctypes.c_void_p * n)(*[_ptr(x) for x in xs])
        self.ys = (ctypes.c_void_p * n)(*[_ptr(y) for y in ys])
        self.out = HLQ_OUT_F32 if out_f32 else HLQ_OUT_F16
        self.ws = ws if ws is not None else alloc_batch_workspace(list(descs), xs[0].device)
        self._keep = (list(packed), list(xs), list(ys))

    def launch(self, stream=None):
        _check("hlq_lut_gemv_batch", lib.hlq_lut_gemv_batch(
            self.n, self.descs, self.packed, self.xs, self.ys, self.out, _ptr(self.ws),
            self.ws.numel(), _stream_ptr(stream)))


class GemmBatch:
    """Pre-marshalled arguments of one hlq_lut_gemm_batch call: Y_i[M, N_i] = X_i[M, K_i] @ W^_i."""

    def __init__(self, descs, packed, Xs, Ys, out_f32=False, ws=None):
        n = len(descs)
        self.n = n
        self.M = int(Xs[0].shape[0])
        self.descs = (HlqDesc * n)(*descs)
        self.packed = (ctypes.c_void_p * n)(*[_ptr(p) for p in packed])
        self.Xs = (ctypes.c_void_p * n)(*[_ptr(x) for x in Xs])
        self.Ys = (ctypes.c_void_p * n)(*[_ptr(y) for y in Ys])
        self.ldx = (ctypes.c_int64 * n)(*[max(int(x.stride(0)), d.K) for x, d in zip(Xs, descs)])
        self.ldy = (ctypes.c_int64 * n)(*[max(int(y.stride(0)), d.N) for y, d in zip(Ys, descs)])
        self.out = HLQ_OUT_F32 if out_f32 else HLQ_OUT_F16
        if ws is None:
            w = ctypes.c_size_t()
            _check("hlq_gemm_batch_workspace_bytes",
                   lib.hlq_gemm_batch_workspace_bytes(n, self.descs, self.M, ctypes.byref(w)))
            ws = _new_workspace(w.value, Xs[0].device)
        self.ws = ws
        self._keep = (list(packed), list(Xs), list(Ys))

    def launch(self, stream=None):
        _check("hlq_lut_gemm_batch", lib.hlq_lut_gemm_batch(
            self.n, self.descs, self.packed, self.Xs, self.M, self.ldx, self.Ys, self.ldy, self.out,
            _ptr(self.ws), self.ws.numel(), _stream_ptr(stream)))


def hlq_lut_gemv(desc: HlqDesc, packed, x, y=None, out_f32: bool = False, ws=None, stream=None):
    """y[N] = x[K] @ W^ ; x fp16 cuda tensor."""
    import torch
    if y is None:
        y = torch.empty(desc.N, dtype=torch.float32 if out_f32 else torch.float16, device=x.device)
    if ws is None:
        ws = alloc_workspace(desc, 1, x.device)
    _check("hlq_lut_gemv", lib.hlq_lut_gemv(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(y),
                                            HLQ_OUT_F32 if out_f32 else HLQ_OUT_F16, _ptr(ws), ws.numel(),
                                            _stream_ptr(stream)))
    return y


STATIC_SCRATCH_BYTES = 131072 + (4 << 20)


def hlq_lut_gemv_static(desc: HlqDesc, packed, x, y, out_f32: bool = False, stream=None):
    """hlq_lut_gemv without a workspace argument (scratch in a fixed array of the library); `y` is
    the caller's output tensor: this call allocates nothing."""
    _check("hlq_lut_gemv_static", lib.hlq_lut_gemv_static(ctypes.byref(desc), _ptr(packed), _ptr(x), _ptr(y),
                                                          HLQ_OUT_F32 if out_f32 else HLQ_OUT_F16, _stream_ptr(stream)))
    return y


def hlq_lut_gemm(desc: HlqDesc, packed, X, Y=None, out_f32: bool = False, ws=None, stream=None):
    """Y[M,N] = X[M,K] @ W^ ; X fp16 cuda tensor, row-major (stride(1) == 1)."""
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, desc.N), dtype=torch.float32 if out_f32 else torch.float16, device=X.device)
    if ws is None:
        ws = alloc_workspace(desc, M, X.device)
    ldx = X.stride(0) if M > 1 else max(X.stride(0), desc.K)
    ldy = Y.stride(0) if M > 1 else max(Y.stride(0), desc.N)
    _check("hlq_lut_gemm", lib.hlq_lut_gemm(ctypes.byref(desc), _ptr(packed), _ptr(X), M, ldx, _ptr(Y), ldy,
                                            HLQ_OUT_F32 if out_f32 else HLQ_OUT_F16, _ptr(ws), ws.numel(),
                                            _stream_ptr(stream)))
    return Y
