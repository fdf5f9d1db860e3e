"""The C-ABI library loads, exports every declared symbol, and does its host-side argument
checks without a GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from oracle import hlq_oracle as O
from paper_2510_19482_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hlq.h")).read()
    return re.findall(r"HLQ_API\s+[\w\s\*]+?\b(hlq_\w+)\s*\(", text)


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert {"hlq_pack", "hlq_unpack", "hlq_lut_gemv", "hlq_lut_gemm", "hlq_packed_bytes",
            "hlq_workspace_bytes", "hlq_status_string", "hlq_layout_version"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("K,N,q,G", [(4096, 4096, 2, 128), (4096, 1024, 3, 128), (14336, 4096, 4, 128),
                                     (8192, 128256, 2, 64), (128, 8, 1, 32), (256, 8, 4, 256)])
def test_packed_bytes_closed_form(K, N, q, G):
    total, bits, meta = B.packed_bytes(B.make_desc(K, N, q, G))
    assert total == O.packed_bytes(K, N, q, G)
    assert bits == K * N * q // 8 and meta == 2 * (q + 1) * (K // G) * N
    assert total * 8 == K * N * O.bits_per_weight(q, G)


def test_baseline_packed_sizes():
    # sizes the benchmark's byte counts rest on
    assert B.packed_bytes(B.make_desc(4096, 4096, 2, 128))[0] == 4_980_736
    from paper_2510_19482_amd import synth
    layer = sum(B.packed_bytes(B.make_desc(s.K, s.N, 2, 128))[0] for s in synth.LLAMA31_8B_LAYER)
    assert layer == 64_749_568
    layer3 = sum(B.packed_bytes(B.make_desc(s.K, s.N, 3, 128))[0] for s in synth.LLAMA31_8B_LAYER)
    assert layer3 == 95_420_416


@pytest.mark.parametrize("K,N,q,G", [(4096, 4096, 0, 128), (4096, 4096, 5, 128), (4096, 4096, 2, 48),
                                     (4096, 4096, 2, 16), (4000, 4096, 2, 128), (4096, 4100, 2, 128),
                                     (0, 4096, 2, 128), (4096, 0, 2, 128), (128, 8, 2, 256)])
def test_bad_descriptors_rejected(K, N, q, G):
    with pytest.raises(B.HlqError) as e:
        B.packed_bytes(B.make_desc(K, N, q, G))
    assert e.value.status == 2


def test_bad_layout_and_null():
    d = B.make_desc(128, 8, 2, 128, layout=123)
    with pytest.raises(B.HlqError) as e:
        B.packed_bytes(d)
    assert e.value.status == 2
    t = ctypes.c_size_t()
    assert B.lib.hlq_packed_bytes(None, ctypes.byref(t), None, None) == 1
    d = B.make_desc(128, 8, 2, 128)
    assert B.lib.hlq_packed_bytes(ctypes.byref(d), None, None, None) == 1
    assert B.lib.hlq_workspace_bytes(ctypes.byref(d), -1, ctypes.byref(t)) == 5


def test_host_side_argument_errors_launch_nothing():
    d = B.make_desc(128, 8, 2, 128)
    dp = ctypes.byref(d)
    fake = 0x1000   # never dereferenced: every call below fails validation first
    total = B.packed_bytes(d)[0]
    assert B.lib.hlq_pack(dp, None, fake, fake, fake, total, None) == 1
    assert B.lib.hlq_pack(dp, fake, fake, fake, fake, total - 1, None) == 4
    assert B.lib.hlq_unpack(dp, None, fake, fake, fake, None) == 1
    assert B.lib.hlq_lut_gemv(dp, fake, None, fake, 0, fake, 1 << 20, None) == 1
    assert B.lib.hlq_lut_gemv(dp, fake, fake, fake, 7, fake, 1 << 20, None) == 3
    assert B.lib.hlq_lut_gemm(dp, fake, fake, 4, 127, fake, 8, 0, fake, 1 << 20, None) == 5
    assert B.lib.hlq_lut_gemm(dp, fake, fake, 4, 128, fake, 7, 0, fake, 1 << 20, None) == 5
    assert B.lib.hlq_lut_gemm(dp, fake, fake, -1, 128, fake, 8, 0, fake, 1 << 20, None) == 5
    assert B.lib.hlq_lut_gemm(dp, fake, fake, 0, 128, fake, 8, 0, fake, 1 << 20, None) == 0   # M=0 no-op
    # workspace too small where one is needed
    big = B.make_desc(4096, 4096, 2, 128)
    need = B.workspace_bytes(big, 1)
    assert need > 0
    assert B.lib.hlq_lut_gemv(ctypes.byref(big), fake, fake, fake, 0, fake, need - 256 - 1, None) == 4
    assert B.lib.hlq_lut_gemv(ctypes.byref(big), fake, fake, fake, 0, None, 0, None) == 1


def test_stream_read_argument_errors_launch_nothing():
    fake = 0x1000
    assert B.lib.hlq_stream_read(None, 4096, 0, fake, 1 << 20, None) == 1
    assert B.lib.hlq_stream_read(fake, 4096, 0, None, 1 << 20, None) == 1
    assert B.lib.hlq_stream_read(fake + 8, 4096, 0, fake, 1 << 20, None) == 5
    assert B.lib.hlq_stream_read(fake, 4100, 0, fake, 1 << 20, None) == 5
    assert B.lib.hlq_stream_read(fake, 4096, -1, fake, 1 << 20, None) == 3
    assert B.lib.hlq_stream_read(fake, 4096, 65537, fake, 1 << 20, None) == 3
    assert B.lib.hlq_stream_read(fake, 1 << 20, 16, fake, 63, None) == 4
    assert B.lib.hlq_stream_read(fake, 0, 0, fake, 0, None) == 0            # nothing to read


def test_mfma_probe_argument_errors_launch_nothing():
    fake = 0x1000
    assert B.lib.hlq_mfma_probe(0, None, 4096, 1, 1, fake, 1024, None, None) == 1
    assert B.lib.hlq_mfma_probe(0, fake, 4096, 1, 1, None, 1024, None, None) == 1
    assert B.lib.hlq_mfma_probe(0, fake + 8, 4096, 1, 1, fake, 1024, None, None) == 5
    assert B.lib.hlq_mfma_probe(0, fake, 4100, 1, 1, fake, 1024, None, None) == 5
    assert B.lib.hlq_mfma_probe(0, fake, 0, 1, 1, fake, 1024, None, None) == 5
    assert B.lib.hlq_mfma_probe(0, fake, 4096, 0, 1, fake, 1024, None, None) == 3
    assert B.lib.hlq_mfma_probe(0, fake, 4096, 1, 0, fake, 1024, None, None) == 3
    assert B.lib.hlq_mfma_probe(0, fake, 4096, 1, 65537, fake, 1 << 30, None, None) == 3
    assert B.lib.hlq_mfma_probe(0, fake, 4096, 1, 2, fake, 2047, None, None) == 4
    assert B.lib.hlq_mfma_probe(2, fake, 4096, 1, 1, fake, 1024, None, None) == 3
    assert B.lib.hlq_mfma_probe(-1, fake, 4096, 1, 1, fake, 1024, None, None) == 3


def test_workspace_sizes_cover_every_path():
    # counters + room for split-K partial sums: K is never cut into slices shorter than four chunks,
    # so (K/128 + 3) // 4 slices of N fp32 values bound every GEMV plan; a few-rows GEMM needs that
    # per row; a grouped launch needs the sum over its problems
    counters = 131072
    t = ctypes.c_size_t()
    for (K, N) in [(4096, 4096), (14336, 4096), (512, 64)]:
        d = B.make_desc(K, N, 2, 128)
        slices = (K // 128 + 3) // 4
        gemv = slices * N * 4 if slices > 1 else 0
        assert B.workspace_bytes(d, 1) >= counters + gemv
        for M in (2, 4, 8):
            assert B.workspace_bytes(d, M) >= counters + M * gemv
        # the size is for exactly M rows (the K split is planned per M): never below the counters
        for M in (33, 64, 512, 2048):
            assert B.workspace_bytes(d, M) >= counters
    descs = [B.make_desc(4096, 4096, 2, 128), B.make_desc(14336, 4096, 2, 128)]
    arr = (B.HlqDesc * 2)(*descs)
    assert B.lib.hlq_gemm_batch_workspace_bytes(2, arr, 4, ctypes.byref(t)) == 0
    single = [B.workspace_bytes(d, 4) - counters for d in descs]
    assert t.value >= counters + sum(single) - 512
    assert B.lib.hlq_gemm_batch_workspace_bytes(2, arr, 1, ctypes.byref(t)) == 0
    assert t.value == B.batch_workspace_bytes(descs)
    assert B.lib.hlq_gemm_batch_workspace_bytes(0, arr, 4, ctypes.byref(t)) == 3
    assert B.lib.hlq_gemm_batch_workspace_bytes(2, arr, -1, ctypes.byref(t)) == 5
    assert B.lib.hlq_gemm_batch_workspace_bytes(2, None, 4, ctypes.byref(t)) == 1


def test_path_knobs_accept_documented_values_only():
    for v in (0, 1, 2, 3, 4, 5, 6):
        assert B.lib.hlq_set_gemv_path(v) == 0
    for v in (0, 1, 2, 3, 4):
        assert B.lib.hlq_set_gemm_path(v) == 0
    assert B.lib.hlq_set_gemv_path(7) == 3
    assert B.lib.hlq_set_gemv_path(-1) == 3
    assert B.lib.hlq_set_gemm_path(5) == 3
    assert B.lib.hlq_set_gemv_path(0) == 0 and B.lib.hlq_set_gemm_path(0) == 0


def test_status_strings():
    seen = set()
    for s in range(0, 7):
        msg = B.status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert B.status_string(99) == "unknown status"
