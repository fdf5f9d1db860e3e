"""hlq_lut_gemv_static (the entry point for callers that cannot allocate: its split-K scratch is a
fixed array inside the library) against hlq_lut_gemv on the same inputs, through the C ABI.

Both calls run the same kernels with the same plan, and the split-K sum is taken in slice order, so
the two outputs must agree bit for bit; the oracle check on top guards against both being wrong.
Two calls in a row share the library's array, the second on a smaller problem: what the first call
left there must not leak into the second.  (The file name sorts after the other tests on purpose: it
runs last.)"""
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


def say(*a):
    print(*a, flush=True)


def make_case(K, N, q, G, key):
    codes, S, Z = synth.make_weight(K, N, q, G, "noalloc", key)
    x = synth.make_x(1, K, "noalloc", key)
    d, packed = pack_on_gpu(codes, S, Z, q, G)
    ref = c_oracle.gemm_f64(x, codes, S, Z, q, G)
    return d, packed, dev(x[0]), ref


def run_pair(case, out_f32):
    d, packed, x, ref = case
    dt = torch.float32 if out_f32 else torch.float16
    # outputs are allocated BEFORE the calls under test; poisoned so that a column nobody writes shows
    y_static = torch.full((d.N,), float("nan"), dtype=dt, device="cuda")
    y_ws = torch.full((d.N,), float("nan"), dtype=dt, device="cuda")
    ws = B.alloc_workspace(d, 1)
    torch.cuda.synchronize()
    rc = B.lib.hlq_lut_gemv_static(ctypes.byref(d), int(packed.data_ptr()), int(x.data_ptr()), int(y_static.data_ptr()),
                                   1 if out_f32 else 0, int(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, B.status_string(rc)
    B.hlq_lut_gemv(d, packed, x, y=y_ws, out_f32=out_f32, ws=ws)
    torch.cuda.synchronize()
    a, b = y_static.cpu().numpy(), y_ws.cpu().numpy()
    assert np.array_equal(a.view(np.uint32 if out_f32 else np.uint16), b.view(np.uint32 if out_f32 else np.uint16)), \
        "static-scratch entry point differs from hlq_lut_gemv"
    err = O.row_rel_err(a.astype(np.float64)[None, :], ref).max()
    say("      row err vs oracle", float(err))
    assert err <= TOL


@pytest.mark.parametrize("path", ["mx", "lut"])
@pytest.mark.parametrize("plan", [(0, 0), (4, 2)], ids=["default-plan", "many-slices"])
def test_static_scratch_two_calls_second_smaller(path, plan):
    B.set_gemv_path(B.GEMV_LUT if path == "lut" else B.GEMV_MX)
    B.set_gemv_plan(0, plan[0], plan[1])
    try:
        # K = 14336 is split across workgroups under every plan (partial sums + counters in the scratch
        # array); the second problem is smaller in K and N, with a ragged last tile
        big = make_case(14336, 4096, 2, 128, "big")
        small = make_case(4096, 1000, 2, 128, "small")
        for p in B.gemv_plan_query([big[0]], 1) + B.gemv_plan_query([small[0]], 1):
            say("   plan: slices", p.slices, "chunks/slice", p.chunks_per_slice, "waves/tile", p.waves_per_tile)
        assert B.gemv_plan_query([big[0]], 1)[0].slices > 1
        for out_f32 in (False, True):
            say("   call 1 (14336 x 4096)", path, plan, "f32" if out_f32 else "f16")
            run_pair(big, out_f32)
            say("   call 2 (4096 x 1000)")
            run_pair(small, out_f32)
            say("   call 3 (14336 x 4096 again)")
            run_pair(big, out_f32)
    finally:
        B.set_gemv_plan(0, 0, 0)
        B.set_gemv_path(B.GEMV_AUTO)


def test_static_scratch_other_formats():
    # three planes with 64-wide groups, then four planes: other instantiations, same scratch array
    for (K, N, q, G) in ((8192, 2048, 3, 64), (2048, 520, 4, 128)):
        say("   ", K, N, q, G)
        run_pair(make_case(K, N, q, G, f"{q}-{G}"), True)


def test_static_scratch_rejects_what_does_not_fit():
    # 16 K slices of a 128256-wide matrix are 8.2 MB of partial sums: more than the array holds.
    # Refused on the host, before any launch (fake pointers are never dereferenced).
    d = B.make_desc(8192, 128256, 2, 128)
    B.set_gemv_plan(0, 1, 1)
    try:
        assert B.gemv_plan_query([d], 1)[0].slices * d.N * 4 > B.STATIC_SCRATCH_BYTES
        rc = B.lib.hlq_lut_gemv_static(ctypes.byref(d), 0x1000, 0x1000, 0x1000, 0, None)
        assert rc == 4, B.status_string(rc)
    finally:
        B.set_gemv_plan(0, 0, 0)
