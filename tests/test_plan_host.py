"""Host logic of the GEMV launch planner, swept without a GPU through hlq_gemv_plan_query.

What the kernels assume about a plan: every K slice starts inside K (a slice's first chunk is used to
form addresses even for a wavefront whose own run is empty), slices cover K, slice boundaries are
even (a 256-wide quant group spans two chunks), the number of partial sums per output stays within
what hlq_workspace_bytes reserves, and the block ranges of the problems of a launch tile the grid."""
import pytest

from paper_2510_19482_amd import binding as B


def check_plan(info, nchunks, what):
    cps, ns = info.chunks_per_slice, info.slices
    assert cps >= 1 and ns >= 1, what
    assert (ns - 1) * cps < nchunks, (what, "a slice starts past K", cps, ns)
    assert ns * cps >= nchunks, (what, "slices do not cover K", cps, ns)
    assert cps % 2 == 0 or ns == 1, (what, "odd slice boundary", cps, ns)
    assert ns <= max(1, (nchunks + 3) // 4), (what, "more partial sums than the workspace holds", ns)
    assert info.blocks == info.tile_groups * ns, what
    wpt = info.waves_per_tile
    assert 1 <= wpt <= info.waves_per_workgroup and info.waves_per_workgroup % wpt == 0, what


def sweep(nchunks_range, plans, paths, Ms, N=512, q=2, G=128):
    try:
        for path in paths:
            B.set_gemv_path(path)
            for (W, cpw) in plans:
                B.set_gemv_plan(0, W, cpw)
                for M in Ms:
                    for nchunks in nchunks_range:
                        d = B.make_desc(128 * nchunks, N, q, G)
                        info = B.gemv_plan_query([d], M)[0]
                        check_plan(info, nchunks, (path, W, cpw, M, nchunks))
    finally:
        B.set_gemv_plan(0, 0, 0)
        B.set_gemv_path(B.GEMV_AUTO)


def test_default_plans_every_k():
    # the built-in choices, every K the library accepts (K = 128 .. 2^21), M = 1 and the few-rows launches
    sweep(range(1, 16385), [(0, 0)], [B.GEMV_MX, B.GEMV_LUT], [1])
    sweep(range(1, 16385), [(0, 0)], [B.GEMV_AUTO], [2, 8])


def test_default_plans_wide_launch():
    # a launch large enough for the planner's long-run regime (units >= 12000 and >= 65536)
    sweep(range(1, 2049, 3), [(0, 0)], [B.GEMV_MX, B.GEMV_LUT], [1, 4], N=128256)


def test_forced_plans():
    # every wavefront count and run length hlq_set_gemv_plan accepts in practice
    plans = [(W, cpw) for W in (1, 2, 3, 4, 8, 16) for cpw in (1, 2, 3, 4, 5, 7, 8, 13)]
    sweep(list(range(1, 700)) + list(range(16000, 16385)), plans, [B.GEMV_MX, B.GEMV_LUT], [1])
    sweep(range(1, 300), plans, [B.GEMV_AUTO], [2, 5, 8])


@pytest.mark.parametrize("G", [32, 64, 256])
def test_other_group_sizes(G):
    rows = {32: [1, 2], 64: [1, 4], 256: [1, 8]}[G]
    sweep([n for n in range(2, 1200, 2)], [(0, 0), (4, 2), (8, 7)], [B.GEMV_AUTO], rows, G=G)


def test_grouped_launch_tiles_the_grid():
    from paper_2510_19482_amd import synth
    descs = [B.make_desc(s.K, s.N, 2, 128) for s in synth.LLAMA31_8B_LAYER]
    infos = B.gemv_plan_query(descs, 1)
    spans = sorted((i.first_block, i.blocks) for i in infos)
    at = 0
    for first, n in spans:
        assert first == at
        at += n
    for d, i in zip(descs, infos):
        check_plan(i, d.K // 128, (d.K, d.N))


def test_plan_query_argument_errors():
    import ctypes
    d = B.make_desc(4096, 4096, 2, 128)
    out = (B.GemvPlanInfo * 1)()
    assert B.lib.hlq_gemv_plan_query(1, None, 1, out) == 1
    assert B.lib.hlq_gemv_plan_query(1, ctypes.byref(d), 1, None) == 1
    assert B.lib.hlq_gemv_plan_query(0, ctypes.byref(d), 1, out) == 3
    assert B.lib.hlq_gemv_plan_query(1, ctypes.byref(d), 0, out) == 3
    assert B.lib.hlq_gemv_plan_query(1, ctypes.byref(d), 1000, out) == 3
