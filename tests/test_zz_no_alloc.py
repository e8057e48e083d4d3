"""conv2d_bwd_weight_noalloc (slice partials in the library's own device array) against
conv2d_bwd_weight (caller workspace), through the C ABI: two calls in a row, the second with a
smaller input, so that what the first call left in the shared array must not reach the second
call's result.  Also against the oracle, at the tolerance of every GPU parity test."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2305_08819_amd as mc
import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _inputs(d, seed):
    k = wl.stream_key("noalloc", seed)
    X = wl.uniform_pm1(k, (d.N, d.IH, d.IW, d.IC))
    G = wl.uniform_pm1(k + 2, (d.N, d.OH, d.OW, d.OC))
    return X, G


def _raw_noalloc(lib, tX, tG, out, d):
    """The entry point through ctypes alone: raw pointers, torch's current stream."""
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return lib.conv2d_bwd_weight_noalloc(ctypes.c_void_p(tX.data_ptr()), ctypes.c_void_p(tG.data_ptr()),
                                         ctypes.c_void_p(out.data_ptr()), ctypes.byref(d), st)


def test_noalloc_matches_workspace_entry_point_twice_in_a_row():
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    mc.conv2d_set_tile(0, 0, -1)
    lib = mc.load()
    mc.conv2d_init()
    assert mc.conv2d_noalloc_scratch_bytes() == 32 << 20
    # first a layer whose partials fill a good part of the array, then a smaller one
    shapes = [(64, 16, 16, 64, 128, 3, 3, 1, 1), (32, 8, 8, 64, 64, 3, 3, 1, 1)]
    needs = []
    for i, shp in enumerate(shapes):
        d = mc.make_desc(*shp)
        pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
        assert pl.split > 1 and 0 < pl.workspace_bytes <= mc.conv2d_noalloc_scratch_bytes()
        needs.append(pl.workspace_bytes)
        X, G = _inputs(d, i)
        tX, tG = gu.nan_fenced(X), gu.nan_fenced(G)
        buf, out = gu.guarded((d.OC, d.FH, d.FW, d.IC))
        before = torch.cuda.memory_allocated()
        rc = _raw_noalloc(lib, tX, tG, out, d)
        assert rc == 0, lib.conv2d_status_string(rc)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert gu.guards_intact(buf)
        got = out.cpu().numpy()
        ref_gpu = gu.run_gpu("bwd_weight", d, X, G)          # existing entry point, caller workspace
        # same plan, same kernels, fixed combine order: the two entry points agree bit for bit,
        # which is inside the bar of every parity test (rel-L2 <= 1e-5, max-abs <= 1e-3)
        rel, mx = gu.errors(got, ref_gpu.astype(np.float64))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (shp, rel, mx)
        assert np.array_equal(got, ref_gpu), shp
        rel, mx = gu.errors(got, gu.run_oracle("bwd_weight", d, X, G))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (shp, rel, mx)
    assert needs[1] < needs[0]


def test_noalloc_rejects_shapes_beyond_its_array():
    lib = mc.load()
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, 64)      # many slices of a 9.4 MB result: far beyond 32 MiB
    try:
        d = mc.make_desc(128, 4, 4, 512, 512, 3, 3, 1, 1)
        assert mc.conv2d_workspace_bytes(mc.OP_BWD_WEIGHT, d) > mc.conv2d_noalloc_scratch_bytes()
        # rejected before any HIP call: dummy (aligned, non-null) pointers are never touched
        rc = lib.conv2d_bwd_weight_noalloc(ctypes.c_void_p(256), ctypes.c_void_p(512), ctypes.c_void_p(768),
                                           ctypes.byref(d), None)
        assert rc == -3
    finally:
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
