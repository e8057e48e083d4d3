"""Host-side tests of the C ABI that need no GPU: the library loads, exports every declared
symbol, validates arguments before any HIP call, and plans sensibly."""
import ctypes
import os
import re

import pytest

import paper_2305_08819_amd as mc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mc.LIB_PATH):
        from paper_2305_08819_amd import build
        build.build()
    return mc.load()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "mi355conv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(conv2d_\w+|deconv2d|matmul_\w+)\s*\(", hdr))
    assert declared == set(mc.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    assert lib.conv2d_status_string(0) == b"ok"
    for code in range(-6, 0):
        assert lib.conv2d_status_string(code) not in (b"ok", b"unknown status")
    assert lib.conv2d_status_string(-99) == b"unknown status"


def _call(lib, name, a, b, c, desc, ws=0, nbytes=0):
    return getattr(lib, name)(ctypes.c_void_p(a), ctypes.c_void_p(b), ctypes.c_void_p(c),
                              ctypes.byref(desc) if desc is not None else None,
                              ctypes.c_void_p(ws), nbytes, None)


@pytest.mark.parametrize("name", ["conv2d_fwd", "conv2d_bwd_data", "deconv2d", "conv2d_bwd_weight"])
def test_argument_errors_before_any_hip_call(lib, name):
    good = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)
    assert _call(lib, name, 0, 256, 512, good) == -1            # null tensor
    assert _call(lib, name, 256, 512, 768, None) == -1          # null desc
    assert _call(lib, name, 256, 512, 772, good) == -4          # misaligned
    for field, val in (("N", 0), ("IC", -1), ("sh", 0), ("pw", -1), ("FH", 0)):
        bad = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)
        setattr(bad, field, val)
        assert _call(lib, name, 256, 512, 768, bad) == -2, field
    assert _call(lib, name, 256, 512, 768, mc.make_desc(1, 2, 2, 4, 4, 5, 5, 1, 0)) == -2   # OH <= 0
    assert _call(lib, name, 256, 512, 768, mc.make_desc(1 << 20, 64, 64, 64, 64, 3, 3, 1, 1)) == -2  # 2^32 elems


def test_bias_act_argument_errors_before_any_hip_call(lib):
    good = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)

    def call(x, w, b, y, desc, slope=0.1):
        return lib.conv2d_fwd_bias_act(ctypes.c_void_p(x), ctypes.c_void_p(w), ctypes.c_void_p(b), ctypes.c_void_p(y),
                                       ctypes.byref(desc), ctypes.c_float(slope), ctypes.c_void_p(0), 0, None)
    assert call(0, 256, 0, 512, good) == -1                      # null tensor (a null bias is allowed)
    assert call(256, 512, 1026, 768, good) == -4                 # bias not 4-byte aligned
    assert call(256, 512, 1024, 772, good) == -4                 # misaligned output
    assert call(256, 512, 1024, 768, good, float("nan")) == -5   # NaN slope
    bad = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)
    bad.OC = 0
    assert call(256, 512, 1024, 768, bad) == -2


def test_fwd_u8_argument_errors_before_any_hip_call(lib):
    def call(x8, w, y, desc, scale=0.5):
        return lib.conv2d_fwd_u8(ctypes.c_void_p(x8), ctypes.c_float(scale), ctypes.c_void_p(w), ctypes.c_void_p(y),
                                 ctypes.byref(desc), None)
    first = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)
    assert call(0, 512, 768, first) == -1                       # null pixels
    assert call(257, 512, 0, first) == -1                       # null output (odd pixel address is fine)
    assert call(257, 516, 768, first) == -4                     # misaligned filter
    assert call(257, 512, 768, first, float("nan")) == -5
    assert call(256, 512, 768, mc.make_desc(4, 8, 8, 64, 16, 3, 3, 1, 1)) == -5   # not a first-layer shape


def test_workspace_errors(lib):
    d = mc.make_desc(128, 2, 2, 512, 512, 3, 3, 1, 1)
    need = mc.conv2d_workspace_bytes(mc.OP_FWD, d)
    assert need > 0
    assert _call(lib, "conv2d_fwd", 256, 512, 768, d, 0, 0) == -3
    assert _call(lib, "conv2d_fwd", 256, 512, 768, d, 1024, need - 1) == -3
    assert _call(lib, "conv2d_fwd", 256, 512, 768, d, 1028, need) == -4


def test_plans(lib):
    q = mc.conv2d_query_plan
    # 3 input channels: first-layer kernels (one MFMA stage, 128 x 64 tile forward; 4 x 32 pixels per
    # workgroup backward-data; 64 x 32 backward-weight); odd output channels: backward-weight goes direct
    p = q(mc.OP_FWD, mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_MFMA and (p.tile_m, p.tile_n, p.split) == (128, 64, 1) and p.grid == 2
    p = q(mc.OP_BWD_DATA, mc.make_desc(128, 32, 32, 3, 64, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_MFMA and p.grid == 128 * 8 and p.workspace_bytes == 0
    p = q(mc.OP_BWD_WEIGHT, mc.make_desc(128, 32, 32, 3, 64, 3, 3, 1, 1))
    assert (p.tile_m, p.tile_n) == (64, 32) and p.split > 1
    # 5 input channels with a 3x3 filter (45 patch columns): element-wise loaders
    p = q(mc.OP_FWD, mc.make_desc(4, 8, 8, 5, 16, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_MFMA and p.tile_n == 32
    p = q(mc.OP_BWD_WEIGHT, mc.make_desc(4, 8, 8, 3, 15, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_DIRECT and p.workspace_bytes == 0
    p = q(mc.OP_FWD, mc.make_desc(128, 32, 32, 64, 128, 3, 3, 2, 1))
    assert p.variant == mc.VARIANT_MFMA and p.split == 1 and p.grid >= 256
    p = q(mc.OP_FWD, mc.make_desc(128, 2, 2, 512, 512, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_MFMA and p.pos_major == 1 and p.split > 1
    assert p.workspace_bytes == p.split * 128 * 2 * 2 * 512 * 4
    p = q(mc.OP_BWD_WEIGHT, mc.make_desc(128, 32, 32, 64, 64, 3, 3, 1, 1))
    assert p.variant == mc.VARIANT_MFMA and p.split > 1
    with pytest.raises(mc.Mi355ConvError):
        q(7, mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1))
    # tuning override
    mc.conv2d_set_tuning(mc.VARIANT_DIRECT, 0)
    try:
        assert q(mc.OP_FWD, mc.make_desc(128, 2, 2, 512, 512, 3, 3, 1, 1)).variant == mc.VARIANT_DIRECT
    finally:
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    with pytest.raises(mc.Mi355ConvError):
        mc.conv2d_set_tuning(5, 0)


def test_longest_first_dealing_is_a_permutation_and_balances(lib):
    """Small maps in (y,x,n) order have workgroups of unequal length; the host deals them to the 256 CUs
    (hardware ids 256 apart share a CU while the grid is resident).  Every id must map to a distinct
    rank, and the busiest CU must stay close to the mean - for grids that are and are not multiples of 256."""
    cases = [(mc.OP_FWD, mc.make_desc(128, 4, 4, 512, 512, 3, 3, 1, 1)),         # 1024 workgroups, taps 9/6/4
             (mc.OP_BWD_DATA, mc.make_desc(128, 4, 4, 256, 512, 3, 3, 1, 1)),
             (mc.OP_BWD_WEIGHT, mc.make_desc(128, 4, 4, 512, 512, 3, 3, 1, 1)),  # 576: 64 CUs hold three
             (mc.OP_BWD_WEIGHT, mc.make_desc(128, 4, 4, 256, 512, 3, 3, 1, 1)),  # 288
             (mc.OP_FWD, mc.make_desc(128, 8, 8, 256, 256, 3, 3, 1, 1))]
    for op, d, region_wise in [c + (1,) for c in cases] + [c + (0,) for c in cases]:
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 1 if op == mc.OP_BWD_WEIGHT else 0)   # backward-weight: one slice
        mc.conv2d_set_order(region_wise)
        pl = mc.conv2d_query_plan(op, d)
        assert pl.pos_major == 1 and pl.grid > 256
        # every XCD owns a group of the tiles unless that is switched off
        want = mc.ORDER_REGIONS if region_wise else mc.ORDER_LONGEST
        assert pl.order == want, (op, region_wise, pl.order)
        seen, load = set(), [0] * 256
        for wg in range(pl.grid):
            rank, work = mc.conv2d_query_workgroup(op, d, wg)
            assert 0 <= rank < pl.grid and rank not in seen
            seen.add(rank)
            load[wg % 256] += work
        mean = sum(load) / 256.0
        if pl.grid <= 1024:     # resident at once (64x64 tiles: four per CU); larger grids refill as workgroups finish
            assert max(load) <= 1.5 * mean if pl.grid < 512 else max(load) <= 1.1 * mean, (op, pl.grid, max(load), mean)
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    mc.conv2d_set_order(1)
    with pytest.raises(mc.Mi355ConvError):
        mc.conv2d_set_order(2)
    # all workgroups alike: identity
    d = mc.make_desc(128, 16, 16, 256, 64, 1, 1, 1, 0)
    assert mc.conv2d_query_workgroup(mc.OP_FWD, d, 5) == (5, 1)
    with pytest.raises(mc.Mi355ConvError):
        mc.conv2d_query_workgroup(mc.OP_FWD, d, 1 << 20)


def _launcher_takes(op, d, pl):
    """The launchers' preconditions, restated from their documentation (not from the planner)."""
    ohow = d.OH * d.OW
    tile = (pl.tile_m, pl.tile_n)
    if pl.kernel == mc.KERNEL_DIRECT:
        return True
    if pl.kernel == mc.KERNEL_FIRST_LAYER:
        ok = d.FH * d.FW * d.IC <= 32
        if op == mc.OP_BWD_DATA:
            ok = ok and d.sh == 1 and d.sw == 1 and d.IC <= 4 and d.OC % 32 == 0 and (d.FH + 3) * (d.FW + 31) <= 224
        return ok
    if pl.kernel == mc.KERNEL_WGRAD_FAST:
        narrow = 32 % d.OW == 0 and (ohow % 32 == 0 or 32 % ohow == 0)
        wide = d.OW > 32 and d.OW % 32 == 0
        if not (narrow or wide) or d.IC % 4 or d.OC % 4:
            return False
        if pl.pos_major and (wide or d.N % 32 or ohow > 64):
            return False
        return tile in ((128, 128), (64, 128), (128, 64), (64, 64), (32, 128))
    if pl.kernel == mc.KERNEL_WGRAD:
        if d.OC % 4:
            return False
        if d.IC % 4:
            return not pl.pos_major and tile in ((64, 64), (128, 64))
        if pl.pos_major and d.N % 32:
            return False
        return tile in ((128, 128), (64, 128), (128, 64), (64, 64))
    if pl.pos_major and d.N % pl.tile_m:
        return False
    if pl.kernel == mc.KERNEL_GATHER_ELEM:
        return tile in ((128, 64), (64, 64), (128, 32))
    src, dst = (d.OC, d.IC) if op == mc.OP_BWD_DATA else (d.IC, d.OC)
    if src % 4:
        return False
    if op == mc.OP_BWD_DATA and dst % 4:
        return tile == (128, 32)
    return tile in ((128, 128), (128, 64), (64, 64), (128, 32))


def test_every_plan_is_one_its_launcher_takes(lib):
    """Sweep of shapes x overrides through the host-only planner: every plan must meet the
    preconditions of the launcher it names (a plan that does not would surface as a launch
    error on the GPU).  Includes one-row maps of 64 pixels, where (oh,ow,n) order and the
    wide-row backward-weight kernel used to be planned together."""
    import itertools
    shapes = []
    for n, (ih, iw), ic, oc, (f, s_, p) in itertools.product(
            (1, 3, 32, 128), ((1, 64), (2, 2), (4, 4), (8, 8), (16, 16), (5, 7), (1, 128), (2, 32), (32, 32), (3, 96)),
            (3, 4, 6, 16, 48, 64), (4, 10, 32, 48, 160),
            ((1, 1, 0), (3, 1, 1), (3, 2, 1), (5, 1, 2), ((1, 3), 1, (0, 1)), ((3, 1), (2, 1), (1, 0)))):
        shapes.append((n, ih, iw, ic, oc) + ((f, f) if isinstance(f, int) else f) + (s_, p))
    overrides = [(0, 0, -1, 0), (0, 0, 1, 0), (0, 0, 0, 3), (128, 128, 1, 2), (32, 128, -1, 0), (128, 64, -1, 5)]
    checked = 0
    try:
        for bm, bn, pm, split in overrides:
            mc.conv2d_set_tile(bm, bn, pm)
            mc.conv2d_set_tuning(mc.VARIANT_AUTO, split)
            for shp in shapes:
                d = mc.make_desc(*shp)
                if d.OH <= 0 or d.OW <= 0:
                    continue
                for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT):
                    pl = mc.conv2d_query_plan(op, d)       # raises if the library itself finds the plan unlaunchable
                    assert _launcher_takes(op, d, pl), (shp, op, (bm, bn, pm, split), pl.kernel, pl.tile_m, pl.tile_n, pl.pos_major)
                    assert pl.split >= 1 and (pl.grid >= 1 or pl.kernel == mc.KERNEL_DIRECT)
                    checked += 1
    finally:
        mc.conv2d_set_tile(0, 0, -1)
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    assert checked > 10000
    # the shape that used to get an unlaunchable plan
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, mc.make_desc(32, 1, 64, 64, 64, 3, 3, 1, 1))
    assert pl.kernel == mc.KERNEL_WGRAD_FAST and pl.pos_major == 0


def test_noalloc_argument_errors_before_any_hip_call(lib):
    good = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)

    def call(x, g, w, desc):
        return lib.conv2d_bwd_weight_noalloc(ctypes.c_void_p(x), ctypes.c_void_p(g), ctypes.c_void_p(w),
                                             ctypes.byref(desc) if desc is not None else None, None)
    assert call(0, 512, 768, good) == -1
    assert call(256, 512, 768, None) == -1
    assert call(256, 516, 768, good) == -4
    bad = mc.make_desc(4, 8, 8, 3, 16, 3, 3, 1, 1)
    bad.N = 0
    assert call(256, 512, 768, bad) == -2
    assert mc.conv2d_noalloc_scratch_bytes() == 32 << 20
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, 64)
    try:
        big = mc.make_desc(128, 4, 4, 512, 512, 3, 3, 1, 1)
        assert mc.conv2d_workspace_bytes(mc.OP_BWD_WEIGHT, big) > mc.conv2d_noalloc_scratch_bytes()
        assert call(256, 512, 768, big) == -3       # needs more than the library's array
    finally:
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)


def test_matmul_argument_errors_and_plans_before_any_hip_call(lib):
    def call(kind, a, b, c, M, N, K):
        return lib.matmul_f32(kind, ctypes.c_void_p(a), ctypes.c_void_p(b), ctypes.c_void_p(c), M, N, K, ctypes.c_void_p(0), 0, None)
    assert call(mc.MATMUL_NT, 0, 512, 768, 4, 4, 4) == -1
    assert call(mc.MATMUL_NN, 256, 516, 768, 4, 4, 4) == -4
    assert call(mc.MATMUL_TN, 256, 512, 768, 0, 4, 4) == -2
    assert call(7, 256, 512, 768, 4, 4, 4) == -5
    assert mc.matmul_workspace_bytes(7, 4, 4, 4) == 0
    # the weight gradient of a 512 -> 10 classifier head over a batch of 128 is a sliced reduction or a single tile
    assert mc.matmul_workspace_bytes(mc.MATMUL_TN, 10, 512, 128) % 16 == 0


def test_region_and_group_wise_orders_map_ids_onto_tiles_one_to_one(lib):
    """Sweep of shapes, tiles and slice counts through the planner: wherever a plan names the region-wise
    (forward, backward-data) or group-wise (backward-weight) order, the kernels' own decode functions
    (conv2d_query_tile runs them on the host) must send the workgroup ids of the launch to every
    (row tile, column tile, slice) exactly once."""
    shapes = []
    for n in (64, 128, 256):
        for hw in ((2, 2), (4, 4), (8, 8), (16, 16), (6, 4), (5, 4), (4, 6), (3, 5), (8, 2)):
            for ic, oc in ((64, 64), (128, 256), (256, 128), (512, 512), (96, 160), (192, 64)):
                shapes.append((n, hw[0], hw[1], ic, oc, 3, 3, 1, 1))
    shapes += [(128, 8, 8, 64, 128, 5, 5, 1, 2), (128, 8, 8, 64, 256, 3, 3, 2, 1), (128, 7, 7, 64, 128, 3, 3, 1, 1),
               (256, 32, 32, 32, 64, 3, 3, 1, 1), (128, 8, 8, 128, 128, 3, 1, 1, (1, 0)), (128, 4, 4, 256, 512, 1, 3, 1, (0, 1))]
    checked = {mc.OP_FWD: 0, mc.OP_BWD_DATA: 0, mc.OP_BWD_WEIGHT: 0}
    try:
        for shp in shapes:
            d = mc.make_desc(*shp)
            for split in (0, 2, 3, 8):
                for tile in ((0, 0), (128, 64)):
                    mc.conv2d_set_tuning(mc.VARIANT_AUTO, split)
                    mc.conv2d_set_tile(tile[0], tile[1], -1)
                    for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT):
                        pl = mc.conv2d_query_plan(op, d)
                        if pl.order != mc.ORDER_REGIONS:
                            if pl.variant == mc.VARIANT_MFMA and pl.grid > 0:
                                with pytest.raises(mc.Mi355ConvError):
                                    mc.conv2d_query_tile(op, d, 0)
                            continue
                        if pl.grid > 4096:      # keep the sweep short
                            continue
                        tiles = [mc.conv2d_query_tile(op, d, wg) for wg in range(pl.grid)]
                        assert len(set(tiles)) == pl.grid, (shp, split, tile, op)
                        rows = {t[0] for t in tiles}
                        cols = {t[1] for t in tiles}
                        slices = {t[2] for t in tiles}
                        assert slices == set(range(pl.split)), (shp, split, op, sorted(slices))
                        assert rows == set(range(len(rows))) and cols == set(range(len(cols)))
                        assert len(rows) * len(cols) * pl.split == pl.grid, (shp, split, op, len(rows), len(cols), pl.split, pl.grid)
                        if op == mc.OP_BWD_WEIGHT:
                            assert len(rows) == -(-d.OC // pl.tile_m) and len(cols) == -(-(d.FH * d.FW * d.IC) // pl.tile_n)
                        else:
                            dst_c = d.IC if op == mc.OP_BWD_DATA else d.OC
                            m = d.N * (d.IH * d.IW if op == mc.OP_BWD_DATA else d.OH * d.OW)
                            assert len(cols) == -(-dst_c // pl.tile_n) and len(rows) == -(-m // pl.tile_m)
                        checked[op] += 1
    finally:
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
        mc.conv2d_set_tile(0, 0, -1)
    assert min(checked.values()) >= 20, checked


def test_plan_queries_from_many_threads(lib):
    """The planner and its plan cache are shared by all threads of a process: eight threads that query
    plans and workspace sizes for interleaved shapes at once (ctypes drops the interpreter lock during a
    call) get exactly what one thread gets."""
    import threading
    shapes = [(128, hw, hw, ic, oc, 3, 3, 1, 1) for hw in (2, 4, 8, 16) for ic in (64, 128, 256) for oc in (64, 256, 512)]
    shapes += [(64, 7, 5, 24, 40, 3, 3, 2, 1), (128, 32, 32, 64, 128, 3, 3, 2, 1), (128, 16, 16, 256, 64, 1, 1, 1, 0)]

    def answers(order):
        out = {}
        for i in order:
            d = mc.make_desc(*shapes[i])
            for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT):
                pl = mc.conv2d_query_plan(op, d)
                out[(i, op)] = (pl.variant, pl.tile_m, pl.tile_n, pl.split, pl.pos_major, pl.grid, pl.workspace_bytes,
                                pl.kernel, pl.order, mc.conv2d_workspace_bytes(op, d),
                                mc.conv2d_query_workgroup(op, d, pl.grid - 1) if pl.grid else None)
        return out

    want = answers(range(len(shapes)))
    got, errors = [None] * 8, []

    def work(t):
        try:
            order = list(range(len(shapes)))
            order = order[3 * t:] + order[:3 * t]      # every thread its own order over all shapes
            if t % 2:
                order.reverse()
            for _ in range(3):
                got[t] = answers(order)
        except Exception as e:      # reported by the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for t in range(8):
        assert got[t] == want, t
