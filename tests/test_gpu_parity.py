"""GPU parity: every operator through the C ABI against the CPU oracle, element by element.

Tolerance (stated for this build): relative L2 <= 1e-5 and max abs <= 1e-3, written in
tests/gpu_util.py.  Small shapes sweep odd sizes, ragged tiles, every variant and forced
reduction splits; the configuration layers run at full size in the launch configuration that
bench.py times.
"""
import sys

import numpy as np
import pytest
import torch

import paper_2305_08819_amd as mc
import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(autouse=True)
def _reset_tuning():
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    mc.conv2d_set_tile(0, 0, -1)
    mc.conv2d_set_order(1)
    yield
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    mc.conv2d_set_tile(0, 0, -1)
    mc.conv2d_set_order(1)


def small_inputs(desc, seed):
    k = wl.stream_key("sweep", seed)
    X = wl.uniform_pm1(k, (desc.N, desc.IH, desc.IW, desc.IC))
    W = wl.uniform_pm1(k + 1, (desc.OC, desc.FH, desc.FW, desc.IC))
    G = wl.uniform_pm1(k + 2, (desc.N, desc.OH, desc.OW, desc.OC))
    return X, W, G


# N, IH, IW, IC, OC, FH, FW, stride, pad  -- channel counts the 16-byte loaders cannot take
ODD_SHAPES = [
    (5, 12, 12, 3, 64, 3, 3, 1, 1),        # first-layer shape, several row tiles
    (2, 9, 7, 24, 40, 3, 3, 2, 1),         # IC % 4 == 0 but not % 32; ragged columns; two phases
    (3, 6, 6, 48, 20, 5, 5, 1, 2),         # more than one reduction stage per tap
    (1, 9, 9, 2, 8, 9, 9, 1, 4),           # 81 taps: beyond the tap-mask width
    (4, 8, 8, 3, 16, 3, 3, 1, 1),          # configuration 1
    (1, 5, 7, 1, 1, 3, 3, 1, 1),
    (3, 9, 6, 5, 2, 3, 2, (2, 1), (0, 1)),
    (2, 7, 7, 24, 10, 5, 5, 1, 2),
    (1, 11, 10, 3, 5, 2, 3, (3, 2), (1, 2)),
    (2, 6, 6, 16, 3, 1, 1, 2, 0),
    (2, 10, 9, 1, 3, 7, 7, 3, 3),
    (1, 3, 3, 2, 2, 3, 3, 1, 0),
    (1, 2, 2, 1, 1, 4, 4, 1, 1),           # filter larger than the map
]


@pytest.mark.parametrize("shp", ODD_SHAPES)
def test_direct_variant_odd_shapes(shp):
    say("direct %s" % (shp,))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_DIRECT, 0)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


@pytest.mark.parametrize("split", [0, 2])
@pytest.mark.parametrize("shp", ODD_SHAPES)
def test_elementwise_mfma_variant_odd_shapes(shp, split):
    """Channel counts that are not a multiple of 4 go through the element-wise MFMA kernels; those
    that are a multiple of 4 but not of 32 (24, 48, 16 here) take the 16-byte loaders with a
    partly empty last stage per tap."""
    say("elem %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    assert mc.conv2d_query_plan(mc.OP_FWD, d).variant == mc.VARIANT_MFMA
    assert mc.conv2d_query_plan(mc.OP_BWD_DATA, d).variant == mc.VARIANT_MFMA
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


# backward-data into few channels of any count (not a multiple of 4) with OC a multiple of 32:
# 16-byte loads of dY, 4-byte loads of the filter (the first layer of the VGG stack is the type)
FEW_CHANNEL_SHAPES = [
    (2, 9, 9, 5, 32, 3, 3, 2, 1),
    (3, 8, 8, 7, 64, 5, 5, 1, 2),
    (2, 6, 6, 30, 32, 3, 3, 1, 1),
    (4, 10, 7, 1, 96, 3, 2, (1, 2), (1, 0)),
]


@pytest.mark.parametrize("split", [0, 3])
@pytest.mark.parametrize("shp", FEW_CHANNEL_SHAPES)
def test_bwd_data_few_channels(shp, split):
    say("few-channel %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    pl = mc.conv2d_query_plan(mc.OP_BWD_DATA, d)
    assert pl.variant == mc.VARIANT_MFMA and (pl.tile_m, pl.tile_n) == (128, 32)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


# backward-data with very few input channels, unit stride: patch-gradient GEMM + col2im kernel
SMALL_IC_SHAPES = [
    (3, 7, 9, 3, 64, 3, 3, 1, 1),
    (2, 33, 35, 3, 32, 3, 3, 1, 1),       # several tiles along both axes, ragged edges
    (2, 9, 40, 4, 96, 3, 2, 1, (2, 0)),   # pad larger than the usual, non-square filter
    (5, 6, 5, 1, 32, 3, 3, 1, 0),         # no padding, one channel
    (2, 8, 8, 2, 64, 1, 1, 1, 0),
    (1, 5, 70, 3, 64, 2, 3, 1, (0, 2)),
]


@pytest.mark.parametrize("shp", SMALL_IC_SHAPES)
def test_bwd_data_small_ic(shp):
    say("small-ic %s" % (shp,))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, 0)
    pl = mc.conv2d_query_plan(mc.OP_BWD_DATA, d)
    assert pl.variant == mc.VARIANT_MFMA and pl.grid == d.N * ((d.IH + 3) // 4) * ((d.IW + 31) // 32)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


@pytest.mark.parametrize("split", [0, 1, 7])
@pytest.mark.parametrize("shp", SMALL_IC_SHAPES + [(3, 9, 9, 3, 32, 3, 3, 2, 1), (2, 11, 8, 1, 100, 5, 5, (1, 2), 2),
                                                   (70, 4, 4, 2, 64, 3, 3, 1, 1)])
def test_bwd_weight_small_ic(shp, split):
    """Backward-weight with at most 32 patch columns (FH*FW*IC): 64 x 32 tile, rows sliced."""
    say("small-ic wgrad %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
    assert pl.variant == mc.VARIANT_MFMA and (pl.tile_m, pl.tile_n) == (64, 32)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), ops=("bwd_weight",), label=str(shp))


# output rows of 64, 96, 128 pixels: the fast backward-weight kernel's wide-row variant
WIDE_ROW_SHAPES = [
    (1, 4, 64, 8, 32, 3, 3, 1, 1),
    (2, 6, 96, 4, 16, 3, 3, 1, 1),
    (1, 8, 128, 8, 8, 3, 3, 2, 1),
    (1, 3, 64, 12, 64, 5, 5, 1, 2),
    (2, 2, 64, 16, 32, 1, 1, 1, 0),
]


@pytest.mark.parametrize("split", [0, 1, 3])
@pytest.mark.parametrize("shp", WIDE_ROW_SHAPES)
def test_bwd_weight_wide_rows(shp, split):
    say("wide rows %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), ops=("bwd_weight",), label=str(shp))


# backward-weight with at most 32 output channels on aligned maps: the 32x128 tile (one block row)
NARROW_OC_SHAPES = [
    (4, 8, 8, 16, 32, 3, 3, 1, 1),
    (2, 16, 16, 8, 24, 5, 5, 1, 2),
    (64, 4, 4, 64, 32, 3, 3, 1, 1),      # (oh,ow,n) order with stage skipping
    (3, 16, 16, 12, 8, 1, 1, 2, 0),
]


@pytest.mark.parametrize("split", [0, 1, 5])
@pytest.mark.parametrize("shp", NARROW_OC_SHAPES)
def test_bwd_weight_narrow_tile(shp, split):
    say("narrow-oc %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    mc.conv2d_set_tile(32, 128, -1)     # the planner keeps small problems like these on 64x64
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
    assert pl.variant == mc.VARIANT_MFMA and (pl.tile_m, pl.tile_n) == (32, 128)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


# shapes the MFMA variants accept, chosen to give ragged row tiles, ragged column tiles,
# several stride phases, non-square filters/strides/pads and more than 32 taps
MFMA_SHAPES = [
    (3, 7, 5, 32, 96, 3, 3, 2, 1),
    (2, 9, 9, 64, 32, 3, 3, 1, 1),
    (5, 6, 7, 32, 160, 1, 1, 1, 0),
    (2, 8, 8, 32, 64, 1, 1, 2, 0),
    (1, 12, 11, 64, 64, 5, 5, 1, 2),
    (2, 13, 9, 32, 32, 3, 2, (2, 1), (0, 1)),
    (2, 10, 10, 32, 64, 7, 7, 3, 3),
    (1, 9, 8, 96, 224, 2, 3, (3, 2), (1, 2)),
    (128, 2, 2, 64, 96, 3, 3, 1, 1),       # position-major rows
    (128, 3, 3, 32, 32, 3, 3, 1, 1),
    (256, 4, 4, 32, 64, 5, 5, 1, 2),
    (128, 4, 4, 64, 32, 3, 3, 2, 1),
    (1, 1, 1, 32, 32, 1, 1, 1, 0),
    (2, 5, 5, 32, 32, 3, 3, 1, 2),         # pad larger than (F-1)/2
]


@pytest.mark.parametrize("split", [0, 1, 3])
@pytest.mark.parametrize("shp", MFMA_SHAPES)
def test_mfma_variant_shapes(shp, split):
    say("mfma %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT):
        assert mc.conv2d_query_plan(op, d).variant == mc.VARIANT_MFMA
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


# ---- every compiled tile, forced ---------------------------------------------------------------
# The planner rarely leaves the 64x64 tile on small problems, so each compiled (tile, row order,
# loader) instantiation is forced here through conv2d_set_tile / conv2d_set_tuning, the plan is
# checked to be the forced one, and the result is compared with the oracle.
GATHER_TILES = [(128, 128), (128, 64), (64, 64), (128, 32)]
GATHER_FORCED_SHAPES = [
    (128, 4, 4, 64, 160, 3, 3, 1, 1),     # channels on the 32-grid, ragged column tiles, (y,x,n) order possible
    (128, 3, 5, 48, 72, 3, 3, 1, 1),      # channel counts off the 32-grid: partly empty last stage per tap
    (128, 6, 6, 32, 64, 3, 3, 2, 1),      # stride phases in backward-data
    (5, 9, 7, 32, 96, 3, 3, 1, 1),        # ragged row tiles (315 rows), (n,y,x) order only
]


@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("pm", [0, 1])
@pytest.mark.parametrize("tile", GATHER_TILES, ids=lambda t: "%dx%d" % t)
@pytest.mark.parametrize("shp", GATHER_FORCED_SHAPES)
def test_forced_gather_tiles(shp, tile, pm, split):
    d = mc.make_desc(*shp)
    if pm and d.N % tile[0] != 0:
        pytest.skip("(y,x,n) order needs a batch that is a multiple of the row tile")
    say("forced gather %s tile %s pm %d split %d" % (shp, tile, pm, split))
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    mc.conv2d_set_tile(tile[0], tile[1], pm)
    for op in (mc.OP_FWD, mc.OP_BWD_DATA):
        pl = mc.conv2d_query_plan(op, d)
        assert pl.kernel == mc.KERNEL_GATHER and (pl.tile_m, pl.tile_n) == tile, (op, pl.tile_m, pl.tile_n)
        # a forced slice count is clamped to half the tile's stages
        assert pl.pos_major == pm and (pl.split == split or 1 < pl.split < split), (op, pl.pos_major, pl.split)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), ops=("fwd", "bwd_data"), label=str(shp))


WGRAD_TILES = [(128, 128), (64, 128), (128, 64), (64, 64), (32, 128)]
# shape, row order, kernel family the plan must name
WGRAD_FORCED_SHAPES = [
    ((8, 8, 8, 64, 160, 3, 3, 1, 1), 0, "fast"),       # aligned map, (n,oh,ow) order, ragged tiles both ways
    ((64, 4, 4, 64, 160, 3, 3, 1, 1), 1, "fast"),      # (oh,ow,n) order with stage skipping
    ((2, 4, 64, 16, 160, 3, 3, 1, 1), 0, "fast"),      # wide rows (OW = 64)
    ((3, 4, 4, 16, 32, 3, 3, 1, 1), 0, "fast"),        # 48 rows: the last 32-row stage is half empty
    ((5, 8, 4, 8, 16, 3, 3, 1, 1), 0, "fast"),         # 160 rows, five stages
    ((3, 7, 5, 32, 160, 3, 3, 1, 1), 0, "generic"),    # map the fast kernel does not take
    ((32, 3, 3, 64, 96, 3, 3, 1, 1), 1, "generic"),    # (oh,ow,n) order in the generic kernel
    ((4, 8, 8, 6, 160, 3, 3, 1, 1), 0, "elem"),        # input channels not a multiple of 4
]


@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("tile", WGRAD_TILES, ids=lambda t: "%dx%d" % t)
@pytest.mark.parametrize("case", WGRAD_FORCED_SHAPES, ids=lambda c: "%s-%s" % (c[2], "x".join(map(str, c[0][:5]))))
def test_forced_wgrad_tiles(case, tile, split):
    shp, pm, family = case
    if tile == (32, 128) and family != "fast":
        pytest.skip("the one-block-row tile exists in the fast kernel only")
    if family == "elem" and tile[1] != 64:
        pytest.skip("the element-wise X loader is compiled for 64-wide tiles")
    say("forced wgrad %s %s tile %s split %d" % (shp, family, tile, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    mc.conv2d_set_tile(tile[0], tile[1], pm)
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
    assert pl.kernel == (mc.KERNEL_WGRAD_FAST if family == "fast" else mc.KERNEL_WGRAD)
    assert (pl.tile_m, pl.tile_n) == tile and pl.pos_major == pm
    assert pl.split == split or (split > 1 and 1 <= pl.split < split), pl.split   # clamped to half the stages
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), ops=("bwd_weight",), label=str(shp))


# partial last stage of the first-layer backward-weight kernel (rows not a multiple of 32, more than 32)
@pytest.mark.parametrize("shp", [(3, 9, 9, 3, 32, 3, 3, 2, 1), (7, 5, 5, 1, 64, 3, 3, 1, 1), (1, 10, 10, 3, 96, 3, 3, 1, 1)])
@pytest.mark.parametrize("split", [1, 2])
def test_bwd_weight_small_ic_partial_last_stage(shp, split):
    say("small-ic wgrad partial stage %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    assert (d.N * d.OH * d.OW) % 32 != 0 and d.N * d.OH * d.OW > 32
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    assert mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d).kernel == mc.KERNEL_FIRST_LAYER
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), ops=("bwd_weight",), label=str(shp))


def test_bwd_weight_one_row_wide_map_keeps_row_major_order():
    """An output map of one row of 64 pixels is small enough for (oh,ow,n) order, but the fast
    kernel's wide-row variant runs in (n,oh,ow) order only: the plan must say so and run."""
    d = mc.make_desc(32, 1, 64, 64, 64, 3, 3, 1, 1)
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
    assert pl.kernel == mc.KERNEL_WGRAD_FAST and pl.pos_major == 0
    gu.check_all_ops(d, *small_inputs(d, 99), label="1x64 map")
    d = mc.make_desc(32, 1, 64, 16, 32, 1, 3, 1, (0, 1))
    assert mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d).pos_major == 0
    gu.check_all_ops(d, *small_inputs(d, 98), label="1x64 map, 1x3 filter")


def test_mfma_and_direct_agree_with_plan_defaults():
    d = mc.make_desc(2, 9, 9, 64, 32, 3, 3, 1, 1)
    gu.check_all_ops(d, *small_inputs(d, 7))


def test_bitwise_reproducible_and_deconv_alias():
    d = mc.make_desc(128, 4, 4, 64, 64, 3, 3, 1, 1)
    X, W, G = small_inputs(d, 11)
    for op in ("fwd", "bwd_data", "bwd_weight"):
        a, b = gu.operands(op, X, W, G)
        r1, r2 = gu.run_gpu(op, d, a, b), gu.run_gpu(op, d, a, b)
        assert np.array_equal(r1, r2), op
    r3 = gu.run_gpu("bwd_data", d, G, W, entry=mc.deconv2d)
    assert np.array_equal(r3, gu.run_gpu("bwd_data", d, G, W))


def test_side_stream():
    d = mc.make_desc(2, 9, 9, 64, 32, 3, 3, 1, 1)
    X, W, G = small_inputs(d, 13)
    st = torch.cuda.Stream()
    for op in ("fwd", "bwd_data", "bwd_weight"):
        a, b = gu.operands(op, X, W, G)
        got = gu.run_gpu(op, d, a, b, stream=st)
        rel, mx = gu.errors(got, gu.run_oracle(op, d, a, b))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL


def test_host_threads_launch_on_their_own_streams():
    """Four host threads, each with its own stream, workspace and shape, enqueue all three operators
    repeatedly at the same time (plan cache, per-device set-up and error text are shared or per thread);
    every result must be the one a single thread gets."""
    import threading
    shapes = [(64, 4, 4, 128, 256, 3, 3, 1, 1), (32, 8, 8, 64, 64, 3, 3, 1, 1), (8, 16, 16, 32, 48, 3, 3, 2, 1),
              (128, 2, 2, 256, 256, 3, 3, 1, 1)]
    jobs = []
    for i, shp in enumerate(shapes):
        d = mc.make_desc(*shp)
        X, W, G = small_inputs(d, 900 + i)
        ref = {op: gu.run_gpu(op, d, *gu.operands(op, X, W, G)) for op in ("fwd", "bwd_data", "bwd_weight")}
        dev = {k: torch.from_numpy(v).cuda() for k, v in (("X", X), ("W", W), ("G", G))}
        need = max(mc.conv2d_workspace_bytes(o, d) for o in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT))
        jobs.append({"d": d, "ref": ref, "dev": dev, "st": torch.cuda.Stream(),
                     "ws": torch.empty(max(need, 16) // 4, dtype=torch.float32, device="cuda"),
                     "Y": torch.empty((d.N, d.OH, d.OW, d.OC), dtype=torch.float32, device="cuda"),
                     "dX": torch.empty((d.N, d.IH, d.IW, d.IC), dtype=torch.float32, device="cuda"),
                     "dW": torch.empty((d.OC, d.FH, d.FW, d.IC), dtype=torch.float32, device="cuda")})
    torch.cuda.synchronize()
    errors = []

    def work(j):
        try:
            for _ in range(20):
                mc.conv2d_fwd(j["dev"]["X"], j["dev"]["W"], j["Y"], j["d"], ws=j["ws"], stream=j["st"])
                mc.conv2d_bwd_data(j["dev"]["G"], j["dev"]["W"], j["dX"], j["d"], ws=j["ws"], stream=j["st"])
                mc.conv2d_bwd_weight(j["dev"]["X"], j["dev"]["G"], j["dW"], j["d"], ws=j["ws"], stream=j["st"])
        except Exception as e:      # reported by the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i, j in enumerate(jobs):
        for op, key in (("fwd", "Y"), ("bwd_data", "dX"), ("bwd_weight", "dW")):
            assert np.array_equal(j[key].cpu().numpy(), j["ref"][op]), (shapes[i], op)


BIAS_ACT_SHAPES = [
    (3, 9, 9, 64, 48, 3, 3, 1, 1),       # 16-byte loaders
    (2, 7, 6, 5, 7, 3, 2, (2, 1), (1, 0)),   # element-wise loaders, odd output count (scalar tail of the combine pass)
    (64, 4, 4, 64, 64, 3, 3, 1, 1),      # (y,x,n) row order
    (2, 8, 8, 32, 10, 1, 1, 1, 0),
]


@pytest.mark.parametrize("variant,split", [(None, 0), (None, 3), ("direct", 0)])
@pytest.mark.parametrize("shp", BIAS_ACT_SHAPES)
def test_fwd_bias_act(shp, variant, split):
    """Biased convolution with leaky-ReLU in the epilogue (unsliced) or in the combine pass (sliced)."""
    say("bias-act %s %s split=%d" % (shp, variant, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_DIRECT if variant == "direct" else mc.VARIANT_MFMA, split)
    X, W, _ = small_inputs(d, hash(shp) & 0xffff)
    bias = wl.uniform_pm1(wl.stream_key("bias", d.OC), (d.OC,))
    tX, tW, tb = torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(bias).cuda()
    for b, tbias, slope in ((bias, tb, 0.125), (None, None, 0.0), (bias, tb, 1.0)):
        buf, out = gu.guarded((d.N, d.OH, d.OW, d.OC))
        mc.conv2d_fwd_bias_act(tX, tW, tbias, out, d, slope)
        torch.cuda.synchronize()
        assert gu.guards_intact(buf)
        rel, mx = gu.errors(out.cpu().numpy(), gu.oracle.conv2d_fwd_bias_act(X, W, b, slope, (d.sh, d.sw), (d.ph, d.pw)))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (slope, rel, mx)
    # no bias, slope 1: exactly the plain forward operator
    buf, out = gu.guarded((d.N, d.OH, d.OW, d.OC))
    mc.conv2d_fwd_bias_act(tX, tW, None, out, d, 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), gu.run_gpu("fwd", d, X, W))


@pytest.mark.parametrize("shp", [(8, 32, 32, 3, 64, 3, 3, 1, 1), (3, 9, 11, 1, 20, 5, 5, 2, 2), (2, 7, 7, 3, 16, 3, 3, (2, 1), 1),
                                 (5, 6, 6, 6, 8, 2, 2, 1, 0)])
def test_fwd_u8_pixels(shp):
    """First-layer forward from 8-bit pixels, converted on load with scale 1/255."""
    say("u8 %s" % (shp,))
    d = mc.make_desc(*shp)
    k = wl.stream_key("u8", *shp[:5])
    X8 = ((wl.uniform_pm1(k, (d.N, d.IH, d.IW, d.IC)).astype(np.float64) + 1.0) * 127.99).astype(np.uint8)
    W = wl.uniform_pm1(k + 1, (d.OC, d.FH, d.FW, d.IC))
    scale = 1.0 / 255.0
    buf, out = gu.guarded((d.N, d.OH, d.OW, d.OC))
    mc.conv2d_fwd_u8(torch.from_numpy(X8).cuda(), scale, torch.from_numpy(W).cuda(), out, d)
    torch.cuda.synchronize()
    assert gu.guards_intact(buf)
    rel, mx = gu.errors(out.cpu().numpy(), gu.oracle.conv2d_fwd_u8(X8, scale, W, (d.sh, d.sw), (d.ph, d.pw)))
    assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (rel, mx)
    assert int(X8.max()) > 200 and int(X8.min()) < 50


def test_fwd_u8_rejects_other_shapes():
    d = mc.make_desc(2, 8, 8, 64, 64, 3, 3, 1, 1)
    x8 = torch.zeros((2, 8, 8, 64), dtype=torch.uint8, device="cuda")
    w = torch.zeros((64, 3, 3, 64), device="cuda")
    y = torch.zeros((2, 8, 8, 64), device="cuda")
    with pytest.raises(mc.Mi355ConvError):
        mc.conv2d_fwd_u8(x8, 1.0, w, y, d)


def test_fully_connected_as_1x1_convolution():
    """The paper's fully-connected layer (Fig. 2 `fullconnect`) is the 1x1 operator on a 1x1 map:
    a CIFAR classifier head, 512 features -> 10 classes, all three operators."""
    d = mc.make_desc(128, 1, 1, 512, 10, 1, 1, 1, 0)
    gu.check_all_ops(d, *small_inputs(d, 77), label="fc 512->10")
    d = mc.make_desc(128, 1, 1, 512, 512, 1, 1, 1, 0)
    gu.check_all_ops(d, *small_inputs(d, 78), label="fc 512->512")


# M, N, K of C[M,N]: classifier head, square, ragged everything, K not a multiple of 4, a long reduction
MATMUL_SHAPES = [(128, 10, 512), (256, 512, 512), (33, 7, 50), (100, 36, 27), (64, 64, 4096), (5, 1000, 64), (1, 1, 1)]


@pytest.mark.parametrize("split", [0, 3])
@pytest.mark.parametrize("shape", MATMUL_SHAPES)
def test_matmul_fully_connected(shape, split):
    """The fully-connected layer's three matrix multiplies (paper Fig. 2 fullconnect; Sec. II matMul /
    matMulT1) through matmul_f32 against the oracle's matrix multiply."""
    M, N, K = shape
    say("matmul %s split=%d" % (shape, split))
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, split)
    k = wl.stream_key("matmul", M, N, K)
    cases = [(mc.MATMUL_NT, (M, K), (N, K), False, True), (mc.MATMUL_NN, (M, K), (K, N), False, False),
             (mc.MATMUL_TN, (K, M), (K, N), True, False)]
    for i, (kind, sa, sb, ta, tb) in enumerate(cases):
        A = wl.uniform_pm1(k + 2 * i, sa)
        B = wl.uniform_pm1(k + 2 * i + 1, sb)
        buf, out = gu.guarded((M, N))
        need = mc.matmul_workspace_bytes(kind, M, N, K)
        ws = torch.full((max(need, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
        mc.matmul_f32(kind, gu.nan_fenced(A), gu.nan_fenced(B), out, ws=ws)
        torch.cuda.synchronize()
        assert gu.guards_intact(buf)
        rel, mx = gu.errors(out.cpu().numpy(), gu.oracle.matmul(A, B, ta, tb))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (kind, rel, mx)


@pytest.mark.parametrize("shp,split", [((128, 5, 3, 64, 256, 3, 3, 1, 1), 8), ((128, 3, 3, 64, 192, 3, 3, 1, 1), 5),
                                       ((64, 6, 6, 32, 128, 5, 5, 1, 2), 4),
                                       # filter larger than the activations and than an XCD's L2: ranks enumerate
                                       # class by class with the (slice, column tile) index slowest
                                       ((64, 3, 3, 256, 512, 3, 3, 1, 1), 8), ((128, 4, 3, 160, 544, 3, 3, 1, 1), 3)])
def test_balanced_dealing_odd_grids(shp, split):
    """(y,x,n) row order with grids that are not multiples of 256 and maps that are not square: the
    longest-first dealing (a permutation of the workgroups) must leave every result intact."""
    say("balanced %s split=%d" % (shp, split))
    d = mc.make_desc(*shp)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    mc.conv2d_set_tile(64, 64, 1)
    grids = []
    for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT):
        pl = mc.conv2d_query_plan(op, d)
        assert pl.pos_major == 1
        grids.append(pl.grid)
        ranks = {mc.conv2d_query_workgroup(op, d, wg)[0] for wg in range(pl.grid)}
        assert ranks == set(range(pl.grid))
    assert max(grids) > 256
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


# shape, tile, forced slices: (y,x,n) launches that the region-wise order takes, chosen so that every
# factor of the division among the XCDs occurs (quarters, halves along one axis only; one or several
# image groups; one or several (slice, column) groups), with slices by source
# channels (slice count divides the 32-channel chunks) and by stages (it does not), grids that are
# resident at once (snake dealing, also with a partial last lap of 32) and grids that are not.
REGION_CASES = [
    ((128, 8, 8, 64, 64, 3, 3, 1, 1), (64, 64), 2),      # quarters x 2 image groups
    ((128, 4, 4, 128, 256, 3, 3, 1, 1), (64, 64), 4),    # small map, filter-heavy: slice/column groups
    ((128, 4, 4, 96, 256, 3, 3, 1, 1), (64, 64), 2),     # 3 chunks per tap, 2 slices: slices by stages
    ((128, 6, 4, 256, 256, 3, 3, 1, 1), (64, 64), 2),    # 6x4 map: regions of 3x2 positions
    ((64, 8, 8, 64, 256, 3, 3, 1, 1), (64, 64), 1),      # one row tile per position: no image groups
    ((128, 5, 4, 64, 256, 3, 3, 1, 1), (64, 64), 2),     # odd height: halves along x only
    ((128, 4, 6, 64, 256, 3, 3, 1, 1), (64, 64), 3),     # slices by stages (3 does not divide the 2 chunks of a tap)
    ((256, 16, 16, 32, 128, 3, 3, 1, 1), (64, 64), 1),   # 2048 workgroups: not resident at once
    ((128, 6, 6, 32, 256, 5, 5, 1, 2), (64, 64), 1),     # 36 workgroups per XCD: partial last lap
    ((256, 8, 8, 64, 128, 3, 3, 1, 1), (128, 64), 2),    # 128-row tiles
    ((128, 8, 8, 64, 64, 3, 3, 1, 1), (128, 32), 2),
]


@pytest.mark.parametrize("case", REGION_CASES, ids=lambda c: "x".join(map(str, c[0][:5])) + "-%dx%d-s%d" % (c[1] + (c[2],)))
def test_region_wise_order(case):
    """The region-wise workgroup order is a permutation of the tiles: results are bitwise those of the
    older order and within tolerance of the oracle."""
    shp, tile, split = case
    say("region-wise order %s tile %s split %d" % (shp, tile, split))
    d = mc.make_desc(*shp)
    X, W, G = small_inputs(d, hash(shp) & 0xffff)
    mc.conv2d_set_tuning(mc.VARIANT_MFMA, split)
    mc.conv2d_set_tile(tile[0], tile[1], 1)
    taken = 0
    for op, name in ((mc.OP_FWD, "fwd"), (mc.OP_BWD_DATA, "bwd_data")):
        a, b = gu.operands(name, X, W, G)
        mc.conv2d_set_order(1)
        pl = mc.conv2d_query_plan(op, d)
        assert pl.pos_major == 1 and pl.kernel == mc.KERNEL_GATHER
        ranks = {mc.conv2d_query_workgroup(op, d, wg)[0] for wg in range(pl.grid)}
        assert ranks == set(range(pl.grid))
        taken += pl.order == mc.ORDER_REGIONS
        got = gu.run_gpu(name, d, a, b)
        mc.conv2d_set_order(0)
        assert mc.conv2d_query_plan(op, d).order != mc.ORDER_REGIONS
        old = gu.run_gpu(name, d, a, b)
        assert np.array_equal(got, old), "%s %s: the two orders differ" % (shp, name)
        rel, mx = gu.errors(got, gu.run_oracle(name, d, a, b))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (shp, name, rel, mx)
    assert taken >= 1, "no operator of %s took the region-wise order" % (shp,)



# shape, forced slices: (oh,ow,n) backward-weight launches that the group-wise order takes, with one or
# several slice groups, grids of one to nine workgroups per CU and an odd slice count
WGRAD_GROUP_CASES = [((128, 4, 4, 256, 512, 3, 3, 1, 1), 0), ((128, 4, 4, 256, 512, 3, 3, 1, 1), 1),
                     ((128, 4, 4, 256, 512, 3, 3, 1, 1), 8), ((128, 8, 8, 128, 256, 3, 3, 1, 1), 0),
                     ((128, 8, 8, 128, 256, 3, 3, 1, 1), 4), ((128, 2, 2, 256, 256, 3, 3, 1, 1), 2),
                     ((96, 4, 4, 192, 192, 3, 3, 1, 1), 8), ((128, 4, 4, 128, 128, 3, 3, 1, 1), 0)]


@pytest.mark.parametrize("case", WGRAD_GROUP_CASES, ids=lambda c: "x".join(map(str, c[0][:5])) + "-s%d" % c[1])
def test_group_wise_order_bwd_weight(case):
    """Backward-weight with every XCD owning a group of output-channel tiles, input-channel tiles and
    slices: a permutation of the workgroups, so results are bitwise those of the older order."""
    shp, split = case
    say("group-wise backward-weight %s split %d" % (shp, split))
    d = mc.make_desc(*shp)
    X, W, G = small_inputs(d, hash(shp) & 0xffff)
    mc.conv2d_set_tuning(mc.VARIANT_AUTO, split)
    a, b = gu.operands("bwd_weight", X, W, G)
    mc.conv2d_set_order(1)
    pl = mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d)
    assert pl.kernel == mc.KERNEL_WGRAD_FAST and pl.pos_major == 1 and pl.order == mc.ORDER_REGIONS, (pl.kernel, pl.order)
    ranks = {mc.conv2d_query_workgroup(mc.OP_BWD_WEIGHT, d, wg)[0] for wg in range(pl.grid)}
    assert ranks == set(range(pl.grid))
    got = gu.run_gpu("bwd_weight", d, a, b)
    mc.conv2d_set_order(0)
    assert mc.conv2d_query_plan(mc.OP_BWD_WEIGHT, d).order != mc.ORDER_REGIONS
    old = gu.run_gpu("bwd_weight", d, a, b)
    assert np.array_equal(got, old), "%s: the two orders differ" % (shp,)
    rel, mx = gu.errors(got, gu.run_oracle("bwd_weight", d, a, b))
    assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, (shp, rel, mx)



def _seeded_shapes(count, seed):
    """A fixed list of shapes drawn once from a seeded generator: every loader, row order, tile and
    slicing rule meets sizes nobody picked by hand."""
    rng = np.random.default_rng(seed)
    chans_in = [1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 48, 64, 96]
    chans_out = [1, 2, 3, 4, 8, 10, 16, 32, 48, 64, 96, 128]
    out = []
    while len(out) < count:
        n = int(rng.choice([1, 2, 3, 5, 8, 32, 64, 128], p=[.2, .2, .15, .1, .1, .1, .1, .05]))
        ih, iw = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        fh, fw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        ic, oc = int(rng.choice(chans_in)), int(rng.choice(chans_out))
        if ih + 2 * ph < fh or iw + 2 * pw < fw:
            continue
        if n * ih * iw * ic > 400000 or n * ih * iw * oc > 400000:
            continue
        out.append((n, ih, iw, ic, oc, fh, fw, (sh, sw), (ph, pw)))
    return out


@pytest.mark.parametrize("shp", _seeded_shapes(48, 20230508))
def test_seeded_random_shapes(shp):
    say("seeded %s" % (shp,))
    d = mc.make_desc(*shp)
    gu.check_all_ops(d, *small_inputs(d, hash(shp) & 0xffff), label=str(shp))


def test_concurrent_streams_inception_branches():
    """Independent operators enqueued on different streams at once (the paper's asynchronous APIs
    run branches of a network in parallel, Sec. III Layer-4 / Sec. IV): the 1x1, 3x3 and 5x5
    branches of configuration 4 on one shared input, then backward-data and backward-weight of one
    layer side by side.  Each operator has its own workspace; results must equal those of the
    same calls made one after the other on one stream bit for bit, and meet the oracle tolerance."""
    n = 16
    branches = [mc.make_desc(n, 16, 16, 256, 64, 1, 1, 1, 0), mc.make_desc(n, 16, 16, 256, 128, 3, 3, 1, 1),
                mc.make_desc(n, 16, 16, 256, 32, 5, 5, 1, 2)]
    k = wl.stream_key("streams")
    X = wl.uniform_pm1(k, (n, 16, 16, 256))
    Ws = [wl.uniform_pm1(k + 1 + i, (d.OC, d.FH, d.FW, d.IC)) for i, d in enumerate(branches)]
    tX = torch.from_numpy(X).cuda()
    tWs = [torch.from_numpy(w).cuda() for w in Ws]

    def launch(streams):
        outs, keep = [], []
        for d, tw, st in zip(branches, tWs, streams):
            y = torch.full((d.N, d.OH, d.OW, d.OC), float("nan"), dtype=torch.float32, device="cuda")
            need = mc.conv2d_workspace_bytes(mc.OP_FWD, d)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            keep.append(ws)
            if st is not None:
                st.wait_stream(torch.cuda.current_stream())
            mc.conv2d_fwd(tX, tw, y, d, ws=ws, stream=st)
            outs.append(y)
        torch.cuda.synchronize()
        return [o.cpu().numpy() for o in outs]

    serial = launch([None, None, None])
    parallel = launch([torch.cuda.Stream() for _ in branches])
    for d, w, a, b in zip(branches, Ws, serial, parallel):
        assert np.array_equal(a, b)
        rel, mx = gu.errors(b, gu.run_oracle("fwd", d, X, w))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL

    # backward-data || backward-weight of the 3x3 branch
    d = branches[1]
    G = wl.uniform_pm1(k + 9, (d.N, d.OH, d.OW, d.OC))
    tG = torch.from_numpy(G).cuda()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    dX = torch.full((d.N, d.IH, d.IW, d.IC), float("nan"), dtype=torch.float32, device="cuda")
    dW = torch.full((d.OC, d.FH, d.FW, d.IC), float("nan"), dtype=torch.float32, device="cuda")
    ws1 = torch.empty(max(mc.conv2d_workspace_bytes(mc.OP_BWD_DATA, d), 16), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(mc.conv2d_workspace_bytes(mc.OP_BWD_WEIGHT, d), 16), dtype=torch.uint8, device="cuda")
    for st in (s1, s2):
        st.wait_stream(torch.cuda.current_stream())
    mc.conv2d_bwd_data(tG, tWs[1], dX, d, ws=ws1, stream=s1)
    mc.conv2d_bwd_weight(tX, tG, dW, d, ws=ws2, stream=s2)
    torch.cuda.synchronize()
    for op, got, (a, b) in (("bwd_data", dX, (G, Ws[1])), ("bwd_weight", dW, (X, G))):
        rel, mx = gu.errors(got.cpu().numpy(), gu.run_oracle(op, d, a, b))
        assert rel <= gu.REL_L2_TOL and mx <= gu.MAX_ABS_TOL, op


def test_hip_graph_replay_matches_eager():
    """The entry points only enqueue kernels (no allocation, no memset, no synchronisation), so a
    sequence of operators can be captured into a HIP graph.  Every replay - with eager launches and
    synchronisations in between - must reproduce the eager results bit for bit."""
    descs = [mc.make_desc(64, 4, 4, 64, 128, 3, 3, 1, 1),      # sliced reductions + combine pass, (y,x,n) order
             mc.make_desc(8, 16, 16, 32, 64, 3, 3, 2, 1),      # stride phases
             mc.make_desc(16, 12, 12, 3, 32, 3, 3, 1, 1)]      # first-layer kernels
    k = wl.stream_key("graph")
    items = []
    for i, d in enumerate(descs):
        X = torch.from_numpy(wl.uniform_pm1(k + 3 * i, (d.N, d.IH, d.IW, d.IC))).cuda()
        W = torch.from_numpy(wl.uniform_pm1(k + 3 * i + 1, (d.OC, d.FH, d.FW, d.IC))).cuda()
        G = torch.from_numpy(wl.uniform_pm1(k + 3 * i + 2, (d.N, d.OH, d.OW, d.OC))).cuda()
        outs = [torch.empty((d.N, d.OH, d.OW, d.OC), device="cuda"), torch.empty_like(X), torch.empty_like(W)]
        wss = [torch.empty(max(mc.conv2d_workspace_bytes(op, d), 16), dtype=torch.uint8, device="cuda")
               for op in (mc.OP_FWD, mc.OP_BWD_DATA, mc.OP_BWD_WEIGHT)]
        items.append((d, X, W, G, outs, wss))

    def enqueue():
        for d, X, W, G, outs, wss in items:
            mc.conv2d_fwd(X, W, outs[0], d, ws=wss[0])
            mc.conv2d_bwd_data(G, W, outs[1], d, ws=wss[1])
            mc.conv2d_bwd_weight(X, G, outs[2], d, ws=wss[2])

    enqueue()
    torch.cuda.synchronize()
    eager = [[o.clone() for o in it[4]] for it in items]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enqueue()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        for it in items:                       # poison, then eager work of the program in between
            for o in it[4]:
                o.fill_(float("nan"))
        scratch = torch.randn(1 << 16, device="cuda").sum().item()
        assert scratch == scratch
        graph.replay()
        torch.cuda.synchronize()
        for it, ref in zip(items, eager):
            for o, r in zip(it[4], ref):
                assert torch.equal(o, r), rep


def _distinct_shapes(layers):
    seen, out = set(), []
    for l in layers:
        key = (l.N, l.IH, l.IW, l.IC, l.OC, l.FH, l.FW, l.stride, l.pad)
        # the VGG-16 stack is kept whole: its inputs come from the chain through the oracle
        if key in seen and l not in wl.CFG5:
            continue
        seen.add(key)
        out.append(l)
    return out


FULL_LAYERS = _distinct_shapes(wl.all_layers())


@pytest.mark.parametrize("layer", FULL_LAYERS, ids=[l.name for l in FULL_LAYERS])
def test_configuration_layers_full_size(layer):
    say("full-size %s" % (layer,))
    d = gu.desc_of(layer)
    # the VGG-16 stack takes its activations from a chain through the oracle (conv, ReLU, pooling)
    t = gu.vgg_chain_inputs(layer) if layer in wl.CFG5 else wl.make_inputs(layer)
    # every operator runs twice: results must be bitwise reproducible
    stats = gu.check_all_ops(d, t["X"], t["W"], t["G"], label=layer.name, twice=True)
    say("  %s" % {k: "rel=%.2e max=%.2e" % v for k, v in stats.items()})
