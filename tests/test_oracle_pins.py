"""Pins for the CPU oracle (oracle/conv_oracle.c): nothing here touches the GPU path.

The paper prints no worked example for its conv\\deconv operators (Sec. III Layer-1, Sec. IV),
so each pin is something mathematics fixes independently of the oracle's loop nest:
hand-written closed forms (tests/golden), delta filters, the 1x1 == GEMM special case
(numpy matmul), second formulations with a different loop structure (pad-and-slice, scatter,
im2col matrix), the adjoint identity, exact finite differences and a library cross-check
(torch CPU fp64).  Shapes use IC != OC, FH != FW, sh != sw, ph != pw so that a transposed
operand, swapped axis, flipped filter or wrong padding side fails at least one pin.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def rnd(*shape):
    return rng.standard_normal(shape).astype(np.float32)


def rel(a, b):
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


# ---- second forms (different loop structure, numpy fp64) --------------------------------
def fwd_pad_slice(X, W, s, p):
    (sh, sw), (ph, pw) = s, p
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    OH, OW = oracle.out_size(IH, FH, sh, ph), oracle.out_size(IW, FW, sw, pw)
    Xp = np.zeros((N, IH + 2 * ph, IW + 2 * pw, IC))
    Xp[:, ph:ph + IH, pw:pw + IW] = X
    Y = np.zeros((N, OH, OW, OC))
    for fh in range(FH):
        for fw in range(FW):
            sl = Xp[:, fh:fh + (OH - 1) * sh + 1:sh, fw:fw + (OW - 1) * sw + 1:sw, :]
            Y += sl @ W[:, fh, fw, :].astype(np.float64).T
    return Y


def bwd_data_scatter(G, W, ihw, s, p):
    (sh, sw), (ph, pw) = s, p
    N, OH, OW, OC = G.shape
    _, FH, FW, IC = W.shape
    IH, IW = ihw
    dXp = np.zeros((N, IH + 2 * ph + FH, IW + 2 * pw + FW, IC))
    for oh in range(OH):
        for ow in range(OW):
            for fh in range(FH):
                for fw in range(FW):
                    dXp[:, oh * sh + fh, ow * sw + fw, :] += \
                        G[:, oh, ow, :].astype(np.float64) @ W[:, fh, fw, :].astype(np.float64)
    return dXp[:, ph:ph + IH, pw:pw + IW, :]


def bwd_weight_im2col(X, G, fhw, s, p):
    (sh, sw), (ph, pw) = s, p
    N, IH, IW, IC = X.shape
    _, OH, OW, OC = G.shape
    FH, FW = fhw
    Xp = np.zeros((N, IH + 2 * ph, IW + 2 * pw, IC))
    Xp[:, ph:ph + IH, pw:pw + IW] = X
    cols = np.zeros((N * OH * OW, FH * FW * IC))
    for fh in range(FH):
        for fw in range(FW):
            sl = Xp[:, fh:fh + (OH - 1) * sh + 1:sh, fw:fw + (OW - 1) * sw + 1:sw, :]
            cols[:, (fh * FW + fw) * IC:(fh * FW + fw + 1) * IC] = sl.reshape(-1, IC)
    return (G.reshape(-1, OC).astype(np.float64).T @ cols).reshape(OC, FH, FW, IC)


SHAPES = [
    # N, IH, IW, IC, OC, FH, FW, (sh,sw), (ph,pw)
    (2, 5, 7, 3, 4, 3, 3, (1, 1), (1, 1)),
    (1, 8, 8, 1, 1, 3, 3, (2, 2), (1, 1)),
    (3, 9, 6, 5, 2, 3, 2, (2, 1), (0, 1)),
    (2, 7, 7, 2, 3, 5, 5, (1, 1), (2, 2)),
    (1, 11, 10, 3, 5, 2, 3, (3, 2), (1, 2)),
    (2, 6, 6, 4, 3, 1, 1, (2, 2), (0, 0)),
    (1, 4, 4, 2, 2, 3, 3, (1, 1), (2, 2)),
    (2, 10, 9, 1, 3, 7, 7, (3, 3), (3, 3)),
    (1, 3, 3, 2, 2, 3, 3, (1, 1), (0, 0)),
]


@pytest.mark.parametrize("shp", SHAPES)
def test_second_forms(shp):
    N, IH, IW, IC, OC, FH, FW, s, p = shp
    X, W = rnd(N, IH, IW, IC), rnd(OC, FH, FW, IC)
    Y = oracle.conv2d_fwd(X, W, s, p)
    assert rel(Y, fwd_pad_slice(X, W, s, p)) < 1e-12
    G = rnd(*Y.shape)
    assert rel(oracle.conv2d_bwd_data(G, W, (IH, IW), s, p),
               bwd_data_scatter(G, W, (IH, IW), s, p)) < 1e-12
    assert rel(oracle.conv2d_bwd_weight(X, G, (FH, FW), s, p),
               bwd_weight_im2col(X, G, (FH, FW), s, p)) < 1e-12


# ---- closed forms -------------------------------------------------------------------------
def test_allones_golden_fwd():
    tbl = np.loadtxt(os.path.join(GOLD, "allones_3x3_s1_p1_4x4.txt"))
    for IC, OC in ((1, 1), (5, 2)):
        Y = oracle.conv2d_fwd(np.ones((2, 4, 4, IC)), np.ones((OC, 3, 3, IC)), 1, 1)
        for n, oc in itertools.product(range(2), range(OC)):
            assert np.array_equal(Y[n, :, :, oc], IC * tbl)


def test_allones_golden_bwd_data_stride2():
    reach = np.loadtxt(os.path.join(GOLD, "bwd_data_reach_32_to_16_3x3_s2_p1.txt"))
    OC, IC = 3, 2
    dX = oracle.conv2d_bwd_data(np.ones((1, 16, 16, OC)), np.ones((OC, 3, 3, IC)), (32, 32), 2, 1)
    expect = OC * np.outer(reach, reach)
    for ic in range(IC):
        assert np.array_equal(dX[0, :, :, ic], expect)


def test_allones_bwd_weight_closed_form():
    N, H, Wd, IC, OC = 3, 6, 5, 2, 4
    dW = oracle.conv2d_bwd_weight(np.ones((N, H, Wd, IC)), np.ones((N, H, Wd, OC)), (3, 3), 1, 1)
    for fh, fw in itertools.product(range(3), range(3)):
        assert np.all(dW[:, fh, fw, :] == N * (H - abs(fh - 1)) * (Wd - abs(fw - 1)))


def test_1x1_stride2_unreached_pixels_are_zero():
    G, W = rnd(2, 4, 4, 3), rnd(3, 1, 1, 5)
    dX = oracle.conv2d_bwd_data(G, W, (8, 8), 2, 0)
    assert np.all(dX[:, 1::2] == 0) and np.all(dX[:, :, 1::2] == 0)
    assert rel(dX[:, ::2, ::2], G.astype(np.float64) @ W[:, 0, 0, :].astype(np.float64)) < 1e-12


# ---- delta filters (pin correlation-not-convolution, padding side, index direction) -------
def test_delta_filter_identity_bitwise():
    C = 4
    X = rnd(2, 6, 5, C)
    for F in (1, 3, 5):
        W = np.zeros((C, F, F, C), np.float32)
        for c in range(C):
            W[c, F // 2, F // 2, c] = 1
        assert np.array_equal(oracle.conv2d_fwd(X, W, 1, F // 2), X.astype(np.float64))


def test_shifted_delta_shifts_input():
    C = 2
    X = rnd(1, 6, 7, C)
    W = np.zeros((C, 3, 3, C), np.float32)
    for c in range(C):
        W[c, 0, 2, c] = 1           # tap (fh=0, fw=2): Y[oh,ow] = X[oh-1, ow+1]
    Y = oracle.conv2d_fwd(X, W, 1, 1)
    expect = np.zeros_like(Y)
    expect[:, 1:, :-1] = X[:, :-1, 1:]
    assert np.array_equal(Y, expect)
    # the adjoint shifts the other way: dX[ih,iw] = G[ih+1, iw-1]
    dX = oracle.conv2d_bwd_data(X, W, (6, 7), 1, 1)
    e2 = np.zeros_like(dX)
    e2[:, :-1, 1:] = X[:, 1:, :-1]
    assert np.array_equal(dX, e2)


# ---- 1x1 stride-1 == GEMM -------------------------------------------------------------------
def test_1x1_is_gemm():
    N, H, Wd, IC, OC = 2, 3, 5, 7, 4
    X, W, G = rnd(N, H, Wd, IC), rnd(OC, 1, 1, IC), rnd(N, H, Wd, OC)
    Xm, Wm, Gm = (a.astype(np.float64) for a in (X.reshape(-1, IC), W.reshape(OC, IC),
                                                 G.reshape(-1, OC)))
    assert rel(oracle.conv2d_fwd(X, W).reshape(-1, OC), Xm @ Wm.T) < 1e-13
    assert rel(oracle.conv2d_bwd_data(G, W, (H, Wd)).reshape(-1, IC), Gm @ Wm) < 1e-13
    assert rel(oracle.conv2d_bwd_weight(X, G, (1, 1)).reshape(OC, IC), Gm.T @ Xm) < 1e-13


# ---- adjoint / trilinear identity ---------------------------------------------------------
@pytest.mark.parametrize("shp", SHAPES)
def test_adjoint_identity(shp):
    N, IH, IW, IC, OC, FH, FW, s, p = shp
    X, W = rnd(N, IH, IW, IC), rnd(OC, FH, FW, IC)
    Y = oracle.conv2d_fwd(X, W, s, p)
    G = rnd(*Y.shape)
    a = float(np.sum(Y * G))
    b = float(np.sum(X.astype(np.float64) * oracle.conv2d_bwd_data(G, W, (IH, IW), s, p)))
    c = float(np.sum(W.astype(np.float64) * oracle.conv2d_bwd_weight(X, G, (FH, FW), s, p)))
    scale = float(np.sum(np.abs(Y * G))) + 1e-300
    assert abs(a - b) / scale < 1e-12 and abs(a - c) / scale < 1e-12


# ---- exact finite differences (the loss <fwd(X,W),G> is linear in W and in X) --------------
def test_finite_difference_bwd_weight_and_data():
    N, IH, IW, IC, OC, FH, FW, s, p = 2, 5, 6, 2, 3, 3, 3, (2, 1), (1, 0)
    X, W = rnd(N, IH, IW, IC), rnd(OC, FH, FW, IC)
    G = rnd(*oracle.conv2d_fwd(X, W, s, p).shape).astype(np.float64)
    dW = oracle.conv2d_bwd_weight(X, G, (FH, FW), s, p)
    for j in range(W.size):
        e = np.zeros(W.size, np.float32)
        e[j] = 1
        fd = float(np.sum(oracle.conv2d_fwd(X, e.reshape(W.shape), s, p) * G))
        assert abs(fd - dW.ravel()[j]) < 1e-10
    dX = oracle.conv2d_bwd_data(G, W, (IH, IW), s, p)
    for j in range(X.size):
        e = np.zeros(X.size, np.float32)
        e[j] = 1
        fd = float(np.sum(oracle.conv2d_fwd(e.reshape(X.shape), W, s, p) * G))
        assert abs(fd - dX.ravel()[j]) < 1e-10


# ---- linearity and per-image independence -------------------------------------------------
def test_linearity_and_batch_permutation():
    X1, X2, W = rnd(3, 6, 6, 2), rnd(3, 6, 6, 2), rnd(4, 3, 3, 2)
    # power-of-two coefficients keep a*X1 + b*X2 exact in fp32
    lhs = oracle.conv2d_fwd((2 * X1 + 0.5 * X2).astype(np.float32), W, 2, 1)
    assert rel(lhs, 2 * oracle.conv2d_fwd(X1, W, 2, 1) + 0.5 * oracle.conv2d_fwd(X2, W, 2, 1)) < 1e-6
    perm = [2, 0, 1]
    assert np.array_equal(oracle.conv2d_fwd(X1[perm], W, 2, 1), oracle.conv2d_fwd(X1, W, 2, 1)[perm])


# ---- library cross-check: torch CPU fp64 -----------------------------------------------------
@pytest.mark.parametrize("shp", SHAPES)
def test_torch_cpu_fp64_crosscheck(shp):
    torch = pytest.importorskip("torch")
    N, IH, IW, IC, OC, FH, FW, s, p = shp
    X, W = rnd(N, IH, IW, IC), rnd(OC, FH, FW, IC)
    xt = torch.tensor(X, dtype=torch.float64).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(W, dtype=torch.float64).permute(0, 3, 1, 2).requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=s, padding=p)
    Y = oracle.conv2d_fwd(X, W, s, p)
    assert rel(Y, yt.detach().permute(0, 2, 3, 1).numpy()) < 1e-12
    G = rnd(*Y.shape)
    yt.backward(torch.tensor(G, dtype=torch.float64).permute(0, 3, 1, 2))
    assert rel(oracle.conv2d_bwd_data(G, W, (IH, IW), s, p),
               xt.grad.permute(0, 2, 3, 1).numpy()) < 1e-12
    assert rel(oracle.conv2d_bwd_weight(X, G, (FH, FW), s, p),
               wt.grad.permute(0, 2, 3, 1).numpy()) < 1e-12


# ---- degenerate cases ---------------------------------------------------------------------
def test_empty_and_filter_larger_than_input():
    assert oracle.conv2d_fwd(rnd(0, 4, 4, 2), rnd(3, 3, 3, 2), 1, 1).shape == (0, 4, 4, 3)
    assert oracle.conv2d_fwd(rnd(1, 2, 2, 2), rnd(3, 5, 5, 2), 1, 0).shape == (1, 0, 0, 3)
    # filter larger than the map but padding makes it fit: one output pixel sees the whole map
    X, W = rnd(1, 2, 2, 1), rnd(1, 4, 4, 1)
    Y = oracle.conv2d_fwd(X, W, 1, 1)
    assert Y.shape == (1, 1, 1, 1)
    assert abs(Y[0, 0, 0, 0] - float(np.sum(X[0, :, :, 0].astype(np.float64) *
                                            W[0, 1:3, 1:3, 0]))) < 1e-13


# ---- the seeded generators (shared by both sides; no conv arithmetic) -----------------------
def test_generators_are_reproducible_and_scaled():
    l = wl.CFG1[0]
    a, b = wl.make_inputs(l), wl.make_inputs(l)
    for k in a:
        assert np.array_equal(a[k], b[k]) and a[k].dtype == np.float32
        assert a[k].min() >= -1 and a[k].max() < 1
    z = wl.normal01(wl.stream_key("t", 1), (200000,))
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    w = wl.make_inputs(wl.Layer("k", 1, 4, 4, 64, 256, 3, 3, 1, 1), ("W",))["W"]
    assert abs(w.std() / np.sqrt(2.0 / 576) - 1) < 0.02
    assert wl.CFG2[0].flops == 2 * 32768 * 128 * 576
    assert sum(l.flops for l in wl.CFG5) == 2 * 128 * 313196544


# ---- biased convolution + leaky-ReLU (Fig. 2 constructors) -----------------------------------
def test_bias_act_hand_values():
    """1x1 input, 1x1 filter: conv is a product; values worked out by hand."""
    X = np.array([2.0, -3.0], dtype=np.float32).reshape(2, 1, 1, 1)
    W = np.array([1.0, -1.0, 0.5], dtype=np.float32).reshape(3, 1, 1, 1)
    bias = np.array([0.25, -1.0, 2.0], dtype=np.float32)
    y = oracle.conv2d_fwd_bias_act(X, W, bias, 0.125)
    # image 0: 2*[1,-1,.5] + b = [2.25, -3, 3] -> leaky: [2.25, -0.375, 3]
    # image 1: -3*[1,-1,.5] + b = [-2.75, 2, 0.5] -> [-0.34375, 2, 0.5]
    want = np.array([[2.25, -0.375, 3.0], [-0.34375, 2.0, 0.5]]).reshape(2, 1, 1, 3)
    assert np.array_equal(y, want)


def test_bias_act_special_cases():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 5, 4, 3)).astype(np.float32)
    W = rng.standard_normal((4, 3, 2, 3)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    plain = oracle.conv2d_fwd(X, W, (1, 2), (1, 0))
    # slope 1: bias only; no bias and slope 1: the convolution itself
    assert np.array_equal(oracle.conv2d_fwd_bias_act(X, W, None, 1.0, (1, 2), (1, 0)), plain)
    assert np.allclose(oracle.conv2d_fwd_bias_act(X, W, b, 1.0, (1, 2), (1, 0)), plain + b.astype(np.float64), rtol=0, atol=0)
    # slope 0: ReLU; the bias shifts channel c only
    relu = oracle.conv2d_fwd_bias_act(X, W, b, 0.0, (1, 2), (1, 0))
    assert np.array_equal(relu, np.maximum(plain + b.astype(np.float64), 0.0))
    # negative slope acts on the negative part only, linearly
    y = oracle.conv2d_fwd_bias_act(X, W, b, 0.3, (1, 2), (1, 0))
    z = plain + b.astype(np.float64)
    assert np.array_equal(y[z > 0], z[z > 0]) and np.allclose(y[z <= 0], 0.3 * z[z <= 0], rtol=1e-15, atol=0)
    # a wrong channel axis for the bias would fail here: only channel 2 gets a bias
    b2 = np.zeros(4, dtype=np.float32); b2[2] = 7.0
    d = oracle.conv2d_fwd_bias_act(X, W, b2, 1.0, (1, 2), (1, 0)) - plain
    assert np.allclose(d[..., 2], 7.0, rtol=0, atol=1e-12) and not d[..., [0, 1, 3]].any()


# ---- forward from 8-bit pixels -------------------------------------------------------------------
def test_fwd_u8_hand_values_and_scale():
    X8 = np.array([[0, 255], [128, 3]], dtype=np.uint8).reshape(1, 2, 2, 1)
    W = np.array([2.0], dtype=np.float32).reshape(1, 1, 1, 1)
    y = oracle.conv2d_fwd_u8(X8, 0.5, W)                      # exact: bytes * 0.5 * 2
    assert np.array_equal(y.reshape(2, 2), np.array([[0.0, 255.0], [128.0, 3.0]]))
    rng = np.random.default_rng(11)
    X8 = rng.integers(0, 256, size=(2, 6, 5, 3), dtype=np.uint8)
    W = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    # scale 1: the plain operator on the bytes as floats
    assert np.array_equal(oracle.conv2d_fwd_u8(X8, 1.0, W, 1, 1), oracle.conv2d_fwd(X8.astype(np.float32), W, 1, 1))
    # a power-of-two scale commutes with every rounding: exact linearity
    assert np.array_equal(oracle.conv2d_fwd_u8(X8, 0.25, W, 2, 1), 0.25 * oracle.conv2d_fwd_u8(X8, 1.0, W, 2, 1))
    # 1/255: each pixel is the fp32 product byte * fp32(1/255), not a double-precision quotient
    y = oracle.conv2d_fwd_u8(X8, 1.0 / 255.0, W, 1, 1)
    x32 = (X8.astype(np.float32) * np.float32(1.0 / 255.0))
    assert x32.dtype == np.float32 and np.array_equal(y, oracle.conv2d_fwd(x32, W, 1, 1))
    assert np.abs(y - oracle.conv2d_fwd(X8.astype(np.float64).astype(np.float32), W, 1, 1) / 255.0).max() < 1e-5


# ---- do the pins bite?  mistakes planted in a copy of the definition, on the CPU -----------------
def _fwd_with_mistake(X, W, s, p, mistake):
    """The forward definition as plain loops, with one plausible mistake switched on."""
    (sh, sw), (ph, pw) = s, p
    N, IH, IW, IC = X.shape
    OC, FH, FW, _ = W.shape
    if mistake == "swapped stride":
        sh, sw = sw, sh
    if mistake == "swapped padding":
        ph, pw = pw, ph
    OH, OW = (IH + 2 * ph - FH) // sh + 1, (IW + 2 * pw - FW) // sw + 1
    Y = np.zeros((N, OH, OW, OC))
    for oh in range(OH):
        for ow in range(OW):
            for fh in range(FH):
                for fw in range(FW):
                    ih, iw = oh * sh - ph + fh, ow * sw - pw + fw
                    if mistake == "padding on the far side":
                        ih, iw = oh * sh + ph - (FH - 1) + fh, ow * sw + pw - (FW - 1) + fw
                    if not (0 <= ih < IH and 0 <= iw < IW):
                        continue
                    if mistake == "dropped last tap" and fh == FH - 1 and fw == FW - 1 and FH * FW > 1:
                        continue
                    wf = W[:, FH - 1 - fh, FW - 1 - fw, :] if mistake == "flipped filter" else \
                        W[:, fw, fh, :] if mistake == "transposed filter" and FH == FW else W[:, fh, fw, :]
                    Y[:, oh, ow, :] += X[:, ih, iw, :].astype(np.float64) @ wf.astype(np.float64).T
    return Y


def _pins_hold(fwd):
    """The forward pins with the implementation passed in: shifted delta, all-ones closed form,
    pad-and-slice second form on an asymmetric shape."""
    C = 2
    X = rnd(1, 6, 7, C)
    W = np.zeros((C, 3, 3, C), np.float32)
    for c in range(C):
        W[c, 0, 2, c] = 1
    expect = np.zeros((1, 6, 7, C))
    expect[:, 1:, :-1] = X[:, :-1, 1:]
    ok = np.array_equal(fwd(X, W, (1, 1), (1, 1)), expect)
    # all ones, 4x5 map, 3x2 filter, stride (1,2), pad (1,0): count of taps inside the image
    Y = fwd(np.ones((1, 4, 5, 3), np.float32), np.ones((2, 3, 2, 3), np.float32), (1, 2), (1, 0))
    rows = np.array([2, 3, 3, 2])
    ok = ok and Y.shape == (1, 4, 2, 2) and np.array_equal(Y[0, :, :, 0], 3.0 * np.outer(rows, [2, 2]))
    Xr, Wr = rnd(2, 7, 5, 3), rnd(4, 3, 2, 3)
    Yr = fwd(Xr, Wr, (2, 1), (0, 1))
    ref = fwd_pad_slice(Xr, Wr, (2, 1), (0, 1))
    return bool(ok and Yr.shape == ref.shape and rel(Yr, ref) < 1e-12)


def test_planted_mistakes_fail_the_pins():
    assert _pins_hold(lambda X, W, s, p: np.asarray(oracle.conv2d_fwd(X, W, s, p)))
    assert _pins_hold(lambda X, W, s, p: _fwd_with_mistake(X, W, s, p, None))
    for mistake in ("flipped filter", "transposed filter", "swapped stride", "swapped padding",
                    "padding on the far side", "dropped last tap"):
        assert not _pins_hold(lambda X, W, s, p: _fwd_with_mistake(X, W, s, p, mistake)), mistake


# ---- matrix multiply of the fully-connected layer -------------------------------------------------
def test_matmul_hand_values_and_closed_forms():
    # values worked out by hand: [[1,2,3],[4,5,6]] x [[1,0],[0,1],[2,-1]] = [[7,-1],[16,-1]]
    A = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    B = np.array([[1, 0], [0, 1], [2, -1]], dtype=np.float32)
    assert np.array_equal(oracle.matmul(A, B), np.array([[7, -1], [16, -1]], dtype=np.float64))
    # the same product with either operand stored transposed
    assert np.array_equal(oracle.matmul(np.ascontiguousarray(A.T), B, transpose_a=True), [[7, -1], [16, -1]])
    assert np.array_equal(oracle.matmul(A, np.ascontiguousarray(B.T), transpose_b=True), [[7, -1], [16, -1]])
    # identity and all-ones closed forms (M, N, K all different, so a swapped extent cannot pass)
    X = wl.uniform_pm1(wl.stream_key("mm-id"), (5, 7))
    assert np.array_equal(oracle.matmul(X, np.eye(7, dtype=np.float32)), X.astype(np.float64))
    assert np.array_equal(oracle.matmul(np.eye(5, dtype=np.float32), X), X.astype(np.float64))
    assert np.array_equal(oracle.matmul(np.ones((3, 11), np.float32), np.ones((11, 4), np.float32)), np.full((3, 4), 11.0))


def test_matmul_against_numpy_and_transposition_identities():
    k = wl.stream_key("mm")
    for i, (M, N, K) in enumerate([(1, 1, 1), (3, 5, 7), (17, 2, 33), (8, 40, 5), (64, 10, 512)]):
        A = wl.uniform_pm1(k + 2 * i, (M, K))
        B = wl.uniform_pm1(k + 2 * i + 1, (K, N))
        ref = A.astype(np.float64) @ B.astype(np.float64)          # library routine
        for ta in (False, True):
            for tb in (False, True):
                a = np.ascontiguousarray(A.T) if ta else A
                b = np.ascontiguousarray(B.T) if tb else B
                got = oracle.matmul(a, b, ta, tb)
                assert got.shape == (M, N)
                assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref))), (M, N, K, ta, tb)
        # (A B)^T = B^T A^T
        assert np.allclose(oracle.matmul(A, B).T, oracle.matmul(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T)), rtol=0, atol=1e-12)


def test_matmul_is_the_1x1_convolution_on_a_1x1_map():
    """Y = X W^T of a fully-connected layer equals the forward convolution of a 1x1 map with a 1x1
    filter, and its two gradients equal backward-data and backward-weight of that convolution."""
    k = wl.stream_key("mm-conv")
    M, K, N = 6, 20, 9
    X = wl.uniform_pm1(k, (M, K))
    W = wl.uniform_pm1(k + 1, (N, K))
    G = wl.uniform_pm1(k + 2, (M, N))
    y = oracle.conv2d_fwd(X.reshape(M, 1, 1, K), W.reshape(N, 1, 1, K)).reshape(M, N)
    assert np.max(np.abs(oracle.matmul(X, W, transpose_b=True) - y)) <= 1e-12
    dx = oracle.conv2d_bwd_data(G.reshape(M, 1, 1, N), W.reshape(N, 1, 1, K), (1, 1)).reshape(M, K)
    assert np.max(np.abs(oracle.matmul(G, W) - dx)) <= 1e-12
    dw = oracle.conv2d_bwd_weight(X.reshape(M, 1, 1, K), G.reshape(M, 1, 1, N), (1, 1)).reshape(N, K)
    assert np.max(np.abs(oracle.matmul(G, X, transpose_a=True) - dw)) <= 1e-12


def test_matmul_planted_mistakes_fail_the_pins():
    """Copies of the definition with one mistake each (wrong transposition flag, swapped extents)
    must disagree with the hand values or numpy."""
    A = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    B = np.array([[1, 0], [0, 1], [2, -1]], dtype=np.float32)
    want = np.array([[7, -1], [16, -1]], dtype=np.float64)

    def mm(A, B, ta, tb, M, N, K):
        C = np.zeros((M, N))
        for i in range(M):
            for j in range(N):
                for kk in range(K):
                    a = A.ravel()[kk * M + i] if ta else A.ravel()[i * K + kk]
                    b = B.ravel()[j * K + kk] if tb else B.ravel()[kk * N + j]
                    C[i, j] += float(a) * float(b)
        return C
    assert np.array_equal(mm(A, B, 0, 0, 2, 2, 3), want)                   # the faithful copy passes
    assert not np.array_equal(mm(A, B, 1, 0, 2, 2, 3), want)               # A read as if stored transposed
    assert not np.array_equal(mm(A, B, 0, 1, 2, 2, 3), want)               # B read as if stored transposed
    A2 = wl.uniform_pm1(wl.stream_key("mm-plant"), (3, 4))
    B2 = wl.uniform_pm1(wl.stream_key("mm-plant") + 1, (4, 5))
    ref = A2.astype(np.float64) @ B2.astype(np.float64)
    assert np.allclose(mm(A2, B2, 0, 0, 3, 5, 4), ref)
    assert not np.allclose(mm(A2, B2, 0, 0, 3, 5, 3), ref)                 # one reduction term dropped
