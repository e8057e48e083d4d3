"""CPU oracle for the three fp32 NHWC convolution operators.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it, and it never imports the product package.

The arithmetic lives in ``conv_oracle.c`` (plain C loop nests, fp64
accumulation); this module only compiles that file with gcc, loads it with
ctypes and marshals numpy arrays.  Pin status: every function here is pinned by
``tests/test_oracle_pins.py`` (closed forms, delta filters, 1x1 == GEMM,
scatter/pad-and-slice second forms, adjoint identity, exact finite
differences, a library cross-check); ``conv2d_fwd_bias_act`` adds the bias add
and leaky-ReLU of the paper's layer constructors on top of ``conv2d_fwd`` in
plain numpy fp64 and is pinned by hand-computed values and its special cases
(slope 1, slope 0, zero bias); ``conv2d_fwd_u8`` converts 8-bit pixels to
fp32 (byte * scale, rounded once to fp32) before ``conv2d_fwd`` and is pinned
by hand values, the scale-1 case and its linearity in the scale; ``matmul``
(the fully-connected layer's matrix multiply, plain C loops in fp64) is pinned
by hand values, identity and all-ones closed forms, its transposition
identities, numpy's fp64 matmul and the 1x1 convolution on a 1x1 map.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_oracle.c into liboracle_conv.so (gcc -O2 -fopenmp, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # ORACLE_CONV_LIB: another build of conv_oracle.c (the sanitizer test's instrumented one)
        path = os.environ.get("ORACLE_CONV_LIB")
        if not path:
            build()
            path = _LIB
        lib = ctypes.CDLL(path)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ints = [ctypes.c_int] * 11
        for name in ("oracle_conv2d_fwd", "oracle_conv2d_bwd_data", "oracle_conv2d_bwd_weight"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, fp, dp] + ints
            fn.restype = None
        lib.oracle_matmul.argtypes = [fp, fp, dp] + [ctypes.c_int] * 5
        lib.oracle_matmul.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops will use."""
    return int(_load().oracle_num_threads())


def out_size(i: int, f: int, stride: int, pad: int) -> int:
    """floor((i + 2*pad - f)/stride) + 1, or 0 when the filter does not fit."""
    span = i + 2 * pad - f
    return span // stride + 1 if span >= 0 else 0


def _pair(v):
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _f32(a, ndim):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == ndim
    return a


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def conv2d_fwd(X, W, stride=1, pad=0):
    """Y[N,OH,OW,OC] in fp64 from X[N,IH,IW,IC], W[OC,FH,FW,IC] (fp32 values)."""
    X, W = _f32(X, 4), _f32(W, 4)
    N, IH, IW, IC = X.shape
    OC, FH, FW, IC2 = W.shape
    assert IC == IC2
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    OH, OW = out_size(IH, FH, sh, ph), out_size(IW, FW, sw, pw)
    Y = np.zeros((N, OH, OW, OC), dtype=np.float64)
    if Y.size:
        _load().oracle_conv2d_fwd(_fp(X), _fp(W), _dp(Y), N, IH, IW, IC, OC, FH, FW, sh, sw, ph, pw)
    return Y


def conv2d_bwd_data(G, W, in_hw, stride=1, pad=0):
    """dX[N,IH,IW,IC] in fp64 from G[N,OH,OW,OC], W[OC,FH,FW,IC]; in_hw=(IH,IW)."""
    G, W = _f32(G, 4), _f32(W, 4)
    IH, IW = _pair(in_hw)
    N, OH, OW, OC = G.shape
    OC2, FH, FW, IC = W.shape
    assert OC == OC2
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    assert OH == out_size(IH, FH, sh, ph) and OW == out_size(IW, FW, sw, pw)
    dX = np.zeros((N, IH, IW, IC), dtype=np.float64)
    if dX.size and G.size:
        _load().oracle_conv2d_bwd_data(_fp(G), _fp(W), _dp(dX), N, IH, IW, IC, OC, FH, FW,
                                       sh, sw, ph, pw)
    return dX


def conv2d_bwd_weight(X, G, filter_hw, stride=1, pad=0):
    """dW[OC,FH,FW,IC] in fp64 from X[N,IH,IW,IC], G[N,OH,OW,OC]; filter_hw=(FH,FW)."""
    X, G = _f32(X, 4), _f32(G, 4)
    FH, FW = _pair(filter_hw)
    N, IH, IW, IC = X.shape
    N2, OH, OW, OC = G.shape
    assert N == N2
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    assert OH == out_size(IH, FH, sh, ph) and OW == out_size(IW, FW, sw, pw)
    dW = np.zeros((OC, FH, FW, IC), dtype=np.float64)
    if dW.size and G.size:
        _load().oracle_conv2d_bwd_weight(_fp(X), _fp(G), _dp(dW), N, IH, IW, IC, OC, FH, FW,
                                         sh, sw, ph, pw)
    return dW


def conv2d_fwd_bias_act(X, W, bias=None, negative_slope=1.0, stride=1, pad=0):
    """act(conv(X, W) + bias[oc]) with act(v) = v if v > 0 else negative_slope * v, in fp64.

    The biased convolution and the leaky-ReLU activation are the paper's layer constructors
    (Fig. 2: ``conv3D(..., biased)``, ``leakyRelu``); the formula is the usual definition of both.
    ``bias`` None means no bias; ``negative_slope`` 1 means no activation.
    """
    y = np.asarray(conv2d_fwd(X, W, stride, pad), dtype=np.float64)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        assert b.shape == (y.shape[3],)
        y = y + b[None, None, None, :]
    return np.where(y > 0.0, y, y * float(negative_slope))


def conv2d_fwd_u8(X8, scale, W, stride=1, pad=0):
    """Forward convolution of 8-bit pixels: x = fp32(byte) * fp32(scale), rounded once to fp32 (the
    paper converts pixel bytes to floats on the device, Sec. III; Table I: pixels / 255), then
    ``conv2d_fwd``.  The conversion is part of the operator, so it is done in the precision the
    operator is defined in (fp32); the sums are fp64 as everywhere in this oracle."""
    x8 = np.ascontiguousarray(X8)
    assert x8.dtype == np.uint8 and x8.ndim == 4
    x = x8.astype(np.float32) * np.float32(scale)
    return conv2d_fwd(x, W, stride, pad)


def matmul(A, B, transpose_a=False, transpose_b=False):
    """C = op(A) @ op(B) in fp64 for fp32 row-major matrices (op = transpose where asked): the matrix
    multiply of the paper's fully-connected layer (Fig. 2 ``fullconnect``; Sec. II ``matMul`` /
    ``matMulT1``), as plain C loops with one fp64 accumulator per output element."""
    A, B = _f32(A, 2), _f32(B, 2)
    M, K = (A.shape[1], A.shape[0]) if transpose_a else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transpose_b else B.shape
    assert K == K2, (A.shape, B.shape, transpose_a, transpose_b)
    C = np.zeros((M, N), dtype=np.float64)
    if C.size and K:
        _load().oracle_matmul(_fp(A), _fp(B), _dp(C), M, N, K, int(bool(transpose_a)), int(bool(transpose_b)))
    return C
