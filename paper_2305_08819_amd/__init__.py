"""MI355X-native fp32 NHWC convolution (forward, deconvolution/backward-data, backward-weight).

Thin ctypes binding over ``libmi355conv.so`` (C ABI in ``include/mi355conv.h``).  The binding
only marshals arguments: shapes into a ``conv2d_desc``, torch CUDA tensors into raw device
pointers, the current torch stream into a ``hipStream_t``.  All arithmetic runs in the HIP
kernels; there is no fallback, and importing the library fails loudly if it was not built.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
# MI355CONV_LIB: another build of the same sources (the sanitizer test's host-instrumented one)
LIB_PATH = os.environ.get("MI355CONV_LIB") or os.path.join(_PKG, "libmi355conv.so")

OP_FWD, OP_BWD_DATA, OP_BWD_WEIGHT = 0, 1, 2
VARIANT_AUTO, VARIANT_DIRECT, VARIANT_MFMA = -1, 0, 1
KERNEL_DIRECT, KERNEL_GATHER, KERNEL_GATHER_ELEM, KERNEL_FIRST_LAYER, KERNEL_WGRAD, KERNEL_WGRAD_FAST = range(6)
ORDER_PLAIN, ORDER_LONGEST, ORDER_REGIONS = range(3)

EXPORTS = ("conv2d_workspace_bytes", "conv2d_query_plan", "conv2d_query_workgroup", "conv2d_query_tile", "conv2d_set_tuning", "conv2d_set_tile", "conv2d_set_order", "conv2d_fwd",
           "conv2d_fwd_bias_act", "conv2d_fwd_u8",
           "conv2d_bwd_data", "deconv2d", "conv2d_bwd_weight", "conv2d_status_string",
           "conv2d_last_hip_error", "conv2d_init", "conv2d_bwd_weight_noalloc", "conv2d_noalloc_scratch_bytes",
           "conv2d_probe_mfma_rate", "matmul_workspace_bytes", "matmul_f32")
MATMUL_NT, MATMUL_NN, MATMUL_TN = 0, 1, 2


class ConvDesc(ctypes.Structure):
    """Mirror of ``conv2d_desc``."""
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "IH", "IW", "IC", "OC", "FH", "FW", "sh", "sw", "ph", "pw")]

    @property
    def OH(self):
        return (self.IH + 2 * self.ph - self.FH) // self.sh + 1

    @property
    def OW(self):
        return (self.IW + 2 * self.pw - self.FW) // self.sw + 1


class PlanInfo(ctypes.Structure):
    """Mirror of ``conv2d_plan_info``."""
    _fields_ = [("variant", ctypes.c_int), ("tile_m", ctypes.c_int), ("tile_n", ctypes.c_int),
                ("split", ctypes.c_int), ("pos_major", ctypes.c_int), ("grid", ctypes.c_int),
                ("workspace_bytes", ctypes.c_size_t), ("kernel", ctypes.c_int), ("order", ctypes.c_int)]


class Mi355ConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        lib = load()
        msg = lib.conv2d_status_string(status).decode()
        hip = lib.conv2d_last_hip_error().decode()
        super().__init__("%s: %s (%d)%s" % (where, msg, status, " [" + hip + "]" if hip else ""))


_lib = None


def load() -> ctypes.CDLL:
    """Load the built library; raise if it is missing (no silent fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s not built: run `python -m paper_2305_08819_amd.build`" % LIB_PATH)
        # torch ships its own HIP runtime; it has to be in the process before this library is, so that
        # both use that one runtime (loaded the other way round, the first operator call fails with
        # "no ROCm-capable device is detected")
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, dp = ctypes.c_void_p, ctypes.POINTER(ConvDesc)
        lib.conv2d_workspace_bytes.argtypes = [ctypes.c_int, dp]
        lib.conv2d_workspace_bytes.restype = ctypes.c_size_t
        lib.conv2d_query_plan.argtypes = [ctypes.c_int, dp, ctypes.POINTER(PlanInfo)]
        lib.conv2d_query_plan.restype = ctypes.c_int
        lib.conv2d_query_workgroup.argtypes = [ctypes.c_int, dp, ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                               ctypes.POINTER(ctypes.c_int)]
        lib.conv2d_query_workgroup.restype = ctypes.c_int
        lib.conv2d_set_tuning.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.conv2d_set_tuning.restype = ctypes.c_int
        lib.conv2d_set_tile.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.conv2d_set_tile.restype = ctypes.c_int
        lib.conv2d_set_order.argtypes = [ctypes.c_int]
        lib.conv2d_set_order.restype = ctypes.c_int
        for name in ("conv2d_fwd", "conv2d_bwd_data", "deconv2d", "conv2d_bwd_weight"):
            fn = getattr(lib, name)
            fn.argtypes = [vp, vp, vp, dp, vp, ctypes.c_size_t, vp]
            fn.restype = ctypes.c_int
        lib.conv2d_fwd_bias_act.argtypes = [vp, vp, vp, vp, dp, ctypes.c_float, vp, ctypes.c_size_t, vp]
        lib.conv2d_fwd_bias_act.restype = ctypes.c_int
        lib.conv2d_fwd_u8.argtypes = [vp, ctypes.c_float, vp, vp, dp, vp]
        lib.conv2d_fwd_u8.restype = ctypes.c_int
        lib.conv2d_init.argtypes = []
        lib.conv2d_init.restype = ctypes.c_int
        lib.conv2d_bwd_weight_noalloc.argtypes = [vp, vp, vp, dp, vp]
        lib.conv2d_bwd_weight_noalloc.restype = ctypes.c_int
        lib.conv2d_noalloc_scratch_bytes.argtypes = []
        lib.conv2d_noalloc_scratch_bytes.restype = ctypes.c_size_t
        lib.conv2d_probe_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        lib.conv2d_probe_mfma_rate.restype = ctypes.c_int
        lib.matmul_workspace_bytes.argtypes = [ctypes.c_int] * 4
        lib.matmul_workspace_bytes.restype = ctypes.c_size_t
        lib.matmul_f32.argtypes = [ctypes.c_int, vp, vp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp]
        lib.matmul_f32.restype = ctypes.c_int
        lib.conv2d_status_string.argtypes = [ctypes.c_int]
        lib.conv2d_status_string.restype = ctypes.c_char_p
        lib.conv2d_last_hip_error.argtypes = []
        lib.conv2d_last_hip_error.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _pair(v):
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def make_desc(N, IH, IW, IC, OC, FH, FW, stride=1, pad=0) -> ConvDesc:
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    return ConvDesc(N, IH, IW, IC, OC, FH, FW, sh, sw, ph, pw)


def conv2d_workspace_bytes(op: int, desc: ConvDesc) -> int:
    return int(load().conv2d_workspace_bytes(op, ctypes.byref(desc)))


def conv2d_query_plan(op: int, desc: ConvDesc) -> PlanInfo:
    info = PlanInfo()
    rc = load().conv2d_query_plan(op, ctypes.byref(desc), ctypes.byref(info))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_query_plan")
    return info


def conv2d_query_workgroup(op: int, desc: ConvDesc, workgroup: int):
    """(rank, work) of hardware workgroup id `workgroup` under the plan's longest-first dealing."""
    rank, work = ctypes.c_int(0), ctypes.c_int(0)
    rc = load().conv2d_query_workgroup(op, ctypes.byref(desc), workgroup, ctypes.byref(rank), ctypes.byref(work))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_query_workgroup")
    return rank.value, work.value


def conv2d_query_tile(op: int, desc: ConvDesc, workgroup: int):
    """(row tile, column tile, slice) of hardware workgroup id `workgroup` of a region-/group-wise launch."""
    a, b, c = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    rc = load().conv2d_query_tile(op, ctypes.byref(desc), workgroup, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_query_tile")
    return a.value, b.value, c.value


def conv2d_set_tuning(variant: int = VARIANT_AUTO, split: int = 0) -> None:
    rc = load().conv2d_set_tuning(variant, split)
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_set_tuning")


def conv2d_set_tile(tile_m: int = 0, tile_n: int = 0, pos_major: int = -1) -> None:
    rc = load().conv2d_set_tile(tile_m, tile_n, pos_major)
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_set_tile")


def conv2d_set_order(region_wise: int = 1) -> None:
    rc = load().conv2d_set_order(region_wise)
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_set_order")


def conv2d_init() -> None:
    """One-time set-up of the current device (needed before stream capture; otherwise optional)."""
    rc = load().conv2d_init()
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_init")


def conv2d_noalloc_scratch_bytes() -> int:
    return int(load().conv2d_noalloc_scratch_bytes())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(t, shape, name):
    import torch
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise ValueError("%s must be a contiguous fp32 CUDA tensor" % name)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))


def _own_workspace(need, like, stream):
    """Workspace for a call that brought none.  The tensor is dropped when the call returns, while
    the kernels may still be running: it is tied to the stream they run on, so torch's caching
    allocator does not hand the block to another stream's allocation before they finish."""
    if not need:
        return None
    import torch
    ws = torch.empty(need, dtype=torch.uint8, device=like.device)
    if stream is not None:
        ws.record_stream(stream)
    return ws


def _call(name, op, a, b, out, desc, ws, stream):
    lib = load()
    if ws is None:      # the library checks the size of a workspace the caller brings
        ws = _own_workspace(conv2d_workspace_bytes(op, desc), out, stream)
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    rc = getattr(lib, name)(_ptr(a), _ptr(b), _ptr(out), ctypes.byref(desc), _ptr(ws), nbytes,
                            _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, name)
    return out


def conv2d_fwd(X, W, Y, desc: ConvDesc, ws=None, stream=None):
    """Y[N,OH,OW,OC] <- conv(X[N,IH,IW,IC], W[OC,FH,FW,IC]); enqueue only."""
    _check(X, (desc.N, desc.IH, desc.IW, desc.IC), "X")
    _check(W, (desc.OC, desc.FH, desc.FW, desc.IC), "W")
    _check(Y, (desc.N, desc.OH, desc.OW, desc.OC), "Y")
    return _call("conv2d_fwd", OP_FWD, X, W, Y, desc, ws, stream)


def conv2d_fwd_bias_act(X, W, bias, Y, desc: ConvDesc, negative_slope=1.0, ws=None, stream=None):
    """Y <- act(conv(X, W) + bias[oc]), act(v) = v if v > 0 else negative_slope * v; bias may be None."""
    _check(X, (desc.N, desc.IH, desc.IW, desc.IC), "X")
    _check(W, (desc.OC, desc.FH, desc.FW, desc.IC), "W")
    _check(Y, (desc.N, desc.OH, desc.OW, desc.OC), "Y")
    if bias is not None:
        _check(bias, (desc.OC,), "bias")
    lib = load()
    if ws is None:
        ws = _own_workspace(conv2d_workspace_bytes(OP_FWD, desc), Y, stream)
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    rc = lib.conv2d_fwd_bias_act(_ptr(X), _ptr(W), _ptr(bias), _ptr(Y), ctypes.byref(desc),
                                 ctypes.c_float(negative_slope), _ptr(ws), nbytes, _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_fwd_bias_act")
    return Y


def conv2d_fwd_u8(X8, scale, W, Y, desc: ConvDesc, stream=None):
    """Y <- conv(float(X8) * scale, W) for uint8 pixels X8[N,IH,IW,IC]; first-layer shapes only."""
    import torch
    if not (X8.is_cuda and X8.dtype == torch.uint8 and X8.is_contiguous()):
        raise ValueError("X8 must be a contiguous uint8 CUDA tensor")
    if tuple(X8.shape) != (desc.N, desc.IH, desc.IW, desc.IC):
        raise ValueError("X8 has shape %s" % (tuple(X8.shape),))
    _check(W, (desc.OC, desc.FH, desc.FW, desc.IC), "W")
    _check(Y, (desc.N, desc.OH, desc.OW, desc.OC), "Y")
    rc = load().conv2d_fwd_u8(_ptr(X8), ctypes.c_float(scale), _ptr(W), _ptr(Y), ctypes.byref(desc),
                              _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_fwd_u8")
    return Y


def conv2d_bwd_data(dY, W, dX, desc: ConvDesc, ws=None, stream=None):
    """dX[N,IH,IW,IC] <- deconv(dY[N,OH,OW,OC], W[OC,FH,FW,IC]); enqueue only."""
    _check(dY, (desc.N, desc.OH, desc.OW, desc.OC), "dY")
    _check(W, (desc.OC, desc.FH, desc.FW, desc.IC), "W")
    _check(dX, (desc.N, desc.IH, desc.IW, desc.IC), "dX")
    return _call("conv2d_bwd_data", OP_BWD_DATA, dY, W, dX, desc, ws, stream)


def deconv2d(dY, W, dX, desc: ConvDesc, ws=None, stream=None):
    """Same as conv2d_bwd_data, through the library's ``deconv2d`` symbol."""
    _check(dY, (desc.N, desc.OH, desc.OW, desc.OC), "dY")
    _check(W, (desc.OC, desc.FH, desc.FW, desc.IC), "W")
    _check(dX, (desc.N, desc.IH, desc.IW, desc.IC), "dX")
    return _call("deconv2d", OP_BWD_DATA, dY, W, dX, desc, ws, stream)


def conv2d_bwd_weight(X, dY, dW, desc: ConvDesc, ws=None, stream=None):
    """dW[OC,FH,FW,IC] <- sum over pixels of dY x X; enqueue only."""
    _check(X, (desc.N, desc.IH, desc.IW, desc.IC), "X")
    _check(dY, (desc.N, desc.OH, desc.OW, desc.OC), "dY")
    _check(dW, (desc.OC, desc.FH, desc.FW, desc.IC), "dW")
    return _call("conv2d_bwd_weight", OP_BWD_WEIGHT, X, dY, dW, desc, ws, stream)


def conv2d_bwd_weight_noalloc(X, dY, dW, desc: ConvDesc, stream=None):
    """conv2d_bwd_weight with the slice partials in the library's own device array: no workspace
    argument, no allocation anywhere (this binding allocates nothing either)."""
    _check(X, (desc.N, desc.IH, desc.IW, desc.IC), "X")
    _check(dY, (desc.N, desc.OH, desc.OW, desc.OC), "dY")
    _check(dW, (desc.OC, desc.FH, desc.FW, desc.IC), "dW")
    rc = load().conv2d_bwd_weight_noalloc(_ptr(X), _ptr(dY), _ptr(dW), ctypes.byref(desc), _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_bwd_weight_noalloc")
    return dW


def conv2d_probe_mfma_rate(valu_per_8_mfma, workgroups, iters, out, stream=None):
    """Launch the register-only fp32 MFMA loop (measurement aid); returns the FLOP it executes."""
    rc = load().conv2d_probe_mfma_rate(valu_per_8_mfma, workgroups, iters, _ptr(out), _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, "conv2d_probe_mfma_rate")
    return workgroups * 4 * iters * 8 * 4096


def matmul_workspace_bytes(kind: int, M: int, N: int, K: int) -> int:
    return int(load().matmul_workspace_bytes(kind, M, N, K))


def matmul_f32(kind, A, B, C, ws=None, stream=None):
    """C[M,N] <- A B^T (MATMUL_NT), A B (MATMUL_NN) or A^T B (MATMUL_TN): the fully-connected layer's
    forward, input gradient and weight gradient; enqueue only."""
    M, N = C.shape
    K = A.shape[0] if kind == MATMUL_TN else A.shape[1]
    _check(A, (K, M) if kind == MATMUL_TN else (M, K), "A")
    _check(B, (N, K) if kind == MATMUL_NT else (K, N), "B")
    _check(C, (M, N), "C")
    if ws is None:
        ws = _own_workspace(matmul_workspace_bytes(kind, M, N, K), C, stream)
    nbytes = ws.numel() * ws.element_size() if ws is not None else 0
    rc = load().matmul_f32(kind, _ptr(A), _ptr(B), _ptr(C), M, N, K, _ptr(ws), nbytes, _stream_handle(stream))
    if rc != 0:
        raise Mi355ConvError(rc, "matmul_f32")
    return C
