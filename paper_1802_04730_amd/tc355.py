"""Thin ctypes binding of libtc355.so: argument marshalling only.

Every function has the name and argument order of the C entry point in
include/tc355.h.  Tensors are torch CUDA tensors (device memory owned by the
caller); extents are read from their shapes; work is enqueued on torch's
current stream unless ``stream`` (a raw hipStream_t value) is given.  A non-zero
status raises ``TcError``.  There is no CPU fallback: if the library cannot be
loaded the import of this module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

_LIB = None

TC_OK = 0
STATUS_NAMES = {0: "TC_OK", 1: "TC_ERR_NULL", 2: "TC_ERR_SHAPE", 3: "TC_ERR_ALIAS", 4: "TC_ERR_ALIGN",
                5: "TC_ERR_WORKSPACE", 6: "TC_ERR_LAUNCH", 7: "TC_ERR_UNSUPPORTED", 8: "TC_ERR_SCRATCH_LIMIT"}
TC_MLP_STATIC_SCRATCH_BYTES = 8 << 20
# tc355_set_option keys and values (include/tc355.h)
TC_OPT_INT8, TC_OPT_MLP_KERNEL, TC_OPT_MLP_SPIN_LIMIT = 0, 1, 2
TC_INT8_AUTO, TC_INT8_OFF, TC_INT8_TEN, TC_INT8_THIRTEEN = 0, 1, 2, 3
TC_MLP_AUTO, TC_MLP_ROWS, TC_MLP_TILES, TC_MLP_PER_LAYER = 0, 1, 2, 3

EXPORTS = ["tc_status_string", "tc355_version", "tc355_set_option", "tc355_get_option", "tc355_last_path", "tc_tbmm", "tc_tbmm_ws", "tc_tbmm_workspace_bytes", "tc_mlp_fcrelu", "tc_mlp_fcrelu_workspace_bytes",
           "tc_mlp_fcrelu_static",
           "tc_group_conv", "tc_group_conv_infer", "tc_kron", "tc_sconv2d", "tc_sconv2d_infer", "tc_lut"]


class TcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


def lib() -> ctypes.CDLL:
    """Load libtc355.so, building it first if it is missing or older than its sources (and hipcc is there)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = _build.LIB
    if not os.path.exists(path) or (_build.is_stale() and _build.have_hipcc()):
        _build.build(force=True)
    L = ctypes.CDLL(path)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    L.tc_status_string.argtypes = [ctypes.c_int]
    L.tc_status_string.restype = ctypes.c_char_p
    L.tc355_version.restype = ctypes.c_int
    L.tc355_set_option.argtypes = [ctypes.c_int, i64]
    L.tc355_set_option.restype = ctypes.c_int
    L.tc355_get_option.argtypes = [ctypes.c_int]
    L.tc355_get_option.restype = i64
    L.tc355_last_path.restype = ctypes.c_char_p
    L.tc_tbmm.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp]
    L.tc_tbmm.restype = ctypes.c_int
    L.tc_tbmm_ws.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp, ctypes.c_size_t, vp]
    L.tc_tbmm_ws.restype = ctypes.c_int
    L.tc_tbmm_workspace_bytes.argtypes = [i64, i64, i64, i64]
    L.tc_tbmm_workspace_bytes.restype = ctypes.c_size_t
    L.tc_mlp_fcrelu.argtypes = [vp, i64, i32, ctypes.POINTER(i64), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                ctypes.POINTER(vp), vp, ctypes.c_size_t, vp]
    L.tc_mlp_fcrelu.restype = ctypes.c_int
    L.tc_mlp_fcrelu_static.argtypes = [vp, i64, i32, ctypes.POINTER(i64), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       ctypes.POINTER(vp), vp]
    L.tc_mlp_fcrelu_static.restype = ctypes.c_int
    L.tc_mlp_fcrelu_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(i64)]
    L.tc_mlp_fcrelu_workspace_bytes.restype = ctypes.c_size_t
    L.tc_group_conv.argtypes = [vp, vp, vp, vp] + [i64] * 8 + [vp]
    L.tc_group_conv.restype = ctypes.c_int
    L.tc_group_conv_infer.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.tc_group_conv_infer.restype = ctypes.c_int
    L.tc_kron.argtypes = [vp, vp, vp, vp] + [i64] * 5 + [vp]
    L.tc_kron.restype = ctypes.c_int
    L.tc_sconv2d.argtypes = [vp, vp, vp, vp] + [i64] * 9 + [vp]
    L.tc_sconv2d.restype = ctypes.c_int
    L.tc_sconv2d_infer.argtypes = [i64] * 6 + [ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.tc_sconv2d_infer.restype = ctypes.c_int
    L.tc_lut.argtypes = [i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64),
                         ctypes.POINTER(i64), i64, i64, vp]
    L.tc_lut.restype = ctypes.c_int
    _LIB = L
    return L


def status_string(status: int) -> str:
    return lib().tc_status_string(int(status)).decode()


def tc355_version() -> int:
    return int(lib().tc355_version())


def set_option(key: int, value: int) -> int:
    """Set an option of the calling host thread (tc355_set_option); returns the previous value."""
    old = int(lib().tc355_get_option(int(key)))
    _check(lib().tc355_set_option(int(key), int(value)), "tc355_set_option")
    return old


def get_option(key: int) -> int:
    return int(lib().tc355_get_option(int(key)))


def last_path() -> str:
    """Kernel family chosen by this thread's most recent entry-point call, e.g. "tbmm:lds" (tc355_last_path)."""
    return lib().tc355_last_path().decode()


class option:
    """Context manager: an option of the calling thread for the duration of a block."""

    def __init__(self, key: int, value: int):
        self.key, self.value = key, value

    def __enter__(self):
        self.old = set_option(self.key, self.value)
        return self

    def __exit__(self, *exc):
        set_option(self.key, self.old)
        return False


def _ptr(t, name: str) -> int:
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch CUDA tensor" % name)
    if t.dtype != torch.float32:
        raise TypeError("%s must be float32, got %s" % (name, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be dense row-major (contiguous)" % name)
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return int(stream)


def _check(status: int, where: str) -> None:
    if status != TC_OK:
        raise TcError(status, where)


def tc_tbmm(X, Y, Z, stream=None) -> None:
    """Z[B,N,M] = sum_k X[B,N,K] * Y[B,M,K]; Z is written in place."""
    B, N, K = X.shape
    B2, M, K2 = Y.shape
    if (B, K) != (B2, K2) or tuple(Z.shape) != (B, N, M):
        raise ValueError("tc_tbmm: shapes X %s Y %s Z %s do not fit" % (tuple(X.shape), tuple(Y.shape), tuple(Z.shape)))
    _check(lib().tc_tbmm(_ptr(X, "X"), _ptr(Y, "Y"), _ptr(Z, "Z"), B, N, M, K, _stream(stream)), "tc_tbmm")


def tc_tbmm_workspace_bytes(B: int, N: int, M: int, K: int) -> int:
    return int(lib().tc_tbmm_workspace_bytes(int(B), int(N), int(M), int(K)))


def tc_tbmm_ws(X, Y, Z, workspace, stream=None) -> None:
    """tc_tbmm with a workspace (a uint8 tensor of at least tc_tbmm_workspace_bytes bytes, or None)."""
    B, N, K = X.shape
    B2, M, K2 = Y.shape
    if (B, K) != (B2, K2) or tuple(Z.shape) != (B, N, M):
        raise ValueError("tc_tbmm_ws: shapes X %s Y %s Z %s do not fit" % (tuple(X.shape), tuple(Y.shape), tuple(Z.shape)))
    wp = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    wn = int(workspace.numel() * workspace.element_size()) if workspace is not None else 0
    _check(lib().tc_tbmm_ws(_ptr(X, "X"), _ptr(Y, "Y"), _ptr(Z, "Z"), B, N, M, K, wp, ctypes.c_size_t(wn), _stream(stream)),
           "tc_tbmm_ws")


def tc_mlp_fcrelu_workspace_bytes(batch: int, dims) -> int:
    n = len(dims) - 1
    arr = (ctypes.c_int64 * (n + 1))(*[int(d) for d in dims])
    return int(lib().tc_mlp_fcrelu_workspace_bytes(int(batch), n, arr))


def _mlp_args(I, W, bias, O, where):
    n = len(W)
    batch, d0 = I.shape
    dims = [d0] + [int(w.shape[0]) for w in W]
    for l in range(n):
        if tuple(W[l].shape) != (dims[l + 1], dims[l]) or tuple(bias[l].shape) != (dims[l + 1],):
            raise ValueError("%s: layer %d shapes do not chain" % (where, l))
        if O[l] is not None and tuple(O[l].shape) != (batch, dims[l + 1]):
            raise ValueError("%s: O[%d] has the wrong shape" % (where, l))
    vp = ctypes.c_void_p
    Wp = (vp * n)(*[_ptr(w, "W[%d]" % l) for l, w in enumerate(W)])
    bp = (vp * n)(*[_ptr(b, "bias[%d]" % l) for l, b in enumerate(bias)])
    Op = (vp * n)(*[_ptr(o, "O[%d]" % l) for l, o in enumerate(O)])
    dm = (ctypes.c_int64 * (n + 1))(*dims)
    return batch, n, dm, Wp, bp, Op


def tc_mlp_fcrelu(I, W, bias, O, workspace=None, stream=None) -> None:
    """Chained fcrelu layers.  W, bias, O are lists (O[l] may be None for l < last).

    ``workspace`` is a torch CUDA uint8 tensor of at least
    tc_mlp_fcrelu_workspace_bytes(batch, dims) bytes (None only when that is 0).
    """
    batch, n, dm, Wp, bp, Op = _mlp_args(I, W, bias, O, "tc_mlp_fcrelu")
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise TypeError("workspace must be a contiguous CUDA tensor")
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(lib().tc_mlp_fcrelu(_ptr(I, "I"), batch, n, dm, Wp, bp, Op, ws_ptr, ws_bytes, _stream(stream)),
           "tc_mlp_fcrelu")


def tc_mlp_fcrelu_static(I, W, bias, O, stream=None) -> None:
    """tc_mlp_fcrelu on the library's static scratch array: no workspace argument, no allocation."""
    batch, n, dm, Wp, bp, Op = _mlp_args(I, W, bias, O, "tc_mlp_fcrelu_static")
    _check(lib().tc_mlp_fcrelu_static(_ptr(I, "I"), batch, n, dm, Wp, bp, Op, _stream(stream)),
           "tc_mlp_fcrelu_static")


def tc_group_conv_infer(H: int, W: int, KH: int, KW: int):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().tc_group_conv_infer(H, W, KH, KW, ctypes.byref(oh), ctypes.byref(ow)), "tc_group_conv_infer")
    return int(oh.value), int(ow.value)


def tc_group_conv(I, W1, bias, O, stream=None) -> None:
    """O[N,G,F,OH,OW] = grouped conv of I[N,G,C,H,W] with W1[G,F,C,KH,KW] plus bias[G*F] (or None)."""
    N, G, C, H, W = I.shape
    G2, F, C2, KH, KW = W1.shape
    if (G, C) != (G2, C2):
        raise ValueError("tc_group_conv: I and W1 disagree on G or C")
    if bias is not None and tuple(bias.shape) != (G * F,):
        raise ValueError("tc_group_conv: bias must be [G*F]")
    if tuple(O.shape) != (N, G, F, H - KH + 1, W - KW + 1):
        raise ValueError("tc_group_conv: O has the wrong shape")
    _check(lib().tc_group_conv(_ptr(I, "I"), _ptr(W1, "W1"), _ptr(bias, "bias"), _ptr(O, "O"),
                               N, G, C, F, H, W, KH, KW, _stream(stream)), "tc_group_conv")


def tc_kron(W1, W2, X, Y, stream=None) -> None:
    """Y[B,I,J] = sum_{k,l} W1[I,K] * W2[J,L] * X[B,K,L]."""
    I, K = W1.shape
    J, L = W2.shape
    B, K2, L2 = X.shape
    if (K, L) != (K2, L2) or tuple(Y.shape) != (B, I, J):
        raise ValueError("tc_kron: shapes do not fit")
    _check(lib().tc_kron(_ptr(W1, "W1"), _ptr(W2, "W2"), _ptr(X, "X"), _ptr(Y, "Y"), B, I, K, J, L,
                         _stream(stream)), "tc_kron")


def tc_sconv2d_infer(H: int, W: int, KH: int, KW: int, sh: int, sw: int):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().tc_sconv2d_infer(H, W, KH, KW, sh, sw, ctypes.byref(oh), ctypes.byref(ow)), "tc_sconv2d_infer")
    return int(oh.value), int(ow.value)


def tc_sconv2d(I, Wt, bias, O, sh: int, sw: int, stream=None) -> None:
    """O[N,F,OH,OW] = bias[F] + convolution of I[N,C,H,W] with Wt[F,C,KH,KW], strides (sh, sw), no padding."""
    N, C, H, W = I.shape
    F, C2, KH, KW = Wt.shape
    if C != C2:
        raise ValueError("tc_sconv2d: I and Wt disagree on C")
    if bias is not None and tuple(bias.shape) != (F,):
        raise ValueError("tc_sconv2d: bias must be [F]")
    if tuple(O.shape) != (N, F) + tc_sconv2d_infer(H, W, KH, KW, sh, sw):
        raise ValueError("tc_sconv2d: O has the wrong shape")
    _check(lib().tc_sconv2d(_ptr(I, "I"), _ptr(Wt, "Wt"), _ptr(bias, "bias"), _ptr(O, "O"),
                            N, C, F, H, W, KH, KW, sh, sw, _stream(stream)), "tc_sconv2d")


def tc_lut(LUT, Idx, O, stream=None) -> None:
    """O[t][B,D] = sum_k LUT[t][Idx[t][B,k], :] for every table t; LUT, Idx, O are lists of equal length."""
    n = len(LUT)
    if n == 0 or len(Idx) != n or len(O) != n:
        raise ValueError("tc_lut: LUT, Idx and O must be lists of the same, non-zero length")
    B, D = O[0].shape
    for t in range(n):
        if Idx[t].dtype != torch.int32 or not Idx[t].is_cuda or not Idx[t].is_contiguous():
            raise TypeError("tc_lut: Idx[%d] must be a contiguous int32 CUDA tensor" % t)
        if LUT[t].shape[1] != D or Idx[t].shape[0] != B or tuple(O[t].shape) != (B, D):
            raise ValueError("tc_lut: table %d shapes do not fit" % t)
    vp = ctypes.c_void_p
    Lp = (vp * n)(*[_ptr(x, "LUT[%d]" % t) for t, x in enumerate(LUT)])
    Ip = (vp * n)(*[x.data_ptr() for x in Idx])
    Op = (vp * n)(*[_ptr(x, "O[%d]" % t) for t, x in enumerate(O)])
    Ev = (ctypes.c_int64 * n)(*[int(x.shape[0]) for x in LUT])
    Lv = (ctypes.c_int64 * n)(*[int(x.shape[1]) for x in Idx])
    _check(lib().tc_lut(n, Lp, Ip, Op, Ev, Lv, D, B, _stream(stream)), "tc_lut")
