"""ctypes binding of oracle/tc_oracle.c (test infrastructure, not product code).

Argument marshalling only: every number comes out of the C loop nests.  Inputs
are numpy float32 arrays (converted with ``ascontiguousarray``), outputs are
freshly allocated float64 arrays.  The shared library is compiled with gcc on
first use if it is not there yet.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tc_oracle.c")
_LIB = os.path.join(_HERE, "libtc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile tc_oracle.c -> libtc_oracle.so (gcc -O2, OpenMP, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.tc_oracle_tbmm.argtypes = [fp, fp, dp, i64, i64, i64, i64]
    lib.tc_oracle_tbmm.restype = ctypes.c_int
    lib.tc_oracle_mlp_fcrelu.argtypes = [fp, i64, i32, ctypes.POINTER(i64),
                                         ctypes.POINTER(fp), ctypes.POINTER(fp),
                                         ctypes.POINTER(dp), i32]
    lib.tc_oracle_mlp_fcrelu.restype = ctypes.c_int
    lib.tc_oracle_group_conv_infer.argtypes = [i64, i64, i64, i64,
                                               ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.tc_oracle_group_conv_infer.restype = ctypes.c_int
    lib.tc_oracle_group_conv.argtypes = [fp, fp, fp, dp] + [i64] * 8
    lib.tc_oracle_group_conv.restype = ctypes.c_int
    lib.tc_oracle_kron.argtypes = [fp, fp, fp, dp] + [i64] * 5
    lib.tc_oracle_kron.restype = ctypes.c_int
    lib.tc_oracle_sconv2d_infer.argtypes = [i64] * 6 + [ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.tc_oracle_sconv2d_infer.restype = ctypes.c_int
    lib.tc_oracle_sconv2d.argtypes = [fp, fp, fp, dp] + [i64] * 9
    lib.tc_oracle_sconv2d.restype = ctypes.c_int
    lib.tc_oracle_lut.argtypes = [fp, ctypes.POINTER(ctypes.c_int32), dp] + [i64] * 4
    lib.tc_oracle_lut.restype = ctypes.c_int
    lib.tc_oracle_set_threads.argtypes = [ctypes.c_int]
    lib.tc_oracle_get_threads.restype = ctypes.c_int
    lib.tc_oracle_max_threads.restype = ctypes.c_int
    _lib = lib
    return lib


def set_threads(n: int) -> None:
    _load().tc_oracle_set_threads(int(n))


def get_threads() -> int:
    return int(_load().tc_oracle_get_threads())


def max_threads() -> int:
    return int(_load().tc_oracle_max_threads())


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are float32 arrays, got %s" % a.dtype)
    return a


def _fp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError("%s: oracle status %d (1 = null pointer, 2 = bad shape, 3 = index outside the table)"
                         % (what, rc))


def tbmm(X, Y) -> np.ndarray:
    """Z[b,n,m] = sum_k X[b,n,k] * Y[b,m,k] in float64."""
    X, Y = _f32(X), _f32(Y)
    B, N, K = X.shape
    B2, M, K2 = Y.shape
    if (B, K) != (B2, K2):
        raise ValueError("tbmm: X %s and Y %s disagree on B or K" % (X.shape, Y.shape))
    Z = np.empty((B, N, M), dtype=np.float64)
    _check(_load().tc_oracle_tbmm(_fp(X), _fp(Y), _dp(Z), B, N, M, K), "tbmm")
    return Z


def mlp_fcrelu(I, Ws, bs, round_intermediates: bool = False) -> list:
    """Chained fcrelu layers; returns [O_0, ..., O_{n-1}] in float64."""
    I = _f32(I)
    Ws = [_f32(w) for w in Ws]
    bs = [_f32(b) for b in bs]
    n = len(Ws)
    if n == 0 or len(bs) != n:
        raise ValueError("mlp_fcrelu: need as many biases as weights, at least one")
    batch, d0 = I.shape
    dims = [d0]
    for l in range(n):
        if Ws[l].ndim != 2 or Ws[l].shape[1] != dims[-1] or bs[l].shape != (Ws[l].shape[0],):
            raise ValueError("mlp_fcrelu: layer %d shapes W %s bias %s do not chain from width %d"
                             % (l, Ws[l].shape, bs[l].shape, dims[-1]))
        dims.append(Ws[l].shape[0])
    Os = [np.empty((batch, dims[l + 1]), dtype=np.float64) for l in range(n)]
    fp, dp = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
    Wp = (fp * n)(*[_fp(w) for w in Ws])
    bp = (fp * n)(*[_fp(b) for b in bs])
    Op = (dp * n)(*[_dp(o) for o in Os])
    dm = (ctypes.c_int64 * (n + 1))(*dims)
    _check(_load().tc_oracle_mlp_fcrelu(_fp(I), batch, n, dm, Wp, bp, Op,
                                        1 if round_intermediates else 0), "mlp_fcrelu")
    return Os


def group_conv_infer(H: int, W: int, KH: int, KW: int):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    _check(_load().tc_oracle_group_conv_infer(H, W, KH, KW, ctypes.byref(oh), ctypes.byref(ow)),
           "group_conv_infer")
    return int(oh.value), int(ow.value)


def group_conv(I, W1, bias=None) -> np.ndarray:
    """O[n,g,o,h,w] = sum_{i,kh,kw} I[n,g,i,h+kh,w+kw] * W1[g,o,i,kh,kw] + bias[g*F+o]."""
    I, W1 = _f32(I), _f32(W1)
    N, G, C, H, W = I.shape
    G2, F, C2, KH, KW = W1.shape
    if (G, C) != (G2, C2):
        raise ValueError("group_conv: I %s and W1 %s disagree on G or C" % (I.shape, W1.shape))
    OH, OW = group_conv_infer(H, W, KH, KW)
    bp = None
    if bias is not None:
        bias = _f32(bias)
        if bias.shape != (G * F,):
            raise ValueError("group_conv: bias must be [G*F]")
        bp = _fp(bias)
    O = np.empty((N, G, F, OH, OW), dtype=np.float64)
    _check(_load().tc_oracle_group_conv(_fp(I), _fp(W1), bp, _dp(O), N, G, C, F, H, W, KH, KW),
           "group_conv")
    return O


def kron(W1, W2, X) -> np.ndarray:
    """Y[b,i,j] = sum_{k,l} W1[i,k] * W2[j,l] * X[b,k,l] (single comprehension)."""
    W1, W2, X = _f32(W1), _f32(W2), _f32(X)
    I, K = W1.shape
    J, L = W2.shape
    B, K2, L2 = X.shape
    if (K, L) != (K2, L2):
        raise ValueError("kron: X %s does not match W1 %s / W2 %s" % (X.shape, W1.shape, W2.shape))
    Y = np.empty((B, I, J), dtype=np.float64)
    _check(_load().tc_oracle_kron(_fp(W1), _fp(W2), _fp(X), _dp(Y), B, I, K, J, L), "kron")
    return Y


def sconv2d_infer(H: int, W: int, KH: int, KW: int, sh: int, sw: int):
    oh, ow = ctypes.c_int64(), ctypes.c_int64()
    _check(_load().tc_oracle_sconv2d_infer(H, W, KH, KW, sh, sw, ctypes.byref(oh), ctypes.byref(ow)),
           "sconv2d_infer")
    return int(oh.value), int(ow.value)


def sconv2d(I, Wt, bias, sh: int, sw: int) -> np.ndarray:
    """O[n,f,h,w] = bias[f] + sum_{c,kh,kw} I[n,c,sh*h+kh,sw*w+kw] * Wt[f,c,kh,kw]."""
    I, Wt = _f32(I), _f32(Wt)
    N, C, H, W = I.shape
    F, C2, KH, KW = Wt.shape
    if C != C2:
        raise ValueError("sconv2d: I %s and W %s disagree on C" % (I.shape, Wt.shape))
    OH, OW = sconv2d_infer(H, W, KH, KW, sh, sw)
    bp = None
    if bias is not None:
        bias = _f32(bias)
        if bias.shape != (F,):
            raise ValueError("sconv2d: bias must be [F]")
        bp = _fp(bias)
    O = np.empty((N, F, OH, OW), dtype=np.float64)
    _check(_load().tc_oracle_sconv2d(_fp(I), _fp(Wt), bp, _dp(O), N, C, F, H, W, KH, KW, sh, sw), "sconv2d")
    return O


def lut(LUT, Idx) -> np.ndarray:
    """O[i,j] = sum_k LUT[Idx[i,k], j] in float64; raises if an index lies outside the table."""
    LUT = _f32(LUT)
    Idx = np.ascontiguousarray(Idx)
    if Idx.dtype != np.int32:
        raise TypeError("lut: indices are int32, got %s" % Idx.dtype)
    E, D = LUT.shape
    B, L = Idx.shape
    O = np.empty((B, D), dtype=np.float64)
    _check(_load().tc_oracle_lut(_fp(LUT), Idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _dp(O),
                                 E, D, B, L), "lut")
    return O
