"""ctypes access to the plain-C oracle (`pb_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
All arithmetic of the method lives in the C file; this wrapper only allocates
numpy arrays and passes pointers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pb_oracle.c")
_LIB = os.path.join(_HERE, "libpb_oracle.so")
_lib = None

c_i64 = ctypes.c_int64
c_int = ctypes.c_int
c_f32 = ctypes.c_float
_P = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction: IEEE fp32 divide and rint)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.pbo_quantize.argtypes = [_P, c_i64, c_int, _P, _P]
        L.pbo_quantize.restype = c_int
        L.pbo_quantize_mode.argtypes = [_P, c_i64, c_int, c_int, _P, _P]
        L.pbo_quantize_mode.restype = c_int
        L.pbo_bitlayers.argtypes = [_P, c_i64, c_int, _P, _P]
        L.pbo_bitlayers.restype = c_int
        L.pbo_scales.argtypes = [c_f32, c_int, _P]
        L.pbo_scales.restype = None
        L.pbo_fixed_point.argtypes = [_P, c_i64, c_int, c_int, _P]
        L.pbo_fixed_point.restype = c_int
        L.pbo_planes.argtypes = [_P, c_i64, c_int, _P, _P]
        L.pbo_planes.restype = c_int
        L.pbo_bit_products.argtypes = [_P, _P, c_i64, c_i64, c_int, _P]
        L.pbo_bit_products.restype = None
        L.pbo_plane_weighting.argtypes = [_P, _P, c_i64, c_int, _P]
        L.pbo_plane_weighting.restype = None
        L.pbo_accumulate.argtypes = [_P, _P, c_int, c_i64, _P]
        L.pbo_accumulate.restype = None
        L.pbo_dequant.argtypes = [_P, _P, c_int, c_i64, c_int, _P]
        L.pbo_dequant.restype = None
        L.pbo_matmul_bitserial.argtypes = [_P, _P, _P, c_int, c_int, c_i64, c_i64, _P, c_i64, c_int, c_int,
                                           _P, _P, _P]
        L.pbo_matmul_bitserial.restype = c_int
        L.pbo_layer_products_direct.argtypes = [_P, c_int, c_i64, c_i64, _P, c_i64, _P]
        L.pbo_layer_products_direct.restype = None
        L.pbo_words_per_row.argtypes = [c_i64]
        L.pbo_words_per_row.restype = c_i64
        L.pbo_pack_words.argtypes = [_P, c_i64, c_i64, _P]
        L.pbo_pack_words.restype = None
        L.pbo_matmul_words.argtypes = [_P, _P, c_int, c_int, c_i64, c_i64, c_i64, c_i64, _P, c_i64, c_int, c_int,
                                       _P, _P]
        L.pbo_matmul_words.restype = c_int
        L.pbo_lstm_pointwise.argtypes = [_P, _P, _P, c_i64, c_i64, _P, _P]
        L.pbo_lstm_pointwise.restype = None
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_P)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def quantize(W, bits):
    """-> (q int32 like W, d float32 scalar)."""
    W = _c(W, np.float32)
    q = np.empty(W.shape, dtype=np.int32)
    d = np.zeros(1, dtype=np.float32)
    rc = lib().pbo_quantize(_ptr(W), W.size, bits, _ptr(q), _ptr(d))
    if rc:
        raise ValueError("pbo_quantize rc=%d" % rc)
    return q, d[0]


QUANT_SYMMETRIC, QUANT_RANGE, QUANT_SIGN, QUANT_CLIP = 0, 1, 2, 3


def quantize_mode(W, bits, mode):
    """Section 3.3's other quantizers (1 = printed range formula, 2 = 1-bit +-1 code, 3 = clipping search)."""
    W = _c(W, np.float32)
    q = np.empty(W.shape, dtype=np.int32)
    d = np.zeros(1, dtype=np.float32)
    rc = lib().pbo_quantize_mode(_ptr(W), W.size, bits, mode, _ptr(q), _ptr(d))
    if rc:
        raise ValueError("pbo_quantize_mode rc=%d" % rc)
    return q, d[0]


def bitlayers(q, bits):
    """-> (layers uint8 [bits, *q.shape], s int64 [bits])."""
    q = _c(q, np.int32)
    layers = np.empty((bits,) + q.shape, dtype=np.uint8)
    s = np.empty(bits, dtype=np.int64)
    rc = lib().pbo_bitlayers(_ptr(q), q.size, bits, _ptr(layers), _ptr(s))
    if rc:
        raise ValueError("pbo_bitlayers rc=%d" % rc)
    return layers, s


def scales(d, bits):
    out = np.empty(bits, dtype=np.float32)
    lib().pbo_scales(c_f32(float(d)), bits, _ptr(out))
    return out


def fixed_point(x, frac_bits=16, act_bits=32):
    x = _c(x, np.float32)
    xq = np.empty(x.shape, dtype=np.int32)
    rc = lib().pbo_fixed_point(_ptr(x), x.size, frac_bits, act_bits, _ptr(xq))
    if rc:
        raise ValueError("pbo_fixed_point rc=%d" % rc)
    return xq


def planes(xq, act_bits=32):
    """xq: 1-D int32 -> (planes uint8 [k, n], c int64 [k])."""
    xq = _c(xq, np.int32)
    assert xq.ndim == 1
    pl = np.empty((act_bits, xq.size), dtype=np.uint8)
    c = np.empty(act_bits, dtype=np.int64)
    rc = lib().pbo_planes(_ptr(xq), xq.size, act_bits, _ptr(pl), _ptr(c))
    if rc:
        raise ValueError("pbo_planes rc=%d" % rc)
    return pl, c


def bit_products(layer, pl):
    layer = _c(layer, np.uint8)
    pl = _c(pl, np.uint8)
    R, C = layer.shape
    k = pl.shape[0]
    assert pl.shape[1] == C
    P = np.empty((R, k), dtype=np.int64)
    lib().pbo_bit_products(_ptr(layer), _ptr(pl), R, C, k, _ptr(P))
    return P


def plane_weighting(P, c):
    P = _c(P, np.int64)
    c = _c(c, np.int64)
    R, k = P.shape
    A = np.empty(R, dtype=np.int64)
    lib().pbo_plane_weighting(_ptr(P), _ptr(c), R, k, _ptr(A))
    return A


def accumulate(A, s, m):
    A = _c(A, np.int64)
    s = _c(s, np.int64)
    R = A.shape[-1]
    assert A.shape[0] >= m
    T = np.empty(R, dtype=np.int64)
    lib().pbo_accumulate(_ptr(A), _ptr(s), m, R, _ptr(T))
    return T


def dequant(A, scales_, m, frac_bits=16):
    A = _c(A, np.int64)
    sc = _c(scales_, np.float32)
    R = A.shape[-1]
    y = np.empty(R, dtype=np.float32)
    lib().pbo_dequant(_ptr(A), _ptr(sc), m, R, frac_bits, _ptr(y))
    return y


def matmul_bitserial(layers, scales_, s, bits_used, X, frac_bits=16, act_bits=32):
    """layers uint8 [B,R,C]; X float32 [N,C] -> (A int64 [m,N,R], T int64 [N,R], Y float32 [N,R])."""
    layers = _c(layers, np.uint8)
    B, R, C = layers.shape
    X = _c(X, np.float32).reshape(-1, C)
    N = X.shape[0]
    sc = _c(scales_, np.float32)
    s = _c(s, np.int64)
    A = np.empty((bits_used, N, R), dtype=np.int64)
    T = np.empty((N, R), dtype=np.int64)
    Y = np.empty((N, R), dtype=np.float32)
    rc = lib().pbo_matmul_bitserial(_ptr(layers), _ptr(sc), _ptr(s), B, bits_used, R, C, _ptr(X), N,
                                    frac_bits, act_bits, _ptr(A), _ptr(T), _ptr(Y))
    if rc:
        raise ValueError("pbo_matmul_bitserial rc=%d" % rc)
    return A, T, Y


def layer_products_direct(layers, bits_used, xq):
    layers = _c(layers, np.uint8)
    B, R, C = layers.shape
    xq = _c(xq, np.int32).reshape(-1, C)
    N = xq.shape[0]
    A = np.empty((bits_used, N, R), dtype=np.int64)
    lib().pbo_layer_products_direct(_ptr(layers), bits_used, R, C, _ptr(xq), N, _ptr(A))
    return A


def pack_words(bits01):
    bits01 = _c(bits01, np.uint8)
    lead = bits01.shape[:-1]
    C = bits01.shape[-1]
    R = int(np.prod(lead)) if lead else 1
    Cw = lib().pbo_words_per_row(C)
    words = np.empty(lead + (Cw,), dtype=np.uint64)
    lib().pbo_pack_words(_ptr(bits01), R, C, _ptr(words))
    return words


def matmul_words(layers_w, scales_, bits_used, C, X, r0=0, r1=None, frac_bits=16, act_bits=32,
                 want_A=True, want_Y=True):
    """Packed-word tier. layers_w uint64 [B,R,Cw]; only rows [r0,r1) are computed (others left 0)."""
    layers_w = _c(layers_w, np.uint64)
    B, R, Cw = layers_w.shape
    assert Cw == lib().pbo_words_per_row(C)
    X = _c(X, np.float32).reshape(-1, C)
    N = X.shape[0]
    if r1 is None:
        r1 = R
    sc = _c(scales_, np.float32)
    A = np.zeros((bits_used, N, R), dtype=np.int64) if want_A else None
    Y = np.zeros((N, R), dtype=np.float32) if want_Y else None
    rc = lib().pbo_matmul_words(_ptr(layers_w), _ptr(sc), B, bits_used, R, C, r0, r1, _ptr(X), N,
                                frac_bits, act_bits, _ptr(A), _ptr(Y))
    if rc:
        raise ValueError("pbo_matmul_words rc=%d" % rc)
    return A, Y


def lstm_pointwise(gates, bias, c_prev):
    gates = _c(gates, np.float32)
    N = gates.shape[0]
    H = gates.shape[1] // 4
    c_prev = _c(c_prev, np.float32).reshape(N, H)
    b = None if bias is None else _c(bias, np.float32)
    h = np.empty((N, H), dtype=np.float32)
    c = np.empty((N, H), dtype=np.float32)
    lib().pbo_lstm_pointwise(_ptr(gates), _ptr(b), _ptr(c_prev), H, N, _ptr(h), _ptr(c))
    return h, c


def prepare(W, bits, mode=0):
    """Algorithm 1 as a whole: -> dict(q, d, layers, s, scales)."""
    q, d = quantize(W, bits) if mode == 0 else quantize_mode(W, bits, mode)
    layers, s = bitlayers(q, bits)
    return {"q": q, "d": d, "layers": layers, "s": s, "scales": scales(d, bits), "bits": bits}
