"""ctypes access to the CPU oracle in qg_oracle.c.

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's cpu_baseline leg may
import this module.  It does argument marshalling only; all arithmetic is in the C file.
Array conventions: W [N,K] fp32, q [N,K] uint8, s [N,K/G] fp32, z [N,K/G] uint8,
canonical packed codes uint32 [K*b/32, N], canonical scales fp32 [K/G, N], canonical packed
zeros uint32 [ceil(K/G*b/32), N].
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.qgo_threads.restype = i32
        L.qgo_set_threads.restype = None
        L.qgo_set_threads.argtypes = [i32]
        L.qgo_code_words.restype = i64
        L.qgo_code_words.argtypes = [i64, i32]
        L.qgo_storage_bits.restype = i64
        L.qgo_storage_bits.argtypes = [i64, i64, i32, i32]
        sigs = {
            "qgo_quantize": [vp, i64, i64, i32, i32, vp, vp, vp],
            "qgo_dequantize": [vp, vp, vp, i64, i64, i32, vp],
            "qgo_pack_codes": [vp, i64, i64, i32, vp],
            "qgo_unpack_codes": [vp, i64, i64, i32, vp],
            "qgo_pack_zeros": [vp, i64, i64, i32, vp],
            "qgo_unpack_zeros": [vp, i64, i64, i32, vp],
            "qgo_transpose_scales": [vp, i64, i64, vp],
            "qgo_matvec": [vp, vp, vp, i64, i64, i32, vp, vp],
            "qgo_matvec_factored": [vp, vp, vp, i64, i64, i32, vp, vp],
            "qgo_matvec_packed": [vp, vp, vp, i64, i64, i32, i32, vp, vp],
            "qgo_matmul_small": [vp, vp, vp, i64, i64, i32, vp, i64, vp],
            "qgo_row_norms": [vp, vp, vp, i64, i64, i32, vp],
        }
        L.qgo_swiglu.restype = None
        L.qgo_swiglu.argtypes = [vp, vp, i64, vp]
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.restype = i32
            fn.argtypes = args
        _LIB = L
    return _LIB


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad argument (code {rc})")


def threads():
    return int(lib().qgo_threads())


def set_threads(n: int):
    lib().qgo_set_threads(int(n))


def quantize(W, bits, group):
    W = _c(W, np.float32)
    N, K = W.shape
    if group <= 0 or K % group:
        raise ValueError("oracle quantize: K must be a multiple of group")
    q = np.empty((N, K), np.uint8)
    s = np.empty((N, K // group), np.float32)
    z = np.empty((N, K // group), np.uint8)
    _check(lib().qgo_quantize(_p(W), N, K, bits, group, _p(q), _p(s), _p(z)), "quantize")
    return q, s, z


def dequantize(q, s, z, group):
    q, s, z = _c(q, np.uint8), _c(s, np.float32), _c(z, np.uint8)
    N, K = q.shape
    out = np.empty((N, K), np.float64)
    _check(lib().qgo_dequantize(_p(q), _p(s), _p(z), N, K, group, _p(out)), "dequantize")
    return out


def pack_codes(q, bits):
    q = _c(q, np.uint8)
    N, K = q.shape
    P = np.empty((int(lib().qgo_code_words(K, bits)), N), np.uint32)
    _check(lib().qgo_pack_codes(_p(q), N, K, bits, _p(P)), "pack_codes")
    return P


def unpack_codes(P, K, bits):
    P = _c(P, np.uint32)
    N = P.shape[1]
    q = np.empty((N, K), np.uint8)
    _check(lib().qgo_unpack_codes(_p(P), N, K, bits, _p(q)), "unpack_codes")
    return q


def pack_zeros(z, bits):
    z = _c(z, np.uint8)
    N, G = z.shape
    Zp = np.empty((int(lib().qgo_code_words(G, bits)), N), np.uint32)
    _check(lib().qgo_pack_zeros(_p(z), N, G, bits, _p(Zp)), "pack_zeros")
    return Zp


def unpack_zeros(Zp, ngroups, bits):
    Zp = _c(Zp, np.uint32)
    N = Zp.shape[1]
    z = np.empty((N, ngroups), np.uint8)
    _check(lib().qgo_unpack_zeros(_p(Zp), N, ngroups, bits, _p(z)), "unpack_zeros")
    return z


def transpose_scales(s):
    s = _c(s, np.float32)
    N, G = s.shape
    St = np.empty((G, N), np.float32)
    _check(lib().qgo_transpose_scales(_p(s), N, G, _p(St)), "transpose_scales")
    return St


def storage_bits(N, K, bits, group):
    return int(lib().qgo_storage_bits(N, K, bits, group))


def matvec(q, s, z, group, x):
    q, s, z, x = _c(q, np.uint8), _c(s, np.float32), _c(z, np.uint8), _c(x, np.float32)
    N, K = q.shape
    y = np.empty(N, np.float64)
    _check(lib().qgo_matvec(_p(q), _p(s), _p(z), N, K, group, _p(x), _p(y)), "matvec")
    return y


def matvec_factored(q, s, z, group, x):
    q, s, z, x = _c(q, np.uint8), _c(s, np.float32), _c(z, np.uint8), _c(x, np.float32)
    N, K = q.shape
    y = np.empty(N, np.float64)
    _check(lib().qgo_matvec_factored(_p(q), _p(s), _p(z), N, K, group, _p(x), _p(y)),
           "matvec_factored")
    return y


def matvec_packed(P, St, Zp, K, bits, group, x):
    P, St, Zp, x = _c(P, np.uint32), _c(St, np.float32), _c(Zp, np.uint32), _c(x, np.float32)
    N = P.shape[1]
    y = np.empty(N, np.float64)
    _check(lib().qgo_matvec_packed(_p(P), _p(St), _p(Zp), N, K, bits, group, _p(x), _p(y)),
           "matvec_packed")
    return y


def matmul_small(q, s, z, group, X):
    q, s, z, X = _c(q, np.uint8), _c(s, np.float32), _c(z, np.uint8), _c(X, np.float32)
    N, K = q.shape
    M = X.shape[0]
    Y = np.empty((M, N), np.float64)
    _check(lib().qgo_matmul_small(_p(q), _p(s), _p(z), N, K, group, _p(X), M, _p(Y)),
           "matmul_small")
    return Y


def row_norms(q, s, z, group):
    q, s, z = _c(q, np.uint8), _c(s, np.float32), _c(z, np.uint8)
    N, K = q.shape
    out = np.empty(N, np.float64)
    _check(lib().qgo_row_norms(_p(q), _p(s), _p(z), N, K, group, _p(out)), "row_norms")
    return out


def swiglu(g, u):
    """h = silu(g) * u in fp64 (the gated combination after the "gate" and "up" products)."""
    g, u = _c(g, np.float64), _c(u, np.float64)
    h = np.empty_like(g)
    lib().qgo_swiglu(_p(g), _p(u), g.size, _p(h))
    return h

