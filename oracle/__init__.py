"""CPU oracle (test infrastructure only): ctypes wrapper over liboracle.so.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import this package.  It shares nothing with the HIP path; inputs are the
unpacked one-value-per-byte tensors in the paper's logical orders.
"""

from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        i64, i32, vp = C.c_int64, C.c_int, C.c_void_p
        _lib.orc_threads.restype = i32
        _lib.orc_decode.argtypes = [vp, i64, i32, i32, vp]
        _lib.orc_gemm.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp]
        _lib.orc_gemm_rows.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, i64, i64, vp]
        _lib.orc_apbit_gemm.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp]
        _lib.orc_conv2d.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, vp]
        _lib.orc_quantize.argtypes = [vp, i64, C.c_float, C.c_float, i32, vp]
        _lib.orc_fold_bn.argtypes = [vp, vp, vp, vp, C.c_double, C.c_double, C.c_double, i64, vp, vp]
        _lib.orc_epilogue.argtypes = [vp, i64, i64, i64, vp, vp, vp, C.c_float, i32, vp, vp]
        _lib.orc_maxpool.argtypes = [vp, i64, i64, i64, i64, i32, i32, i32, vp]
        _lib.orc_sumpool.argtypes = [vp, i64, i64, i64, vp]
        _lib.orc_gridpool.argtypes = [vp, i64, i64, i64, i64, i32, i32, vp]
    return _lib


class OracleError(RuntimeError):
    NAMES = {1: "bad argument", 2: "stored value outside its encoding", 3: "int32 overflow", 4: "out of memory"}

    def __init__(self, code):
        super().__init__(f"oracle error {code}: {self.NAMES.get(code, '?')}")
        self.code = code


def _chk(rc):
    if rc:
        raise OracleError(rc)


def _bytes(a):
    a = np.ascontiguousarray(a)
    assert a.dtype in (np.uint8, np.int8), a.dtype
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return lib().orc_threads()


def decode(stored, bits, enc):
    s = _bytes(stored)
    out = np.empty(s.shape, np.int32)
    _chk(lib().orc_decode(_p(s), s.size, bits, enc, _p(out)))
    return out


def gemm(W, encW, p, X, encX, q):
    W, X = _bytes(W), _bytes(X)
    M, K = W.shape
    N, K2 = X.shape
    assert K == K2
    Y = np.zeros((M, N), np.int32)
    _chk(lib().orc_gemm(_p(W), encW, p, _p(X), encX, q, M, N, K, _p(Y)))
    return Y


def gemm_rows(W, encW, p, X, encX, q, m0, m1):
    """Rows m0..m1-1 of the product (returned as an (m1-m0) x N array)."""
    W, X = _bytes(W), _bytes(X)
    M, K = W.shape
    N, _ = X.shape
    Y = np.zeros((M, N), np.int32)
    _chk(lib().orc_gemm_rows(_p(W), encW, p, _p(X), encX, q, M, N, K, m0, m1, _p(Y)))
    return Y[m0:m1]


def apbit_gemm(W, encW, p, X, encX, q):
    W, X = _bytes(W), _bytes(X)
    M, K = W.shape
    N, _ = X.shape
    Y = np.zeros((M, N), np.int32)
    _chk(lib().orc_apbit_gemm(_p(W), encW, p, _p(X), encX, q, M, N, K, _p(Y)))
    return Y


def conv2d(W, encW, p, X, encX, q, stride, pad):
    """W: Cout x Cin x R x S, X: BS x Cin x H x W  ->  BS x Cout x Ho x Wo int32."""
    W, X = _bytes(W), _bytes(X)
    Cout, Cin, R, S = W.shape
    BS, Cin2, H, Wd = X.shape
    assert Cin == Cin2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (Wd + 2 * pad - S) // stride + 1
    Y = np.zeros((BS, Cout, Ho, Wo), np.int32)
    _chk(lib().orc_conv2d(_p(W), encW, p, _p(X), encX, q, BS, Cin, H, Wd, Cout, R, S, stride, pad, _p(Y)))
    return Y


def quantize(x, zero, step, bits):
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint8)
    _chk(lib().orc_quantize(_p(x), x.size, zero, step, bits, _p(out)))
    return out


def fold_bn(gamma, beta, mean, var, eps, z, s):
    g, b, m, v = (np.ascontiguousarray(a, np.float64) for a in (gamma, beta, mean, var))
    scale, bias = np.empty(g.shape, np.float32), np.empty(g.shape, np.float32)
    _chk(lib().orc_fold_bn(_p(g), _p(b), _p(m), _p(v), eps, z, s, g.size, _p(scale), _p(bias)))
    return scale, bias


def epilogue(Y, scale, bias, q_out, res=None, res_scale=0.0, want_t=False):
    """Y: BS x C x ... int32 -> (codes uint8 or None, t fp32 or None)."""
    Y = np.ascontiguousarray(Y, np.int32)
    BS, Cc = Y.shape[0], Y.shape[1]
    HW = int(np.prod(Y.shape[2:])) if Y.ndim > 2 else 1
    scale = np.ascontiguousarray(scale, np.float32)
    bias = np.ascontiguousarray(bias, np.float32)
    assert scale.size == Cc and bias.size == Cc
    if res is not None:
        res = _bytes(res)
        assert res.shape == Y.shape
    codes = np.empty(Y.shape, np.uint8) if q_out else None
    t = np.empty(Y.shape, np.float32) if want_t else None
    _chk(lib().orc_epilogue(_p(Y), BS, Cc, HW, _p(scale), _p(bias), _p(res), res_scale, q_out, _p(t), _p(codes)))
    return codes, t


def maxpool(codes, k, stride, pad):
    c = _bytes(codes)
    BS, Cc, H, Wd = c.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    out = np.empty((BS, Cc, Ho, Wo), np.uint8)
    _chk(lib().orc_maxpool(_p(c), BS, Cc, H, Wd, k, stride, pad, _p(out)))
    return out


def sumpool(codes):
    c = _bytes(codes)
    BS, Cc = c.shape[:2]
    out = np.empty((BS, Cc), np.uint8)
    _chk(lib().orc_sumpool(_p(c), BS, Cc, c.size // max(BS * Cc, 1), _p(out)))
    return out


POOL_MAX, POOL_SUM = 1, 2


def gridpool(Y, k, mode):
    """k x k grid pooling of int32 results BS x C x H x W (maximum or sum per grid; Sec. 5.2)."""
    Y = np.ascontiguousarray(Y, np.int32)
    BS, Cc, H, Wd = Y.shape
    out = np.empty((BS, Cc, H // k, Wd // k), np.int32)
    _chk(lib().orc_gridpool(_p(Y), BS, Cc, H, Wd, k, mode, _p(out)))
    return out
