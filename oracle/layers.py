"""ctypes front of the C oracle (oracle/bs_oracle.c) -- TEST INFRASTRUCTURE.

One Python function per layer of Section 2 of the paper (element-wise:
normalisation, ReLU, residual add; pooling: max, average).  Every function
takes and returns whole NCHW float32 numpy arrays.  Nothing here is used by
the HIP library or its binding.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = None

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_i32p = C.POINTER(C.c_int32)
_i64 = C.c_int64


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.bso_round_bf16.argtypes = [_f32p, _i64]
        L.bso_round_f16.argtypes = [_f32p, _i64]
        L.bso_bn_fold.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_double, _i64, _f32p, _f32p]
        L.bso_batchnorm.argtypes = [_f32p, _f32p, _i64, _i64, _i64, _i64, _f32p, _f32p]
        L.bso_batchnorm_textbook_f64.argtypes = [_f32p, _f64p, _i64, _i64, _i64, _i64,
                                                 _f32p, _f32p, _f32p, _f32p, C.c_double]
        L.bso_relu.argtypes = [_f32p, _f32p, _i64]
        L.bso_add.argtypes = [_f32p, _f32p, _f32p, _i64]
        L.bso_leaky_relu.argtypes = [_f32p, _f32p, _i64, C.c_float]
        L.bso_clamp.argtypes = [_f32p, _f32p, _i64, C.c_float, C.c_float]
        L.bso_pool_out.argtypes = [_i64] * 4 + [C.c_int]
        L.bso_pool_out.restype = _i64
        L.bso_maxpool.argtypes = [_f32p, _f32p, _i32p] + [_i64] * 10 + [C.c_int]
        L.bso_avgpool.argtypes = [_f32p, _f32p] + [_i64] * 10 + [C.c_int, C.c_int]
        for f in (L.bso_round_bf16, L.bso_round_f16, L.bso_bn_fold, L.bso_batchnorm, L.bso_batchnorm_textbook_f64,
                  L.bso_relu, L.bso_add, L.bso_maxpool, L.bso_avgpool, L.bso_leaky_relu, L.bso_clamp):
            f.restype = None
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a: np.ndarray):
    return a.ctypes.data_as(_f32p)


def _nchw(x):
    if x.ndim != 4:
        raise ValueError("expected an NCHW tensor")
    return tuple(int(v) for v in x.shape)


def round_bf16(x) -> np.ndarray:
    y = _f32(x).copy()
    lib().bso_round_bf16(_p(y), y.size)
    return y


def round_f16(x) -> np.ndarray:
    y = _f32(x).copy()
    lib().bso_round_f16(_p(y), y.size)
    return y


def round_to(x, dtype: str) -> np.ndarray:
    """Storage rounding of a layer output: none for "f32", bfloat16 / binary16 otherwise."""
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "f16":
        return round_f16(x)
    return x


def bn_fold(gamma, beta, mean, var, eps):
    gamma, beta, mean, var = (_f32(v) for v in (gamma, beta, mean, var))
    c = gamma.size
    scale = np.empty(c, np.float32)
    shift = np.empty(c, np.float32)
    lib().bso_bn_fold(_p(gamma), _p(beta), _p(mean), _p(var), float(eps), c, _p(scale), _p(shift))
    return scale, shift


def batchnorm(x, gamma, beta, mean, var, eps) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = _nchw(x)
    if any(np.asarray(v).size != c for v in (gamma, beta, mean, var)):
        raise ValueError("BatchNorm parameter length must equal C")
    scale, shift = bn_fold(gamma, beta, mean, var, eps)
    y = np.empty_like(x)
    lib().bso_batchnorm(_p(x), _p(y), n, c, h, w, _p(scale), _p(shift))
    return y


def batchnorm_textbook_f64(x, gamma, beta, mean, var, eps) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = _nchw(x)
    gamma, beta, mean, var = (_f32(v) for v in (gamma, beta, mean, var))
    y = np.empty(x.shape, np.float64)
    lib().bso_batchnorm_textbook_f64(_p(x), y.ctypes.data_as(_f64p), n, c, h, w, _p(gamma),
                                     _p(beta), _p(mean), _p(var), float(eps))
    return y


def relu(x) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().bso_relu(_p(x), _p(y), x.size)
    return y


def leaky_relu(x, slope) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().bso_leaky_relu(_p(x), _p(y), x.size, float(np.float32(slope)))
    return y


def clamp(x, lo, hi) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().bso_clamp(_p(x), _p(y), x.size, float(np.float32(lo)), float(np.float32(hi)))
    return y


def add(a, r) -> np.ndarray:
    a, r = _f32(a), _f32(r)
    if a.shape != r.shape:
        raise ValueError("residual shape differs from the activation's")
    y = np.empty_like(a)
    lib().bso_add(_p(a), _p(r), _p(y), a.size)
    return y


def pool_out(size, k, s, p, ceil_mode=False) -> int:
    return int(lib().bso_pool_out(int(size), int(k), int(s), int(p), 1 if ceil_mode else 0))


def maxpool(x, k, s, p, return_indices=False, ceil_mode=False):
    x = _f32(x)
    n, c, h, w = _nchw(x)
    ho, wo = pool_out(h, k[0], s[0], p[0], ceil_mode), pool_out(w, k[1], s[1], p[1], ceil_mode)
    if ho < 1 or wo < 1:
        raise ValueError("pool output would be empty")
    y = np.empty((n, c, ho, wo), np.float32)
    idx = np.empty((n, c, ho, wo), np.int32)
    lib().bso_maxpool(_p(x), _p(y), idx.ctypes.data_as(_i32p), n, c, h, w,
                      k[0], k[1], s[0], s[1], p[0], p[1], 1 if ceil_mode else 0)
    return (y, idx) if return_indices else y


def avgpool(x, k, s, p, count_include_pad=True, ceil_mode=False) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = _nchw(x)
    ho, wo = pool_out(h, k[0], s[0], p[0], ceil_mode), pool_out(w, k[1], s[1], p[1], ceil_mode)
    if ho < 1 or wo < 1:
        raise ValueError("pool output would be empty")
    y = np.empty((n, c, ho, wo), np.float32)
    lib().bso_avgpool(_p(x), _p(y), n, c, h, w, k[0], k[1], s[0], s[1], p[0], p[1],
                      1 if count_include_pad else 0, 1 if ceil_mode else 0)
    return y


def set_threads(n: int) -> None:
    """Limit the OpenMP team of the C oracle (used by the CPU-baseline timing)."""
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def max_threads() -> int:
    return int(C.CDLL("libgomp.so.1").omp_get_max_threads())

