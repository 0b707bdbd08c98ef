"""ctypes binding of the C oracle (oracle/mbq_oracle.c).  TEST AND BENCHMARK INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmbq_oracle.so")
_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            from . import build as b

            b.build()
        lib = ctypes.CDLL(LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.mbq_oracle_max_threads.restype = ctypes.c_int
        lib.mbq_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.mbq_oracle_encode.argtypes = [p, i64, i64, p, p, p]
        lib.mbq_oracle_route.argtypes = [p, i64, i64, p, p, p, p, p]
        lib.mbq_oracle_bucket.argtypes = [p, i64, p, p]
        lib.mbq_oracle_linear.argtypes = [p, i64, i64, p, p, p, i64, p, p]
        for f in (lib.mbq_oracle_set_threads, lib.mbq_oracle_encode, lib.mbq_oracle_route, lib.mbq_oracle_bucket,
                  lib.mbq_oracle_linear):
            f.restype = None
        _lib = lib
    return _lib


def _p(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def max_threads() -> int:
    return int(load().mbq_oracle_max_threads())


def set_threads(n: int) -> None:
    load().mbq_oracle_set_threads(int(n))


def encode(W: np.ndarray):
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    codes = np.empty((4, N, K), dtype=np.uint8)
    s0 = np.empty((N, K // 128), dtype=np.float32)
    z0 = np.empty((N, K // 128), dtype=np.float32)
    load().mbq_oracle_encode(_p(W), N, K, _p(codes), _p(s0), _p(z0))
    return codes, s0, z0


def route(x_bits: np.ndarray, Wr: np.ndarray, br: np.ndarray):
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    Wr = np.ascontiguousarray(Wr, dtype=np.float32)
    br = np.ascontiguousarray(br, dtype=np.float32)
    T, K = x_bits.shape
    S = np.empty((T, 4), dtype=np.float64)
    prec = np.empty(T, dtype=np.int32)
    gap = np.empty(T, dtype=np.float64)
    load().mbq_oracle_route(_p(x_bits), T, K, _p(Wr), _p(br), _p(S), _p(prec), _p(gap))
    return S, prec, gap


def bucket(prec: np.ndarray):
    prec = np.ascontiguousarray(prec, dtype=np.int32)
    perm = np.empty(len(prec), dtype=np.int32)
    offsets = np.empty(5, dtype=np.int32)
    load().mbq_oracle_bucket(_p(prec), len(prec), _p(perm), _p(offsets))
    return perm, offsets


def linear(x_bits: np.ndarray, codes: np.ndarray, s0: np.ndarray, z0: np.ndarray, prec: np.ndarray) -> np.ndarray:
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    s0 = np.ascontiguousarray(s0, dtype=np.float32)
    z0 = np.ascontiguousarray(z0, dtype=np.float32)
    prec = np.ascontiguousarray(prec, dtype=np.int32)
    T, K = x_bits.shape
    N = codes.shape[1]
    Y = np.empty((T, N), dtype=np.float64)
    load().mbq_oracle_linear(_p(x_bits), T, K, _p(codes), _p(s0), _p(z0), N, _p(prec), _p(Y))
    return Y
