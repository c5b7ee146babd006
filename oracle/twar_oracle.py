"""ctypes loader for the C reference of the Three-Way AR transform (TEST INFRASTRUCTURE ONLY, see
twar_oracle.h).  Marshals numpy arrays; no arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "twar_oracle.c")
_LIB = os.path.join(_HERE, "libtwar_oracle.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class Params(C.Structure):
    _fields_ = [("w", (C.c_int16 * 3) * 3), ("bias", C.c_int32 * 3)]


def make_params(weights, bias) -> Params:
    """weights: 3x3 integers (Q2.14), bias: 3 integers (Q8.14)."""
    p = Params()
    for c in range(3):
        for k in range(3):
            p.w[c][k] = int(weights[c][k])
        p.bias[c] = int(bias[c])
    return p


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u8p, pp = C.POINTER(C.c_uint8), C.POINTER(Params)
        L.twar_oracle_predict.restype = C.c_int
        L.twar_oracle_predict.argtypes = [pp, C.c_int, C.c_int, C.c_int, C.c_int]
        for f in (L.twar_oracle_forward, L.twar_oracle_inverse):
            f.restype = None
            f.argtypes = [pp, C.c_uint32, C.c_uint32, C.c_uint32, u8p, u8p]
        _lib = L
    return _lib


def predict(p: Params, channel: int, a: int, b: int, c: int) -> int:
    return int(lib().twar_oracle_predict(C.byref(p), channel, a, b, c))


def _run(fn, p: Params, arr):
    a = np.ascontiguousarray(arr, dtype=np.uint8)
    assert a.ndim == 4 and a.shape[3] == 3
    out = np.zeros_like(a)
    if a.size:
        fn(C.byref(p), a.shape[0], a.shape[1], a.shape[2], a.ctypes.data_as(C.POINTER(C.c_uint8)),
           out.ctypes.data_as(C.POINTER(C.c_uint8)))
    return out


def forward(p: Params, img):
    return _run(lib().twar_oracle_forward, p, img)


def inverse(p: Params, res):
    return _run(lib().twar_oracle_inverse, p, res)
