"""ctypes loader for the mixture-of-logistics C oracle (TEST INFRASTRUCTURE ONLY, see
mix_oracle.h).  Marshals numpy arrays; no arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from .pilc_oracle import Geom, make_geom, OK, E_ARG, E_CAPACITY, E_TOO_LARGE, E_FORMAT, E_CORRUPT  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "mix_oracle.c"), os.path.join(_HERE, "pilc_oracle.c")]
_LIB = os.path.join(_HERE, "libmix_oracle.so")


def build(force: bool = False) -> str:
    newest = max(os.path.getmtime(s) for s in _SRCS + [os.path.join(_HERE, "mix_oracle.h"),
                                                       os.path.join(_HERE, "pilc_oracle.h")])
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", tmp]
                              + _SRCS + ["-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.mix_oracle_cum.restype = C.c_uint32
        L.mix_oracle_max_coded_bytes.restype = C.c_uint64
        for f in (L.mix_oracle_symbol_tables, L.mix_oracle_encode, L.mix_oracle_decode):
            f.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _prep(g, k, mu, log_scale, weight, chan_coef):
    mu = np.ascontiguousarray(mu, dtype=np.uint16)
    ls = np.ascontiguousarray(log_scale, dtype=np.int16)
    wt = np.ascontiguousarray(weight, dtype=np.uint16)
    cf = np.ascontiguousarray(chan_coef, dtype=np.int16)
    px = g.n * g.h * g.w
    if 1 <= k <= 16:  # other K are for the C side to reject
        assert mu.size == 3 * px * k and ls.size == 3 * px * k and wt.size == px * k and cf.size == 3 * g.n
    return mu, ls, wt, cf


def cum(mu_eff, log_scale, weight, prec_bits, k):
    me = np.ascontiguousarray(mu_eff, dtype=np.int64)
    ls = np.ascontiguousarray(log_scale, dtype=np.int16)
    wt = np.ascontiguousarray(weight, dtype=np.uint16)
    return int(lib().mix_oracle_cum(_p(me), _p(ls), _p(wt), C.c_int(len(me)), C.c_int(prec_bits), C.c_int(k)))


def symbol_tables(g, k, img, mu, log_scale, weight, chan_coef):
    mu, ls, wt, cf = _prep(g, k, mu, log_scale, weight, chan_coef)
    img = np.ascontiguousarray(img, dtype=np.uint8)
    cum_out = np.zeros(img.size, dtype=np.uint32)
    freq_out = np.zeros(img.size, dtype=np.uint32)
    rc = lib().mix_oracle_symbol_tables(C.byref(g), C.c_int(k), _p(img), _p(mu), _p(ls), _p(wt), _p(cf),
                                        _p(cum_out), _p(freq_out))
    return rc, cum_out.reshape(img.shape), freq_out.reshape(img.shape)


def max_coded_bytes(g):
    return int(lib().mix_oracle_max_coded_bytes(C.byref(g)))


def encode(g, k, img, mu, log_scale, weight, chan_coef, capacity=None):
    mu, ls, wt, cf = _prep(g, k, mu, log_scale, weight, chan_coef)
    img = np.ascontiguousarray(img, dtype=np.uint8)
    cap = max_coded_bytes(g) if capacity is None else capacity
    coded = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_uint64(0)
    rc = lib().mix_oracle_encode(C.byref(g), C.c_int(k), _p(img), _p(mu), _p(ls), _p(wt), _p(cf), _p(coded),
                                 C.c_uint64(cap), C.byref(nbytes))
    return rc, coded[: nbytes.value].copy()


def decode(g, k, coded, mu, log_scale, weight, chan_coef):
    mu, ls, wt, cf = _prep(g, k, mu, log_scale, weight, chan_coef)
    coded = np.ascontiguousarray(coded, dtype=np.uint8)
    out = np.zeros((g.n, g.h, g.w, 3), dtype=np.uint8)
    rc = lib().mix_oracle_decode(C.byref(g), C.c_int(k), _p(coded), C.c_uint64(coded.size), _p(mu), _p(ls),
                                 _p(wt), _p(cf), _p(out))
    return rc, out
