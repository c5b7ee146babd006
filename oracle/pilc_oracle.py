"""ctypes loader for the C oracle (TEST INFRASTRUCTURE ONLY, see pilc_oracle.h).

Marshals numpy arrays into the plain-C reference.  No arithmetic of the method
lives here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pilc_oracle.c")
_LIB = os.path.join(_HERE, "libpilc_oracle.so")

OK = 0
E_ARG = -1
E_CAPACITY = -3
E_TOO_LARGE = -4
E_FORMAT = -5
E_CORRUPT = -6


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no -march tricks).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


class Geom(C.Structure):
    _fields_ = [
        ("n", C.c_uint32),
        ("h", C.c_uint32),
        ("w", C.c_uint32),
        ("prec_bits", C.c_uint32),
        ("lane_mode", C.c_uint32),
        ("lane_a", C.c_uint32),
        ("lane_b", C.c_uint32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u8p, u16p, i16p, u32p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_int16, C.c_uint32))
        gp = C.POINTER(Geom)
        L.pilc_oracle_table_sigmoid.restype = u32p
        L.pilc_oracle_table_exp_hi.restype = u32p
        L.pilc_oracle_table_exp_lo.restype = u32p
        L.pilc_oracle_lane_count.restype = C.c_uint64
        L.pilc_oracle_lane_count.argtypes = [gp]
        L.pilc_oracle_lane_pixels.restype = C.c_uint64
        L.pilc_oracle_lane_pixels.argtypes = [gp, C.c_uint64]
        L.pilc_oracle_lane_pixel_index.restype = C.c_uint64
        L.pilc_oracle_lane_pixel_index.argtypes = [gp, C.c_uint64, C.c_uint64]
        L.pilc_oracle_mean_shift.restype = None
        L.pilc_oracle_mean_shift.argtypes = [u8p, u16p, i16p, C.POINTER(C.c_int64)]
        L.pilc_oracle_inv_scale.restype = C.c_int64
        L.pilc_oracle_inv_scale.argtypes = [C.c_int32]
        L.pilc_oracle_edge_cdf.restype = C.c_uint32
        L.pilc_oracle_edge_cdf.argtypes = [C.c_int64, C.c_int64, C.c_int]
        L.pilc_oracle_cum.restype = C.c_uint32
        L.pilc_oracle_cum.argtypes = [C.c_int64, C.c_int32, C.c_int, C.c_int]
        L.pilc_oracle_symbol_tables.restype = C.c_int
        L.pilc_oracle_symbol_tables.argtypes = [gp, u8p, u16p, i16p, i16p, u32p, u32p]
        L.pilc_oracle_cross_entropy_bits.restype = C.c_double
        L.pilc_oracle_cross_entropy_bits.argtypes = [gp, u8p, u16p, i16p, i16p]
        L.pilc_oracle_rans_encode_tables.restype = C.c_int
        L.pilc_oracle_rans_encode_tables.argtypes = [
            u32p, u32p, C.c_uint64, C.c_int, u16p, C.POINTER(C.c_uint64), u32p]
        L.pilc_oracle_rans_decode_tables.restype = C.c_int
        L.pilc_oracle_rans_decode_tables.argtypes = [
            u32p, C.c_uint64, C.c_int, u16p, C.c_uint64, C.c_uint32, u8p]
        L.pilc_oracle_max_coded_bytes.restype = C.c_uint64
        L.pilc_oracle_max_coded_bytes.argtypes = [gp]
        L.pilc_oracle_encode.restype = C.c_int
        L.pilc_oracle_encode.argtypes = [gp, u8p, u16p, i16p, i16p, u8p, C.c_uint64,
                                         C.POINTER(C.c_uint64)]
        L.pilc_oracle_decode.restype = C.c_int
        L.pilc_oracle_decode.argtypes = [gp, u8p, C.c_uint64, u16p, i16p, i16p, u8p]
        _lib = L
    return _lib


def _ptr(a: np.ndarray, ctype):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ctype))


def make_geom(n, h, w, prec_bits, lane_mode, lane_a, lane_b=0) -> Geom:
    return Geom(int(n), int(h), int(w), int(prec_bits), int(lane_mode), int(lane_a), int(lane_b))


def _check_inputs(g: Geom, img, mu, log_scale, chan_coef):
    sym = g.n * g.h * g.w * 3
    assert img is None or (img.dtype == np.uint8 and img.size == sym)
    assert mu.dtype == np.uint16 and mu.size == sym
    assert log_scale.dtype == np.int16 and log_scale.size == sym
    assert chan_coef.dtype == np.int16 and chan_coef.size == g.n * 3


def tables() -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    L = lib()
    t = np.ctypeslib.as_array(L.pilc_oracle_table_sigmoid(), shape=(2049,)).copy()
    eh = np.ctypeslib.as_array(L.pilc_oracle_table_exp_hi(), shape=(640,)).copy()
    el = np.ctypeslib.as_array(L.pilc_oracle_table_exp_lo(), shape=(64,)).copy()
    return t, eh, el


def lane_count(g: Geom) -> int:
    return int(lib().pilc_oracle_lane_count(C.byref(g)))


def lane_pixels(g: Geom, lane: int) -> int:
    return int(lib().pilc_oracle_lane_pixels(C.byref(g), lane))


def lane_pixel_index(g: Geom, lane: int, t: int) -> int:
    return int(lib().pilc_oracle_lane_pixel_index(C.byref(g), lane, t))


def mean_shift(x, mu, coef):
    xa = np.ascontiguousarray(x, dtype=np.uint8)
    ma = np.ascontiguousarray(mu, dtype=np.uint16)
    ca = np.ascontiguousarray(coef, dtype=np.int16)
    out = np.zeros(3, dtype=np.int64)
    lib().pilc_oracle_mean_shift(_ptr(xa, C.c_uint8), _ptr(ma, C.c_uint16), _ptr(ca, C.c_int16),
                                 _ptr(out, C.c_int64))
    return [int(v) for v in out]


def inv_scale(log_scale_q: int) -> int:
    return int(lib().pilc_oracle_inv_scale(int(log_scale_q)))


def edge_cdf(mu_eff: int, inv_s: int, k: int) -> int:
    return int(lib().pilc_oracle_edge_cdf(int(mu_eff), int(inv_s), int(k)))


def cum(mu_eff: int, log_scale_q: int, prec_bits: int, k: int) -> int:
    return int(lib().pilc_oracle_cum(int(mu_eff), int(log_scale_q), int(prec_bits), int(k)))


def symbol_tables(g: Geom, img, mu, log_scale, chan_coef):
    _check_inputs(g, img, mu, log_scale, chan_coef)
    sym = g.n * g.h * g.w * 3
    cum_out = np.empty(sym, dtype=np.uint32)
    freq_out = np.empty(sym, dtype=np.uint32)
    rc = lib().pilc_oracle_symbol_tables(
        C.byref(g), _ptr(img, C.c_uint8), _ptr(mu, C.c_uint16), _ptr(log_scale, C.c_int16),
        _ptr(chan_coef, C.c_int16), _ptr(cum_out, C.c_uint32), _ptr(freq_out, C.c_uint32))
    if rc != OK:
        raise ValueError("oracle symbol_tables rc=%d" % rc)
    return cum_out, freq_out


def cross_entropy_bits(g: Geom, img, mu, log_scale, chan_coef) -> float:
    _check_inputs(g, img, mu, log_scale, chan_coef)
    return float(lib().pilc_oracle_cross_entropy_bits(
        C.byref(g), _ptr(img, C.c_uint8), _ptr(mu, C.c_uint16), _ptr(log_scale, C.c_int16),
        _ptr(chan_coef, C.c_int16)))


def rans_encode_tables(cum_a, freq_a, prec_bits: int):
    cum_a = np.ascontiguousarray(cum_a, dtype=np.uint32)
    freq_a = np.ascontiguousarray(freq_a, dtype=np.uint32)
    n = cum_a.size
    words = np.zeros(max(n, 1), dtype=np.uint16)
    nwords = C.c_uint64(0)
    state = C.c_uint32(0)
    rc = lib().pilc_oracle_rans_encode_tables(
        _ptr(cum_a, C.c_uint32), _ptr(freq_a, C.c_uint32), n, int(prec_bits),
        _ptr(words, C.c_uint16), C.byref(nwords), C.byref(state))
    if rc != OK:
        raise ValueError("oracle rans_encode_tables rc=%d" % rc)
    return words[: nwords.value].copy(), int(state.value)


def rans_decode_tables(table_cum, prec_bits: int, words, state: int):
    table_cum = np.ascontiguousarray(table_cum, dtype=np.uint32)
    assert table_cum.ndim == 2 and table_cum.shape[1] == 257
    words = np.ascontiguousarray(words, dtype=np.uint16)
    n = table_cum.shape[0]
    sym = np.zeros(max(n, 1), dtype=np.uint8)
    wbuf = words if words.size else np.zeros(1, dtype=np.uint16)
    rc = lib().pilc_oracle_rans_decode_tables(
        _ptr(table_cum, C.c_uint32), n, int(prec_bits), _ptr(wbuf, C.c_uint16), words.size,
        int(state), _ptr(sym, C.c_uint8))
    return rc, sym[:n].copy()


def max_coded_bytes(g: Geom) -> int:
    return int(lib().pilc_oracle_max_coded_bytes(C.byref(g)))


def encode(g: Geom, img, mu, log_scale, chan_coef, capacity: int | None = None):
    """Returns (rc, container bytes as a uint8 array)."""
    _check_inputs(g, img, mu, log_scale, chan_coef)
    cap = max_coded_bytes(g) if capacity is None else int(capacity)
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_uint64(0)
    rc = lib().pilc_oracle_encode(
        C.byref(g), _ptr(img, C.c_uint8), _ptr(mu, C.c_uint16), _ptr(log_scale, C.c_int16),
        _ptr(chan_coef, C.c_int16), _ptr(out, C.c_uint8), cap, C.byref(nbytes))
    return rc, out[: nbytes.value].copy() if rc == OK else out[:0]


def decode(g: Geom, coded, mu, log_scale, chan_coef):
    """Returns (rc, image uint8 [n,h,w,3])."""
    _check_inputs(g, None, mu, log_scale, chan_coef)
    coded = np.ascontiguousarray(coded, dtype=np.uint8)
    img = np.zeros((g.n, g.h, g.w, 3), dtype=np.uint8)
    cbuf = coded if coded.size else np.zeros(1, dtype=np.uint8)
    rc = lib().pilc_oracle_decode(
        C.byref(g), _ptr(cbuf, C.c_uint8), coded.size, _ptr(mu, C.c_uint16),
        _ptr(log_scale, C.c_int16), _ptr(chan_coef, C.c_int16), _ptr(img, C.c_uint8))
    return rc, img
