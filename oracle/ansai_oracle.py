"""ctypes loader for the C reference of the table-driven coder (TEST INFRASTRUCTURE ONLY, see
ansai_oracle.h).  Marshals numpy arrays; no arithmetic of the method lives here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ansai_oracle.c")
_LIB = os.path.join(_HERE, "libansai_oracle.so")

OK, E_ARG, E_CAPACITY, E_FORMAT, E_CORRUPT = 0, -1, -3, -5, -6


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class Model(C.Structure):
    _fields_ = [("prec_bits", C.c_int), ("num_dist", C.c_int), ("num_sym", C.c_int),
                ("mass", C.POINTER(C.c_uint32))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u8p, u16p, u32p, i32p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_uint32, C.c_int32))
        mp = C.POINTER(Model)
        L.ansai_oracle_build_tables.restype = C.c_int
        L.ansai_oracle_build_tables.argtypes = [mp, i32p, u32p, u8p, u8p, u16p]
        L.ansai_oracle_encode_piece_direct.restype = C.c_int64
        L.ansai_oracle_encode_piece_direct.argtypes = [mp, u8p, u8p, C.c_int64, u8p, u32p]
        L.ansai_oracle_decode_piece_direct.restype = C.c_int
        L.ansai_oracle_decode_piece_direct.argtypes = [mp, u8p, C.c_int64, u8p, C.c_int64, C.c_uint32, u8p]
        L.ansai_oracle_max_coded_bytes.restype = C.c_uint64
        L.ansai_oracle_max_coded_bytes.argtypes = [C.c_uint32, C.c_uint32, C.c_int]
        L.ansai_oracle_encode.restype = C.c_int
        L.ansai_oracle_encode.argtypes = [mp, C.c_uint32, C.c_uint32, u8p, u8p, u8p, C.c_uint64,
                                          C.POINTER(C.c_uint64)]
        L.ansai_oracle_decode.restype = C.c_int
        L.ansai_oracle_decode.argtypes = [mp, C.c_uint32, C.c_uint32, u8p, u8p, C.c_uint64, u8p]
        L.ansai_oracle_center.restype = None
        L.ansai_oracle_center.argtypes = [u8p, u8p, C.c_uint64, C.c_int, u8p]
        _lib = L
    return _lib


def _ptr(a: np.ndarray, ctype):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(ctype))


class _Held:
    """A Model plus the array its pointer refers to."""

    def __init__(self, prec_bits: int, mass):
        self.mass = np.ascontiguousarray(mass, dtype=np.uint32)
        assert self.mass.ndim == 2
        self.c = Model(int(prec_bits), self.mass.shape[0], self.mass.shape[1], _ptr(self.mass, C.c_uint32))

    @property
    def ref(self):
        return C.byref(self.c)


def build_tables(prec_bits: int, mass):
    md = _Held(prec_bits, mass)
    d, x = md.mass.shape
    top = 1 << prec_bits
    delta = np.zeros((d, x), dtype=np.int32)
    phi = np.zeros((d, x), dtype=np.uint32)
    theta = np.zeros((d, top), dtype=np.uint8)
    nbits = np.zeros((d, top), dtype=np.uint8)
    nxt = np.zeros((d, top), dtype=np.uint16)
    rc = lib().ansai_oracle_build_tables(md.ref, _ptr(delta, C.c_int32), _ptr(phi, C.c_uint32),
                                         _ptr(theta, C.c_uint8), _ptr(nbits, C.c_uint8), _ptr(nxt, C.c_uint16))
    if rc != OK:
        raise ValueError("ansai build_tables rc=%d" % rc)
    return delta, phi, theta, nbits, nxt


def encode_piece_direct(prec_bits: int, mass, sym, dist):
    md = _Held(prec_bits, mass)
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    dist = np.ascontiguousarray(dist, dtype=np.uint8)
    assert sym.shape == dist.shape and sym.ndim == 1
    bits = np.zeros(max(sym.size * prec_bits, 1), dtype=np.uint8)
    state = C.c_uint32(0)
    n = lib().ansai_oracle_encode_piece_direct(md.ref, _ptr(sym, C.c_uint8), _ptr(dist, C.c_uint8), sym.size,
                                              _ptr(bits, C.c_uint8), C.byref(state))
    if n < 0:
        raise ValueError("ansai encode_piece_direct rc=%d" % n)
    return bits[:n].copy(), int(state.value)


def decode_piece_direct(prec_bits: int, mass, dist, bits, state: int):
    md = _Held(prec_bits, mass)
    dist = np.ascontiguousarray(dist, dtype=np.uint8)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    out = np.zeros(max(dist.size, 1), dtype=np.uint8)
    bbuf = bits if bits.size else np.zeros(1, dtype=np.uint8)
    rc = lib().ansai_oracle_decode_piece_direct(md.ref, _ptr(dist, C.c_uint8), dist.size, _ptr(bbuf, C.c_uint8),
                                               bits.size, int(state), _ptr(out, C.c_uint8))
    return rc, out[: dist.size].copy()


def max_coded_bytes(pieces: int, count: int, prec_bits: int) -> int:
    return int(lib().ansai_oracle_max_coded_bytes(pieces, count, prec_bits))


def encode(prec_bits: int, mass, sym, dist, capacity: int | None = None):
    """sym, dist: uint8 [pieces, count].  Returns (rc, container bytes)."""
    md = _Held(prec_bits, mass)
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    dist = np.ascontiguousarray(dist, dtype=np.uint8)
    assert sym.ndim == 2 and sym.shape == dist.shape
    pieces, count = sym.shape
    cap = max_coded_bytes(pieces, count, prec_bits) if capacity is None else int(capacity)
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_uint64(0)
    rc = lib().ansai_oracle_encode(md.ref, pieces, count, _ptr(sym, C.c_uint8), _ptr(dist, C.c_uint8),
                                   _ptr(out, C.c_uint8), cap, C.byref(nbytes))
    return rc, out[: nbytes.value].copy() if rc == OK else out[:0]


def decode(prec_bits: int, mass, dist, coded):
    md = _Held(prec_bits, mass)
    dist = np.ascontiguousarray(dist, dtype=np.uint8)
    coded = np.ascontiguousarray(coded, dtype=np.uint8)
    assert dist.ndim == 2
    pieces, count = dist.shape
    out = np.zeros((pieces, count), dtype=np.uint8)
    cbuf = coded if coded.size else np.zeros(1, dtype=np.uint8)
    rc = lib().ansai_oracle_decode(md.ref, pieces, count, _ptr(dist, C.c_uint8), _ptr(cbuf, C.c_uint8),
                                   coded.size, _ptr(out, C.c_uint8))
    return rc, out


def center(values, mu, inverse: bool = False):
    """(r - mu + 128) mod 256, or its inverse (Sec. 3.3)."""
    a = np.ascontiguousarray(values, dtype=np.uint8)
    m = np.ascontiguousarray(mu, dtype=np.uint8)
    assert a.shape == m.shape
    out = np.zeros(max(a.size, 1), dtype=np.uint8)
    if a.size:
        lib().ansai_oracle_center(_ptr(a.reshape(-1), C.c_uint8), _ptr(m.reshape(-1), C.c_uint8), a.size,
                                  1 if inverse else 0, _ptr(out, C.c_uint8))
    return out[: a.size].reshape(a.shape)
