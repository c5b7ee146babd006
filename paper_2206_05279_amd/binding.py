"""Thin Python binding of libpilc's C ABI: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device
memory and streams.  There is no CPU fallback: if the library has not been built, or
no GPU is present, the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpilc.so")

PILC_OK = 0
PILC_E_ARG = -1
PILC_E_WORKSPACE = -2
PILC_E_CAPACITY = -3
PILC_E_TOO_LARGE = -4
PILC_E_FORMAT = -5
PILC_E_CORRUPT = -6
PILC_E_HIP = -7
PILC_E_TIMEOUT = -8

EXPORTS = [
    "pilc_lane_count", "pilc_workspace_size", "pilc_encode", "pilc_encode_static", "pilc_decode",
    "pilc_symbol_tables",
    "pilc_set_timing", "pilc_set_kernel_policy", "pilc_set_one_pass_wait", "pilc_set_ansai_decode_waves", "pilc_last_timing", "pilc_timing_name", "pilc_strerror",
    "pilc_last_hip_error", "pilc_version",
    "pilc_ansai_table_bytes", "pilc_ansai_build_tables", "pilc_ansai_workspace_size", "pilc_ansai_encode",
    "pilc_ansai_decode", "pilc_ansai_center", "pilc_twar_forward", "pilc_twar_inverse",
    "pilc_mix_encode", "pilc_mix_decode",
]


class pilc_geom(C.Structure):
    _fields_ = [("n", C.c_uint32), ("h", C.c_uint32), ("w", C.c_uint32), ("prec_bits", C.c_uint32),
                ("lane_mode", C.c_uint32), ("lane_a", C.c_uint32), ("lane_b", C.c_uint32)]


class pilc_params(C.Structure):
    _fields_ = [("mu", C.c_void_p), ("log_scale", C.c_void_p), ("chan_coef", C.c_void_p)]


class pilc_mix_params(C.Structure):
    _fields_ = [("mu", C.c_void_p), ("log_scale", C.c_void_p), ("weight", C.c_void_p),
                ("chan_coef", C.c_void_p), ("num_comp", C.c_uint32)]


class pilc_ansai_shape(C.Structure):
    _fields_ = [("pieces", C.c_uint32), ("count", C.c_uint32), ("prec_bits", C.c_uint32),
                ("num_dist", C.c_uint32), ("num_sym", C.c_uint32)]


class pilc_twar_params(C.Structure):
    _fields_ = [("w", (C.c_int16 * 3) * 3), ("bias", C.c_int32 * 3)]


class PilcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().pilc_strerror(code).decode()
        if code == PILC_E_HIP:
            msg += ": " + lib().pilc_last_hip_error().decode()
        super().__init__("%s failed: %s (%d)" % (where, msg, code))


_lib = None


def lib():
    """Loads libpilc.so (building it first only if no built library exists; a library older than
    its sources is loaded with a warning: `python -m paper_2206_05279_amd.build` rebuilds it)."""
    global _lib
    if _lib is None:
        from . import build
        if not os.path.exists(LIB_PATH):
            build.build_lib()
        elif build.built_digest() != build.source_digest():
            import warnings
            warnings.warn("libpilc.so was not built from the current csrc/ and include/pilc.h: "
                          "run `python -m paper_2206_05279_amd.build`", RuntimeWarning, stacklevel=2)
        L = C.CDLL(LIB_PATH)
        gp, pp = C.POINTER(pilc_geom), C.POINTER(pilc_params)
        L.pilc_lane_count.restype = C.c_uint64
        L.pilc_lane_count.argtypes = [gp]
        L.pilc_workspace_size.restype = C.c_int
        L.pilc_workspace_size.argtypes = [gp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.pilc_encode.restype = C.c_int
        L.pilc_encode.argtypes = [gp, C.c_void_p, pp, C.c_void_p, C.c_size_t, C.c_void_p,
                                  C.c_size_t, C.POINTER(C.c_uint64), C.c_void_p]
        L.pilc_encode_static.restype = C.c_int
        L.pilc_encode_static.argtypes = [gp, C.c_void_p, pp, C.c_void_p, C.c_size_t,
                                         C.POINTER(C.c_uint64), C.c_void_p]
        L.pilc_decode.restype = C.c_int
        L.pilc_decode.argtypes = [gp, C.c_void_p, C.c_size_t, pp, C.c_void_p, C.c_size_t,
                                  C.c_void_p, C.c_void_p]
        L.pilc_symbol_tables.restype = C.c_int
        L.pilc_symbol_tables.argtypes = [gp, C.c_void_p, pp, C.c_void_p, C.c_void_p, C.c_void_p]
        L.pilc_set_timing.restype = None
        L.pilc_set_timing.argtypes = [C.c_int]
        L.pilc_set_kernel_policy.restype = C.c_int
        L.pilc_set_kernel_policy.argtypes = [C.c_int]
        L.pilc_set_ansai_decode_waves.restype = C.c_int
        L.pilc_set_ansai_decode_waves.argtypes = [C.c_int]
        L.pilc_set_one_pass_wait.restype = None
        L.pilc_set_one_pass_wait.argtypes = [C.c_uint64, C.c_int]
        L.pilc_last_timing.restype = C.c_int
        L.pilc_last_timing.argtypes = [C.POINTER(C.c_float), C.c_int]
        L.pilc_timing_name.restype = C.c_char_p
        L.pilc_timing_name.argtypes = [C.c_int]
        L.pilc_strerror.restype = C.c_char_p
        L.pilc_strerror.argtypes = [C.c_int]
        L.pilc_last_hip_error.restype = C.c_char_p
        L.pilc_version.restype = C.c_uint32
        sp = C.POINTER(pilc_ansai_shape)
        L.pilc_ansai_table_bytes.restype = C.c_size_t
        L.pilc_ansai_table_bytes.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.pilc_ansai_build_tables.restype = C.c_int
        L.pilc_ansai_build_tables.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
        L.pilc_ansai_workspace_size.restype = C.c_int
        L.pilc_ansai_workspace_size.argtypes = [sp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.pilc_ansai_encode.restype = C.c_int
        L.pilc_ansai_encode.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                        C.c_void_p, C.c_size_t, C.POINTER(C.c_uint64), C.c_void_p]
        tp = C.POINTER(pilc_twar_params)
        for f in (L.pilc_twar_forward, L.pilc_twar_inverse):
            f.restype = C.c_int
            f.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, tp, C.c_void_p, C.c_void_p]
        L.pilc_ansai_center.restype = C.c_int
        L.pilc_ansai_center.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int, C.c_void_p, C.c_void_p]
        L.pilc_ansai_decode.restype = C.c_int
        L.pilc_ansai_decode.argtypes = [sp, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_size_t, C.c_void_p, C.c_void_p]
        mp = C.POINTER(pilc_mix_params)
        L.pilc_mix_encode.restype = C.c_int
        L.pilc_mix_encode.argtypes = [gp, C.c_void_p, mp, C.c_void_p, C.c_size_t, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_uint64), C.c_void_p]
        L.pilc_mix_decode.restype = C.c_int
        L.pilc_mix_decode.argtypes = [gp, C.c_void_p, C.c_size_t, mp, C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def make_geom(n, h, w, prec_bits, lane_mode, lane_a, lane_b=0) -> pilc_geom:
    return pilc_geom(int(n), int(h), int(w), int(prec_bits), int(lane_mode), int(lane_a), int(lane_b))


def _dev_ptr(t: Optional[torch.Tensor], dtype, what: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous %s device tensor" % (what, dtype))
    return t.data_ptr()


def _params(mu, log_scale, chan_coef) -> pilc_params:
    return pilc_params(_dev_ptr(mu, torch.uint16, "mu"), _dev_ptr(log_scale, torch.int16, "log_scale"),
                       _dev_ptr(chan_coef, torch.int16, "chan_coef"))


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def pilc_lane_count(geom: pilc_geom) -> int:
    return int(lib().pilc_lane_count(C.byref(geom)))


def pilc_workspace_size(geom: pilc_geom) -> Tuple[int, int]:
    """Returns (workspace_bytes, max_coded_bytes)."""
    ws, mc = C.c_size_t(0), C.c_size_t(0)
    rc = lib().pilc_workspace_size(C.byref(geom), C.byref(ws), C.byref(mc))
    if rc != PILC_OK:
        raise PilcError(rc, "pilc_workspace_size")
    return int(ws.value), int(mc.value)


def pilc_encode(geom: pilc_geom, img, mu, log_scale, chan_coef, workspace, coded,
                stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> Tuple[int, int]:
    """Runs pilc_encode; returns (rc, coded_bytes).  workspace / coded are uint8 device tensors."""
    nbytes = C.c_uint64(0)
    par = _params(mu, log_scale, chan_coef)
    rc = lib().pilc_encode(C.byref(geom), _dev_ptr(img, torch.uint8, "img"), C.byref(par),
                           _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                           _dev_ptr(coded, torch.uint8, "coded"), coded.numel(), C.byref(nbytes),
                           _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_encode")
    return rc, int(nbytes.value)


PILC_STATIC_SCRATCH_BYTES = 16 << 20


def pilc_encode_static(geom: pilc_geom, img, mu, log_scale, chan_coef, coded,
                       stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> Tuple[int, int]:
    """Runs pilc_encode_static (the library's own scratch array instead of a workspace)."""
    nbytes = C.c_uint64(0)
    par = _params(mu, log_scale, chan_coef)
    rc = lib().pilc_encode_static(C.byref(geom), _dev_ptr(img, torch.uint8, "img"), C.byref(par),
                                  _dev_ptr(coded, torch.uint8, "coded"), coded.numel(), C.byref(nbytes),
                                  _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_encode_static")
    return rc, int(nbytes.value)


def pilc_decode(geom: pilc_geom, coded, coded_bytes: int, mu, log_scale, chan_coef, workspace,
                img_out, stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> int:
    par = _params(mu, log_scale, chan_coef)
    rc = lib().pilc_decode(C.byref(geom), _dev_ptr(coded, torch.uint8, "coded"), int(coded_bytes),
                           C.byref(par), _dev_ptr(workspace, torch.uint8, "workspace"),
                           workspace.numel(), _dev_ptr(img_out, torch.uint8, "img_out"),
                           _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_decode")
    return rc


def pilc_symbol_tables(geom: pilc_geom, img, mu, log_scale, chan_coef, cum_out, freq_out,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
    par = _params(mu, log_scale, chan_coef)
    rc = lib().pilc_symbol_tables(C.byref(geom), _dev_ptr(img, torch.uint8, "img"), C.byref(par),
                                  _dev_ptr(cum_out, torch.uint32, "cum_out"),
                                  _dev_ptr(freq_out, torch.uint32, "freq_out"), _stream_handle(stream))
    if rc != PILC_OK:
        raise PilcError(rc, "pilc_symbol_tables")


def pilc_set_timing(enabled: bool) -> None:
    lib().pilc_set_timing(1 if enabled else 0)


def pilc_set_kernel_policy(policy: int) -> None:
    rc = lib().pilc_set_kernel_policy(int(policy))
    if rc != PILC_OK:
        raise PilcError(rc, "pilc_set_kernel_policy")


def pilc_set_ansai_decode_waves(waves: int) -> None:
    rc = lib().pilc_set_ansai_decode_waves(int(waves))
    if rc != PILC_OK:
        raise PilcError(rc, "pilc_set_ansai_decode_waves")


def pilc_set_one_pass_wait(ticks: int = 0, withhold_first: bool = False) -> None:
    lib().pilc_set_one_pass_wait(int(ticks), int(bool(withhold_first)))


def pilc_last_timing() -> List[Tuple[str, float]]:
    buf = (C.c_float * 16)()
    k = lib().pilc_last_timing(buf, 16)
    return [(lib().pilc_timing_name(i).decode(), float(buf[i])) for i in range(k)]


def pilc_strerror(code: int) -> str:
    return lib().pilc_strerror(int(code)).decode()


def pilc_version() -> int:
    return int(lib().pilc_version())


# ---------------------------------------------------------------- the table-driven coder (ANS-AI)
def make_ansai_shape(pieces, count, prec_bits, num_dist, num_sym=256) -> pilc_ansai_shape:
    return pilc_ansai_shape(int(pieces), int(count), int(prec_bits), int(num_dist), int(num_sym))


def pilc_ansai_table_bytes(prec_bits: int, num_dist: int, num_sym: int = 256) -> int:
    return int(lib().pilc_ansai_table_bytes(int(prec_bits), int(num_dist), int(num_sym)))


def pilc_ansai_build_tables(prec_bits: int, num_dist: int, num_sym: int, mass, tables,
                            stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> int:
    """mass: uint32 device tensor [D, X]; tables: uint8 device tensor of pilc_ansai_table_bytes()."""
    rc = lib().pilc_ansai_build_tables(int(prec_bits), int(num_dist), int(num_sym),
                                       _dev_ptr(mass, torch.uint32, "mass"),
                                       _dev_ptr(tables, torch.uint8, "tables"), tables.numel(),
                                       _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_ansai_build_tables")
    return rc


def pilc_ansai_workspace_size(shape: pilc_ansai_shape) -> Tuple[int, int]:
    """Returns (workspace_bytes, max_coded_bytes)."""
    ws, mc = C.c_size_t(0), C.c_size_t(0)
    rc = lib().pilc_ansai_workspace_size(C.byref(shape), C.byref(ws), C.byref(mc))
    if rc != PILC_OK:
        raise PilcError(rc, "pilc_ansai_workspace_size")
    return int(ws.value), int(mc.value)


def pilc_ansai_encode(shape: pilc_ansai_shape, sym, dist, tables, workspace, coded,
                      stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> Tuple[int, int]:
    nbytes = C.c_uint64(0)
    rc = lib().pilc_ansai_encode(C.byref(shape), _dev_ptr(sym, torch.uint8, "sym"),
                                 _dev_ptr(dist, torch.uint8, "dist"), _dev_ptr(tables, torch.uint8, "tables"),
                                 _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                 _dev_ptr(coded, torch.uint8, "coded"), coded.numel(), C.byref(nbytes),
                                 _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_ansai_encode")
    return rc, int(nbytes.value)


def pilc_ansai_decode(shape: pilc_ansai_shape, coded, coded_bytes: int, dist, tables, workspace, sym_out,
                      stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> int:
    rc = lib().pilc_ansai_decode(C.byref(shape), _dev_ptr(coded, torch.uint8, "coded"), int(coded_bytes),
                                 _dev_ptr(dist, torch.uint8, "dist"), _dev_ptr(tables, torch.uint8, "tables"),
                                 _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                 _dev_ptr(sym_out, torch.uint8, "sym_out"), _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_ansai_decode")
    return rc


def pilc_ansai_center(values, mu, out, inverse: bool = False,
                      stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> int:
    """out = (values - mu + 128) mod 256, or with inverse (values + mu - 128) mod 256; uint8 tensors."""
    rc = lib().pilc_ansai_center(_dev_ptr(values, torch.uint8, "values"), _dev_ptr(mu, torch.uint8, "mu"),
                                 values.numel(), 1 if inverse else 0, _dev_ptr(out, torch.uint8, "out"),
                                 _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_ansai_center")
    return rc


# ---------------------------------------------------------------- Three-Way AR residual transform
def make_twar_params(weights, bias) -> pilc_twar_params:
    """weights: 3x3 integers (Q2.14), bias: 3 integers (Q8.14)."""
    p = pilc_twar_params()
    for c in range(3):
        for k in range(3):
            p.w[c][k] = int(weights[c][k])
        p.bias[c] = int(bias[c])
    return p


def _twar(fn, name, params, src, dst, stream, check):
    n, h, w, ch = src.shape
    assert ch == 3 and dst.shape == src.shape
    rc = fn(n, h, w, _dev_ptr(src, torch.uint8, "src"), C.byref(params), _dev_ptr(dst, torch.uint8, "dst"),
            _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, name)
    return rc


def pilc_twar_forward(params: pilc_twar_params, img, res, stream: Optional[torch.cuda.Stream] = None,
                      check: bool = True) -> int:
    return _twar(lib().pilc_twar_forward, "pilc_twar_forward", params, img, res, stream, check)


def pilc_twar_inverse(params: pilc_twar_params, res, img, stream: Optional[torch.cuda.Stream] = None,
                      check: bool = True) -> int:
    return _twar(lib().pilc_twar_inverse, "pilc_twar_inverse", params, res, img, stream, check)


# ---- mixture of K logistic laws per subpixel ------------------------------------------------
def _mix_params(num_comp, mu, log_scale, weight, chan_coef) -> pilc_mix_params:
    return pilc_mix_params(_dev_ptr(mu, torch.uint16, "mu"), _dev_ptr(log_scale, torch.int16, "log_scale"),
                           _dev_ptr(weight, torch.uint16, "weight"),
                           _dev_ptr(chan_coef, torch.int16, "chan_coef"), int(num_comp))


def pilc_mix_encode(geom: pilc_geom, num_comp: int, img, mu, log_scale, weight, chan_coef, workspace,
                    coded, stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> Tuple[int, int]:
    """Runs pilc_mix_encode; returns (rc, coded_bytes)."""
    nbytes = C.c_uint64(0)
    par = _mix_params(num_comp, mu, log_scale, weight, chan_coef)
    rc = lib().pilc_mix_encode(C.byref(geom), _dev_ptr(img, torch.uint8, "img"), C.byref(par),
                               _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                               _dev_ptr(coded, torch.uint8, "coded"), coded.numel(), C.byref(nbytes),
                               _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_mix_encode")
    return rc, int(nbytes.value)


def pilc_mix_decode(geom: pilc_geom, num_comp: int, coded, coded_bytes: int, mu, log_scale, weight,
                    chan_coef, workspace, img_out, stream: Optional[torch.cuda.Stream] = None,
                    check: bool = True) -> int:
    par = _mix_params(num_comp, mu, log_scale, weight, chan_coef)
    rc = lib().pilc_mix_decode(C.byref(geom), _dev_ptr(coded, torch.uint8, "coded"), int(coded_bytes),
                               C.byref(par), _dev_ptr(workspace, torch.uint8, "workspace"),
                               workspace.numel(), _dev_ptr(img_out, torch.uint8, "img_out"),
                               _stream_handle(stream))
    if check and rc != PILC_OK:
        raise PilcError(rc, "pilc_mix_decode")
    return rc
