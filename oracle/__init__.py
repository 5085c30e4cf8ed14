"""CPU oracle for the butterfly + quantisation path (TEST INFRASTRUCTURE ONLY).

Thin ctypes front end to `bq_oracle.c` plus the dense definitional builder in `dense.py`.  Nothing
in the product package imports this; only tests, the smoke check and the benchmark's cpu_baseline
leg do.  It shares no code with the HIP library.

All transform entry points take float64 arrays `[rows, heads*n]` (exact values of the stored
inputs) and float32 `theta` of layout `[heads][log2 n][n/2]`, and return float64.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build
from .dense import dense_butterfly, dense_layer, pair_indices  # noqa: F401
from .hadamard import hadamard  # noqa: F401

_LIB = None


def lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            path = _build.build()
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        L.bq_oracle_fwd.argtypes = [dp, dp, fp, ctypes.c_long, ctypes.c_int, ctypes.c_int]
        L.bq_oracle_inv.argtypes = [dp, dp, fp, ctypes.c_long, ctypes.c_int, ctypes.c_int]
        L.bq_oracle_bwd.argtypes = [dp, dp, fp, dp, dp, dp, ctypes.c_long, ctypes.c_int, ctypes.c_int]
        L.bq_oracle_quant.argtypes = [fp, ctypes.c_long, ctypes.c_long, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.POINTER(ctypes.c_int8), fp]
        L.bq_oracle_pack_codes.argtypes = [ctypes.POINTER(ctypes.c_int8), ctypes.c_long, ctypes.c_long,
                                           ctypes.c_int, ctypes.POINTER(ctypes.c_uint8)]
        L.bq_oracle_f32_to_f16_bits.argtypes = [ctypes.c_float]
        L.bq_oracle_f32_to_f16_bits.restype = ctypes.c_uint16
        L.bq_oracle_f16_bits_to_f32.argtypes = [ctypes.c_uint16]
        L.bq_oracle_f16_bits_to_f32.restype = ctypes.c_float
        L.bq_oracle_num_threads.restype = ctypes.c_int
        L.bq_oracle_dequant.argtypes = [ctypes.POINTER(ctypes.c_int8), fp, ctypes.c_long, ctypes.c_long, ctypes.c_int, fp]
        L.bq_oracle_bin_histogram.argtypes = [ctypes.POINTER(ctypes.c_int8), ctypes.c_long, ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_uint64)]
        L.bq_oracle_uniformity_kl.argtypes = [ctypes.POINTER(ctypes.c_uint64), ctypes.c_int]
        L.bq_oracle_uniformity_kl.restype = ctypes.c_double
        _LIB = L
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _theta_check(theta, n, heads):
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    k = int(n).bit_length() - 1
    if theta.size != heads * k * (n // 2):
        raise ValueError(f"theta has {theta.size} angles, expected {heads * k * (n // 2)}")
    return theta


def _rows2d(x, n, heads):
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.ndim == 1:
        x = x[None, :]
    if x.ndim != 2 or x.shape[1] != n * heads:
        raise ValueError(f"expected [rows, {n * heads}], got {x.shape}")
    return x


def forward(x, theta, n, heads=1):
    """y = B(theta) x, row by row (layer 1 first)."""
    x = _rows2d(x, n, heads)
    theta = _theta_check(theta, n, heads)
    y = np.empty_like(x)
    rc = lib().bq_oracle_fwd(_p(x, ctypes.c_double), _p(y, ctypes.c_double), _p(theta, ctypes.c_float),
                             x.shape[0], n, heads)
    if rc:
        raise ValueError("bq_oracle_fwd: bad shape")
    return y


def inverse(y, theta, n, heads=1):
    """x = B(theta)^T y."""
    y = _rows2d(y, n, heads)
    theta = _theta_check(theta, n, heads)
    x = np.empty_like(y)
    rc = lib().bq_oracle_inv(_p(y, ctypes.c_double), _p(x, ctypes.c_double), _p(theta, ctypes.c_float),
                             y.shape[0], n, heads)
    if rc:
        raise ValueError("bq_oracle_inv: bad shape")
    return x


def backward(x, dy, theta, n, heads=1, want_abs=True):
    """Returns (dx [rows, heads*n], dtheta [heads, k, n/2], absacc or None), all float64."""
    x = _rows2d(x, n, heads)
    dy = _rows2d(dy, n, heads)
    theta = _theta_check(theta, n, heads)
    k = int(n).bit_length() - 1
    dx = np.empty_like(x)
    dth = np.empty((heads, k, n // 2), dtype=np.float64)
    ab = np.empty_like(dth) if want_abs else None
    rc = lib().bq_oracle_bwd(_p(x, ctypes.c_double), _p(dy, ctypes.c_double), _p(theta, ctypes.c_float),
                             _p(dx, ctypes.c_double), _p(dth, ctypes.c_double),
                             _p(ab, ctypes.c_double) if want_abs else None, x.shape[0], n, heads)
    if rc:
        raise ValueError("bq_oracle_bwd: bad shape")
    return dx, dth, ab


def quantize(y32, group, bits, scale_dtype="f32"):
    """Symmetric uniform quantiser on float32 rows.  Returns (codes int8 [rows,width],
    scales float32 [rows, width/group])."""
    y32 = np.ascontiguousarray(y32, dtype=np.float32)
    if y32.ndim == 1:
        y32 = y32[None, :]
    rows, width = y32.shape
    codes = np.empty((rows, width), dtype=np.int8)
    scales = np.empty((rows, width // group), dtype=np.float32)
    rc = lib().bq_oracle_quant(_p(y32, ctypes.c_float), rows, width, group, bits,
                               1 if scale_dtype == "f16" else 0, _p(codes, ctypes.c_int8),
                               _p(scales, ctypes.c_float))
    if rc:
        raise ValueError("bq_oracle_quant: bad argument")
    return codes, scales


def dequantize(codes, scales, group):
    """Dequant(q) = s * q in float32.  codes int8 [rows,width], scales float32 [rows,width/group]."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    rows, width = codes.shape
    yq = np.empty((rows, width), dtype=np.float32)
    rc = lib().bq_oracle_dequant(_p(codes, ctypes.c_int8), _p(scales, ctypes.c_float), rows, width, group,
                                 _p(yq, ctypes.c_float))
    if rc:
        raise ValueError("bq_oracle_dequant: bad argument")
    return yq


def bin_histogram(codes, bits):
    """Occupancy of the 2^bits code bins: hist[c] = #(code == c - 2^(bits-1)), uint64."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    hist = np.zeros(1 << bits, dtype=np.uint64)
    rc = lib().bq_oracle_bin_histogram(_p(codes, ctypes.c_int8), codes.size, bits, _p(hist, ctypes.c_uint64))
    if rc:
        raise ValueError("bq_oracle_bin_histogram: bad argument")
    return hist


def uniformity_kl(hist, bits):
    """D_KL(P_bins || uniform) of a bin histogram (natural log)."""
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    assert hist.size == 1 << bits
    return float(lib().bq_oracle_uniformity_kl(_p(hist, ctypes.c_uint64), bits))


def pack_codes(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    rows, width = codes.shape
    out = np.empty((rows, width * bits // 8), dtype=np.uint8)
    rc = lib().bq_oracle_pack_codes(_p(codes, ctypes.c_int8), rows, width, bits, _p(out, ctypes.c_uint8))
    if rc:
        raise ValueError("bq_oracle_pack_codes: bad argument")
    return out


def unpack_codes(packed, bits):
    """Inverse of pack_codes (numpy; test helper)."""
    packed = np.asarray(packed, dtype=np.uint8)
    per = 8 // bits
    fields = [(packed >> (e * bits)) & ((1 << bits) - 1) for e in range(per)]
    u = np.stack(fields, axis=-1).reshape(packed.shape[0], -1).astype(np.int16)
    u = np.where(u >= (1 << (bits - 1)), u - (1 << bits), u)
    return u.astype(np.int8)


def f32_to_f16_bits(v: float) -> int:
    return int(lib().bq_oracle_f32_to_f16_bits(ctypes.c_float(v)))


def f16_bits_to_f32(h: int) -> float:
    return float(lib().bq_oracle_f16_bits_to_f32(ctypes.c_uint16(h)))


def num_threads() -> int:
    return int(lib().bq_oracle_num_threads())
