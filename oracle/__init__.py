"""ctypes access to the CPU reference solver (test infrastructure only).

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this package; the GPU product path never does.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "squant_oracle.cpp")
_LIB = os.path.join(_HERE, "libsquant_oracle.so")

MODE_E, MODE_EK, MODE_EKC, MODE_EC = 0, 1, 2, 3
ONE = 1 << 23
HALF = 1 << 22

CXXFLAGS = ["-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
            "-pthread"]


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB):
        subprocess.check_call(["g++", *CXXFLAGS, _SRC, "-o", _LIB])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        L.squant_oracle_quantize.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp]
        L.squant_oracle_quantize_mt.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, i32]
        L.squant_oracle_quantize_trace.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp] + [vp] * 7
        i64 = ctypes.c_int64
        L.squant_oracle_pack_int4.argtypes = [vp, i64, i64, vp]
        L.squant_oracle_dequantize.argtypes = [vp, vp, i64, i64, vp]
        L.squant_oracle_dequantize_bf16.argtypes = [vp, vp, i64, i64, vp]
        L.squant_oracle_dequantize_bf16.restype = ctypes.c_int
        L.squant_oracle_activation_range.argtypes = [vp, vp, i64, ctypes.c_float, i32, i32, vp]
        L.squant_oracle_activation_range.restype = ctypes.c_int
        L.squant_oracle_widen_f16.argtypes = [vp, i64, vp]
        L.squant_oracle_widen_bf16.argtypes = [vp, i64, vp]
        for f in (L.squant_oracle_pack_int4, L.squant_oracle_dequantize,
                  L.squant_oracle_widen_f16, L.squant_oracle_widen_bf16):
            f.restype = ctypes.c_int
        for f in (L.squant_oracle_quantize, L.squant_oracle_quantize_mt,
                  L.squant_oracle_quantize_trace, L.squant_oracle_hardware_threads):
            f.restype = ctypes.c_int
        _lib = L
    return _lib


def _prep(w):
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim == 2:
        w = w[:, :, None, None]
    if w.ndim == 3:
        w = w[:, :, :, None]
    assert w.ndim == 4
    return w


def quantize(w, bits: int, mode: int = MODE_EKC, threads: int = 1):
    """Returns (codes int8 [same shape as w], scales float32 [cout])."""
    w4 = _prep(w)
    cout, cin, kh, kw = w4.shape
    codes = np.empty(w4.shape, dtype=np.int8)
    scales = np.empty(cout, dtype=np.float32)
    if threads > 1:
        rc = lib().squant_oracle_quantize_mt(w4.ctypes.data, cout, cin, kh, kw, bits, mode,
                                             codes.ctypes.data, scales.ctypes.data, threads)
    else:
        rc = lib().squant_oracle_quantize(w4.ctypes.data, cout, cin, kh, kw, bits, mode,
                                          codes.ctypes.data, scales.ctypes.data)
    if rc != 0:
        raise ValueError(f"squant_oracle_quantize failed with status {rc}")
    return codes, scales


def quantize_trace(w, bits: int, mode: int = MODE_EKC):
    """Returns (codes, scales, trace dict of the intermediate decisions, Q23 integers)."""
    w4 = _prep(w)
    cout, cin, kh, kw = w4.shape
    codes = np.empty(w4.shape, dtype=np.int8)
    scales = np.empty(cout, dtype=np.float32)
    tr = {
        "kernel_k": np.empty((cout, cin), np.int32),
        "kernel_sum": np.empty((cout, cin), np.int32),
        "cand_index": np.empty((cout, cin), np.int32),
        "cand_value": np.empty((cout, cin), np.int32),
        "channel_sum": np.empty(cout, np.int64),
        "channel_k": np.empty(cout, np.int32),
        "perturbation": np.empty((cout, cin, kh * kw), np.int32),
    }
    rc = lib().squant_oracle_quantize_trace(
        w4.ctypes.data, cout, cin, kh, kw, bits, mode, codes.ctypes.data, scales.ctypes.data,
        *[tr[k].ctypes.data for k in ("kernel_k", "kernel_sum", "cand_index", "cand_value",
                                      "channel_sum", "channel_k", "perturbation")])
    if rc != 0:
        raise ValueError(f"squant_oracle_quantize_trace failed with status {rc}")
    return codes, scales, tr


def hardware_threads() -> int:
    return int(lib().squant_oracle_hardware_threads())


def pack_int4(codes):
    """codes int8 [cout, ...] with |code| <= 7 -> uint8 [cout, (len + 1) // 2], two per byte."""
    c = np.ascontiguousarray(codes, dtype=np.int8)
    cout = c.shape[0]
    n = c.size // cout
    out = np.empty((cout, (n + 1) // 2), dtype=np.uint8)
    rc = lib().squant_oracle_pack_int4(c.ctypes.data, cout, n, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"squant_oracle_pack_int4 failed with status {rc}")
    return out


def dequantize(codes, scales):
    """code * scale of its output channel, float32, same shape as codes."""
    c = np.ascontiguousarray(codes, dtype=np.int8)
    s = np.ascontiguousarray(scales, dtype=np.float32)
    cout = c.shape[0]
    assert s.shape == (cout,)
    out = np.empty(c.shape, dtype=np.float32)
    rc = lib().squant_oracle_dequantize(c.ctypes.data, s.ctypes.data, cout, c.size // cout,
                                        out.ctypes.data)
    if rc != 0:
        raise ValueError(f"squant_oracle_dequantize failed with status {rc}")
    return out


def dequantize_bf16(codes, scales):
    """code * scale rounded to bfloat16, as uint16 bit patterns, same shape as codes."""
    c = np.ascontiguousarray(codes, dtype=np.int8)
    s = np.ascontiguousarray(scales, dtype=np.float32)
    cout = c.shape[0]
    out = np.empty(c.shape, dtype=np.uint16)
    rc = lib().squant_oracle_dequantize_bf16(c.ctypes.data, s.ctypes.data, cout, c.size // cout,
                                             out.ctypes.data)
    if rc != 0:
        raise ValueError(f"squant_oracle_dequantize_bf16 failed with status {rc}")
    return out


def widen(bits16, wtype: str):
    """uint16 bit patterns of binary16 ("f16") or bfloat16 ("bf16") weights -> float32."""
    h = np.ascontiguousarray(bits16, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    fn = {"f16": lib().squant_oracle_widen_f16, "bf16": lib().squant_oracle_widen_bf16}[wtype]
    rc = fn(h.ctypes.data, h.size, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"widen failed with status {rc}")
    return out


def activation_range(gamma, beta, n_sigma: float, relu: bool, bits: int):
    """(lo, hi, scale, zero_point) of the batch-norm based per-tensor activation range."""
    g = np.ascontiguousarray(gamma, dtype=np.float32)
    b = np.ascontiguousarray(beta, dtype=np.float32)
    assert g.shape == b.shape and g.ndim == 1
    out = np.empty(4, dtype=np.float32)
    rc = lib().squant_oracle_activation_range(g.ctypes.data, b.ctypes.data, g.size, float(n_sigma),
                                              int(bool(relu)), bits, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"squant_oracle_activation_range failed with status {rc}")
    return np.float32(out[0]), np.float32(out[1]), np.float32(out[2]), int(out[3])
