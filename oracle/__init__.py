"""CPU oracle for the ultra-low-bit GEMM / convolution path (arXiv 2207.08820, Sections IV-V).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.  It shares nothing with the HIP library and never
imports it.  The arithmetic lives in ``dlrt_oracle.c`` (plain C loops on the unpacked
integer values, int32 accumulation); this module only marshals numpy arrays.

Parity pins for every function are in ``tests/test_oracle_pins.py``; no function here is
"parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dlrt_oracle.c")
_LIB = os.path.join(_HERE, "libdlrt_oracle.so")

UNSIGNED, TWOS, BIPOLAR = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no fp contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_num_threads.restype = i32
        lib.oracle_set_threads.argtypes = [i32]
        lib.oracle_gemm_i32.argtypes = [vp, vp, vp, i64, i64, i64]
        lib.oracle_conv2d_i32.argtypes = [vp, vp, vp] + [i32] * 11
        lib.oracle_quantize.argtypes = [vp, vp, i32, i64, i64, ctypes.c_float, ctypes.c_float, vp]
        lib.oracle_quantize_bipolar.argtypes = [vp, vp, i32, i64, i64, vp]
        lib.oracle_epilogue_f32.argtypes = [vp, vp, vp, i64, i32, vp, vp, i32]
        lib.oracle_pack_bitplanes.argtypes = [vp, i64, i64, i32, i32, vp]
        lib.oracle_pack_conv_weights.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp]
        for name in ("oracle_set_threads", "oracle_gemm_i32", "oracle_conv2d_i32", "oracle_quantize",
                     "oracle_quantize_bipolar", "oracle_epilogue_f32", "oracle_pack_bitplanes", "oracle_pack_conv_weights"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _values(a, name) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != np.int8:
        if a.size and (a.min() < -128 or a.max() > 127):
            raise ValueError(f"{name}: values do not fit int8")
        a = a.astype(np.int8)
    return np.ascontiguousarray(a)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def gemm_i32(a, w) -> np.ndarray:
    """C[m, n] = sum_k a[m, k] * w[n, k] on integer values (Section V)."""
    a, w = _values(a, "a"), _values(w, "w")
    M, K = a.shape
    N, K2 = w.shape
    if K != K2:
        raise ValueError("reduction lengths differ")
    c = np.empty((M, N), dtype=np.int32)
    _load().oracle_gemm_i32(_p(a), _p(w), _p(c), M, N, K)
    return c


def conv_out_size(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def conv2d_i32(x, w, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Direct NHWC x OHWI convolution with zero padding, int32 NHWC output."""
    x, w = _values(x, "x"), _values(w, "w")
    N, H, W, Ci = x.shape
    Co, KH, KW, Ci2 = w.shape
    if Ci != Ci2:
        raise ValueError("channel counts differ")
    Ho = conv_out_size(H, KH, stride[0], pad[0])
    Wo = conv_out_size(W, KW, stride[1], pad[1])
    y = np.empty((N, Ho, Wo, Co), dtype=np.int32)
    _load().oracle_conv2d_i32(_p(x), _p(w), _p(y), N, H, W, Ci, Co, KH, KW,
                              stride[0], stride[1], pad[0], pad[1])
    return y


def value_range(bits: int, enc: int):
    """Closed range of representable values for an encoding (Section IV's Q_N, Q_P when signed)."""
    if enc == UNSIGNED:
        return 0, (1 << bits) - 1
    if enc == TWOS:
        return -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    return -1, 1


def quantize(x, scale, bits: int, enc: int) -> np.ndarray:
    """round(clip(x / s, lo, hi)), ties to even, fp32 (Section IV).  scale: scalar or one per row.
    Bipolar (+1 / -1, no zero level): the sign of x / s, zero counted as +1."""
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    x2 = x.reshape(-1, x.shape[-1])
    scale = np.ascontiguousarray(np.asarray(scale, dtype=np.float32).reshape(-1))
    per_row = int(scale.size != 1)
    if per_row and scale.size != x2.shape[0]:
        raise ValueError("scale must have one value or one per row")
    lo, hi = value_range(bits, enc)
    q = np.empty(x2.shape, dtype=np.int8)
    if enc == BIPOLAR:
        _load().oracle_quantize_bipolar(_p(x2), _p(scale), per_row, x2.shape[0], x2.shape[1], _p(q))
        return q.reshape(x.shape)
    _load().oracle_quantize(_p(x2), _p(scale), per_row, x2.shape[0], x2.shape[1], float(lo), float(hi), _p(q))
    return q.reshape(x.shape)


def epilogue_f32(acc, scale, bias=None, qbits: int | None = None):
    """y = fma(float(acc), scale[c], bias[c]); optional q = clamp(round(y), 0, 2^qbits - 1) as uint8."""
    acc = np.ascontiguousarray(np.asarray(acc, dtype=np.int32))
    C = acc.shape[-1]
    rows = acc.size // C if C else 0
    scale = np.ascontiguousarray(np.asarray(scale, dtype=np.float32))
    assert scale.shape == (C,)
    if bias is not None:
        bias = np.ascontiguousarray(np.asarray(bias, dtype=np.float32))
        assert bias.shape == (C,)
    y = np.empty(acc.shape, dtype=np.float32)
    q = np.empty(acc.shape, dtype=np.uint8) if qbits is not None else None
    _load().oracle_epilogue_f32(_p(acc), _p(scale), _p(bias) if bias is not None else None, rows, C,
                                _p(y), _p(q) if q is not None else None, int(qbits or 1))
    return y, q


def packed_words(rows: int, K: int, bits: int) -> int:
    return rows * bits * ((K + 31) // 32)


def pack_bitplanes(q, bits: int, enc: int) -> np.ndarray:
    """values [rows, K] -> uint32 [rows, bits, ceil(K/32)], LSB-first along K, zero padded."""
    q = _values(q, "q")
    rows, K = q.shape
    dst = np.empty((rows, bits, (K + 31) // 32), dtype=np.uint32)
    _load().oracle_pack_bitplanes(_p(q), rows, K, bits, enc, _p(dst))
    return dst


def pack_conv_weights(w, bits: int, enc: int) -> np.ndarray:
    """OHWI values -> uint32 [Co, bits, KH*KW*ceil(Ci/32)], each tap padded to whole words."""
    w = _values(w, "w")
    Co, KH, KW, Ci = w.shape
    dst = np.empty((Co, bits, KH * KW * ((Ci + 31) // 32)), dtype=np.uint32)
    _load().oracle_pack_conv_weights(_p(w), Co, KH, KW, Ci, bits, enc, _p(dst))
    return dst
