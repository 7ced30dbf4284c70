"""ctypes front end of the CPU oracle (``iflow_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU package never imports this module and this module
never imports the GPU package.

The C file follows Section 3 of arXiv 2401.08294 (Eq.1-5, Table 3's formats and the remark that
two FP16 numbers are stored per block); this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "iflow_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

Q8_B32, Q8_B64, Q4_B32, Q4_B64, Q3H_B64, Q6_B64, Q5_B64, Q3_B32, Q2_B32 = range(9)
FORMATS = {"Q8_B32": Q8_B32, "Q8_B64": Q8_B64, "Q4_B32": Q4_B32, "Q4_B64": Q4_B64, "Q3H_B64": Q3H_B64,
           "Q6_B64": Q6_B64, "Q5_B64": Q5_B64, "Q3_B32": Q3_B32, "Q2_B32": Q2_B32}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: strict IEEE fp32, no contraction, OpenMP for the row-parallel sum."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i64, p = C.c_int64, C.c_void_p
        L.orc_packed_bytes.restype = i64
        L.orc_packed_bytes.argtypes = [C.c_int, i64, i64]
        L.orc_f16_to_f32.restype = C.c_float
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        L.orc_f64_to_f16.restype = C.c_uint16
        L.orc_f64_to_f16.argtypes = [C.c_double]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_quantize_block.restype = None
        L.orc_quantize_block.argtypes = [p, C.c_int, C.c_int, p, p, p]
        L.orc_quantize.argtypes = [C.c_int, p, i64, i64, p, p, p]
        L.orc_pair_encode.argtypes = [C.c_int, C.c_int]
        L.orc_pair_decode.restype = None
        L.orc_pair_decode.argtypes = [C.c_int, p, p]
        L.orc_dequant_value.restype = C.c_uint16
        L.orc_dequant_value.argtypes = [C.c_int, C.c_uint16, C.c_uint16]
        L.orc_pack_canonical.argtypes = [C.c_int, p, p, p, i64, i64, p]
        L.orc_unpack_canonical.argtypes = [C.c_int, p, i64, i64, p, p, p]
        L.orc_pack_device.argtypes = [C.c_int, p, p, p, i64, i64, p]
        L.orc_dequant.argtypes = [C.c_int, p, p, p, i64, i64, p]
        L.orc_gemm.argtypes = [p, i64, i64, p, i64, p, C.c_int]
        L.orc_gemm_f32.restype = None
        L.orc_gemm_f32.argtypes = [p, i64, i64, p, i64, p]
        L.orc_qgemm_canonical.argtypes = [C.c_int, p, i64, i64, p, i64, p, C.c_int]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def levels(fmt: int) -> int:
    return lib().orc_format_levels(fmt)


def block_size(fmt: int) -> int:
    return lib().orc_format_block(fmt)


def packed_bytes(fmt: int, rows: int, cols: int) -> int:
    return int(lib().orc_packed_bytes(fmt, rows, cols))


def f32_to_f16_bits(x) -> np.ndarray:
    x = _c(x, np.float32).ravel()
    return np.array([lib().orc_f32_to_f16(float(v)) for v in x], dtype=np.uint16)


def f64_to_f16_bits(x) -> np.ndarray:
    x = _c(x, np.float64).ravel()
    return np.array([lib().orc_f64_to_f16(float(v)) for v in x], dtype=np.uint16)


def f16_bits_to_f32(h) -> np.ndarray:
    h = _c(h, np.uint16).ravel()
    return np.array([lib().orc_f16_to_f32(int(v)) for v in h], dtype=np.float32)


def quantize_block(w, L: int):
    """Eq.1 / Eq.3 on one block of any length: returns (levels uint8[n], scale bits, offset bits)."""
    w = _c(w, np.float32).ravel()
    q = np.zeros(w.size, np.uint8)
    s = np.zeros(1, np.uint16)
    o = np.zeros(1, np.uint16)
    lib().orc_quantize_block(_ptr(w), w.size, L, _ptr(q), _ptr(s), _ptr(o))
    return q, int(s[0]), int(o[0])


def quantize(fmt: int, w):
    """Whole matrix [rows][cols] fp32 -> (levels uint8 [rows][cols], scale u16 [rows][nbk], offset u16 [rows][nbk])."""
    w = _c(w, np.float32)
    rows, cols = w.shape
    nbk = cols // block_size(fmt)
    q = np.zeros((rows, cols), np.uint8)
    s = np.zeros((rows, nbk), np.uint16)
    o = np.zeros((rows, nbk), np.uint16)
    rc = lib().orc_quantize(fmt, _ptr(w), rows, cols, _ptr(q), _ptr(s), _ptr(o))
    if rc != 0:
        raise ValueError("oracle: bad format or shape")
    return q, s, o


def pair_encode(q_even: int, q_odd: int) -> int:
    return lib().orc_pair_encode(q_even, q_odd)


def pair_decode(c: int):
    a, b = C.c_int(), C.c_int()
    lib().orc_pair_decode(c, C.byref(a), C.byref(b))
    return a.value, b.value


def dequant_value(q: int, scale_bits: int, offset_bits: int) -> int:
    return lib().orc_dequant_value(q, scale_bits, offset_bits)


def _pack(fn, fmt, q, s, o):
    q = _c(q, np.uint8)
    s = _c(s, np.uint16)
    o = _c(o, np.uint16)
    rows, cols = q.shape
    out = np.zeros(packed_bytes(fmt, rows, cols), np.uint8)
    if fn(fmt, _ptr(q), _ptr(s), _ptr(o), rows, cols, _ptr(out)) != 0:
        raise ValueError("oracle: bad format or shape")
    return out


def pack_canonical(fmt, q, s, o) -> np.ndarray:
    return _pack(lib().orc_pack_canonical, fmt, q, s, o)


def pack_device(fmt, q, s, o) -> np.ndarray:
    return _pack(lib().orc_pack_device, fmt, q, s, o)


def unpack_canonical(fmt, packed, rows, cols):
    packed = _c(packed, np.uint8)
    nbk = cols // block_size(fmt)
    q = np.zeros((rows, cols), np.uint8)
    s = np.zeros((rows, nbk), np.uint16)
    o = np.zeros((rows, nbk), np.uint16)
    if lib().orc_unpack_canonical(fmt, _ptr(packed), rows, cols, _ptr(q), _ptr(s), _ptr(o)) != 0:
        raise ValueError("oracle: bad format or shape")
    return q, s, o


def dequant(fmt, q, s, o) -> np.ndarray:
    """Eq.2 with the stored pair -> fp16 bit patterns [rows][cols]."""
    q = _c(q, np.uint8)
    s = _c(s, np.uint16)
    o = _c(o, np.uint16)
    rows, cols = q.shape
    out = np.zeros((rows, cols), np.uint16)
    if lib().orc_dequant(fmt, _ptr(q), _ptr(s), _ptr(o), rows, cols, _ptr(out)) != 0:
        raise ValueError("oracle: bad format or shape")
    return out


def gemm(w16_bits, x16_bits, threads: int = 1) -> np.ndarray:
    """Y[b][n] = sum_k W'[n][k] X[b][k] in fp64; inputs are fp16 bit patterns; returns fp64 [batch][rows]."""
    w = _c(w16_bits, np.uint16)
    x = _c(x16_bits, np.uint16)
    if x.ndim == 1:
        x = x[None, :]
    rows, cols = w.shape
    batch = x.shape[0]
    assert x.shape[1] == cols
    y = np.zeros((batch, rows), np.float64)
    used = lib().orc_gemm(_ptr(w), rows, cols, _ptr(x), batch, _ptr(y), threads)
    if used < 0:
        raise MemoryError
    return y


def gemm_f32(w16_bits, x16_bits) -> np.ndarray:
    w = _c(w16_bits, np.uint16)
    x = _c(x16_bits, np.uint16)
    if x.ndim == 1:
        x = x[None, :]
    rows, cols = w.shape
    y = np.zeros((x.shape[0], rows), np.uint16)
    lib().orc_gemm_f32(_ptr(w), rows, cols, _ptr(x), x.shape[0], _ptr(y))
    return y


def qgemm_canonical(fmt, packed, rows, cols, x16_bits, threads: int = 1):
    """Unpack + dequantize + multiply from a canonical packed record; returns (Y fp64, threads used)."""
    packed = _c(packed, np.uint8)
    x = _c(x16_bits, np.uint16)
    if x.ndim == 1:
        x = x[None, :]
    y = np.zeros((x.shape[0], rows), np.float64)
    used = lib().orc_qgemm_canonical(fmt, _ptr(packed), rows, cols, _ptr(x), x.shape[0], _ptr(y), threads)
    if used < 0:
        raise ValueError("oracle: bad arguments")
    return y, used
