"""ctypes loader for ``gptq_oracle.c`` (plain C, host only).

Each function marshals numpy arrays to the C routine of the same name (prefix
``oracle_``) and returns numpy arrays.  The arithmetic lives in the C file; see its
header for the definition (steps O1..O7 and Q) and the passages of the paper
(Opt4GPTQ, Section 3, Eq. 14-15; Section 4.4) it follows.  fp16 arrays are passed
as ``numpy.float16`` and handed to C as their uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gptq_oracle.c")
_LIB = os.path.join(_HERE, "libgptq_oracle.so")
# The mutation test of the pins (tests/test_oracle_mutants.py) points this at a library built from a patched copy
# of the C file; nothing else sets it.
_OVERRIDE = os.environ.get("GPTQ_ORACLE_LIB_OVERRIDE")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the path of the library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if _OVERRIDE:
            _lib = ctypes.CDLL(_OVERRIDE)
        else:
            build(force=False)
            _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    return a


def _bits(a):
    """fp16 array -> contiguous uint16 view of its bit patterns."""
    return _c(a, np.float16).view(np.uint16)


def _gidx(g_idx):
    return None if g_idx is None else _c(g_idx, np.int32)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"oracle_{name}: invalid argument (code {rc})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def half_bits_to_double(h: np.ndarray) -> np.ndarray:
    h = _c(h, np.uint16)
    out = np.empty(h.shape, np.float64)
    _load().oracle_half_to_double(_p(h), _p(out), ctypes.c_longlong(h.size))
    return out


def double_to_half_bits(v: np.ndarray) -> np.ndarray:
    v = _c(v, np.float64)
    out = np.empty(v.shape, np.uint16)
    _load().oracle_double_to_half(_p(v), _p(out), ctypes.c_longlong(v.size))
    return out


def unpack_qweight(qweight: np.ndarray) -> np.ndarray:
    """O1: int32 [K/8, N] -> uint8 codes [K, N]."""
    qweight = _c(qweight, np.int32)
    kw, n = qweight.shape
    out = np.empty((kw * 8, n), np.uint8)
    _check(_load().oracle_unpack_qweight(_p(qweight), _p(out), kw * 8, n), "unpack_qweight")
    return out


def unpack_qzeros(qzeros: np.ndarray) -> np.ndarray:
    """O2: int32 [G, N/8] -> uint8 zero points [G, N]."""
    qzeros = _c(qzeros, np.int32)
    g, nw = qzeros.shape
    out = np.empty((g, nw * 8), np.uint8)
    _check(_load().oracle_unpack_qzeros(_p(qzeros), _p(out), g, nw * 8), "unpack_qzeros")
    return out


def pack_qweight(q: np.ndarray) -> np.ndarray:
    q = _c(q, np.uint8)
    k, n = q.shape
    out = np.empty((k // 8, n), np.int32)
    _check(_load().oracle_pack_qweight(_p(q), _p(out), k, n), "pack_qweight")
    return out


def pack_qzeros(z: np.ndarray) -> np.ndarray:
    z = _c(z, np.uint8)
    g, n = z.shape
    out = np.empty((g, n // 8), np.int32)
    _check(_load().oracle_pack_qzeros(_p(z), _p(out), g, n), "pack_qzeros")
    return out


def dequant(qweight, qzeros, scales, g_idx, group_size: int) -> np.ndarray:
    """O1..O5: fp16 weights [K, N]."""
    qweight = _c(qweight, np.int32)
    qzeros = _c(qzeros, np.int32)
    sb = _bits(scales)
    gi = _gidx(g_idx)
    k, n = qweight.shape[0] * 8, qweight.shape[1]
    _expect_shapes(qzeros, sb, gi, k, n, group_size)
    out = np.empty((k, n), np.uint16)
    rc = _load().oracle_dequant(_p(qweight), _p(qzeros), _p(sb), None if gi is None else _p(gi), _p(out),
                                k, n, group_size)
    _check(rc, "dequant")
    return out.view(np.float16)


def quantize(w16, scales, z, g_idx, group_size: int) -> np.ndarray:
    """Q: codes uint8 [K, N] from fp16 weights, fp16 scales [G, N] and unpacked zeros uint8 [G, N]."""
    wb = _bits(w16)
    sb = _bits(scales)
    z = _c(z, np.uint8)
    gi = _gidx(g_idx)
    k, n = wb.shape
    out = np.empty((k, n), np.uint8)
    rc = _load().oracle_quantize(_p(wb), _p(sb), _p(z), None if gi is None else _p(gi), _p(out), k, n, group_size)
    _check(rc, "quantize")
    return out


def _expect_shapes(qzeros, sb, gi, k, n, group_size):
    if group_size <= 0 or k % group_size:
        raise ValueError("K must be a positive multiple of group_size")
    g = k // group_size
    if qzeros.shape != (g, n // 8) or n % 8:
        raise ValueError(f"qzeros must be [{g}, {n // 8}], got {qzeros.shape}")
    if sb.shape != (g, n):
        raise ValueError(f"scales must be [{g}, {n}], got {sb.shape}")
    if gi is not None and gi.shape != (k,):
        raise ValueError(f"g_idx must be [{k}], got {gi.shape}")


def gemm_ref(x, qweight, qzeros, scales, g_idx, group_size: int) -> np.ndarray:
    """O6: fp64 reference [M, N] of x @ dequant(...)."""
    xb = _bits(x)
    qweight = _c(qweight, np.int32)
    qzeros = _c(qzeros, np.int32)
    sb = _bits(scales)
    gi = _gidx(g_idx)
    m, k = xb.shape
    n = qweight.shape[1]
    if qweight.shape[0] * 8 != k:
        raise ValueError("x and qweight disagree on K")
    _expect_shapes(qzeros, sb, gi, k, n, group_size)
    out = np.empty((m, n), np.float64)
    rc = _load().oracle_gemm_ref(_p(xb), _p(qweight), _p(qzeros), _p(sb), None if gi is None else _p(gi),
                                 _p(out), m, k, n, group_size)
    _check(rc, "gemm_ref")
    return out


def gemm_ref_sampled(x, qweight, qzeros, scales, g_idx, group_size: int, m_idx, n_idx) -> np.ndarray:
    """O6 at the sampled positions (m_idx[i], n_idx[i]) only."""
    xb = _bits(x)
    qweight = _c(qweight, np.int32)
    qzeros = _c(qzeros, np.int32)
    sb = _bits(scales)
    gi = _gidx(g_idx)
    m_idx = _c(m_idx, np.int32)
    n_idx = _c(n_idx, np.int32)
    m, k = xb.shape
    n = qweight.shape[1]
    if qweight.shape[0] * 8 != k:
        raise ValueError("x and qweight disagree on K")
    _expect_shapes(qzeros, sb, gi, k, n, group_size)
    out = np.empty(m_idx.shape, np.float64)
    rc = _load().oracle_gemm_ref_sampled(_p(xb), _p(qweight), _p(qzeros), _p(sb), None if gi is None else _p(gi),
                                         _p(m_idx), _p(n_idx), ctypes.c_longlong(m_idx.size), _p(out),
                                         m, k, n, group_size)
    _check(rc, "gemm_ref_sampled")
    return out
