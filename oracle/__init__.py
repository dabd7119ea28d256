"""CPU oracle for the AnyBCQ bit-plane product.  TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper over ``bcq_oracle.c`` (plain C, IEEE double) plus the
acceptance tolerance.  It is independent of the HIP library: the two share no
code and neither imports the other.  Only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product path
must never route through it.

The oracle is the plain definition of what the method computes (paper
section 2.2: W = sum_i alpha_i B_i with B_i in {-1,+1}; section 1 / Fig. 1(b):
precision p uses the scale set of precision p with the first p planes;
section 3.1: stored 0 -> -alpha_i, stored 1 -> +alpha_i), followed by an
ordinary matrix-vector product in float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcq_oracle.c")
_SRC_QUANT = os.path.join(_HERE, "bcq_quant_oracle.c")
_LIB = os.path.join(_HERE, "libbcq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``bcq_oracle.c`` and ``bcq_quant_oracle.c`` with gcc into ``libbcq_oracle.so`` beside them."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_QUANT))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-o", _LIB, _SRC, _SRC_QUANT, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.bcq_oracle_pack.argtypes = [vp, vp, i32, i64, i64]
        lib.bcq_oracle_unpack.argtypes = [vp, vp, i32, i64, i64]
        lib.bcq_oracle_dequant.argtypes = [vp, vp, i32, i64, i64, i64, vp]
        lib.bcq_oracle_gemv.argtypes = [vp, vp, i32, vp, vp, vp, i64, i64, i64, i64]
        lib.bcq_oracle_gemm_mixed.argtypes = [vp, vp, vp, i32, vp, vp, vp, i64, i64, i64, i64]
        lib.bcq_oracle_dequant_offset.argtypes = [vp, vp, vp, i32, i64, i64, i64, vp]
        lib.bcq_oracle_gemv_offset.argtypes = [vp, vp, vp, i32, vp, vp, vp, i64, i64, i64, i64]
        lib.bcq_oracle_gemm_mixed_offset.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, i64, i64, i64, i64]
        lib.bcq_oracle_quantize.argtypes = [vp, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp]
        lib.bcq_oracle_quantize.restype = i32
        lib.bcq_oracle_num_threads.restype = i32
        lib.bcq_oracle_set_num_threads.argtypes = [i32]
        for f in (lib.bcq_oracle_pack, lib.bcq_oracle_unpack, lib.bcq_oracle_dequant,
                  lib.bcq_oracle_gemv, lib.bcq_oracle_gemm_mixed, lib.bcq_oracle_dequant_offset,
                  lib.bcq_oracle_gemv_offset, lib.bcq_oracle_gemm_mixed_offset):
            f.restype = i32
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"expected dtype {np.dtype(dtype)}, got {a.dtype}")
    return a


def _half_bits(a) -> np.ndarray:
    """float16 array -> its raw uint16 bit patterns (no value conversion)."""
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError(f"scales/activations must be float16, got {a.dtype}")
    return a.view(np.uint16)


def num_threads() -> int:
    return int(_load().bcq_oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().bcq_oracle_set_num_threads(int(t))


def pack(codes: np.ndarray) -> np.ndarray:
    """int8 codes [P][m][n] (>0 means +1) -> uint32 planes [P][m][n/32]."""
    codes = _c(codes, np.int8)
    P, m, n = codes.shape
    planes = np.empty((P, m, n // 32), dtype=np.uint32)
    if _load().bcq_oracle_pack(_ptr(codes), _ptr(planes), P, m, n) != 0:
        raise ValueError("bcq_oracle_pack: bad shape (n must be a multiple of 32)")
    return planes


def unpack(planes: np.ndarray) -> np.ndarray:
    """uint32 planes [P][m][n/32] -> int8 codes [P][m][n] in {-1,+1}."""
    planes = _c(planes, np.uint32)
    P, m, words = planes.shape
    codes = np.empty((P, m, words * 32), dtype=np.int8)
    if _load().bcq_oracle_unpack(_ptr(planes), _ptr(codes), P, m, words * 32) != 0:
        raise ValueError("bcq_oracle_unpack: bad shape")
    return codes


def _offset_bits(offsets, m, ngroups):
    if offsets is None:
        return None
    z = _half_bits(offsets)
    if z.shape != (m, ngroups):
        raise ValueError(f"offset set has shape {z.shape}, expected {(m, ngroups)}")
    return z


def dequant(planes: np.ndarray, scales_p: np.ndarray, group: int = 128, offsets=None) -> np.ndarray:
    """W_p as float64 [m][n]; p is ``scales_p.shape[0]`` (small shapes only).

    ``offsets`` (float16 [m][n/group]) adds the asymmetric scheme's offset of every (row, group)."""
    planes = _c(planes, np.uint32)
    s = _half_bits(scales_p)
    p, m, ngroups = s.shape
    n = planes.shape[2] * 32
    if planes.shape[0] < p or planes.shape[1] != m or ngroups * group != n:
        raise ValueError("shape mismatch between planes and scales")
    z = _offset_bits(offsets, m, ngroups)
    w = np.empty((m, n), dtype=np.float64)
    zp = _ptr(z) if z is not None else None
    if _load().bcq_oracle_dequant_offset(_ptr(planes), _ptr(s), zp, p, m, n, group, _ptr(w)) != 0:
        raise ValueError("bcq_oracle_dequant: bad argument")
    return w


def gemv(planes: np.ndarray, scales_p: np.ndarray, x: np.ndarray, group: int = 128, offsets=None):
    """Uniform precision p = ``scales_p.shape[0]``; ``offsets`` as for :func:`dequant`.

    Returns ``(y, abs)`` as float64 [batch][m]: y = W_p x, abs = sum_j |W_p[r,j] x_j|.
    """
    planes = _c(planes, np.uint32)
    s = _half_bits(scales_p)
    xb = _half_bits(x)
    p, m, ngroups = s.shape
    batch, n = xb.shape
    if planes.shape[0] < p or planes.shape[1] != m or planes.shape[2] * 32 != n or ngroups * group != n:
        raise ValueError("shape mismatch")
    z = _offset_bits(offsets, m, ngroups)
    zp = _ptr(z) if z is not None else None
    y = np.zeros((batch, m), dtype=np.float64)
    a = np.zeros((batch, m), dtype=np.float64)
    if _load().bcq_oracle_gemv_offset(_ptr(planes), _ptr(s), zp, p, _ptr(xb), _ptr(y), _ptr(a), m, n, batch, group) != 0:
        raise ValueError("bcq_oracle_gemv: bad argument")
    return y, a


def gemm_mixed(planes: np.ndarray, scales_by_p: dict, p_req, x: np.ndarray, group: int = 128, offsets_by_p=None):
    """Per-request precision.  ``scales_by_p[q]`` is the float16 set [q][m][n/group];
    ``offsets_by_p[q]`` (optional) the float16 offsets [m][n/group] of precision q."""
    planes = _c(planes, np.uint32)
    xb = _half_bits(x)
    p_req = np.ascontiguousarray(np.asarray(p_req, dtype=np.int32))
    p_max, m, words = planes.shape
    batch, n = xb.shape
    if words * 32 != n or p_req.shape != (batch,):
        raise ValueError("shape mismatch")
    keep = []
    ptrs = (ctypes.c_void_p * (p_max + 1))()
    for q, s in scales_by_p.items():
        if not 1 <= q <= p_max:
            raise ValueError("scale set for a precision outside [1, p_max]")
        sb = _half_bits(s)
        if sb.shape != (q, m, n // group):
            raise ValueError(f"scale set {q} has shape {sb.shape}")
        keep.append(sb)
        ptrs[q] = sb.ctypes.data
    optrs = (ctypes.c_void_p * (p_max + 1))()
    for q, zq in (offsets_by_p or {}).items():
        if not 1 <= q <= p_max:
            raise ValueError("offset set for a precision outside [1, p_max]")
        zb = _offset_bits(zq, m, n // group)
        keep.append(zb)
        optrs[q] = zb.ctypes.data
    y = np.zeros((batch, m), dtype=np.float64)
    a = np.zeros((batch, m), dtype=np.float64)
    rc = _load().bcq_oracle_gemm_mixed_offset(_ptr(planes), ctypes.cast(ptrs, ctypes.c_void_p),
                                              ctypes.cast(optrs, ctypes.c_void_p) if offsets_by_p else None, _ptr(p_req), p_max,
                                              _ptr(xb), _ptr(y), _ptr(a), m, n, batch, group)
    if rc != 0:
        raise ValueError("bcq_oracle_gemm_mixed: bad argument")
    return y, a


def quantize(w: np.ndarray, p_low: int, p_high: int, cycles: int, group: int = 128, with_offset: bool = False,
             literal_residual: bool = False) -> dict:
    """Algorithm 1 on float16 weights [m][n], every (row, group) on its own.

    Returns ``{"codes": int8 [p_high][m][n] in {-1,+1}, "scales": {p: float64 [p][m][n/group]},
    "offsets": {p: float64 [m][n/group]} or None}`` for p = p_low..p_high, unrounded.
    ``group`` may be any divisor of n here (the packed format needs a multiple of 32).
    """
    wb = _half_bits(w)
    m, n = wb.shape
    if n % group:
        raise ValueError("n must be a multiple of group")
    ng = n // group
    nsets = p_high - p_low + 1
    codes = np.zeros((p_high, m, n), dtype=np.int8)
    flat = np.zeros(sum(p * m * ng for p in range(p_low, p_high + 1)), dtype=np.float64)
    offs = np.zeros((nsets, m, ng), dtype=np.float64)
    rc = _load().bcq_oracle_quantize(_ptr(wb), m, n, group, p_low, p_high, cycles, int(with_offset), int(literal_residual),
                                     _ptr(codes), _ptr(flat), _ptr(offs))
    if rc != 0:
        raise ValueError("bcq_oracle_quantize: bad argument")
    scales, at = {}, 0
    for p in range(p_low, p_high + 1):
        scales[p] = flat[at:at + p * m * ng].reshape(p, m, ng).copy()
        at += p * m * ng
    offsets = {p: offs[p - p_low].copy() for p in range(p_low, p_high + 1)} if with_offset else None
    return {"codes": codes, "scales": scales, "offsets": offsets}


def ulp16(v) -> np.ndarray:
    """Spacing of binary16 at |v|: 2^(max(floor(log2|v|), -14) - 10), at least 2^-24."""
    v = np.abs(np.asarray(v, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(v, 2.0 ** -14)))
    return np.exp2(np.maximum(e, -14.0) - 10.0)


def tolerance(y_ref, abs_ref) -> np.ndarray:
    """Acceptance bound: |y - y_ref| <= 4e-3 * sum_j|W_p[r,j] x_j| + one binary16 ulp at y_ref."""
    return 4e-3 * np.asarray(abs_ref, dtype=np.float64) + ulp16(y_ref)
