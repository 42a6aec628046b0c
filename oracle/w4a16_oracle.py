"""Python face of the CPU oracle (TEST INFRASTRUCTURE, never the product path).

Loads ``libw4a16_oracle.so`` built from ``w4a16_oracle.c`` in this folder and
exposes its functions on numpy arrays.  The arithmetic lives in the C file:
the plain definition C = A * s(W - z) of Section 3, Eq. 2, summed in binary64.
Only tests, the smoke check and the benchmark's host-baseline leg may import
this module; it imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w4a16_oracle.c")
_LIB = os.path.join(_HERE, "libw4a16_oracle.so")
# The mutation test points this at a deliberately broken build to prove that the pins notice.
_OVERRIDE = os.environ.get("W4A16_ORACLE_LIB_OVERRIDE")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over output columns)."""
    if _OVERRIDE:
        return _OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.w4a16_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.w4a16_oracle_half_to_float.restype = ctypes.c_float
        lib.w4a16_oracle_unpack_codes.argtypes = [u32p, ci, ci, u8p]
        lib.w4a16_oracle_unpack_zeros.argtypes = [u32p, ci, ci, u8p]
        lib.w4a16_oracle_dequant.argtypes = [u32p, u16p, u32p, ci, ci, ci, f32p]
        lib.w4a16_oracle_gemm.argtypes = [u16p, u32p, u16p, u32p, ci, ci, ci, ci, f64p]
        lib.w4a16_oracle_gemm_columns.argtypes = [u16p, u32p, u16p, u32p, ci, ci, ci, ci, i32p, ci, f64p]
        lib.w4a16_oracle_dequant_symmetric.argtypes = [u32p, u16p, ci, ci, ci, f32p]
        lib.w4a16_oracle_gemm_symmetric.argtypes = [u16p, u32p, u16p, ci, ci, ci, ci, f64p]
        lib.w4a16_oracle_bfloat_to_float.argtypes = [ctypes.c_uint16]
        lib.w4a16_oracle_bfloat_to_float.restype = ctypes.c_float
        lib.w4a16_oracle_gemm_bf16.argtypes = [u16p, u32p, u16p, u32p, ci, ci, ci, ci, f64p]
        lib.w4a16_oracle_threads.argtypes = []
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _u16(a):
    """fp16 array (or raw uint16 bit patterns) -> contiguous uint16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError("expected float16 or uint16, got %s" % a.dtype)


def _u32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint32:
        raise TypeError("expected uint32, got %s" % a.dtype)
    return a


def half_to_float(bits: int) -> np.float32:
    """binary16 bit pattern -> binary32 value, by the oracle's own conversion."""
    return np.float32(_load().w4a16_oracle_half_to_float(int(bits) & 0xFFFF))


def unpack_codes(Wp: np.ndarray) -> np.ndarray:
    """Wp[K/8, N] uint32 -> q[K, N] uint8 in 0..15 (storage reading of Section 2.2)."""
    Wp = _u32(Wp)
    R, N = Wp.shape
    q = np.empty((R * 8, N), np.uint8)
    rc = _load().w4a16_oracle_unpack_codes(_ptr(Wp, ctypes.c_uint32), R * 8, N, _ptr(q, ctypes.c_uint8))
    if rc:
        raise ValueError("bad shape for unpack_codes: %r" % (Wp.shape,))
    return q


def unpack_zeros(Zp: np.ndarray) -> np.ndarray:
    """Zp[G, N/8] uint32 -> z[G, N] uint8 in 0..15."""
    Zp = _u32(Zp)
    G, C = Zp.shape
    z = np.empty((G, C * 8), np.uint8)
    rc = _load().w4a16_oracle_unpack_zeros(_ptr(Zp, ctypes.c_uint32), G, C * 8, _ptr(z, ctypes.c_uint8))
    if rc:
        raise ValueError("bad shape for unpack_zeros: %r" % (Zp.shape,))
    return z


def _check(Wp, scales, Zp, group):
    Wp, s, Zp = _u32(Wp), _u16(scales), _u32(Zp)
    R, N = Wp.shape
    K = R * 8
    if group < 1 or K % group or N % 8:
        raise ValueError("bad group/shape: K=%d N=%d group=%d" % (K, N, group))
    G = K // group
    if s.shape != (G, N) or Zp.shape != (G, N // 8):
        raise ValueError("scales %r / zeros %r do not fit K=%d N=%d group=%d" % (s.shape, Zp.shape, K, N, group))
    return Wp, s, Zp, K, N


def dequant(Wp, scales, Zp, group: int) -> np.ndarray:
    """Dequant(W) = s (W - z) of Eq. 2 as binary32 [K, N] (exact products)."""
    Wp, s, Zp, K, N = _check(Wp, scales, Zp, group)
    w = np.empty((K, N), np.float32)
    rc = _load().w4a16_oracle_dequant(
        _ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16), _ptr(Zp, ctypes.c_uint32), group, K, N,
        _ptr(w, ctypes.c_float))
    if rc:
        raise ValueError("oracle rejected the shape")
    return w


def gemm(X, Wp, scales, Zp, group: int, cols=None) -> np.ndarray:
    """ref = A * Dequant(W) (Eq. 2) in binary64: [M, N], or [M, len(cols)] on chosen columns."""
    Wp, s, Zp, K, N = _check(Wp, scales, Zp, group)
    X = _u16(X)
    if X.ndim != 2 or X.shape[1] != K:
        raise ValueError("X %r does not fit K=%d" % (X.shape, K))
    M = X.shape[0]
    lib = _load()
    if cols is None:
        ref = np.empty((M, N), np.float64)
        rc = lib.w4a16_oracle_gemm(
            _ptr(X, ctypes.c_uint16), _ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16),
            _ptr(Zp, ctypes.c_uint32), group, M, N, K, _ptr(ref, ctypes.c_double))
    else:
        cols = np.ascontiguousarray(cols, dtype=np.int32)
        ref = np.empty((M, cols.size), np.float64)
        rc = lib.w4a16_oracle_gemm_columns(
            _ptr(X, ctypes.c_uint16), _ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16),
            _ptr(Zp, ctypes.c_uint32), group, M, N, K, _ptr(cols, ctypes.c_int32), int(cols.size),
            _ptr(ref, ctypes.c_double))
    if rc:
        raise ValueError("oracle rejected the arguments")
    return ref


def _check_symmetric(Wp, scales, group):
    Wp, s = _u32(Wp), _u16(scales)
    R, N = Wp.shape
    K = R * 8
    if group < 1 or K % group or N % 8 or s.shape != (K // group, N):
        raise ValueError("scales %r do not fit K=%d N=%d group=%d" % (s.shape, K, N, group))
    return Wp, s, K, N


def dequant_symmetric(Wp, scales, group: int) -> np.ndarray:
    """Symmetric reading of Section 2.1 (z = 0 on signed codes = stored code - 8): s (W - 8) as binary32 [K, N]."""
    Wp, s, K, N = _check_symmetric(Wp, scales, group)
    w = np.empty((K, N), np.float32)
    if _load().w4a16_oracle_dequant_symmetric(_ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16), group, K, N,
                                              _ptr(w, ctypes.c_float)):
        raise ValueError("oracle rejected the shape")
    return w


def gemm_symmetric(X, Wp, scales, group: int) -> np.ndarray:
    """ref = A * s (W - 8) in binary64 [M, N]: Eq. 2 without a zero-point tensor."""
    Wp, s, K, N = _check_symmetric(Wp, scales, group)
    X = _u16(X)
    if X.ndim != 2 or X.shape[1] != K:
        raise ValueError("X %r does not fit K=%d" % (X.shape, K))
    ref = np.empty((X.shape[0], N), np.float64)
    if _load().w4a16_oracle_gemm_symmetric(_ptr(X, ctypes.c_uint16), _ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16),
                                           group, X.shape[0], N, K, _ptr(ref, ctypes.c_double)):
        raise ValueError("oracle rejected the arguments")
    return ref


def bfloat_to_float(bits: int) -> np.float32:
    """bfloat16 bit pattern -> binary32 value, by the oracle's own field-by-field decoding."""
    return np.float32(_load().w4a16_oracle_bfloat_to_float(int(bits) & 0xFFFF))


def gemm_bf16(Xb, Wp, scales, Zp, group: int) -> np.ndarray:
    """ref = A * Dequant(W) (Eq. 2) in binary64 [M, N], A given as bfloat16 bit patterns (uint16 [M, K])."""
    Wp, s, Zp, K, N = _check(Wp, scales, Zp, group)
    Xb = np.ascontiguousarray(Xb)
    if Xb.dtype != np.uint16 or Xb.ndim != 2 or Xb.shape[1] != K:
        raise ValueError("X must be uint16 bfloat16 bit patterns [M, %d], got %s %r" % (K, Xb.dtype, Xb.shape))
    ref = np.empty((Xb.shape[0], N), np.float64)
    if _load().w4a16_oracle_gemm_bf16(_ptr(Xb, ctypes.c_uint16), _ptr(Wp, ctypes.c_uint32), _ptr(s, ctypes.c_uint16),
                                      _ptr(Zp, ctypes.c_uint32), group, Xb.shape[0], N, K, _ptr(ref, ctypes.c_double)):
        raise ValueError("oracle rejected the arguments")
    return ref


def to_bf16_bits(ref: np.ndarray) -> np.ndarray:
    """Final cast of Section 3 for a bfloat16 output: binary64 -> bfloat16 bit patterns, one rounding
    (to nearest, ties to even), written out on the value: v = f 2^e with 1/2 <= |f| < 1 keeps 8 significant
    bits, i.e. a multiple of 2^(e-8); below the normal range the spacing stays 2^-133; beyond the largest
    finite bfloat16 the result is an infinity."""
    v = np.asarray(ref, dtype=np.float64)
    out = np.zeros(v.shape, np.uint16)
    sign = np.signbit(v).astype(np.uint16) << 15
    a = np.abs(v)
    nan = np.isnan(v)
    with np.errstate(invalid="ignore", over="ignore"):
        f, e = np.frexp(np.where(np.isfinite(a), a, 0.0))
        e = np.maximum(e, -125)                      # normal range starts at 2^-126 = 0.5 * 2^-125
        steps = np.rint(np.ldexp(a, 8 - e))          # multiples of the spacing 2^(e-8); rint is ties-to-even
        steps = np.where(np.isfinite(a), steps, 0.0).astype(np.int64)
    # steps in 0..256: 0..127 subnormal (e = -125), 128..255 the significand, 256 = carry into the next binade
    carry = steps == 256
    e = np.where(carry, e + 1, e)
    steps = np.where(carry, 128, steps)
    biased = np.where(steps < 128, 0, e + 126)       # value = steps * 2^(e-8) = (128 + mant) 2^(biased-134)
    mant = np.where(steps < 128, steps, steps - 128)
    inf = np.isinf(a) | (biased >= 255)
    bits = (biased.astype(np.int64) << 7) | mant
    bits = np.where(inf, 0x7F80, bits)
    bits = np.where(nan, 0x7FC0, bits)
    out[...] = bits.astype(np.uint16) | sign
    return out


def to_fp16(ref: np.ndarray) -> np.ndarray:
    """Final cast of Section 3 (wide sum -> FP16), read as round-to-nearest-even."""
    with np.errstate(over="ignore"):
        return np.asarray(ref, dtype=np.float64).astype(np.float16)


def threads() -> int:
    """Host threads the gemm spreads its output columns over."""
    return int(_load().w4a16_oracle_threads())
