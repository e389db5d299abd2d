"""CPU oracle for the MXFP4 weight-only-quantised linear layer (arXiv 2503.13565,
section 3.4.3) -- TEST INFRASTRUCTURE, not the product.

This package wraps ``mxfp4_oracle.c`` (plain C, FP64, index-order loops) with
``ctypes``.  Only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import it.  It shares nothing with the HIP path and
never imports it.

Arrays are numpy: BF16 values travel as their 16-bit patterns (``uint16``),
packed nibbles and scale bytes as ``uint8``, results as ``float64``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mxfp4_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

BLOCK = 32


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP on) and return the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_direct_cast.argtypes = [vp, i64, i64, i64, vp, vp, i32]
        lib.oracle_direct_cast.restype = i32
        lib.oracle_dequant.argtypes = [vp, vp, i64, i64, vp]
        lib.oracle_dequant.restype = i32
        lib.oracle_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32]
        lib.oracle_woq_gemm.restype = i32
        lib.oracle_woq_gemm_late_scaled.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp]
        lib.oracle_woq_gemm_late_scaled.restype = i32
        lib.oracle_bf16_gemm.argtypes = [vp, i64, i64, vp, i64, i64, i64, vp, vp, i32]
        lib.oracle_bf16_gemm.restype = i32
        f64 = ctypes.c_double
        lib.oracle_greedy_accept.argtypes = [vp, vp, i64, vp]
        lib.oracle_greedy_accept.restype = i32
        lib.oracle_sd_speedup.argtypes = [f64, f64, f64]
        lib.oracle_sd_speedup.restype = f64
        lib.oracle_sd_speedup_alpha.argtypes = [f64, f64, f64]
        lib.oracle_sd_speedup_alpha.restype = f64
        lib.oracle_sd_speedup_two_level.argtypes = [f64] * 6
        lib.oracle_sd_speedup_two_level.restype = f64
        lib.oracle_e4m3_direct_cast.argtypes = [vp, i64, i64, i64, vp, vp, i32]
        lib.oracle_e4m3_direct_cast.restype = i32
        lib.oracle_e4m3_dequant.argtypes = [vp, vp, i64, i64, vp]
        lib.oracle_e4m3_dequant.restype = i32
        lib.oracle_e4m3_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32]
        lib.oracle_e4m3_woq_gemm.restype = i32
        lib.oracle_e4m3_magnitude.argtypes = [i32]
        lib.oracle_e4m3_magnitude.restype = ctypes.c_double
        lib.oracle_e2m3_direct_cast.argtypes = [vp, i64, i64, i64, vp, vp, i32]
        lib.oracle_e2m3_direct_cast.restype = i32
        lib.oracle_e2m3_dequant.argtypes = [vp, vp, i64, i64, vp]
        lib.oracle_e2m3_dequant.restype = i32
        lib.oracle_e2m3_woq_gemm.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp, i32]
        lib.oracle_e2m3_woq_gemm.restype = i32
        lib.oracle_e2m3_magnitude.argtypes = [i32]
        lib.oracle_e2m3_magnitude.restype = ctypes.c_double
        lib.oracle_woq_gemm_t.argtypes = [vp, i64, i64, vp, vp, i64, i64, vp, vp]
        lib.oracle_woq_gemm_t.restype = i32
        lib.oracle_mx_block_bytes.argtypes = [i32]
        lib.oracle_mx_block_bytes.restype = i32
        lib.oracle_mx_magnitude.argtypes = [i32, i32]
        lib.oracle_mx_magnitude.restype = ctypes.c_double
        lib.oracle_mx_direct_cast.argtypes = [i32, vp, i64, i64, i64, vp, vp, i32]
        lib.oracle_mx_direct_cast.restype = i32
        lib.oracle_mx_dequant.argtypes = [i32, vp, vp, i64, i64, vp]
        lib.oracle_mx_dequant.restype = i32
        lib.oracle_mx_woq_gemm.argtypes = [i32, vp, i64, i64, vp, vp, i64, i64, vp, vp, i32]
        lib.oracle_mx_woq_gemm.restype = i32
        lib.oracle_epilogue.argtypes = [vp, vp, i64, i64, vp, vp, i64, i32, vp, vp]
        lib.oracle_epilogue.restype = i32
        lib.oracle_argmax.argtypes = [vp, i64, i64, vp, vp]
        lib.oracle_argmax.restype = i32
        lib.oracle_e2m1_magnitude.argtypes = [i32]
        lib.oracle_e2m1_magnitude.restype = ctypes.c_double
        lib.oracle_max_threads.argtypes = []
        lib.oracle_max_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _as(a, dtype, ndim) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if a.ndim != ndim:
        raise ValueError("expected %d dimensions, got shape %r" % (ndim, a.shape))
    return a


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def e2m1_magnitude(code: int) -> float:
    return float(_load().oracle_e2m1_magnitude(int(code)))


def direct_cast(w_bits, threads: int = 0):
    """BF16 bit patterns ``[N,K]`` (uint16) -> (q ``[N,K/2]`` uint8, s ``[N,K/32]`` uint8)."""
    w = _as(w_bits, np.uint16, 2)
    n, k = w.shape
    if k % BLOCK:
        raise ValueError("K must be a multiple of 32")
    q = np.empty((n, k // 2), np.uint8)
    s = np.empty((n, k // BLOCK), np.uint8)
    rc = _load().oracle_direct_cast(_ptr(w), n, k, k, _ptr(q), _ptr(s), threads)
    if rc:
        raise RuntimeError("oracle_direct_cast failed: %d" % rc)
    return q, s


def dequant(q, s) -> np.ndarray:
    """Packed nibbles + scale bytes -> float64 ``[N,K]``."""
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    n, k = q.shape[0], q.shape[1] * 2
    if s.shape != (n, k // BLOCK) or k % BLOCK:
        raise ValueError("scale shape %r does not match q shape %r" % (s.shape, q.shape))
    out = np.empty((n, k), np.float64)
    rc = _load().oracle_dequant(_ptr(q), _ptr(s), n, k, _ptr(out))
    if rc:
        raise RuntimeError("oracle_dequant failed: %d" % rc)
    return out


def woq_gemm(x_bits, q, s, threads: int = 0, want_abs: bool = True):
    """FP64 product ``y[m,n] = sum_k x[m,k] * w_hat[n,k]`` and, if asked, the sum of
    absolute products (for the tolerance).  ``x_bits`` is uint16 ``[M,K]``."""
    x = _as(x_bits, np.uint16, 2)
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, k = x.shape
    n = q.shape[0]
    if q.shape[1] * 2 != k or s.shape != (n, k // BLOCK) or k % BLOCK:
        raise ValueError("shape mismatch: x %r q %r s %r" % (x.shape, q.shape, s.shape))
    y = np.empty((m, n), np.float64)
    a = np.empty((m, n), np.float64) if want_abs else None
    rc = _load().oracle_woq_gemm(_ptr(x), m, k, _ptr(q), _ptr(s), n, k, _ptr(y),
                                 _ptr(a) if want_abs else None, threads)
    if rc:
        raise RuntimeError("oracle_woq_gemm failed: %d" % rc)
    return (y, a) if want_abs else y


def bf16_gemm(x_bits, w_bits, threads: int = 0, want_abs: bool = True):
    """FP64 product with unquantised BF16 weights: ``y[m,n] = sum_k x[m,k] * w[n,k]`` and the sum of
    absolute products.  Both inputs are uint16 BF16 bit patterns, ``[M,K]`` and ``[N,K]``."""
    x = _as(x_bits, np.uint16, 2)
    w = _as(w_bits, np.uint16, 2)
    m, k = x.shape
    n = w.shape[0]
    if w.shape[1] != k:
        raise ValueError("shape mismatch: x %r w %r" % (x.shape, w.shape))
    y = np.empty((m, n), np.float64)
    a = np.empty((m, n), np.float64) if want_abs else None
    rc = _load().oracle_bf16_gemm(_ptr(x), m, k, _ptr(w), n, k, k, _ptr(y), _ptr(a) if want_abs else None,
                                  threads)
    if rc:
        raise RuntimeError("oracle_bf16_gemm failed: %d" % rc)
    return (y, a) if want_abs else y


def woq_gemm_t(x_bits, q, s, want_abs: bool = True):
    """FP64 product along the rows of the stored tensor, ``y[m,k] = sum_n x[m,n] * w_hat[n,k]``, and the
    sum of absolute products.  ``x_bits`` is uint16 ``[M,N]``."""
    x = _as(x_bits, np.uint16, 2)
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, n = x.shape
    k = q.shape[1] * 2
    if q.shape[0] != n or s.shape != (n, k // BLOCK) or k % BLOCK:
        raise ValueError("shape mismatch: x %r q %r s %r" % (x.shape, q.shape, s.shape))
    y = np.empty((m, k), np.float64)
    a = np.empty((m, k), np.float64) if want_abs else None
    rc = _load().oracle_woq_gemm_t(_ptr(x), m, n, _ptr(q), _ptr(s), n, k, _ptr(y), _ptr(a) if want_abs else None)
    if rc:
        raise RuntimeError("oracle_woq_gemm_t failed: %d" % rc)
    return (y, a) if want_abs else y


def woq_gemm_late_scaled(x_bits, q, s) -> np.ndarray:
    """The product with the scale applied once per 32-block partial sum (Eq. 2)."""
    x = _as(x_bits, np.uint16, 2)
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, k = x.shape
    n = q.shape[0]
    y = np.empty((m, n), np.float64)
    rc = _load().oracle_woq_gemm_late_scaled(_ptr(x), m, k, _ptr(q), _ptr(s), n, k, _ptr(y))
    if rc:
        raise RuntimeError("oracle_woq_gemm_late_scaled failed: %d" % rc)
    return y


def e4m3_magnitude(code: int) -> float:
    return float(_load().oracle_e4m3_magnitude(int(code)))


def e4m3_direct_cast(w_bits, threads: int = 0):
    """BF16 bit patterns ``[N, K]`` -> (``q8 [N, K]`` E4M3 bytes, ``s [N, K/32]`` E8M0 scale bytes)."""
    w = _as(w_bits, np.uint16, 2)
    n, k = w.shape
    if k % BLOCK:
        raise ValueError("K must be a multiple of 32")
    q8 = np.empty((n, k), np.uint8)
    s = np.empty((n, k // BLOCK), np.uint8)
    rc = _load().oracle_e4m3_direct_cast(_ptr(w), n, k, k, _ptr(q8), _ptr(s), threads)
    if rc:
        raise RuntimeError("oracle_e4m3_direct_cast failed: %d" % rc)
    return q8, s


def e4m3_dequant(q8, s) -> np.ndarray:
    q8 = _as(q8, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    n, k = q8.shape
    if s.shape != (n, k // BLOCK):
        raise ValueError("shape mismatch: q8 %r s %r" % (q8.shape, s.shape))
    out = np.empty((n, k), np.float64)
    rc = _load().oracle_e4m3_dequant(_ptr(q8), _ptr(s), n, k, _ptr(out))
    if rc:
        raise RuntimeError("oracle_e4m3_dequant failed: %d" % rc)
    return out


def e4m3_woq_gemm(x_bits, q8, s, threads: int = 0, want_abs: bool = True):
    """FP64 product with 8-bit (E4M3 + E8M0) weights and the sum of absolute products."""
    x = _as(x_bits, np.uint16, 2)
    q8 = _as(q8, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, k = x.shape
    n = q8.shape[0]
    if q8.shape[1] != k or s.shape != (n, k // BLOCK):
        raise ValueError("shape mismatch: x %r q8 %r s %r" % (x.shape, q8.shape, s.shape))
    y = np.empty((m, n), np.float64)
    a = np.empty((m, n), np.float64) if want_abs else None
    rc = _load().oracle_e4m3_woq_gemm(_ptr(x), m, k, _ptr(q8), _ptr(s), n, k, _ptr(y),
                                      _ptr(a) if want_abs else None, threads)
    if rc:
        raise RuntimeError("oracle_e4m3_woq_gemm failed: %d" % rc)
    return (y, a) if want_abs else y


def e2m3_magnitude(code: int) -> float:
    return float(_load().oracle_e2m3_magnitude(int(code)))


def e2m3_direct_cast(w_bits, threads: int = 0):
    """BF16 bit patterns ``[N, K]`` -> (``q6 [N, K/32*24]`` packed 6-bit codes, ``s [N, K/32]`` scale bytes)."""
    w = _as(w_bits, np.uint16, 2)
    n, k = w.shape
    if k % BLOCK:
        raise ValueError("K must be a multiple of 32")
    q6 = np.empty((n, k // BLOCK * 24), np.uint8)
    s = np.empty((n, k // BLOCK), np.uint8)
    rc = _load().oracle_e2m3_direct_cast(_ptr(w), n, k, k, _ptr(q6), _ptr(s), threads)
    if rc:
        raise RuntimeError("oracle_e2m3_direct_cast failed: %d" % rc)
    return q6, s


def e2m3_dequant(q6, s) -> np.ndarray:
    q6 = _as(q6, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    n, nblk = s.shape
    if q6.shape != (n, nblk * 24):
        raise ValueError("shape mismatch: q6 %r s %r" % (q6.shape, s.shape))
    out = np.empty((n, nblk * BLOCK), np.float64)
    rc = _load().oracle_e2m3_dequant(_ptr(q6), _ptr(s), n, nblk * BLOCK, _ptr(out))
    if rc:
        raise RuntimeError("oracle_e2m3_dequant failed: %d" % rc)
    return out


def e2m3_woq_gemm(x_bits, q6, s, threads: int = 0, want_abs: bool = True):
    """FP64 product with 6-bit (E2M3 + E8M0) weights and the sum of absolute products."""
    x = _as(x_bits, np.uint16, 2)
    q6 = _as(q6, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, k = x.shape
    n = q6.shape[0]
    if q6.shape[1] != k // BLOCK * 24 or s.shape != (n, k // BLOCK):
        raise ValueError("shape mismatch: x %r q6 %r s %r" % (x.shape, q6.shape, s.shape))
    y = np.empty((m, n), np.float64)
    a = np.empty((m, n), np.float64) if want_abs else None
    rc = _load().oracle_e2m3_woq_gemm(_ptr(x), m, k, _ptr(q6), _ptr(s), n, k, _ptr(y),
                                      _ptr(a) if want_abs else None, threads)
    if rc:
        raise RuntimeError("oracle_e2m3_woq_gemm failed: %d" % rc)
    return (y, a) if want_abs else y


FMT_E5M2, FMT_E3M2, FMT_T2 = 1, 2, 3


def mx_block_bytes(fmt: int) -> int:
    return int(_load().oracle_mx_block_bytes(int(fmt)))


def mx_magnitude(fmt: int, code: int) -> float:
    return float(_load().oracle_mx_magnitude(int(fmt), int(code)))


def mx_direct_cast(fmt: int, w_bits, threads: int = 0):
    """BF16 bit patterns ``[N, K]`` -> (``q [N, K/32 * block bytes]`` packed codes, ``s [N, K/32]`` scale
    bytes) in one of the generic formats (``FMT_E5M2``, ``FMT_E3M2``, ``FMT_T2``)."""
    w = _as(w_bits, np.uint16, 2)
    n, k = w.shape
    bb = mx_block_bytes(fmt)
    if k % BLOCK or not bb:
        raise ValueError("K must be a multiple of 32 and fmt a known format")
    q = np.empty((n, k // BLOCK * bb), np.uint8)
    s = np.empty((n, k // BLOCK), np.uint8)
    rc = _load().oracle_mx_direct_cast(int(fmt), _ptr(w), n, k, k, _ptr(q), _ptr(s), threads)
    if rc:
        raise RuntimeError("oracle_mx_direct_cast failed: %d" % rc)
    return q, s


def mx_dequant(fmt: int, q, s) -> np.ndarray:
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    n, nblk = s.shape
    bb = mx_block_bytes(fmt)
    if q.shape != (n, nblk * bb):
        raise ValueError("shape mismatch: q %r s %r" % (q.shape, s.shape))
    out = np.empty((n, nblk * BLOCK), np.float64)
    rc = _load().oracle_mx_dequant(int(fmt), _ptr(q), _ptr(s), n, nblk * BLOCK, _ptr(out))
    if rc:
        raise RuntimeError("oracle_mx_dequant failed: %d" % rc)
    return out


def mx_woq_gemm(fmt: int, x_bits, q, s, threads: int = 0, want_abs: bool = True):
    """FP64 product with weights in a generic format and the sum of absolute products."""
    x = _as(x_bits, np.uint16, 2)
    q = _as(q, np.uint8, 2)
    s = _as(s, np.uint8, 2)
    m, k = x.shape
    n = q.shape[0]
    bb = mx_block_bytes(fmt)
    if q.shape[1] != k // BLOCK * bb or s.shape != (n, k // BLOCK):
        raise ValueError("shape mismatch: x %r q %r s %r" % (x.shape, q.shape, s.shape))
    y = np.empty((m, n), np.float64)
    a = np.empty((m, n), np.float64) if want_abs else None
    rc = _load().oracle_mx_woq_gemm(int(fmt), _ptr(x), m, k, _ptr(q), _ptr(s), n, k, _ptr(y),
                                    _ptr(a) if want_abs else None, threads)
    if rc:
        raise RuntimeError("oracle_mx_woq_gemm failed: %d" % rc)
    return (y, a) if want_abs else y


ACT_NONE, ACT_SWIGLU = 0, 1


def epilogue(y, a, bias_bits=None, residual_bits=None, act: int = ACT_NONE):
    """Bias, gated activation and residual add on an exact product ``y`` with its sum of absolute
    products ``a`` (both ``[M, N]``): returns ``(out, a_out)``, ``[M, N]`` or ``[M, N/2]`` for
    ``ACT_SWIGLU`` (weight rows interleaved gate, up, gate, up...).  ``bias_bits`` is ``[N]``,
    ``residual_bits`` ``[M, C]`` (any row stride), both BF16 bit patterns; ``tolerance(out, a_out)``
    is the parity bar of the fused call."""
    y = _as(y, np.float64, 2)
    a = _as(a, np.float64, 2)
    if y.shape != a.shape:
        raise ValueError("y %r and a %r differ in shape" % (y.shape, a.shape))
    m, n = y.shape
    c = n // 2 if act == ACT_SWIGLU else n
    b = None if bias_bits is None else _as(bias_bits, np.uint16, 1)
    if b is not None and b.shape[0] != n:
        raise ValueError("bias must have N = %d entries" % n)
    r, ldr = None, 0
    if residual_bits is not None:
        r = np.asarray(residual_bits)
        if r.dtype != np.uint16 or r.ndim != 2 or r.shape != (m, c) or (m > 1 and r.strides[1] != 2):
            raise ValueError("residual must be uint16 [M, %d]" % c)
        if m > 1 and r.strides[0] % 2 == 0 and r.strides[0] >= 2 * c and r.strides[1] == 2:
            ldr = r.strides[0] // 2
        else:
            r = np.ascontiguousarray(r)
            ldr = c
    out = np.empty((m, c), np.float64)
    a_out = np.empty((m, c), np.float64)
    rc = _load().oracle_epilogue(_ptr(y), _ptr(a), m, n, _ptr(b) if b is not None else None,
                                 _ptr(r) if r is not None else None, ldr, int(act), _ptr(out), _ptr(a_out))
    if rc:
        raise RuntimeError("oracle_epilogue failed: %d" % rc)
    return out, a_out


def argmax(y):
    """Row-wise index of the maximum (lowest index among equals) and its value."""
    y = _as(y, np.float64, 2)
    m, n = y.shape
    idx = np.empty((m,), np.int32)
    val = np.empty((m,), np.float64)
    rc = _load().oracle_argmax(_ptr(y), m, n, _ptr(idx), _ptr(val))
    if rc:
        raise RuntimeError("oracle_argmax failed: %d" % rc)
    return idx, val


def greedy_accept(target_tokens, draft_tokens):
    """(G, next token): G leading draft tokens equal the target's picks; the round then emits the
    target's own pick at position G.  ``target_tokens`` has one entry more than ``draft_tokens``."""
    t = _as(target_tokens, np.int32, 1)
    d = _as(draft_tokens, np.int32, 1)
    if t.shape[0] != d.shape[0] + 1:
        raise ValueError("need N + 1 target picks for N draft tokens")
    out = np.zeros(2, np.int32)
    rc = _load().oracle_greedy_accept(_ptr(t), _ptr(d) if d.size else None, d.shape[0], _ptr(out))
    if rc:
        raise RuntimeError("oracle_greedy_accept failed: %d" % rc)
    return int(out[0]), int(out[1])


def sd_speedup(g: float, n_draft: float, s: float) -> float:
    return float(_load().oracle_sd_speedup(g, n_draft, s))


def sd_speedup_alpha(alpha: float, n_draft: float, s: float) -> float:
    return float(_load().oracle_sd_speedup_alpha(alpha, n_draft, s))


def sd_speedup_two_level(alpha_mid, n_mid, s_mid, alpha_last, n_last, s_last) -> float:
    return float(_load().oracle_sd_speedup_two_level(alpha_mid, n_mid, s_mid, alpha_last, n_last, s_last))


def bf16_ulp(y) -> np.ndarray:
    """Spacing of BF16 numbers at |y|: 2^(floor(log2|y|) - 7) for normal numbers, 2^-133 for
    zero and throughout the subnormal range (the format has no finer step there).  This is
    the '+1 BF16 ulp of |y_ref|' term of the output tolerance."""
    y = np.abs(np.asarray(y, np.float64))
    _, ex = np.frexp(y)                       # y = f * 2^ex, f in [0.5, 1)
    ulp = np.ldexp(1.0, np.maximum(ex - 1, -126) - 7)
    return np.where(y == 0.0, np.ldexp(1.0, -126 - 7), ulp)


def tolerance(y_ref, a_ref) -> np.ndarray:
    """|y_gpu - y_ref| <= 1e-3 * sum_k |x_k w_k| + one BF16 ulp of |y_ref|."""
    return 1e-3 * np.asarray(a_ref, np.float64) + bf16_ulp(y_ref)
