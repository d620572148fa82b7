"""ctypes loader for oracle/tw_oracle.c (TEST INFRASTRUCTURE, see the C file's
header for what is followed and which readings are taken).

Arrays of bf16 travel as numpy uint16 bit patterns. Expected values come back
as float64, unrounded.
"""
import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tw_oracle.c")
_LIB = os.path.join(_HERE, "libtw_oracle.so")
_lock = threading.Lock()
_lib = None

_u16p = ctypes.POINTER(ctypes.c_uint16)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64p = ctypes.POINTER(ctypes.c_int64)


def build(force=True):
    """Compile tw_oracle.c with gcc into oracle/libtw_oracle.so."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
           "-o", tmp, _SRC, "-lm", "-lpthread"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        fused_args = [ctypes.POINTER(_u16p), _u16p, _u16p, ctypes.c_float,
                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int, _f64p, _f64p]
        for name in ("tw_oracle_fused", "tw_oracle_fused_rounded_x", "tw_oracle_unfused",
                     "tw_oracle_unfused_f32sum"):
            fn = getattr(lib, name)
            fn.argtypes = fused_args
            fn.restype = ctypes.c_int
        lib.tw_oracle_fused_mt.argtypes = fused_args + [ctypes.c_int]
        lib.tw_oracle_fused_mt.restype = ctypes.c_int
        lib.tw_oracle_gemm.argtypes = [_u16p, _u16p] + [ctypes.c_int64] * 5 + [_f64p]
        lib.tw_oracle_gemm.restype = ctypes.c_int
        lib.tw_oracle_gemm_samples.argtypes = (
            [_u16p, _u16p] + [ctypes.c_int64] * 5 + [_i64p, _i64p, ctypes.c_int64, _f64p])
        lib.tw_oracle_gemm_samples.restype = ctypes.c_int
        lib.tw_oracle_bf16_to_f64_array.argtypes = [_u16p, ctypes.c_int64, _f64p]
        lib.tw_oracle_bf16_to_f64_array.restype = None
        lib.tw_oracle_f64_to_bf16_array.argtypes = [_f64p, ctypes.c_int64, _u16p]
        lib.tw_oracle_f64_to_bf16_array.restype = None
        _lib = lib
        return lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 arrays are passed as uint16 bit patterns, got %s" % a.dtype)
    return a


def _ptr(a, ty):
    return a.ctypes.data_as(ty)


def _fused_call(name, partials, residual, weight, eps, nthreads=None):
    lib = _load()
    residual = _u16(residual)
    weight = _u16(weight)
    if residual.ndim != 2:
        raise ValueError("residual must be [N, H]")
    N, H = residual.shape
    if weight.shape != (H,):
        raise ValueError("weight must be [H]")
    parts = [_u16(p) for p in partials]
    for p in parts:
        if p.shape != (N, H):
            raise ValueError("every partial must be [N, H]")
    P = len(parts)
    arr = (_u16p * max(P, 1))(*[_ptr(p, _u16p) for p in parts])
    ref_out = np.empty((N, H), dtype=np.float64)
    ref_res = np.empty((N, H), dtype=np.float64)
    args = [arr, _ptr(residual, _u16p), _ptr(weight, _u16p), ctypes.c_float(eps),
            N, H, P, _ptr(ref_out, _f64p), _ptr(ref_res, _f64p)]
    if nthreads is not None:
        args.append(int(nthreads))
    rc = getattr(lib, name)(*args)
    if rc != 0:
        raise RuntimeError("%s failed (rc=%d)" % (name, rc))
    return ref_out, ref_res


def fused(partials, residual, weight, eps):
    """Unrounded fp64 (out, residual_out) of the fused path; the oracle proper."""
    return _fused_call("tw_oracle_fused", partials, residual, weight, eps)


def fused_rounded_x(partials, residual, weight, eps):
    """Alternative reading: the bf16-rounded sum feeds the norm."""
    return _fused_call("tw_oracle_fused_rounded_x", partials, residual, weight, eps)


def unfused(partials, residual, weight, eps):
    """The three-pass pipeline (all-reduce to bf16 = the exact sum rounded once, residual add + sum of
    squares, scale from the stored bf16 residual stream). Returns (ref_out, ref_res) like fused()."""
    return _fused_call("tw_oracle_unfused", partials, residual, weight, eps)


def unfused_f32sum(partials, residual, weight, eps):
    """Second reading of the same pipeline: the all-reduce accumulates in binary32 in rank order
    before its one rounding to bf16."""
    return _fused_call("tw_oracle_unfused_f32sum", partials, residual, weight, eps)


def fused_mt(partials, residual, weight, eps, nthreads):
    """Row-parallel run of the same per-row code (for timing on all host cores)."""
    return _fused_call("tw_oracle_fused_mt", partials, residual, weight, eps, nthreads)


def _b_strides(B, K, N, b_layout):
    if b_layout == "kn":      # B stored [K, N] row-major
        if B.shape != (K, N):
            raise ValueError("B must be [K, N] for layout 'kn'")
        return N, 1
    if b_layout == "nk":      # B stored [N, K] row-major (a Linear layer's weight)
        if B.shape != (N, K):
            raise ValueError("B must be [N, K] for layout 'nk'")
        return 1, K
    raise ValueError("b_layout must be 'kn' or 'nk'")


def gemm(A, B, b_layout):
    """fp64 C[M, N] = A[M, K] * B(k, n); B's storage order named by b_layout."""
    lib = _load()
    A = _u16(A)
    B = _u16(B)
    M, K = A.shape
    N = B.shape[1] if b_layout == "kn" else B.shape[0]
    sk, sn = _b_strides(B, K, N, b_layout)
    C = np.empty((M, N), dtype=np.float64)
    rc = lib.tw_oracle_gemm(_ptr(A, _u16p), _ptr(B, _u16p), M, N, K, sk, sn, _ptr(C, _f64p))
    if rc != 0:
        raise RuntimeError("tw_oracle_gemm failed")
    return C


def gemm_samples(A, B, b_layout, ms, ns):
    """The same product evaluated at the listed (m, n) pairs only."""
    lib = _load()
    A = _u16(A)
    B = _u16(B)
    M, K = A.shape
    N = B.shape[1] if b_layout == "kn" else B.shape[0]
    sk, sn = _b_strides(B, K, N, b_layout)
    ms = np.ascontiguousarray(ms, dtype=np.int64)
    ns = np.ascontiguousarray(ns, dtype=np.int64)
    vals = np.empty(ms.shape[0], dtype=np.float64)
    rc = lib.tw_oracle_gemm_samples(_ptr(A, _u16p), _ptr(B, _u16p), M, N, K, sk, sn,
                                    _ptr(ms, _i64p), _ptr(ns, _i64p), ms.shape[0],
                                    _ptr(vals, _f64p))
    if rc != 0:
        raise RuntimeError("tw_oracle_gemm_samples failed")
    return vals


def bf16_to_f64(a):
    lib = _load()
    a = _u16(a)
    out = np.empty(a.shape, dtype=np.float64)
    lib.tw_oracle_bf16_to_f64_array(_ptr(a, _u16p), a.size, _ptr(out, _f64p))
    return out


def f64_to_bf16(a):
    lib = _load()
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty(a.shape, dtype=np.uint16)
    lib.tw_oracle_f64_to_bf16_array(_ptr(a, _f64p), a.size, _ptr(out, _u16p))
    return out
