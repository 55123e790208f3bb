"""CPU oracle for AMULET's matrix-multiplication-like tasks (test infrastructure).

This package is the slow, plain definition of what the GPU library computes:
the triple loop of the paper's Fig. 1 / Fig. 2 / "Test Queries" figure with a
single fp32-rounded product per (i, j, k), a strict fp32 comparison, and double
accumulation in increasing k.  The arithmetic lives in ``amulet_oracle.c``
(plain C, built with gcc); this module only marshals numpy arrays into it.

It shares no code with the HIP path and must never be imported by the product
package: only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

IDENTITY, DISCOUNT, BOOST, COUNT_GT = 0, 1, 2, 3
THRES_COL, THRES_ROW, THRES_CONST, THRES_ELEM = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "amulet_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile amulet_oracle.c into liboracle.so with gcc; returns the path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
             "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # AMULET_ORACLE_LIB: a build of amulet_oracle.c made elsewhere (the sanitizer test's)
        lib = ctypes.CDLL(os.environ.get("AMULET_ORACLE_LIB") or build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_mmlike_f32.restype = i32
        lib.oracle_mmlike_f32.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, vp, i64,
                                          vp, i32, ctypes.POINTER(i32)]
        lib.oracle_mmlike_f32_general.restype = i32
        lib.oracle_mmlike_f32_general.argtypes = [i32, i32, i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64,
                                                  vp, vp, i64, vp, i32, ctypes.POINTER(i32)]
        lib.oracle_mmlike_f64_general.restype = i32
        lib.oracle_mmlike_f64_general.argtypes = lib.oracle_mmlike_f32_general.argtypes
        lib.oracle_count_i8.restype = i32
        lib.oracle_count_i8.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32,
                                        ctypes.POINTER(i32)]
        _lib = lib
    return _lib


def _rowmajor(x: np.ndarray, dtype) -> np.ndarray:
    if x.ndim == 2 and x.size == 0 and x.dtype == dtype:
        return np.zeros((x.shape[0], max(x.shape[1], 1)), dtype)[:, :x.shape[1]]
    if x.dtype != dtype or x.ndim != 2:
        raise ValueError("oracle wants a 2-D %s array with unit column stride" % np.dtype(dtype).name)
    if x.shape[0] == 1 or x.shape[1] == 1:
        # numpy keeps arbitrary strides along axes of length 1: give such arrays the plain layout
        return np.array(x, dtype=dtype, order="C", copy=True).reshape(x.shape)
    if x.strides[1] != x.itemsize or x.strides[0] % x.itemsize:
        raise ValueError("oracle wants a 2-D %s array with unit column stride" % np.dtype(dtype).name)
    return x


def _n_params(task: int) -> int:
    return {IDENTITY: 0, DISCOUNT: 2, BOOST: 1, COUNT_GT: 1}[task]


def mmlike_f32(task: int, A: np.ndarray, B: np.ndarray, params, R_in=None, *, threads: int = 0,
               want_abs: bool = True):
    """R_in + sum_k g(fl32(A[i,k]*B[k,j]), params[:, j]) by the plain triple loop.

    A is M x K, B is K x N (fp32, rows may be strided views); ``params`` is an
    (n_param, N) fp32 array: rows (thres, dis) for DISCOUNT, (thres,) for BOOST
    and COUNT_GT, ignored for IDENTITY.  Returns (R, abs_sum, threads_used),
    with R fp32 M x N and abs_sum the double sum_k |term| (None if not wanted).
    """
    lib = _load()
    A = _rowmajor(A, np.float32)
    B = _rowmajor(B, np.float32)
    M, K = A.shape
    K2, N = B.shape
    if K2 != K:
        raise ValueError("inner dimensions differ")
    npar = _n_params(task)
    if npar:
        P = np.ascontiguousarray(np.asarray(params, dtype=np.float32).reshape(npar, N))
        pptr = P.ctypes.data
    else:
        pptr = None
    R = np.zeros((M, N), np.float32) if R_in is None else np.array(R_in, dtype=np.float32, order="C")
    if R.shape != (M, N):
        raise ValueError("R_in has the wrong shape")
    abs_sum = np.zeros((M, N), np.float64) if want_abs else None
    used = ctypes.c_int(0)
    rc = lib.oracle_mmlike_f32(task, M, N, K, A.ctypes.data, A.strides[0] // 4,
                               B.ctypes.data, B.strides[0] // 4, pptr, R.ctypes.data, N,
                               abs_sum.ctypes.data if want_abs else None, threads,
                               ctypes.byref(used))
    if rc != 0:
        raise ValueError("oracle_mmlike_f32 returned %d" % rc)
    return R, abs_sum, used.value


def mmlike_f64_general(task: int, A: np.ndarray, B: np.ndarray, thres=None, dis=None, R_in=None, *,
                       thres_form: int = THRES_COL, trans_a: bool = False, trans_b: bool = False,
                       threads: int = 0):
    """The general test-query form in the paper's own element type: fp64 operands, one fp64
    product per (i, j, k), strict fp64 comparison, long-double accumulation.
    Returns (R fp64, abs_sum fp64, threads_used)."""
    return _general(np.float64, "oracle_mmlike_f64_general", task, A, B, thres, dis, R_in, thres_form,
                    trans_a, trans_b, threads)


def mmlike_f32_general(task: int, A: np.ndarray, B: np.ndarray, thres=None, dis=None, R_in=None, *,
                       thres_form: int = THRES_COL, trans_a: bool = False, trans_b: bool = False,
                       threads: int = 0):
    """The general test-query form: operands optionally stored transposed (A as K x M,
    B as N x K) and the threshold operand as thres[j], thres[i], a constant or thres[i][j].
    Returns (R, abs_sum, threads_used)."""
    return _general(np.float32, "oracle_mmlike_f32_general", task, A, B, thres, dis, R_in, thres_form,
                    trans_a, trans_b, threads)


def _general(dtype, fn_name, task, A, B, thres, dis, R_in, thres_form, trans_a, trans_b, threads):
    lib = _load()
    es = np.dtype(dtype).itemsize
    A = _rowmajor(A, dtype)
    B = _rowmajor(B, dtype)
    M, K = (A.shape[1], A.shape[0]) if trans_a else A.shape
    K2, N = (B.shape[1], B.shape[0]) if trans_b else B.shape
    if K2 != K:
        raise ValueError("inner dimensions differ")
    tptr, ldt, T = None, 0, None
    if task != IDENTITY:
        want = {THRES_COL: (N,), THRES_ROW: (M,), THRES_CONST: (1,), THRES_ELEM: (M, N)}[thres_form]
        T = np.ascontiguousarray(np.asarray(thres, dtype=dtype).reshape(want))
        tptr, ldt = T.ctypes.data, (N if thres_form == THRES_ELEM else 0)
    D = None
    if task == DISCOUNT:
        D = np.ascontiguousarray(np.asarray(dis, dtype=dtype).reshape(N))
    R = np.zeros((M, N), dtype) if R_in is None else np.array(R_in, dtype=dtype, order="C")
    if R.shape != (M, N):
        raise ValueError("R_in has the wrong shape")
    abs_sum = np.zeros((M, N), np.float64)
    used = ctypes.c_int(0)
    rc = getattr(lib, fn_name)(task, thres_form, int(trans_a), int(trans_b), M, N, K,
                               A.ctypes.data, A.strides[0] // es, B.ctypes.data, B.strides[0] // es,
                               tptr, ldt, D.ctypes.data if D is not None else None,
                               R.ctypes.data, N, abs_sum.ctypes.data, threads, ctypes.byref(used))
    if rc != 0:
        raise ValueError("%s returned %d" % (fn_name, rc))
    return R, abs_sum, used.value


def count_i8(A: np.ndarray, B: np.ndarray, R_in=None, *, threads: int = 0):
    """R_in + A @ B for int8 A (M x K), B (K x N), exact in int32 (join count as matmul)."""
    lib = _load()
    A = _rowmajor(A, np.int8)
    B = _rowmajor(B, np.int8)
    M, K = A.shape
    K2, N = B.shape
    if K2 != K:
        raise ValueError("inner dimensions differ")
    R = np.zeros((M, N), np.int32) if R_in is None else np.array(R_in, dtype=np.int32, order="C")
    used = ctypes.c_int(0)
    rc = lib.oracle_count_i8(M, N, K, A.ctypes.data, A.strides[0], B.ctypes.data, B.strides[0],
                             R.ctypes.data, N, threads, ctypes.byref(used))
    if rc != 0:
        raise OverflowError("oracle_count_i8: a result left the int32 range")
    return R, used.value
