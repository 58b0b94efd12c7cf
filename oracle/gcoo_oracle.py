"""ctypes front end of the CPU oracle in gcoo_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's reported CPU baseline.  Nothing of the GPU library is imported here.
The C file is compiled with gcc on first use when no built library is present.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gcoo_oracle.c")
_LIB = os.path.join(_HERE, "libgcoo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gcoo_oracle.c into libgcoo_oracle.so (plain gcc, -O2, OpenMP).

    With GCOO_ORACLE_SANITIZE=1 in the environment the library is libgcoo_oracle_san.so instead, built with
    -O0 -g -fsanitize=address,undefined: a checking build for one pass of the CPU tests,
        GCOO_ORACLE_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
            UBSAN_OPTIONS=halt_on_error=1 python -m pytest tests -m "not gpu" -q
    (the address sanitizer's runtime has to be loaded before the interpreter's own libraries)."""
    sanitize = os.environ.get("GCOO_ORACLE_SANITIZE", "") == "1"
    out = os.path.join(_HERE, "libgcoo_oracle_san.so") if sanitize else _LIB
    flags = ["-O0", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        tmp = out + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, out)
    return out


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        i64, i32, f64 = C.c_int64, C.c_int32, C.c_double
        vp = C.c_void_p
        L = _lib
        L.oracle_group_count.restype = i64
        L.oracle_group_count.argtypes = [i64, i64]
        L.oracle_last_group_width.restype = i64
        L.oracle_last_group_width.argtypes = [i64, i64]
        L.oracle_gcoo_footprint_elems.restype = i64
        L.oracle_gcoo_footprint_elems.argtypes = [i64, i64, i64]
        L.oracle_num_threads.restype = C.c_int
        L.oracle_coo_from_dense.restype = i64
        L.oracle_coo_from_dense.argtypes = [i64, i64, vp, i64, vp, vp, vp]
        L.oracle_gcoo_from_csr.restype = C.c_int
        L.oracle_gcoo_from_csr.argtypes = [i64, i64, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        L.oracle_gcoo_count_dense.restype = i64
        L.oracle_gcoo_count_dense.argtypes = [i64, i64, vp, i64, i32, vp, vp]
        L.oracle_gcoo_fill_dense.restype = None
        L.oracle_gcoo_fill_dense.argtypes = [i64, i64, vp, i64, i32, vp, vp, vp, vp]
        L.oracle_spdm_csr.restype = None
        L.oracle_spdm_csr.argtypes = [i64, i64, vp, vp, vp, vp, i64, i64, i64, vp, vp]
        L.oracle_spdm_gcoo.restype = None
        L.oracle_spdm_gcoo.argtypes = [i64, i64, i64, vp, vp, vp, vp, i64, vp]
        L.oracle_dense_gemm.restype = None
        L.oracle_dense_gemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp]
        L.oracle_count_runs.restype = i64
        L.oracle_count_runs.argtypes = [i64, vp, vp]
        L.oracle_max_scaled_error.restype = f64
        L.oracle_max_scaled_error.argtypes = [i64, i64, vp, i64, vp, vp, vp]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _as(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


class Gcoo:
    """The five arrays of the format (gIdxes carries one extra sentinel entry)."""

    def __init__(self, m, k, p, values, rows, cols, gIdxes, nnzPerGroup):
        self.m, self.k, self.p = m, k, p
        self.values, self.rows, self.cols = values, rows, cols
        self.gIdxes, self.nnzPerGroup = gIdxes, nnzPerGroup

    @property
    def nnz(self):
        return int(self.values.shape[0])

    @property
    def g(self):
        return int(self.nnzPerGroup.shape[0])


def group_count(n, p):
    return int(lib().oracle_group_count(n, p))


def last_group_width(n, p):
    return int(lib().oracle_last_group_width(n, p))


def footprint_elems(n, p, nnz):
    return int(lib().oracle_gcoo_footprint_elems(n, p, nnz))


def num_threads():
    return int(lib().oracle_num_threads())


def coo_from_dense(A):
    A = _as(A, np.float32)
    m, k = A.shape
    nnz = lib().oracle_coo_from_dense(m, k, _p(A), k, None, None, None)
    v = np.empty(nnz, np.float32)
    r = np.empty(nnz, np.int32)
    c = np.empty(nnz, np.int32)
    lib().oracle_coo_from_dense(m, k, _p(A), k, _p(v), _p(r), _p(c))
    return v, r, c


def gcoo_from_csr(m, k, row_ptr, col_idx, vals, p) -> Gcoo:
    row_ptr = _as(row_ptr, np.int32)
    col_idx = _as(col_idx, np.int32)
    vals = _as(vals, np.float32)
    nnz = int(row_ptr[m]) if m > 0 else 0
    g = group_count(m, p)
    v = np.empty(nnz, np.float32)
    r = np.empty(nnz, np.int32)
    c = np.empty(nnz, np.int32)
    gi = np.empty(g + 1, np.int32)
    npg = np.empty(g, np.int32)
    rc = lib().oracle_gcoo_from_csr(m, k, _p(row_ptr), _p(col_idx), _p(vals), p,
                                    _p(v), _p(r), _p(c), _p(gi), _p(npg))
    if rc != 0:
        raise ValueError("oracle_gcoo_from_csr: malformed input")
    return Gcoo(m, k, p, v, r, c, gi, npg)


def gcoo_from_dense(A, p) -> Gcoo:
    A = _as(A, np.float32)
    m, k = A.shape
    g = group_count(m, p)
    gi = np.empty(g + 1, np.int32)
    npg = np.empty(g, np.int32)
    nnz = lib().oracle_gcoo_count_dense(m, k, _p(A), k, p, _p(gi), _p(npg))
    v = np.empty(nnz, np.float32)
    r = np.empty(nnz, np.int32)
    c = np.empty(nnz, np.int32)
    lib().oracle_gcoo_fill_dense(m, k, _p(A), k, p, _p(gi), _p(v), _p(r), _p(c))
    return Gcoo(m, k, p, v, r, c, gi, npg)


def spdm_csr(k, N, row_ptr, col_idx, vals, B, r0=0, r1=None, want_scale=True):
    """Rows [r0, r1) of C in fp64 and, optionally, of the scale |A|.|B|."""
    row_ptr = _as(row_ptr, np.int32)
    col_idx = _as(col_idx, np.int32)
    vals = _as(vals, np.float32)
    B = _as(B, np.float32)
    m = row_ptr.shape[0] - 1
    if r1 is None:
        r1 = m
    ldb = B.shape[1] if B.ndim == 2 else N
    C64 = np.empty((r1 - r0, N), np.float64)
    D64 = np.empty((r1 - r0, N), np.float64) if want_scale else None
    lib().oracle_spdm_csr(k, N, _p(row_ptr), _p(col_idx), _p(vals), _p(B), ldb, r0, r1, _p(C64), _p(D64))
    return C64, D64


def spdm_gcoo(G: Gcoo, B, N):
    B = _as(B, np.float32)
    C64 = np.empty((G.m, N), np.float64)
    lib().oracle_spdm_gcoo(G.m, N, G.nnz, _p(G.values), _p(G.rows), _p(G.cols), _p(B), B.shape[1], _p(C64))
    return C64


def dense_gemm(A, B):
    A = _as(A, np.float32)
    B = _as(B, np.float32)
    m, k = A.shape
    N = B.shape[1]
    C64 = np.empty((m, N), np.float64)
    lib().oracle_dense_gemm(m, k, N, _p(A), k, _p(B), N, _p(C64))
    return C64


def count_runs(G: Gcoo):
    return int(lib().oracle_count_runs(G.g, _p(G.gIdxes), _p(G.cols)))


def max_scaled_error(Cf32, C64, D64):
    """(max |C - C64| / D64 over D64 > 0, number of NaNs or nonzeros where D64 == 0)."""
    Cf32 = _as(Cf32, np.float32)
    rows, N = C64.shape
    bad = C.c_int64(0)
    e = lib().oracle_max_scaled_error(rows, N, _p(Cf32), Cf32.shape[1], _p(C64), _p(D64), C.byref(bad))
    return float(e), int(bad.value)
