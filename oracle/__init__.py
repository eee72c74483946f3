"""CPU oracle for the packed structured contractions -- TEST INFRASTRUCTURE ONLY.

This package wraps ``dastac_oracle.c`` (plain C, double-precision accumulation,
packed positions obtained by walking the iteration domain with a running
counter; see the header of that file for the passages of the paper it
follows).  It shares no code with the GPU library.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the GPU library and
its Python binding never do.

All arrays are host NumPy arrays.  ``build()`` compiles the C file with gcc.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dastac_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

DOM_TRIU, DOM_TRIL, DOM_TET, DOM_UHC, DOM_BAND = 0, 1, 2, 3, 4

_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, no fast-math: the loop order is the definition)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        L.oracle_count_preceding.restype = _i64
        L.oracle_count_preceding.argtypes = [ctypes.c_int, _ip, _ip]
        L.oracle_count_domain.restype = _i64
        L.oracle_count_domain.argtypes = [ctypes.c_int, _ip]
        L.oracle_point_at.restype = ctypes.c_int
        L.oracle_point_at.argtypes = [ctypes.c_int, _ip, _i64, _ip]
        L.oracle_triu_row_starts.restype = None
        L.oracle_triu_row_starts.argtypes = [_i64, _ip]
        L.oracle_tet_fibre_starts.restype = _i64
        L.oracle_tet_fibre_starts.argtypes = [_i64, _ip]
        L.oracle_triu_position.restype = _i64
        L.oracle_triu_position.argtypes = [_i64, _i64, _i64]
        L.oracle_tet_position.restype = _i64
        L.oracle_tet_position.argtypes = [_i64, _i64, _i64, _i64]
        L.oracle_triu_point_at.restype = ctypes.c_int
        L.oracle_triu_point_at.argtypes = [_i64, _i64, _ip, _ip]
        L.oracle_tet_point_at.restype = ctypes.c_int
        L.oracle_tet_point_at.argtypes = [_i64, _i64, _ip, _ip, _ip]
        L.oracle_pack_triu_f32.argtypes = [_i64, _fp, _i64, _fp]
        L.oracle_unpack_triu_f32.argtypes = [_i64, _fp, _fp, _i64]
        L.oracle_pack_tet_f32.argtypes = [_i64, _fp, _fp]
        L.oracle_unpack_tet_f32.argtypes = [_i64, _fp, _fp]
        L.oracle_pack_band_f32.argtypes = [_i64, _i64, _fp, _i64, _fp]
        L.oracle_unpack_band_f32.argtypes = [_i64, _i64, _fp, _fp, _i64]
        L.oracle_trmv_f32.argtypes = [_i64, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_trmm_f32.argtypes = [_i64, _i64, _fp, _fp, _i64, _fp, _i64, _dp, _i64, _i64]
        L.oracle_band_spmv_f32.argtypes = [_i64, _i64, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_tet_ttv_f32.argtypes = [_i64, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_tet_mttkrp_f32.argtypes = [_i64, _i64, _fp, _fp, _i64, _fp, _i64, _fp, _i64, _dp, _i64, _i64]
        L.oracle_pack_uhc_f32.argtypes = [_i64, _i64, _i64, _fp, _fp]
        L.oracle_unpack_uhc_f32.argtypes = [_i64, _i64, _i64, _fp, _fp]
        L.oracle_trimv_f32.argtypes = [_i64, ctypes.c_int, ctypes.c_int, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_pack_tril_f32.argtypes = [_i64, _fp, _i64, _fp]
        L.oracle_unpack_tril_f32.argtypes = [_i64, _fp, _fp, _i64]
        L.oracle_ttm_ut_f32.argtypes = [_i64, _i64, _i64, _fp, _fp, _i64, _fp, _dp, _i64, _i64]
        L.oracle_pack_triu_f64.argtypes = [_i64, _dp, _i64, _dp]
        L.oracle_unpack_triu_f64.argtypes = [_i64, _dp, _dp, _i64]
        L.oracle_pack_tet_f64.argtypes = [_i64, _dp, _dp]
        L.oracle_unpack_tet_f64.argtypes = [_i64, _dp, _dp]
        L.oracle_pack_band_f64.argtypes = [_i64, _i64, _dp, _i64, _dp]
        L.oracle_unpack_band_f64.argtypes = [_i64, _i64, _dp, _dp, _i64]
        L.oracle_trmv_f64.argtypes = [_i64, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_band_spmv_f64.argtypes = [_i64, _i64, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_tet_ttv_f64.argtypes = [_i64, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_pack_uhc_f64.argtypes = [_i64, _i64, _i64, _dp, _dp]
        L.oracle_unpack_uhc_f64.argtypes = [_i64, _i64, _i64, _dp, _dp]
        L.oracle_ttm_ut_f64.argtypes = [_i64, _i64, _i64, _dp, _dp, _i64, _dp, _dp, _i64, _i64]
        L.oracle_pr_a2_f64.argtypes = [_i64, _i64, _dp, _i64, _dp, _dp, _i64, _i64]
        L.oracle_pr_a3_f64.argtypes = [_i64, _i64, _dp, _i64, _dp, _dp, _i64, _i64]
        L.oracle_tet_mttkrp_f64.argtypes = [_i64, _i64, _dp, _dp, _i64, _dp, _i64, _dp, _i64, _dp, _i64, _i64]
        L.oracle_symm_f64.argtypes = [_i64, _i64, _dp, _dp, _i64, _dp, _i64, _dp, _i64, _i64]
        L.oracle_trmm_f64.argtypes = [_i64, _i64, _dp, _dp, _i64, _dp, _i64, _dp, _i64, _i64]
        L.oracle_pr_a2_f32.argtypes = [_i64, _i64, _fp, _i64, _fp, _dp, _i64, _i64]
        L.oracle_pr_a3_f32.argtypes = [_i64, _i64, _fp, _i64, _fp, _dp, _i64, _i64]
        L.oracle_symm_f32.argtypes = [_i64, _i64, _fp, _fp, _i64, _fp, _i64, _dp, _i64, _i64]
        L.oracle_pack_sband_f32.argtypes = [_i64, _i64, _i64, _fp, _i64, _fp]
        L.oracle_unpack_sband_f32.argtypes = [_i64, _i64, _i64, _fp, _fp, _i64]
        L.oracle_sband_spmv_f32.argtypes = [_i64, _i64, _i64, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_pack_subtri_f32.argtypes = [_i64, _i64, _fp, _i64, _fp]
        L.oracle_unpack_subtri_f32.argtypes = [_i64, _i64, _fp, _fp, _i64]
        L.oracle_subtri_spmv_f32.argtypes = [_i64, _i64, _fp, _fp, _fp, _dp, _i64, _i64]
        L.oracle_pack_leslie_f32.argtypes = [_i64, _fp, _i64, _fp, _fp]
        L.oracle_unpack_leslie_f32.argtypes = [_i64, _fp, _fp, _fp, _i64]
        L.oracle_leslie_spmv_f32.argtypes = [_i64, _fp, _fp, _fp, _fp, _dp]
        L.oracle_trimv_f64.argtypes = [_i64, ctypes.c_int, ctypes.c_int, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_pack_tril_f64.argtypes = [_i64, _dp, _i64, _dp]
        L.oracle_unpack_tril_f64.argtypes = [_i64, _dp, _dp, _i64]
        L.oracle_pack_sband_f64.argtypes = [_i64, _i64, _i64, _dp, _i64, _dp]
        L.oracle_unpack_sband_f64.argtypes = [_i64, _i64, _i64, _dp, _dp, _i64]
        L.oracle_sband_spmv_f64.argtypes = [_i64, _i64, _i64, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_pack_subtri_f64.argtypes = [_i64, _i64, _dp, _i64, _dp]
        L.oracle_unpack_subtri_f64.argtypes = [_i64, _i64, _dp, _dp, _i64]
        L.oracle_subtri_spmv_f64.argtypes = [_i64, _i64, _dp, _dp, _dp, _dp, _i64, _i64]
        L.oracle_pack_leslie_f64.argtypes = [_i64, _dp, _i64, _dp, _dp]
        L.oracle_unpack_leslie_f64.argtypes = [_i64, _dp, _dp, _dp, _i64]
        L.oracle_leslie_spmv_f64.argtypes = [_i64, _dp, _dp, _dp, _dp, _dp]
        for name in ("pack_triu", "unpack_triu", "pack_tet", "unpack_tet", "pack_band", "unpack_band",
                     "trmv", "trmm", "band_spmv", "tet_ttv", "tet_mttkrp"):
            getattr(L, "oracle_%s_f32" % name).restype = None
        _lib = L
    return _lib


def _f(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_fp)


def _d(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def _i(a: np.ndarray):
    assert a.dtype == np.int64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_ip)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# ---- counting definition -----------------------------------------------------

def count_preceding(dom: int, params, idx) -> int:
    p = np.asarray(list(params) + [0, 0, 0], dtype=np.int64)
    x = np.asarray(list(idx) + [0, 0, 0], dtype=np.int64)
    return int(lib().oracle_count_preceding(dom, _i(p), _i(x)))


def count_domain(dom: int, params) -> int:
    p = np.asarray(list(params) + [0, 0, 0], dtype=np.int64)
    return int(lib().oracle_count_domain(dom, _i(p)))


def point_at(dom: int, params, p: int):
    prm = np.asarray(list(params) + [0, 0, 0], dtype=np.int64)
    out = np.zeros(3, dtype=np.int64)
    rc = lib().oracle_point_at(dom, _i(prm), int(p), _i(out))
    if rc != 0:
        return None
    rank = 3 if dom in (DOM_TET, DOM_UHC) else 2
    return tuple(int(t) for t in out[:rank])


def triu_row_starts(n: int) -> np.ndarray:
    s = np.zeros(n + 1, dtype=np.int64)
    lib().oracle_triu_row_starts(n, _i(s))
    return s


def tet_fibre_starts(n: int):
    s = np.zeros(n * n, dtype=np.int64) if n > 0 else np.zeros(1, dtype=np.int64)
    total = int(lib().oracle_tet_fibre_starts(n, _i(s)))
    return s[: n * n].reshape(n, n), total


def triu_position(n, i, j) -> int:
    return int(lib().oracle_triu_position(n, i, j))


def tet_position(n, i, j, k) -> int:
    return int(lib().oracle_tet_position(n, i, j, k))


def triu_point_at(n, p):
    i, j = _i64(), _i64()
    rc = lib().oracle_triu_point_at(n, int(p), ctypes.byref(i), ctypes.byref(j))
    return None if rc else (i.value, j.value)


def tet_point_at(n, p):
    i, j, k = _i64(), _i64(), _i64()
    rc = lib().oracle_tet_point_at(n, int(p), ctypes.byref(i), ctypes.byref(j), ctypes.byref(k))
    return None if rc else (i.value, j.value, k.value)


# ---- compression / decompression --------------------------------------------

def pack_triu(dense: np.ndarray) -> np.ndarray:
    dense = _f32(dense)
    n = dense.shape[0]
    out = np.empty(int(triu_row_starts(n)[n]), dtype=np.float32)
    lib().oracle_pack_triu_f32(n, _f(dense), dense.shape[1], _f(out))
    return out


def unpack_triu(n: int, packed: np.ndarray) -> np.ndarray:
    packed = _f32(packed)
    out = np.full((n, n), np.nan, dtype=np.float32)
    lib().oracle_unpack_triu_f32(n, _f(packed), _f(out), n)
    return out


def pack_tet(dense: np.ndarray) -> np.ndarray:
    dense = _f32(dense)
    n = dense.shape[0]
    _, total = tet_fibre_starts(n)
    out = np.empty(total, dtype=np.float32)
    lib().oracle_pack_tet_f32(n, _f(dense), _f(out))
    return out


def unpack_tet(n: int, packed: np.ndarray) -> np.ndarray:
    packed = _f32(packed)
    out = np.full((n, n, n), np.nan, dtype=np.float32)
    lib().oracle_unpack_tet_f32(n, _f(packed), _f(out))
    return out


def pack_band(dense: np.ndarray, w: int) -> np.ndarray:
    dense = _f32(dense)
    n = dense.shape[0]
    out = np.empty((2 * w + 1) * n, dtype=np.float32)
    lib().oracle_pack_band_f32(n, w, _f(dense), dense.shape[1], _f(out))
    return out


def unpack_band(n: int, w: int, diag: np.ndarray) -> np.ndarray:
    diag = _f32(diag)
    out = np.full((n, n), np.nan, dtype=np.float32)
    lib().oracle_unpack_band_f32(n, w, _f(diag), _f(out), n)
    return out


# ---- contractions: return (result fp32, scale fp64); rows outside the window are NaN ----

def _window(n, rows):
    return (0, n) if rows is None else (int(rows[0]), int(rows[1]))


def trmv(n, Up, x, rows=None):
    Up, x = _f32(Up), _f32(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float32)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_trmv_f32(n, _f(Up), _f(x), _f(y), _d(sc), lo, hi)
    return y, sc


def trmm(n, m, Up, B, rows=None):
    Up, B = _f32(Up), _f32(B)
    lo, hi = _window(n, rows)
    C = np.full((n, m), np.nan, dtype=np.float32)
    sc = np.full((n, m), np.nan, dtype=np.float64)
    lib().oracle_trmm_f32(n, m, _f(Up), _f(B), B.shape[1] if B.ndim == 2 else m, _f(C), m, _d(sc), lo, hi)
    return C, sc


def band_spmv(n, w, D, x, rows=None):
    D, x = _f32(D), _f32(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float32)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_band_spmv_f32(n, w, _f(D), _f(x), _f(y), _d(sc), lo, hi)
    return y, sc


def tet_ttv(n, Ap, v, rows=None):
    Ap, v = _f32(Ap), _f32(v)
    lo, hi = _window(n, rows)
    cnt = int(triu_row_starts(n)[n])
    M = np.full(cnt, np.nan, dtype=np.float32)
    sc = np.full(cnt, np.nan, dtype=np.float64)
    lib().oracle_tet_ttv_f32(n, _f(Ap), _f(v), _f(M), _d(sc), lo, hi)
    return M, sc


def tet_mttkrp(n, R, Ap, B, C, rows=None):
    Ap, B, C = _f32(Ap), _f32(B), _f32(C)
    lo, hi = _window(n, rows)
    M = np.full((n, R), np.nan, dtype=np.float32)
    sc = np.full((n, R), np.nan, dtype=np.float64)
    lib().oracle_tet_mttkrp_f32(n, R, _f(Ap), _f(B), B.shape[1], _f(C), C.shape[1], _f(M), R, _d(sc), lo, hi)
    return M, sc


def pack_uhc(dense: np.ndarray) -> np.ndarray:
    """dense is M x N x Q; returns the points with i<=j in iteration order (i,j,l)."""
    dense = _f32(dense)
    M, N, Q = dense.shape
    cnt = sum(N - i for i in range(min(M, N))) * Q
    packed = np.empty(cnt, dtype=np.float32)
    lib().oracle_pack_uhc_f32(M, N, Q, _f(dense), _f(packed))
    return packed


def unpack_uhc(M: int, N: int, Q: int, packed: np.ndarray) -> np.ndarray:
    packed = _f32(packed)
    dense = np.empty((M, N, Q), dtype=np.float32)
    lib().oracle_unpack_uhc_f32(M, N, Q, _f(packed), _f(dense))
    return dense


def ttm_ut(n, Q, K, Bp, C, rows=None):
    """A(i,j,k) := B(i,j,l)*C(k,l), i<=j; packed in, packed out.  `rows` windows the (i,j) pairs."""
    Bp, C = _f32(Bp), _f32(C)
    pairs = int(triu_row_starts(n)[n])
    lo, hi = (0, pairs) if rows is None else (int(rows[0]), int(rows[1]))
    A = np.full(pairs * K, np.nan, dtype=np.float32)
    sc = np.full(pairs * K, np.nan, dtype=np.float64)
    lib().oracle_ttm_ut_f32(n, Q, K, _f(Bp), _f(C), C.shape[1] if C.ndim == 2 else Q, _f(A), _d(sc), lo, hi)
    return A, sc


def trimv(n, Tp, x, lower=False, mode=0, rows=None):
    """mode 0: T x; 1: T^T x; 2: S x with S symmetric and T its unique triangle (upper, or lower)."""
    Tp, x = _f32(Tp), _f32(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float32)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_trimv_f32(n, int(bool(lower)), int(mode), _f(Tp), _f(x), _f(y), _d(sc), lo, hi)
    return y, sc


def symv(n, Up, x, rows=None):
    """y = S x, S symmetric with its upper triangle packed in Up."""
    return trimv(n, Up, x, lower=False, mode=2, rows=rows)


def pack_tril(dense: np.ndarray) -> np.ndarray:
    dense = _f32(dense)
    n = dense.shape[0]
    packed = np.empty(n * (n + 1) // 2, dtype=np.float32)
    lib().oracle_pack_tril_f32(n, _f(dense), dense.shape[1], _f(packed))
    return packed


def unpack_tril(n: int, packed: np.ndarray) -> np.ndarray:
    packed = _f32(packed)
    dense = np.empty((n, n), dtype=np.float32)
    lib().oracle_unpack_tril_f32(n, _f(packed), _f(dense), n)
    return dense


# ---- further domains (Section 6.4, Table 2 SpMV_L) ---------------------------

def pack_sband(dense: np.ndarray, w: int, s: int) -> np.ndarray:
    dense = _f32(dense)
    n = dense.shape[0]
    out = np.empty((2 * w + 1) * n, dtype=np.float32)
    lib().oracle_pack_sband_f32(n, w, s, _f(dense), dense.shape[1], _f(out))
    return out


def unpack_sband(n: int, w: int, s: int, diag: np.ndarray) -> np.ndarray:
    diag = _f32(diag)
    out = np.empty((n, n), dtype=np.float32)
    lib().oracle_unpack_sband_f32(n, w, s, _f(diag), _f(out), n)
    return out


def sband_spmv(n, w, s, D, x, rows=None):
    D, x = _f32(D), _f32(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float32)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_sband_spmv_f32(n, w, s, _f(D), _f(x), _f(y), _d(sc), lo, hi)
    return y, sc


def pack_subtri(dense: np.ndarray, k: int) -> np.ndarray:
    dense = _f32(dense)
    N = dense.shape[0]
    out = np.empty(k * (k + 1) // 2, dtype=np.float32)
    lib().oracle_pack_subtri_f32(N, k, _f(dense), dense.shape[1], _f(out))
    return out


def unpack_subtri(N: int, k: int, packed: np.ndarray) -> np.ndarray:
    packed = _f32(packed)
    out = np.empty((N, N), dtype=np.float32)
    lib().oracle_unpack_subtri_f32(N, k, _f(packed), _f(out), N)
    return out


def subtri_spmv(N, k, Ap, x, rows=None):
    Ap, x = _f32(Ap), _f32(x)
    lo, hi = _window(N, rows)
    y = np.full(N, np.nan, dtype=np.float32)
    sc = np.full(N, np.nan, dtype=np.float64)
    lib().oracle_subtri_spmv_f32(N, k, _f(Ap), _f(x), _f(y), _d(sc), lo, hi)
    return y, sc


def pack_leslie(dense: np.ndarray):
    dense = _f32(dense)
    n = dense.shape[0]
    R = np.empty(n, dtype=np.float32)
    S = np.empty(max(n - 1, 0), dtype=np.float32)
    lib().oracle_pack_leslie_f32(n, _f(dense), dense.shape[1], _f(R), _f(S))
    return R, S


def unpack_leslie(n: int, R: np.ndarray, S: np.ndarray) -> np.ndarray:
    R, S = _f32(R), _f32(S)
    out = np.empty((n, n), dtype=np.float32)
    lib().oracle_unpack_leslie_f32(n, _f(R), _f(S), _f(out), n)
    return out


def leslie_spmv(n, R, S, x):
    R, S, x = _f32(R), _f32(S), _f32(x)
    y = np.full(n, np.nan, dtype=np.float32)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_leslie_spmv_f32(n, _f(R), _f(S), _f(x), _f(y), _d(sc))
    return y, sc


def symm(n, m, Up, B, rows=None):
    """C = S B, S symmetric with its upper triangle packed in Up; B is n x m."""
    Up, B = _f32(Up), _f32(B)
    lo, hi = _window(n, rows)
    C = np.full((n, m), np.nan, dtype=np.float32)
    sc = np.full((n, m), np.nan, dtype=np.float64)
    lib().oracle_symm_f32(n, m, _f(Up), _f(B), B.shape[1] if B.ndim == 2 else m, _f(C), m, _d(sc), lo, hi)
    return C, sc


def _shifted(a: np.ndarray, ptr_type, lo: int):
    """Pointer to where element 0 of the full array would be when `a` holds its elements lo.. only (the C
    functions touch nothing outside the window they are given)."""
    return ctypes.cast(a.ctypes.data - lo * a.itemsize, ptr_type)


def _pr(fn, count, B, window, compact=False):
    B = _f32(B)
    N, d = B.shape
    lo, hi = (0, count) if window is None else (int(window[0]), int(window[1]))
    assert 0 <= lo <= hi <= count
    if compact:  # only the window is allocated and returned (the full tensor may not fit in host memory)
        out = np.full(hi - lo, np.nan, dtype=np.float32)
        sc = np.full(hi - lo, np.nan, dtype=np.float64)
        fn(N, d, _f(B), d, _shifted(out, _fp, lo), _shifted(sc, _dp, lo), lo, hi)
        return out, sc
    out = np.full(count, np.nan, dtype=np.float32)
    sc = np.full(count, np.nan, dtype=np.float64)
    fn(N, d, _f(B), d, _f(out), _d(sc), lo, hi)
    return out, sc


def pr_a2(B, window=None, compact=False):
    """A2(i,j) = sum_x B(x,i) B(x,j), i<=j, packed; `window` selects packed positions [lo, hi) (with
    `compact` only those are returned)."""
    d = B.shape[1]
    return _pr(lib().oracle_pr_a2_f32, d * (d + 1) // 2, B, window, compact)


def pr_a3(B, window=None, compact=False):
    """A3(i,j,k) = sum_x B(x,i) B(x,j) B(x,k), i<=j<=k, packed."""
    d = B.shape[1]
    return _pr(lib().oracle_pr_a3_f32, d * (d + 1) * (d + 2) // 6, B, window, compact)


# ---- double precision ---------------------------------------------------------

def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def pack_triu_f64(dense):
    dense = _f64(dense)
    n = dense.shape[0]
    out = np.empty(n * (n + 1) // 2, dtype=np.float64)
    lib().oracle_pack_triu_f64(n, _d(dense), dense.shape[1], _d(out))
    return out


def unpack_triu_f64(n, packed):
    packed = _f64(packed)
    out = np.empty((n, n), dtype=np.float64)
    lib().oracle_unpack_triu_f64(n, _d(packed), _d(out), n)
    return out


def pack_tet_f64(dense):
    dense = _f64(dense)
    n = dense.shape[0]
    out = np.empty(n * (n + 1) * (n + 2) // 6, dtype=np.float64)
    lib().oracle_pack_tet_f64(n, _d(dense), _d(out))
    return out


def unpack_tet_f64(n, packed):
    packed = _f64(packed)
    out = np.empty((n, n, n), dtype=np.float64)
    lib().oracle_unpack_tet_f64(n, _d(packed), _d(out))
    return out


def pack_band_f64(dense, w):
    dense = _f64(dense)
    n = dense.shape[0]
    out = np.empty((2 * w + 1) * n, dtype=np.float64)
    lib().oracle_pack_band_f64(n, w, _d(dense), dense.shape[1], _d(out))
    return out


def unpack_band_f64(n, w, diag):
    diag = _f64(diag)
    out = np.empty((n, n), dtype=np.float64)
    lib().oracle_unpack_band_f64(n, w, _d(diag), _d(out), n)
    return out


def trmv_f64(n, Up, x, rows=None):
    Up, x = _f64(Up), _f64(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float64)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_trmv_f64(n, _d(Up), _d(x), _d(y), _d(sc), lo, hi)
    return y, sc


def band_spmv_f64(n, w, D, x, rows=None):
    D, x = _f64(D), _f64(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float64)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_band_spmv_f64(n, w, _d(D), _d(x), _d(y), _d(sc), lo, hi)
    return y, sc


def tet_ttv_f64(n, Ap, v, rows=None):
    Ap, v = _f64(Ap), _f64(v)
    lo, hi = _window(n, rows)
    cnt = n * (n + 1) // 2
    M = np.full(cnt, np.nan, dtype=np.float64)
    sc = np.full(cnt, np.nan, dtype=np.float64)
    lib().oracle_tet_ttv_f64(n, _d(Ap), _d(v), _d(M), _d(sc), lo, hi)
    return M, sc


def trmm_f64(n, m, Up, B, rows=None):
    Up, B = _f64(Up), _f64(B)
    lo, hi = _window(n, rows)
    C = np.full((n, m), np.nan, dtype=np.float64)
    sc = np.full((n, m), np.nan, dtype=np.float64)
    lib().oracle_trmm_f64(n, m, _d(Up), _d(B), B.shape[1] if B.ndim == 2 else m, _d(C), m, _d(sc), lo, hi)
    return C, sc


def symm_f64(n, m, Up, B, rows=None):
    Up, B = _f64(Up), _f64(B)
    lo, hi = _window(n, rows)
    C = np.full((n, m), np.nan, dtype=np.float64)
    sc = np.full((n, m), np.nan, dtype=np.float64)
    lib().oracle_symm_f64(n, m, _d(Up), _d(B), B.shape[1] if B.ndim == 2 else m, _d(C), m, _d(sc), lo, hi)
    return C, sc


def pack_uhc_f64(dense):
    dense = _f64(dense)
    M, N, Q = dense.shape
    packed = np.empty(sum(N - i for i in range(min(M, N))) * Q, dtype=np.float64)
    lib().oracle_pack_uhc_f64(M, N, Q, _d(dense), _d(packed))
    return packed


def unpack_uhc_f64(M, N, Q, packed):
    packed = _f64(packed)
    dense = np.empty((M, N, Q), dtype=np.float64)
    lib().oracle_unpack_uhc_f64(M, N, Q, _d(packed), _d(dense))
    return dense


def ttm_ut_f64(n, Q, K, Bp, C, rows=None):
    Bp, C = _f64(Bp), _f64(C)
    pairs = n * (n + 1) // 2
    lo, hi = (0, pairs) if rows is None else (int(rows[0]), int(rows[1]))
    A = np.full(pairs * K, np.nan, dtype=np.float64)
    sc = np.full(pairs * K, np.nan, dtype=np.float64)
    lib().oracle_ttm_ut_f64(n, Q, K, _d(Bp), _d(C), C.shape[1] if C.ndim == 2 else Q, _d(A), _d(sc), lo, hi)
    return A, sc


def _pr64(fn, count, B, window, compact=False):
    B = _f64(B)
    N, d = B.shape
    lo, hi = (0, count) if window is None else (int(window[0]), int(window[1]))
    assert 0 <= lo <= hi <= count
    if compact:
        out = np.full(hi - lo, np.nan, dtype=np.float64)
        sc = np.full(hi - lo, np.nan, dtype=np.float64)
        fn(N, d, _d(B), d, _shifted(out, _dp, lo), _shifted(sc, _dp, lo), lo, hi)
        return out, sc
    out = np.full(count, np.nan, dtype=np.float64)
    sc = np.full(count, np.nan, dtype=np.float64)
    fn(N, d, _d(B), d, _d(out), _d(sc), lo, hi)
    return out, sc


def pr_a2_f64(B, window=None, compact=False):
    d = B.shape[1]
    return _pr64(lib().oracle_pr_a2_f64, d * (d + 1) // 2, B, window, compact)


def pr_a3_f64(B, window=None, compact=False):
    d = B.shape[1]
    return _pr64(lib().oracle_pr_a3_f64, d * (d + 1) * (d + 2) // 6, B, window, compact)


def tet_mttkrp_f64(n, R, Ap, B, C, rows=None):
    Ap, B, C = _f64(Ap), _f64(B), _f64(C)
    lo, hi = _window(n, rows)
    M = np.full((n, R), np.nan, dtype=np.float64)
    sc = np.full((n, R), np.nan, dtype=np.float64)
    lib().oracle_tet_mttkrp_f64(n, R, _d(Ap), _d(B), B.shape[1], _d(C), C.shape[1], _d(M), R, _d(sc), lo, hi)
    return M, sc


def trimv_f64(n, Tp, x, lower=False, mode=0, rows=None):
    """mode 0: T x; 1: T^T x; 2: S x with S symmetric and T its unique triangle (upper, or lower)."""
    Tp, x = _f64(Tp), _f64(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float64)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_trimv_f64(n, int(bool(lower)), int(mode), _d(Tp), _d(x), _d(y), _d(sc), lo, hi)
    return y, sc


def pack_tril_f64(dense):
    dense = _f64(dense)
    n = dense.shape[0]
    out = np.empty(n * (n + 1) // 2, dtype=np.float64)
    lib().oracle_pack_tril_f64(n, _d(dense), dense.shape[1], _d(out))
    return out


def unpack_tril_f64(n, packed):
    packed = _f64(packed)
    out = np.empty((n, n), dtype=np.float64)
    lib().oracle_unpack_tril_f64(n, _d(packed), _d(out), n)
    return out


def pack_sband_f64(dense, w, s):
    dense = _f64(dense)
    n = dense.shape[0]
    out = np.empty((2 * w + 1) * n, dtype=np.float64)
    lib().oracle_pack_sband_f64(n, w, s, _d(dense), dense.shape[1], _d(out))
    return out


def unpack_sband_f64(n, w, s, diag):
    diag = _f64(diag)
    out = np.empty((n, n), dtype=np.float64)
    lib().oracle_unpack_sband_f64(n, w, s, _d(diag), _d(out), n)
    return out


def sband_spmv_f64(n, w, s, D, x, rows=None):
    D, x = _f64(D), _f64(x)
    lo, hi = _window(n, rows)
    y = np.full(n, np.nan, dtype=np.float64)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_sband_spmv_f64(n, w, s, _d(D), _d(x), _d(y), _d(sc), lo, hi)
    return y, sc


def pack_subtri_f64(dense, k):
    dense = _f64(dense)
    N = dense.shape[0]
    out = np.empty(k * (k + 1) // 2, dtype=np.float64)
    lib().oracle_pack_subtri_f64(N, k, _d(dense), dense.shape[1], _d(out))
    return out


def unpack_subtri_f64(N, k, packed):
    packed = _f64(packed)
    out = np.empty((N, N), dtype=np.float64)
    lib().oracle_unpack_subtri_f64(N, k, _d(packed), _d(out), N)
    return out


def subtri_spmv_f64(N, k, Ap, x, rows=None):
    Ap, x = _f64(Ap), _f64(x)
    lo, hi = _window(N, rows)
    y = np.full(N, np.nan, dtype=np.float64)
    sc = np.full(N, np.nan, dtype=np.float64)
    lib().oracle_subtri_spmv_f64(N, k, _d(Ap), _d(x), _d(y), _d(sc), lo, hi)
    return y, sc


def pack_leslie_f64(dense):
    dense = _f64(dense)
    n = dense.shape[0]
    R = np.empty(n, dtype=np.float64)
    S = np.empty(max(n - 1, 0), dtype=np.float64)
    lib().oracle_pack_leslie_f64(n, _d(dense), dense.shape[1], _d(R), _d(S))
    return R, S


def unpack_leslie_f64(n, R, S):
    R, S = _f64(R), _f64(S)
    out = np.empty((n, n), dtype=np.float64)
    lib().oracle_unpack_leslie_f64(n, _d(R), _d(S), _d(out), n)
    return out


def leslie_spmv_f64(n, R, S, x):
    R, S, x = _f64(R), _f64(S), _f64(x)
    y = np.full(n, np.nan, dtype=np.float64)
    sc = np.full(n, np.nan, dtype=np.float64)
    lib().oracle_leslie_spmv_f64(n, _d(R), _d(S), _d(x), _d(y), _d(sc))
    return y, sc
