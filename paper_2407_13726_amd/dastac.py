"""ctypes binding over libdastac_hip.so -- argument marshalling only.

Every function has the name and argument order of the C entry point in
``include/dastac.h`` (minus the ``dastac_`` prefix and ``_f32`` suffix kept as
is).  Device operands are ``torch`` tensors on a HIP device (used for their
memory and for the current stream, nothing else); outputs are passed in by the
caller.  A non-zero status raises ``DastacError``.  There is no fallback: if
the library is not built, importing this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdastac_hip.so")

OK, EINVAL, ENULL, EOVERFLOW, EALIAS, EHIP = 0, 1, 2, 3, 4, 5

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p

# name -> (restype, argtypes); this table is also what the symbol-export test walks.
SIGNATURES = {
    "dastac_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "dastac_tri_count": (_i64, [_i64]),
    "dastac_tet_count": (_i64, [_i64]),
    "dastac_band_count": (_i64, [_i64, _i64]),
    "dastac_tri_offset": (_i64, [_i64, _i64, _i64]),
    "dastac_tet_offset": (_i64, [_i64, _i64, _i64, _i64]),
    "dastac_band_offset": (_i64, [_i64, _i64, _i64, _i64]),
    "dastac_tri_inverse": (ctypes.c_int, [_i64, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]),
    "dastac_tet_inverse": (ctypes.c_int, [_i64, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64),
                                          ctypes.POINTER(_i64)]),
    "dastac_pack_triu_f32": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_triu_f32": (ctypes.c_int, [_i64, _vp, _vp, _i64, _vp]),
    "dastac_pack_tet_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp]),
    "dastac_unpack_tet_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp]),
    "dastac_pack_band_f32": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_band_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_trmv_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmm_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp]),
    "dastac_band_spmv_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_tet_ttv_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_tet_mttkrp_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp, _i64, _vp]),
    "dastac_symv_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_t_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_lower_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_lower_t_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_symv_lower_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_tril_offset": (_i64, [_i64, _i64, _i64]),
    "dastac_pack_tril_f32": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_tril_f32": (ctypes.c_int, [_i64, _vp, _vp, _i64, _vp]),
    "dastac_uhc_count": (_i64, [_i64, _i64]),
    "dastac_uhc_offset": (_i64, [_i64, _i64, _i64, _i64, _i64]),
    "dastac_pack_uhc_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp]),
    "dastac_unpack_uhc_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp]),
    "dastac_ttm_ut_f32": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _i64, _vp, _vp]),
    "dastac_symm_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp]),
    "dastac_pr_a2_f32": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_pr_a3_f32": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_pack_triu_f64": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_triu_f64": (ctypes.c_int, [_i64, _vp, _vp, _i64, _vp]),
    "dastac_pack_tet_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp]),
    "dastac_unpack_tet_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp]),
    "dastac_pack_band_f64": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_band_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_trmv_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_band_spmv_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_tet_ttv_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmm_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp]),
    "dastac_symm_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp]),
    "dastac_pack_uhc_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp]),
    "dastac_unpack_uhc_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp]),
    "dastac_ttm_ut_f64": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _i64, _vp, _vp]),
    "dastac_pr_a2_f64": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_pr_a3_f64": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_tet_mttkrp_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp, _i64, _vp]),
    "dastac_pack_tril_f64": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_tril_f64": (ctypes.c_int, [_i64, _vp, _vp, _i64, _vp]),
    "dastac_symv_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_t_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_symv_lower_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_lower_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_trmv_lower_t_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp]),
    "dastac_pack_sband_f64": (ctypes.c_int, [_i64, _i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_sband_f64": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_sband_spmv_f64": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_pack_subtri_f64": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_subtri_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_subtri_spmv_f64": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_pack_leslie_f64": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp, _vp]),
    "dastac_unpack_leslie_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _i64, _vp]),
    "dastac_leslie_spmv_f64": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp, _vp]),
    "dastac_subtri_offset": (_i64, [_i64, _i64, _i64, _i64]),
    "dastac_pack_sband_f32": (ctypes.c_int, [_i64, _i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_sband_f32": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_pack_subtri_f32": (ctypes.c_int, [_i64, _i64, _vp, _i64, _vp, _vp]),
    "dastac_unpack_subtri_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _i64, _vp]),
    "dastac_pack_leslie_f32": (ctypes.c_int, [_i64, _vp, _i64, _vp, _vp, _vp]),
    "dastac_unpack_leslie_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _i64, _vp]),
    "dastac_sband_spmv_f32": (ctypes.c_int, [_i64, _i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_subtri_spmv_f32": (ctypes.c_int, [_i64, _i64, _vp, _vp, _vp, _vp]),
    "dastac_leslie_spmv_f32": (ctypes.c_int, [_i64, _vp, _vp, _vp, _vp, _vp]),
    "dastac_stream_sum_f32": (ctypes.c_int, [_i64, _vp, _vp, _i64, _vp]),
}


class DastacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, strerror(status)))


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library; raise if it is missing (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libdastac_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().dastac_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise DastacError(status, where)


def _ptr(t):
    """Device address of a tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if t.dtype.__str__() != "torch.float32":
        raise ValueError("float32 tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _ptr64(t):
    """Device address of a float64 tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if t.dtype.__str__() != "torch.float64":
        raise ValueError("float64 tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


# ---- index polynomials (host) -------------------------------------------------

def tri_count(n): return int(lib().dastac_tri_count(n))
def tet_count(n): return int(lib().dastac_tet_count(n))
def band_count(n, w): return int(lib().dastac_band_count(n, w))
def tri_offset(n, i, j): return int(lib().dastac_tri_offset(n, i, j))
def tet_offset(n, i, j, k): return int(lib().dastac_tet_offset(n, i, j, k))
def band_offset(n, w, d, i): return int(lib().dastac_band_offset(n, w, d, i))


def tri_inverse(n, p):
    i, j = _i64(), _i64()
    _check(lib().dastac_tri_inverse(n, p, ctypes.byref(i), ctypes.byref(j)), "tri_inverse")
    return i.value, j.value


def tet_inverse(n, p):
    i, j, k = _i64(), _i64(), _i64()
    _check(lib().dastac_tet_inverse(n, p, ctypes.byref(i), ctypes.byref(j), ctypes.byref(k)), "tet_inverse")
    return i.value, j.value, k.value


# ---- device operations -----------------------------------------------------------

def pack_triu_f32(n, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_triu_f32(n, _ptr(dense), ld, _ptr(packed), _stream(stream)), "pack_triu_f32")


def unpack_triu_f32(n, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_triu_f32(n, _ptr(packed), _ptr(dense), ld, _stream(stream)), "unpack_triu_f32")


def pack_tet_f32(n, dense, packed, stream=None):
    _check(lib().dastac_pack_tet_f32(n, _ptr(dense), _ptr(packed), _stream(stream)), "pack_tet_f32")


def unpack_tet_f32(n, packed, dense, stream=None):
    _check(lib().dastac_unpack_tet_f32(n, _ptr(packed), _ptr(dense), _stream(stream)), "unpack_tet_f32")


def pack_band_f32(n, w, dense, ld, diag_major, stream=None):
    _check(lib().dastac_pack_band_f32(n, w, _ptr(dense), ld, _ptr(diag_major), _stream(stream)), "pack_band_f32")


def unpack_band_f32(n, w, diag_major, dense, ld, stream=None):
    _check(lib().dastac_unpack_band_f32(n, w, _ptr(diag_major), _ptr(dense), ld, _stream(stream)),
           "unpack_band_f32")


def trmv_f32(n, Up, x, y, stream=None):
    _check(lib().dastac_trmv_f32(n, _ptr(Up), _ptr(x), _ptr(y), _stream(stream)), "trmv_f32")


def trmm_f32(n, m, Up, B, ldb, C, ldc, stream=None):
    _check(lib().dastac_trmm_f32(n, m, _ptr(Up), _ptr(B), ldb, _ptr(C), ldc, _stream(stream)), "trmm_f32")


def band_spmv_f32(n, w, D, x, y, stream=None):
    _check(lib().dastac_band_spmv_f32(n, w, _ptr(D), _ptr(x), _ptr(y), _stream(stream)), "band_spmv_f32")


def tet_ttv_f32(n, Ap, v, Mp, stream=None):
    _check(lib().dastac_tet_ttv_f32(n, _ptr(Ap), _ptr(v), _ptr(Mp), _stream(stream)), "tet_ttv_f32")


def tet_mttkrp_f32(n, R, Ap, B, ldb, C, ldc, M, ldm, stream=None):
    _check(lib().dastac_tet_mttkrp_f32(n, R, _ptr(Ap), _ptr(B), ldb, _ptr(C), ldc, _ptr(M), ldm, _stream(stream)),
           "tet_mttkrp_f32")


def uhc_count(n, Q): return int(lib().dastac_uhc_count(n, Q))
def uhc_offset(n, Q, i, j, l): return int(lib().dastac_uhc_offset(n, Q, i, j, l))


def pack_uhc_f32(n, Q, dense, packed, stream=None):
    _check(lib().dastac_pack_uhc_f32(n, Q, _ptr(dense), _ptr(packed), _stream(stream)), "pack_uhc_f32")


def unpack_uhc_f32(n, Q, packed, dense, stream=None):
    _check(lib().dastac_unpack_uhc_f32(n, Q, _ptr(packed), _ptr(dense), _stream(stream)), "unpack_uhc_f32")


def ttm_ut_f32(n, Q, K, Bp, C, ldc, Ap, stream=None):
    _check(lib().dastac_ttm_ut_f32(n, Q, K, _ptr(Bp), _ptr(C), ldc, _ptr(Ap), _stream(stream)), "ttm_ut_f32")


def symv_f32(n, Up, x, y, stream=None):
    _check(lib().dastac_symv_f32(n, _ptr(Up), _ptr(x), _ptr(y), _stream(stream)), "symv_f32")


def trmv_t_f32(n, Up, x, y, stream=None):
    _check(lib().dastac_trmv_t_f32(n, _ptr(Up), _ptr(x), _ptr(y), _stream(stream)), "trmv_t_f32")


def trmv_lower_f32(n, Lp, x, y, stream=None):
    _check(lib().dastac_trmv_lower_f32(n, _ptr(Lp), _ptr(x), _ptr(y), _stream(stream)), "trmv_lower_f32")


def trmv_lower_t_f32(n, Lp, x, y, stream=None):
    _check(lib().dastac_trmv_lower_t_f32(n, _ptr(Lp), _ptr(x), _ptr(y), _stream(stream)), "trmv_lower_t_f32")


def symv_lower_f32(n, Lp, x, y, stream=None):
    _check(lib().dastac_symv_lower_f32(n, _ptr(Lp), _ptr(x), _ptr(y), _stream(stream)), "symv_lower_f32")


def tril_offset(n, i, j): return int(lib().dastac_tril_offset(n, i, j))


def pack_tril_f32(n, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_tril_f32(n, _ptr(dense), ld, _ptr(packed), _stream(stream)), "pack_tril_f32")


def unpack_tril_f32(n, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_tril_f32(n, _ptr(packed), _ptr(dense), ld, _stream(stream)), "unpack_tril_f32")



def subtri_offset(N, k, i, j): return int(lib().dastac_subtri_offset(N, k, i, j))


def pack_sband_f32(n, w, s, dense, ld, diag_major, stream=None):
    _check(lib().dastac_pack_sband_f32(n, w, s, _ptr(dense), ld, _ptr(diag_major), _stream(stream)),
           "pack_sband_f32")


def unpack_sband_f32(n, w, s, diag_major, dense, ld, stream=None):
    _check(lib().dastac_unpack_sband_f32(n, w, s, _ptr(diag_major), _ptr(dense), ld, _stream(stream)),
           "unpack_sband_f32")


def pack_subtri_f32(N, k, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_subtri_f32(N, k, _ptr(dense), ld, _ptr(packed), _stream(stream)), "pack_subtri_f32")


def unpack_subtri_f32(N, k, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_subtri_f32(N, k, _ptr(packed), _ptr(dense), ld, _stream(stream)),
           "unpack_subtri_f32")


def pack_leslie_f32(n, dense, ld, R, S, stream=None):
    _check(lib().dastac_pack_leslie_f32(n, _ptr(dense), ld, _ptr(R), _ptr(S), _stream(stream)), "pack_leslie_f32")


def unpack_leslie_f32(n, R, S, dense, ld, stream=None):
    _check(lib().dastac_unpack_leslie_f32(n, _ptr(R), _ptr(S), _ptr(dense), ld, _stream(stream)),
           "unpack_leslie_f32")


def sband_spmv_f32(n, w, s, D, x, y, stream=None):
    _check(lib().dastac_sband_spmv_f32(n, w, s, _ptr(D), _ptr(x), _ptr(y), _stream(stream)), "sband_spmv_f32")


def subtri_spmv_f32(N, k, Ap, x, y, stream=None):
    _check(lib().dastac_subtri_spmv_f32(N, k, _ptr(Ap), _ptr(x), _ptr(y), _stream(stream)), "subtri_spmv_f32")


def leslie_spmv_f32(n, R, S, x, y, stream=None):
    _check(lib().dastac_leslie_spmv_f32(n, _ptr(R), _ptr(S), _ptr(x), _ptr(y), _stream(stream)), "leslie_spmv_f32")


def stream_sum_f32(count, src, partial, npartial, stream=None):
    _check(lib().dastac_stream_sum_f32(count, _ptr(src), _ptr(partial), npartial, _stream(stream)), "stream_sum_f32")


def symm_f32(n, m, Up, B, ldb, C, ldc, stream=None):
    _check(lib().dastac_symm_f32(n, m, _ptr(Up), _ptr(B), ldb, _ptr(C), ldc, _stream(stream)), "symm_f32")


def pr_a2_f32(N, d, B, ldb, A2p, stream=None):
    _check(lib().dastac_pr_a2_f32(N, d, _ptr(B), ldb, _ptr(A2p), _stream(stream)), "pr_a2_f32")


def pr_a3_f32(N, d, B, ldb, A3p, stream=None):
    _check(lib().dastac_pr_a3_f32(N, d, _ptr(B), ldb, _ptr(A3p), _stream(stream)), "pr_a3_f32")


# ---- double precision ---------------------------------------------------------

def pack_triu_f64(n, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_triu_f64(n, _ptr64(dense), ld, _ptr64(packed), _stream(stream)), "pack_triu_f64")


def unpack_triu_f64(n, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_triu_f64(n, _ptr64(packed), _ptr64(dense), ld, _stream(stream)), "unpack_triu_f64")


def pack_tet_f64(n, dense, packed, stream=None):
    _check(lib().dastac_pack_tet_f64(n, _ptr64(dense), _ptr64(packed), _stream(stream)), "pack_tet_f64")


def unpack_tet_f64(n, packed, dense, stream=None):
    _check(lib().dastac_unpack_tet_f64(n, _ptr64(packed), _ptr64(dense), _stream(stream)), "unpack_tet_f64")


def pack_band_f64(n, w, dense, ld, diag_major, stream=None):
    _check(lib().dastac_pack_band_f64(n, w, _ptr64(dense), ld, _ptr64(diag_major), _stream(stream)), "pack_band_f64")


def unpack_band_f64(n, w, diag_major, dense, ld, stream=None):
    _check(lib().dastac_unpack_band_f64(n, w, _ptr64(diag_major), _ptr64(dense), ld, _stream(stream)),
           "unpack_band_f64")


def trmv_f64(n, Up, x, y, stream=None):
    _check(lib().dastac_trmv_f64(n, _ptr64(Up), _ptr64(x), _ptr64(y), _stream(stream)), "trmv_f64")


def band_spmv_f64(n, w, D, x, y, stream=None):
    _check(lib().dastac_band_spmv_f64(n, w, _ptr64(D), _ptr64(x), _ptr64(y), _stream(stream)), "band_spmv_f64")


def tet_ttv_f64(n, Ap, v, Mp, stream=None):
    _check(lib().dastac_tet_ttv_f64(n, _ptr64(Ap), _ptr64(v), _ptr64(Mp), _stream(stream)), "tet_ttv_f64")


def trmm_f64(n, m, Up, B, ldb, C, ldc, stream=None):
    _check(lib().dastac_trmm_f64(n, m, _ptr64(Up), _ptr64(B), ldb, _ptr64(C), ldc, _stream(stream)), "trmm_f64")


def symm_f64(n, m, Up, B, ldb, C, ldc, stream=None):
    _check(lib().dastac_symm_f64(n, m, _ptr64(Up), _ptr64(B), ldb, _ptr64(C), ldc, _stream(stream)), "symm_f64")


def pack_uhc_f64(n, Q, dense, packed, stream=None):
    _check(lib().dastac_pack_uhc_f64(n, Q, _ptr64(dense), _ptr64(packed), _stream(stream)), "pack_uhc_f64")


def unpack_uhc_f64(n, Q, packed, dense, stream=None):
    _check(lib().dastac_unpack_uhc_f64(n, Q, _ptr64(packed), _ptr64(dense), _stream(stream)), "unpack_uhc_f64")


def ttm_ut_f64(n, Q, K, Bp, C, ldc, Ap, stream=None):
    _check(lib().dastac_ttm_ut_f64(n, Q, K, _ptr64(Bp), _ptr64(C), ldc, _ptr64(Ap), _stream(stream)), "ttm_ut_f64")


def pr_a2_f64(N, d, B, ldb, A2p, stream=None):
    _check(lib().dastac_pr_a2_f64(N, d, _ptr64(B), ldb, _ptr64(A2p), _stream(stream)), "pr_a2_f64")


def pr_a3_f64(N, d, B, ldb, A3p, stream=None):
    _check(lib().dastac_pr_a3_f64(N, d, _ptr64(B), ldb, _ptr64(A3p), _stream(stream)), "pr_a3_f64")


def tet_mttkrp_f64(n, R, Ap, B, ldb, C, ldc, M, ldm, stream=None):
    _check(lib().dastac_tet_mttkrp_f64(n, R, _ptr64(Ap), _ptr64(B), ldb, _ptr64(C), ldc, _ptr64(M), ldm,
                                       _stream(stream)), "tet_mttkrp_f64")


def pack_tril_f64(n, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_tril_f64(n, _ptr64(dense), ld, _ptr64(packed), _stream(stream)), "pack_tril_f64")


def unpack_tril_f64(n, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_tril_f64(n, _ptr64(packed), _ptr64(dense), ld, _stream(stream)), "unpack_tril_f64")


def symv_f64(n, Up, x, y, stream=None):
    _check(lib().dastac_symv_f64(n, _ptr64(Up), _ptr64(x), _ptr64(y), _stream(stream)), "symv_f64")


def trmv_t_f64(n, Up, x, y, stream=None):
    _check(lib().dastac_trmv_t_f64(n, _ptr64(Up), _ptr64(x), _ptr64(y), _stream(stream)), "trmv_t_f64")


def symv_lower_f64(n, Lp, x, y, stream=None):
    _check(lib().dastac_symv_lower_f64(n, _ptr64(Lp), _ptr64(x), _ptr64(y), _stream(stream)), "symv_lower_f64")


def trmv_lower_f64(n, Lp, x, y, stream=None):
    _check(lib().dastac_trmv_lower_f64(n, _ptr64(Lp), _ptr64(x), _ptr64(y), _stream(stream)), "trmv_lower_f64")


def trmv_lower_t_f64(n, Lp, x, y, stream=None):
    _check(lib().dastac_trmv_lower_t_f64(n, _ptr64(Lp), _ptr64(x), _ptr64(y), _stream(stream)), "trmv_lower_t_f64")


def pack_sband_f64(n, w, s, dense, ld, diag_major, stream=None):
    _check(lib().dastac_pack_sband_f64(n, w, s, _ptr64(dense), ld, _ptr64(diag_major), _stream(stream)),
           "pack_sband_f64")


def unpack_sband_f64(n, w, s, diag_major, dense, ld, stream=None):
    _check(lib().dastac_unpack_sband_f64(n, w, s, _ptr64(diag_major), _ptr64(dense), ld, _stream(stream)),
           "unpack_sband_f64")


def sband_spmv_f64(n, w, s, D, x, y, stream=None):
    _check(lib().dastac_sband_spmv_f64(n, w, s, _ptr64(D), _ptr64(x), _ptr64(y), _stream(stream)), "sband_spmv_f64")


def pack_subtri_f64(N, k, dense, ld, packed, stream=None):
    _check(lib().dastac_pack_subtri_f64(N, k, _ptr64(dense), ld, _ptr64(packed), _stream(stream)), "pack_subtri_f64")


def unpack_subtri_f64(N, k, packed, dense, ld, stream=None):
    _check(lib().dastac_unpack_subtri_f64(N, k, _ptr64(packed), _ptr64(dense), ld, _stream(stream)),
           "unpack_subtri_f64")


def subtri_spmv_f64(N, k, Ap, x, y, stream=None):
    _check(lib().dastac_subtri_spmv_f64(N, k, _ptr64(Ap), _ptr64(x), _ptr64(y), _stream(stream)), "subtri_spmv_f64")


def pack_leslie_f64(n, dense, ld, R, S, stream=None):
    _check(lib().dastac_pack_leslie_f64(n, _ptr64(dense), ld, _ptr64(R), _ptr64(S), _stream(stream)),
           "pack_leslie_f64")


def unpack_leslie_f64(n, R, S, dense, ld, stream=None):
    _check(lib().dastac_unpack_leslie_f64(n, _ptr64(R), _ptr64(S), _ptr64(dense), ld, _stream(stream)),
           "unpack_leslie_f64")


def leslie_spmv_f64(n, R, S, x, y, stream=None):
    _check(lib().dastac_leslie_spmv_f64(n, _ptr64(R), _ptr64(S), _ptr64(x), _ptr64(y), _stream(stream)),
           "leslie_spmv_f64")
