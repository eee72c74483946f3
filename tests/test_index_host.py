"""Host-side checks of the C-ABI library that need no GPU: the index-polynomial
module against the oracle's counting definition, the exported symbols, and the
argument validation of every device entry point (all of which return before any
HIP call is made).
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2407_13726_amd import dastac

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "dastac.h")).read()
    declared = set(re.findall(r"\b(dastac_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(dastac.SIGNATURES), declared ^ set(dastac.SIGNATURES)
    L = dastac.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_binding_signatures_follow_the_header():
    """Every prototype in the header against the argument list the binding marshals: the same number of
    parameters, 64-bit integers where the header says int64_t, pointers where it says pointer."""
    hdr = open(os.path.join(ROOT, "include", "dastac.h")).read()
    hdr = re.sub(r"/\*.*?\*/", " ", hdr, flags=re.S)  # comments mention the entry points too
    protos = re.findall(r"\b([a-z_0-9]+\s*\*?)\s*\b(dastac_[a-z0-9_]+)\s*\(([^)]*)\)\s*;", hdr)
    assert {name for _, name, _ in protos} == set(dastac.SIGNATURES)
    for ret, name, params in protos:
        res, args = dastac.SIGNATURES[name]
        params = [q.strip() for q in params.split(",") if q.strip() and q.strip() != "void"]
        assert len(params) == len(args), name
        for decl, ctype in zip(params, args):
            if "*" in decl:
                assert ctype in (ctypes.c_void_p,) or issubclass(ctype, ctypes._Pointer), (name, decl)
            elif decl.startswith("int64_t"):
                assert ctype is ctypes.c_int64, (name, decl)
            else:
                assert decl.startswith("int ") and ctype is ctypes.c_int, (name, decl)
        if "char" in ret:
            assert res is ctypes.c_char_p, name
        elif ret.strip() == "int64_t":
            assert res is ctypes.c_int64, name
        else:
            assert ret.strip() == "int" and res is ctypes.c_int, name


def test_strerror_names_every_code():
    names = {dastac.strerror(c) for c in range(6)}
    assert len(names) == 6 and "unknown status" not in names
    assert dastac.strerror(99) == "unknown status"


@pytest.mark.parametrize("n", [0, 1, 2, 3, 7, 12, 25])
def test_tri_forward_and_inverse_match_counting(oracle, n):
    assert dastac.tri_count(n) == oracle.count_domain(oracle.DOM_TRIU, [n])
    p = 0
    for i in range(n):
        for j in range(i, n):
            assert dastac.tri_offset(n, i, j) == p == oracle.triu_position(n, i, j)
            assert dastac.tri_inverse(n, p) == (i, j)
            p += 1
    assert dastac.tri_offset(n, 1, 0) == -1 and dastac.tri_offset(n, 0, n) == -1
    for bad in (-1, p):
        with pytest.raises(dastac.DastacError) as e:
            dastac.tri_inverse(n, bad)
        assert e.value.status == dastac.EINVAL


@pytest.mark.parametrize("n", [0, 1, 2, 3, 6, 11])
def test_tet_forward_and_inverse_match_counting(oracle, n):
    assert dastac.tet_count(n) == oracle.count_domain(oracle.DOM_TET, [n])
    p = 0
    for i in range(n):
        for j in range(i, n):
            for k in range(j, n):
                assert dastac.tet_offset(n, i, j, k) == p
                assert oracle.count_preceding(oracle.DOM_TET, [n], [i, j, k]) == p
                assert dastac.tet_inverse(n, p) == (i, j, k)
                p += 1
    assert dastac.tet_offset(n, 0, 1, 0) == -1 and dastac.tet_offset(n, 0, 0, n) == -1
    for bad in (-1, p):
        with pytest.raises(dastac.DastacError):
            dastac.tet_inverse(n, bad)


@pytest.mark.parametrize("n,w", [(1, 0), (5, 2), (7, 16)])
def test_band_offsets_match_counting(oracle, n, w):
    assert dastac.band_count(n, w) == oracle.count_domain(oracle.DOM_BAND, [n, w]) == (2 * w + 1) * n
    for d in range(-w, w + 1):
        for i in range(n):
            assert dastac.band_offset(n, w, d, i) == oracle.count_preceding(oracle.DOM_BAND, [n, w], [d, i])
    assert dastac.band_offset(n, w, w + 1, 0) == -1 and dastac.band_offset(n, w, 0, n) == -1
    assert dastac.band_count(-1, 0) == -1 and dastac.band_count(1, -1) == -1


@pytest.mark.parametrize("n", [1, 2, 6, 11])
def test_tril_offsets_match_counting_and_paper_polynomial(oracle, n):
    """tril(n,i,j) = i/2 + i^2/2 + j (Section 4, Eq. 2 after the fusion of its two pieces)."""
    rows = {(i, j): p for i, j, p in
            (tuple(int(t) for t in ln.split()) for ln in open(os.path.join(
                os.path.dirname(__file__), "golden", "lower_triangle_fused_polynomial.txt"))
             if ln.strip() and not ln.startswith("#"))}
    for i in range(n):
        for j in range(i + 1):
            got = dastac.tril_offset(n, i, j)
            assert got == oracle.count_preceding(oracle.DOM_TRIL, [n], [i, j])
            if n == 6:
                assert got == rows[(i, j)]  # the values printed from the paper's polynomial
    assert dastac.tril_offset(n, 0, 1) == -1 and dastac.tril_offset(n, n, 0) == -1 and dastac.tril_offset(-1, 0, 0) == -1


@pytest.mark.parametrize("n,Q", [(1, 1), (4, 3), (6, 2), (5, 7)])
def test_uhc_offsets_match_counting_and_paper_polynomial(oracle, n, Q):
    """uhc(n,Q,i,j,l) is the number of preceding points of the running example's buffer B, i.e. the
    printed P_B(i,j,l) = (((N-1/2) Q i - 1/2 Q i^2) + Q j) + l."""
    from fractions import Fraction
    assert dastac.uhc_count(n, Q) == oracle.count_domain(oracle.DOM_UHC, [n, n, Q]) == n * (n + 1) // 2 * Q
    for i in range(n):
        for j in range(i, n):
            for l in range(Q):
                got = dastac.uhc_offset(n, Q, i, j, l)
                assert got == oracle.count_preceding(oracle.DOM_UHC, [n, n, Q], [i, j, l])
                assert got == (n - Fraction(1, 2)) * Q * i - Fraction(1, 2) * Q * i * i + Q * j + l
    assert dastac.uhc_offset(n, Q, 0, 0, Q) == -1 and dastac.uhc_offset(n, Q, n - 1, n, 0) == -1
    assert dastac.uhc_count(-1, 1) == -1 and dastac.uhc_count(4, 0) == -1 and dastac.uhc_count(2 ** 20, 2 ** 24) == -1


def test_benchmark_sizes_row_and_slice_boundaries(oracle):
    """Forward and inverse at every row start of the large triangle and every fibre start of
    the large tetrahedron, against the oracle's running-counter walk."""
    n = 16384
    starts = oracle.triu_row_starts(n)
    assert dastac.tri_count(n) == starts[n] == 134225920
    for i in list(range(0, n, 97)) + [n - 2, n - 1]:
        assert dastac.tri_offset(n, i, i) == starts[i]
        assert dastac.tri_inverse(n, int(starts[i])) == (i, i)
        assert dastac.tri_inverse(n, int(starts[i + 1]) - 1) == (i, n - 1)
    n = 1024
    fs, total = oracle.tet_fibre_starts(n)
    assert dastac.tet_count(n) == total == 179481600
    rng = np.random.default_rng(5)
    for i in list(range(0, n, 61)) + [n - 1]:
        for j in sorted({i, min(i + 1, n - 1), n - 1, int(rng.integers(i, n))}):
            assert dastac.tet_offset(n, i, j, j) == fs[i, j]
            assert dastac.tet_inverse(n, int(fs[i, j])) == (i, j, j)
            assert dastac.tet_inverse(n, int(fs[i, j]) + (n - 1 - j)) == (i, j, n - 1)


def test_inverse_round_trip_random_positions():
    rng = np.random.default_rng(11)
    for n in (512, 16384, 100003, 2 ** 31 - 1):
        cnt = dastac.tri_count(n)
        for p in [0, cnt - 1] + [int(v) for v in rng.integers(0, cnt, 200)]:
            i, j = dastac.tri_inverse(n, p)
            assert 0 <= i <= j < n and dastac.tri_offset(n, i, j) == p
    for n in (512, 1024, 4099, 2 ** 20):
        cnt = dastac.tet_count(n)
        for p in [0, cnt - 1] + [int(v) for v in rng.integers(0, cnt, 200)]:
            i, j, k = dastac.tet_inverse(n, p)
            assert 0 <= i <= j <= k < n and dastac.tet_offset(n, i, j, k) == p


def test_guards():
    assert dastac.tri_count(-1) == -1 and dastac.tri_count(2 ** 31) == -1
    assert dastac.tri_count(2 ** 31 - 1) == (2 ** 31 - 1) * 2 ** 30
    assert dastac.tet_count(-1) == -1 and dastac.tet_count(2 ** 20 + 1) == -1
    n = 2 ** 20
    assert dastac.tet_count(n) == n * (n + 1) * (n + 2) // 6


# ---- argument validation of the device entry points (no launch happens) --------

def _p(v):
    return ctypes.c_void_p(v)

@pytest.mark.parametrize("N,k", [(1, 1), (5, 0), (6, 4), (9, 9), (12, 5)])
def test_subtri_offsets_match_a_walk_of_the_domain(N, k):
    """subtri(N,k,i,j) is the number of points with j-i >= N-k that precede (i,j) in iteration
    order (Section 6.4, sub-triangular structure), counted here by a plain walk."""
    p = 0
    for i in range(N):
        for j in range(N):
            if j - i >= N - k:
                assert dastac.subtri_offset(N, k, i, j) == p
                p += 1
            else:
                assert dastac.subtri_offset(N, k, i, j) == -1
    assert p == dastac.tri_count(k)
    assert dastac.subtri_offset(N, N + 1, 0, 0) == -1 and dastac.subtri_offset(N, k, 0, N) == -1


def test_new_domain_entry_points_reject_bad_arguments():
    L = dastac.lib()
    assert L.dastac_symm_f32(4, 0, _p(A), _p(B), 4, _p(C), 4, None) == dastac.EINVAL
    assert L.dastac_symm_f32(4, 8, _p(A), _p(B), 7, _p(C), 8, None) == dastac.EINVAL
    assert L.dastac_symm_f32(2 ** 24 + 1, 8, _p(A), _p(B), 8, _p(C), 8, None) == dastac.EOVERFLOW
    assert L.dastac_symm_f32(4, 2, _p(A), None, 2, _p(C), 2, None) == dastac.ENULL
    assert L.dastac_symm_f32(4, 2, _p(A), _p(B), 2, _p(B + 8), 2, None) == dastac.EALIAS
    assert L.dastac_symm_f32(0, 2, None, None, 2, None, 2, None) == dastac.OK
    for fn, dmax in ((L.dastac_pr_a2_f32, 65536), (L.dastac_pr_a3_f32, 8192), (L.dastac_pr_a2_f64, 65536),
                     (L.dastac_pr_a3_f64, 8192)):
        assert fn(-1, 4, _p(A), 4, _p(B), None) == dastac.EINVAL
        assert fn(10, -1, _p(A), 4, _p(B), None) == dastac.EINVAL
        assert fn(10, 4, _p(A), 3, _p(B), None) == dastac.EINVAL
        assert fn(10, dmax + 1, _p(A), dmax + 1, _p(B), None) == dastac.EOVERFLOW
        assert fn(2 ** 31 + 1, 4, _p(A), 4, _p(B), None) == dastac.EOVERFLOW
        assert fn(10, 4, None, 4, _p(B), None) == dastac.ENULL
        assert fn(10, 4, _p(A), 4, None, None) == dastac.ENULL
        assert fn(10, 4, _p(A), 4, _p(A + 32), None) == dastac.EALIAS
        assert fn(10, 0, None, 0, None, None) == dastac.OK
    for fn, nmax in ((L.dastac_trmv_f64, 2 ** 31 - 1), (L.dastac_tet_ttv_f64, 8192), (L.dastac_symv_f64, 262144),
                     (L.dastac_trmv_t_f64, 262144), (L.dastac_symv_lower_f64, 262144),
                     (L.dastac_trmv_lower_f64, 262144), (L.dastac_trmv_lower_t_f64, 262144)):
        assert fn(-1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
        assert fn(nmax + 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
        assert fn(4, None, _p(B), _p(C), None) == dastac.ENULL
        assert fn(4, _p(A), _p(B), _p(B + 16), None) == dastac.EALIAS
        assert fn(0, None, None, None, None) == dastac.OK
    assert L.dastac_trmm_f64(4, 0, _p(A), _p(B), 4, _p(C), 4, None) == dastac.EINVAL
    assert L.dastac_trmm_f64(4, 8, _p(A), _p(B), 8, _p(C), 7, None) == dastac.EINVAL
    assert L.dastac_trmm_f64(4, 2, _p(A), _p(B), 2, None, 2, None) == dastac.ENULL
    assert L.dastac_trmm_f64(4, 2, _p(A), _p(B), 2, _p(B + 56), 2, None) == dastac.EALIAS
    assert L.dastac_trmm_f64(0, 2, None, None, 2, None, 2, None) == dastac.OK
    assert L.dastac_symm_f64(4, 0, _p(A), _p(B), 4, _p(C), 4, None) == dastac.EINVAL
    assert L.dastac_symm_f64(4, 2, None, _p(B), 2, _p(C), 2, None) == dastac.ENULL
    assert L.dastac_symm_f64(4, 2, _p(A), _p(B), 2, _p(B + 56), 2, None) == dastac.EALIAS
    assert L.dastac_symm_f64(0, 2, None, None, 2, None, 2, None) == dastac.OK
    assert L.dastac_ttm_ut_f64(4, 0, 4, _p(A), _p(B), 4, _p(C), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f64(4, 8, 4, _p(A), _p(B), 7, _p(C), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f64(4, 4, 4, _p(A), None, 4, _p(C), None) == dastac.ENULL
    assert L.dastac_ttm_ut_f64(4, 4, 4, _p(A), _p(B), 4, _p(A + 64), None) == dastac.EALIAS
    assert L.dastac_ttm_ut_f64(0, 4, 4, None, None, 4, None, None) == dastac.OK
    assert L.dastac_pack_uhc_f64(4, 0, _p(A), _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_uhc_f64(4, 2, _p(A), None, None) == dastac.ENULL
    assert L.dastac_tet_mttkrp_f64(4, 0, _p(A), _p(B), 4, _p(C), 4, _p(D), 4, None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f64(4, 2 ** 20 + 1, _p(A), _p(B), 2 ** 21, _p(C), 2 ** 21, _p(D), 2 ** 21, None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f64(4, 8, _p(A), _p(B), 8, _p(C), 8, _p(D), 7, None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f64(4, 2, _p(A), _p(B), 2, None, 2, _p(D), 2, None) == dastac.ENULL
    assert L.dastac_tet_mttkrp_f64(0, 2, None, None, 2, None, 2, None, 2, None) == dastac.OK
    assert L.dastac_band_spmv_f64(4, 2 ** 20 + 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_band_spmv_f64(4, 1, _p(A), _p(B), _p(B + 24), None) == dastac.EALIAS
    assert L.dastac_pack_triu_f64(8, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_tet_f64(4, _p(A), None, None) == dastac.ENULL
    assert L.dastac_pack_band_f64(4, -1, _p(A), 4, _p(B), None) == dastac.EINVAL
    # 8-byte elements: two 6-element double vectors 40 bytes apart overlap (two float vectors would not)
    assert L.dastac_trmv_f64(6, _p(A), _p(B), _p(B + 40), None) == dastac.EALIAS
    assert L.dastac_pack_tril_f64(8, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_tril_f64(4, None, _p(B), 4, None) == dastac.ENULL
    assert L.dastac_pack_tril_f64(4, _p(A), 4, _p(A + 120), None) == dastac.EALIAS  # 16 doubles reach byte 128
    assert L.dastac_sband_spmv_f64(4, 1, 0, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_sband_spmv_f64(4, 2 ** 20 + 1, 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_sband_spmv_f64(4, 1, 2, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_sband_spmv_f64(4, 1, 2, _p(A), _p(B), _p(B + 24), None) == dastac.EALIAS
    assert L.dastac_sband_spmv_f64(0, 1, 2, None, None, None, None) == dastac.OK
    assert L.dastac_pack_sband_f64(8, 1, 2, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_sband_f64(8, 1, 2, None, _p(B), 8, None) == dastac.ENULL
    assert L.dastac_subtri_spmv_f64(4, 5, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_subtri_spmv_f64(4, 2, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_subtri_spmv_f64(4, 2, _p(A), _p(B), _p(B + 24), None) == dastac.EALIAS
    assert L.dastac_subtri_spmv_f64(0, 0, None, None, None, None) == dastac.OK
    assert L.dastac_pack_subtri_f64(8, 9, _p(A), 8, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_subtri_f64(8, 4, _p(A), None, 8, None) == dastac.ENULL
    assert L.dastac_leslie_spmv_f64(-1, _p(A), _p(B), _p(C), _p(D), None) == dastac.EINVAL
    assert L.dastac_leslie_spmv_f64(4, _p(A), None, _p(C), _p(D), None) == dastac.ENULL
    assert L.dastac_leslie_spmv_f64(4, _p(A), _p(B), _p(C), _p(A + 24), None) == dastac.EALIAS
    assert L.dastac_leslie_spmv_f64(0, None, None, None, None, None) == dastac.OK
    assert L.dastac_pack_leslie_f64(4, _p(A), 3, _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_unpack_leslie_f64(4, None, _p(B), _p(C), 4, None) == dastac.ENULL
    assert L.dastac_sband_spmv_f32(-1, 1, 1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_sband_spmv_f32(4, 1, 0, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_sband_spmv_f32(4, 2 ** 20 + 1, 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_sband_spmv_f32(4, 1, 2 ** 41, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_sband_spmv_f32(4, 1, 2, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_sband_spmv_f32(4, 1, 2, _p(A), _p(B), _p(B + 4), None) == dastac.EALIAS
    assert L.dastac_sband_spmv_f32(0, 1, 2, None, None, None, None) == dastac.OK
    assert L.dastac_pack_sband_f32(8, 1, 0, _p(A), 8, _p(B), None) == dastac.EINVAL
    assert L.dastac_pack_sband_f32(8, 1, 2, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_sband_f32(8, 1, 2, None, _p(B), 8, None) == dastac.ENULL
    assert L.dastac_subtri_spmv_f32(4, 5, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_subtri_spmv_f32(4, -1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_subtri_spmv_f32(2 ** 20, 524289, _p(D), _p(A), _p(B), None) == dastac.EOVERFLOW
    assert L.dastac_subtri_spmv_f32(4, 2, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_subtri_spmv_f32(4, 2, _p(A), _p(B), _p(B + 8), None) == dastac.EALIAS
    assert L.dastac_subtri_spmv_f32(0, 0, None, None, None, None) == dastac.OK
    assert L.dastac_pack_subtri_f32(8, 9, _p(A), 8, _p(B), None) == dastac.EINVAL
    assert L.dastac_pack_subtri_f32(8, 4, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_subtri_f32(8, 4, _p(A), None, 8, None) == dastac.ENULL
    assert L.dastac_leslie_spmv_f32(-1, _p(A), _p(B), _p(C), _p(D), None) == dastac.EINVAL
    assert L.dastac_leslie_spmv_f32(4, _p(A), None, _p(C), _p(D), None) == dastac.ENULL
    assert L.dastac_leslie_spmv_f32(4, _p(A), _p(B), _p(C), _p(A + 4), None) == dastac.EALIAS
    assert L.dastac_leslie_spmv_f32(0, None, None, None, None, None) == dastac.OK
    assert L.dastac_pack_leslie_f32(4, _p(A), 3, _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_pack_leslie_f32(4, _p(A), 4, _p(B), _p(B + 8), None) == dastac.EALIAS
    assert L.dastac_unpack_leslie_f32(4, None, _p(B), _p(C), 4, None) == dastac.ENULL


A, B, C, D = 0x10000, 0x20000000, 0x40000000, 0x60000000  # fake, never dereferenced


def test_device_entry_points_reject_bad_arguments():
    L = dastac.lib()
    # negative sizes / bad leading dimensions / unsupported m, R, w
    assert L.dastac_pack_triu_f32(-1, _p(A), 4, _p(B), None) == dastac.EINVAL
    assert L.dastac_pack_triu_f32(8, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_triu_f32(8, _p(A), _p(B), 7, None) == dastac.EINVAL
    assert L.dastac_pack_tet_f32(-3, _p(A), _p(B), None) == dastac.EINVAL
    assert L.dastac_pack_band_f32(4, -1, _p(A), 4, _p(B), None) == dastac.EINVAL
    assert L.dastac_trmv_f32(-1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_trmm_f32(4, 0, _p(A), _p(B), 4, _p(C), 4, None) == dastac.EINVAL
    assert L.dastac_trmm_f32(4, 8, _p(A), _p(B), 7, _p(C), 8, None) == dastac.EINVAL
    assert L.dastac_band_spmv_f32(4, -1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_band_spmv_f32(4, 2 ** 20 + 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_tet_ttv_f32(-1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f32(4, 0, _p(A), _p(B), 4, _p(C), 4, _p(D), 4, None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f32(4, 2 ** 20 + 1, _p(A), _p(B), 2 ** 21, _p(C), 2 ** 21, _p(D), 2 ** 21, None) == dastac.EINVAL
    assert L.dastac_tet_mttkrp_f32(4, 8, _p(A), _p(B), 8, _p(C), 8, _p(D), 7, None) == dastac.EINVAL
    for fn in (L.dastac_trmv_t_f32, L.dastac_trmv_lower_f32, L.dastac_trmv_lower_t_f32, L.dastac_symv_lower_f32):
        assert fn(-1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
        assert fn(524289, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
        assert fn(4, None, _p(B), _p(C), None) == dastac.ENULL
        assert fn(4, _p(A), _p(B), _p(B), None) == dastac.EALIAS
        assert fn(0, None, None, None, None) == dastac.OK
    assert L.dastac_pack_tril_f32(8, _p(A), 7, _p(B), None) == dastac.EINVAL
    assert L.dastac_unpack_tril_f32(4, None, _p(B), 4, None) == dastac.ENULL
    assert L.dastac_symv_f32(-1, _p(A), _p(B), _p(C), None) == dastac.EINVAL
    assert L.dastac_symv_f32(524289, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_symv_f32(4, _p(A), None, _p(C), None) == dastac.ENULL
    assert L.dastac_symv_f32(4, _p(A), _p(B), _p(A + 8), None) == dastac.EALIAS
    assert L.dastac_symv_f32(0, None, None, None, None) == dastac.OK
    assert L.dastac_ttm_ut_f32(-1, 4, 4, _p(A), _p(B), 4, _p(C), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f32(4, 0, 4, _p(A), _p(B), 4, _p(C), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f32(4, 4, 0, _p(A), _p(B), 4, _p(C), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f32(4, 8, 4, _p(A), _p(B), 7, _p(C), None) == dastac.EINVAL
    assert L.dastac_pack_uhc_f32(4, 0, _p(A), _p(B), None) == dastac.EINVAL
    assert L.dastac_ttm_ut_f32(2 ** 20, 2 ** 24, 4, _p(A), _p(B), 2 ** 24, _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_ttm_ut_f32(4, 4, 4, None, _p(B), 4, _p(C), None) == dastac.ENULL
    assert L.dastac_ttm_ut_f32(4, 4, 4, _p(A), _p(B), 4, None, None) == dastac.ENULL
    assert L.dastac_unpack_uhc_f32(4, 2, _p(A), None, None) == dastac.ENULL
    assert L.dastac_ttm_ut_f32(4, 4, 4, _p(A), _p(B), 4, _p(A + 16), None) == dastac.EALIAS
    assert L.dastac_ttm_ut_f32(0, 4, 4, None, None, 4, None, None) == dastac.OK
    # overflow guards
    assert L.dastac_tet_ttv_f32(2 ** 20 + 1, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_trmv_f32(2 ** 31, _p(A), _p(B), _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_pack_tet_f32(2 ** 14, _p(A), _p(B), None) == dastac.EOVERFLOW
    # NULL pointers
    assert L.dastac_trmv_f32(4, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_trmv_f32(4, _p(A), None, _p(C), None) == dastac.ENULL
    assert L.dastac_trmv_f32(4, _p(A), _p(B), None, None) == dastac.ENULL
    assert L.dastac_trmm_f32(4, 2, _p(A), None, 2, _p(C), 2, None) == dastac.ENULL
    assert L.dastac_band_spmv_f32(4, 1, None, _p(B), _p(C), None) == dastac.ENULL
    assert L.dastac_tet_ttv_f32(4, _p(A), _p(B), None, None) == dastac.ENULL
    assert L.dastac_tet_mttkrp_f32(4, 2, _p(A), _p(B), 2, None, 2, _p(D), 2, None) == dastac.ENULL
    assert L.dastac_pack_triu_f32(4, None, 4, _p(B), None) == dastac.ENULL
    assert L.dastac_unpack_tet_f32(4, _p(A), None, None) == dastac.ENULL
    assert L.dastac_unpack_band_f32(4, 1, None, _p(B), 4, None) == dastac.ENULL
    # output overlapping an input
    assert L.dastac_trmv_f32(4, _p(A), _p(B), _p(A + 8), None) == dastac.EALIAS
    assert L.dastac_trmv_f32(4, _p(A), _p(B), _p(B), None) == dastac.EALIAS
    assert L.dastac_trmm_f32(4, 2, _p(A), _p(B), 2, _p(B + 4), 2, None) == dastac.EALIAS
    assert L.dastac_band_spmv_f32(4, 1, _p(A), _p(B), _p(A + 44), None) == dastac.EALIAS
    assert L.dastac_tet_ttv_f32(4, _p(A), _p(B), _p(A + 76), None) == dastac.EALIAS
    assert L.dastac_tet_mttkrp_f32(4, 2, _p(A), _p(B), 2, _p(C), 2, _p(C), 2, None) == dastac.EALIAS
    assert L.dastac_pack_triu_f32(4, _p(A), 4, _p(A + 60), None) == dastac.EALIAS
    # n == 0 is a successful no-op, pointers not needed
    assert L.dastac_trmv_f32(0, None, None, None, None) == dastac.OK
    assert L.dastac_trmm_f32(0, 3, None, None, 3, None, 3, None) == dastac.OK
    assert L.dastac_band_spmv_f32(0, 16, None, None, None, None) == dastac.OK
    assert L.dastac_tet_ttv_f32(0, None, None, None, None) == dastac.OK
    assert L.dastac_tet_mttkrp_f32(0, 4, None, None, 4, None, 4, None, 4, None) == dastac.OK
    assert L.dastac_pack_triu_f32(0, None, 0, None, None) == dastac.OK
    assert L.dastac_unpack_tet_f32(0, None, None, None) == dastac.OK
    assert L.dastac_pack_band_f32(0, 2, None, 0, None, None) == dastac.OK


def test_row_strides_are_bounded_and_views_end_at_their_last_used_element():
    """Row strides above DASTAC_MAX_LD (2^28 elements) are refused before any product with them is formed, and a
    strided matrix occupies the bytes up to the last used element of its last row -- not a whole further row."""
    L = dastac.lib()
    big = 2 ** 28 + 1
    assert L.dastac_trmm_f32(4, 2, _p(A), _p(B), big, _p(C), 2, None) == dastac.EOVERFLOW
    assert L.dastac_trmm_f64(4, 2, _p(A), _p(B), 2, _p(C), big, None) == dastac.EOVERFLOW
    assert L.dastac_symm_f32(4, 2, _p(A), _p(B), 2 ** 62, _p(C), 2, None) == dastac.EOVERFLOW
    assert L.dastac_symm_f64(4, 2, _p(A), _p(B), big, _p(C), 2, None) == dastac.EOVERFLOW
    assert L.dastac_tet_mttkrp_f32(4, 2, _p(A), _p(B), 2, _p(C), big, _p(D), 2, None) == dastac.EOVERFLOW
    assert L.dastac_tet_mttkrp_f64(4, 2, _p(A), _p(B), 2, _p(C), 2, _p(D), 2 ** 62, None) == dastac.EOVERFLOW
    assert L.dastac_pack_triu_f32(4, _p(A), big, _p(B), None) == dastac.EOVERFLOW
    assert L.dastac_unpack_tril_f64(4, _p(A), _p(B), big, None) == dastac.EOVERFLOW
    assert L.dastac_pack_band_f32(4, 1, _p(A), 2 ** 62, _p(B), None) == dastac.EOVERFLOW
    assert L.dastac_pr_a2_f32(10, 4, _p(A), big, _p(B), None) == dastac.EOVERFLOW
    assert L.dastac_ttm_ut_f32(4, 4, 4, _p(A), _p(B), big, _p(C), None) == dastac.EOVERFLOW
    assert L.dastac_pack_subtri_f32(8, 4, _p(A), big, _p(B), None) == dastac.EOVERFLOW
    assert L.dastac_pack_leslie_f64(8, _p(A), big, _p(B), _p(C), None) == dastac.EOVERFLOW
    # C is 4 x 2 with row stride 8: its last used element ends at byte (3*8+2)*4 = 104, so an input whose
    # range begins before that byte overlaps it (the accepting case, an input that begins AT byte 104, needs
    # real memory and is in the GPU tests)
    assert L.dastac_trmm_f32(4, 2, _p(A), _p(B + 100), 2, _p(B), 8, None) == dastac.EALIAS
    assert L.dastac_tet_mttkrp_f32(4, 2, _p(A), _p(B + 100), 2, _p(C), 2, _p(B), 8, None) == dastac.EALIAS


def test_stream_sum_rejects_bad_arguments():
    L = dastac.lib()
    assert L.dastac_stream_sum_f32(-1, _p(A), _p(B), 4, None) == dastac.EINVAL
    assert L.dastac_stream_sum_f32(16, _p(A), _p(B), 0, None) == dastac.EINVAL
    assert L.dastac_stream_sum_f32(16, _p(A), _p(B), 2 ** 24 + 1, None) == dastac.EINVAL
    assert L.dastac_stream_sum_f32(2 ** 40 + 1, _p(A), _p(B), 4, None) == dastac.EOVERFLOW
    assert L.dastac_stream_sum_f32(16, None, _p(B), 4, None) == dastac.ENULL
    assert L.dastac_stream_sum_f32(16, _p(A), None, 4, None) == dastac.ENULL
    assert L.dastac_stream_sum_f32(16, _p(A), _p(A + 32), 4, None) == dastac.EALIAS
