"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on
the same seeded inputs.

Bars (stated here, used everywhere below):
  * packed layouts and every copied value: bit-exact;
  * floating outputs: |gpu - oracle| <= 1e-4 * sum|products| per element, the scale
    coming from the oracle; with small-integer inputs every partial sum is exact in
    fp32, so the GPU must then equal the oracle bit for bit whatever its summation order.
"""
import numpy as np
import pytest

from paper_2407_13726_amd import inputs

pytestmark = pytest.mark.gpu

TOL = 1e-4


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


def assert_within(got, want, scale, what):
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    scale = np.asarray(scale, dtype=np.float64).ravel()
    assert np.isfinite(got).all(), what + ": non-finite output"
    err = np.abs(got - want)
    bad = err > TOL * scale
    assert not bad.any(), "%s: %d of %d outside tolerance, worst err/scale %.3g at %d" % (
        what, bad.sum(), bad.size, (err / np.maximum(scale, 1e-300)).max(), int(np.argmax(err - TOL * scale)))


# ------------------------------------------------------------ pack / unpack ----

@pytest.mark.parametrize("n,ld", [(1, 1), (2, 5), (17, 17), (255, 255), (256, 300), (257, 257), (700, 704)])
def test_pack_unpack_triu_bit_exact(gpu, oracle, n, ld):
    D = inputs.uniform(10 + n, n, ld)
    want = oracle.pack_triu(np.ascontiguousarray(D[:, :n]))
    dD, dP = gpu.up(D), gpu.empty(tri(n))
    gpu.d.pack_triu_f32(n, dD, ld, dP)
    got = gpu.down(dP)
    assert got.tobytes() == want.tobytes()
    dU = gpu.empty(n, ld)
    gpu.d.unpack_triu_f32(n, dP, dU, ld)
    U = gpu.down(dU)
    assert U[:, :n].tobytes() == oracle.unpack_triu(n, want).tobytes()
    assert np.isnan(U[:, n:]).all()  # padding columns of the dense buffer are not touched


@pytest.mark.parametrize("n", [1, 2, 9, 33, 70])
def test_pack_unpack_tet_bit_exact(gpu, oracle, n):
    D = inputs.uniform(20 + n, n, n, n)
    want = oracle.pack_tet(D)
    dP = gpu.empty(tet(n))
    gpu.d.pack_tet_f32(n, gpu.up(D), dP)
    assert gpu.down(dP).tobytes() == want.tobytes()
    dU = gpu.empty(n, n, n)
    gpu.d.unpack_tet_f32(n, dP, dU)
    assert gpu.down(dU).tobytes() == oracle.unpack_tet(n, want).tobytes()


@pytest.mark.parametrize("n,w", [(1, 0), (1, 4), (40, 16), (300, 16), (257, 3), (64, 100)])
def test_pack_unpack_band_bit_exact(gpu, oracle, n, w):
    D = inputs.uniform(30 + n, n, n)
    want = oracle.pack_band(D, w)
    dP = gpu.empty((2 * w + 1) * n)
    gpu.d.pack_band_f32(n, w, gpu.up(D), n, dP)
    assert gpu.down(dP).tobytes() == want.tobytes()
    dU = gpu.empty(n, n)
    gpu.d.unpack_band_f32(n, w, dP, dU, n)
    assert gpu.down(dU).tobytes() == oracle.unpack_band(n, w, want).tobytes()


# --------------------------------------------------------------------- TRMV ----

TRMV_SIZES = [1, 2, 3, 4, 5, 63, 64, 65, 129, 257, 512, 1000, 2049, 4100, 8192, 8193, 11111]


@pytest.mark.parametrize("n", TRMV_SIZES)
def test_trmv_parity(gpu, oracle, n):
    Up, x = inputs.uniform(40 + n, tri(n)), inputs.uniform(41 + n, n)
    want, scale = oracle.trmv(n, Up, x)
    y = gpu.empty(n)
    gpu.d.trmv_f32(n, gpu.up(Up), gpu.up(x), y)
    assert_within(gpu.down(y), want, scale, "trmv n=%d" % n)


@pytest.mark.parametrize("n", [1, 7, 130, 515, 1500, 9000])
def test_trmv_integer_inputs_bit_exact(gpu, oracle, n):
    Up, x = inputs.small_int(50 + n, -3, 3, tri(n)), inputs.small_int(51 + n, -3, 3, n)
    want, _ = oracle.trmv(n, Up, x)
    y = gpu.empty(n)
    gpu.d.trmv_f32(n, gpu.up(Up), gpu.up(x), y)
    assert gpu.down(y).tobytes() == want.tobytes()


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_trmv_and_ttv_zero_factor_drops_a_non_finite_element(gpu, oracle, bad):
    """The documented exception to IEEE propagation (dastac.h, "Non-finite inputs"): in these two kernels a
    product with a zero factor contributes nothing.  An Inf/NaN element of the packed operand that meets a zero
    of x therefore gives the result the oracle computes with that element removed -- while the same element
    meeting a non-zero of x poisons its output as the plain rule says."""
    n = 300
    tri, tet = n * (n + 1) // 2, n * (n + 1) * (n + 2) // 6
    x = inputs.uniform(91, n).copy()
    x[17] = 0.0
    U = inputs.uniform(92, tri).copy()
    # row 5, column 17 (meets the zero) and row 9, column 40 (meets a non-zero)
    at = lambda i, j: i * n - i * (i - 1) // 2 + (j - i)
    U[at(5, 17)] = bad
    U[at(9, 40)] = bad
    clean = U.copy()
    clean[at(5, 17)] = 0.0
    clean[at(9, 40)] = 0.0
    want, scale = oracle.trmv(n, clean, x)
    y = gpu.empty(n)
    gpu.d.trmv_f32(n, gpu.up(U), gpu.up(x), y)
    got = gpu.down(y)
    assert not np.isfinite(got[9])
    keep = np.arange(n) != 9
    assert_within(got[keep], want[keep], scale[keep], "trmv with a dropped non-finite element")
    # the same triangle as slice 0 of a tetrahedron
    A = inputs.uniform(93, tet).copy()
    A[:tri] = U
    cleanA = A.copy()
    cleanA[:tri] = clean
    want, scale = oracle.tet_ttv(n, cleanA, x)
    M = gpu.empty(tri)
    gpu.d.tet_ttv_f32(n, gpu.up(A), gpu.up(x), M)
    got = gpu.down(M)
    assert not np.isfinite(got[9])  # M(0,9) is output 9
    keep = np.arange(tri) != 9
    assert_within(got[keep], want[keep], scale[keep], "tet_ttv with a dropped non-finite element")


def test_trmv_unaligned_operands(gpu, oracle):
    """Pointers that are only 4-byte aligned are accepted."""
    n = 777
    Up, x = inputs.uniform(60, tri(n)), inputs.uniform(61, n)
    want, scale = oracle.trmv(n, Up, x)
    dU, dx, dy = gpu.empty(tri(n) + 3), gpu.empty(n + 3), gpu.empty(n + 3)
    dU[1:1 + tri(n)] = gpu.up(Up)
    dx[3:] = gpu.up(x)
    gpu.d.trmv_f32(n, dU[1:], dx[3:], dy[1:])
    out = gpu.down(dy)
    assert_within(out[1:1 + n], want, scale, "trmv unaligned")
    assert np.isnan(out[0]) and np.isnan(out[1 + n:]).all()


# ---------------------------------------------------------------------- TTV ----

@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 17, 64, 65, 130, 200, 300])
def test_tet_ttv_parity(gpu, oracle, n):
    Ap, v = inputs.uniform(70 + n, tet(n)), inputs.uniform(71 + n, n)
    want, scale = oracle.tet_ttv(n, Ap, v)
    M = gpu.empty(tri(n))
    gpu.d.tet_ttv_f32(n, gpu.up(Ap), gpu.up(v), M)
    assert_within(gpu.down(M), want, scale, "ttv n=%d" % n)


@pytest.mark.parametrize("n", [6, 131, 260])
def test_tet_ttv_integer_inputs_bit_exact(gpu, oracle, n):
    Ap, v = inputs.small_int(80 + n, -3, 3, tet(n)), inputs.small_int(81 + n, -3, 3, n)
    want, _ = oracle.tet_ttv(n, Ap, v)
    M = gpu.empty(tri(n))
    gpu.d.tet_ttv_f32(n, gpu.up(Ap), gpu.up(v), M)
    assert gpu.down(M).tobytes() == want.tobytes()


# --------------------------------------------------------------------- band ----

@pytest.mark.parametrize("n,w", [(1, 0), (1, 16), (5, 16), (31, 16), (33, 16), (1023, 16), (1024, 16), (1025, 16),
                                 (5000, 16), (4099, 0), (3000, 2), (3001, 4), (2500, 8), (2000, 1), (1500, 7),
                                 (900, 64), (10, 40), (700, 65), (2300, 200), (50, 1000)])
def test_band_spmv_parity(gpu, oracle, n, w):
    D, x = inputs.band_normal(90 + n, n, w), inputs.normal(91 + n, n)
    want, scale = oracle.band_spmv(n, w, D.ravel(), x)
    y = gpu.empty(n)
    gpu.d.band_spmv_f32(n, w, gpu.up(D.ravel()), gpu.up(x), y)
    assert_within(gpu.down(y), want, scale, "band n=%d w=%d" % (n, w))


@pytest.mark.parametrize("n,w", [(40, 16), (2100, 16), (300, 5)])
def test_band_spmv_ignores_padding_and_is_exact_on_integers(gpu, oracle, n, w):
    D = inputs.band_normal(100 + n, n, w, kind="small_int")
    x = inputs.small_int(101 + n, -3, 3, n)
    want, _ = oracle.band_spmv(n, w, D.ravel(), x)
    for d in range(-w, w + 1):  # poison every padding slot
        for i in range(n):
            if not 0 <= i + d < n:
                D[d + w, i] = np.nan
    y = gpu.empty(n)
    gpu.d.band_spmv_f32(n, w, gpu.up(D.ravel()), gpu.up(x), y)
    assert gpu.down(y).tobytes() == want.tobytes()


# --------------------------------------------------------------------- TRMM ----

@pytest.mark.parametrize("n,m", [(1, 1), (2, 3), (31, 7), (64, 64), (65, 33), (127, 128), (130, 129), (200, 256),
                                 (300, 40), (515, 70)])
def test_trmm_parity(gpu, oracle, n, m):
    Up, B = inputs.uniform(110 + n, tri(n)), inputs.uniform(111 + n, n, m)
    want, scale = oracle.trmm(n, m, Up, B)
    C = gpu.empty(n, m)
    gpu.d.trmm_f32(n, m, gpu.up(Up), gpu.up(B), m, C, m)
    assert_within(gpu.down(C), want, scale, "trmm n=%d m=%d" % (n, m))


def test_trmm_leading_dimensions_and_integer_exactness(gpu, oracle):
    n, m, ldb, ldc = 150, 37, 45, 41
    Up = inputs.small_int(120, -3, 3, tri(n))
    B = inputs.small_int(121, -3, 3, n, ldb)
    want, _ = oracle.trmm(n, m, Up, np.ascontiguousarray(B[:, :m]))
    C = gpu.empty(n, ldc)
    gpu.d.trmm_f32(n, m, gpu.up(Up), gpu.up(B), ldb, C, ldc)
    out = gpu.down(C)
    assert out[:, :m].tobytes() == want.tobytes()
    assert np.isnan(out[:, m:]).all()


def test_trmm_shares_of_the_k_range_exact_on_integers(gpu, oracle):
    """Few columns on a tall triangle: the k-steps of every row-block pair are cut into shares, one workgroup
    each, which add into a zeroed C.  Integer inputs make the result independent of the order of those adds;
    the padding columns of C must survive the clearing; a second call must not add onto the first."""
    n, m, ldb, ldc = 2100, 40, 44, 43
    Up = inputs.small_int(122, -2, 2, tri(n))
    B = inputs.small_int(123, -2, 2, n, ldb)
    want, _ = oracle.trmm(n, m, Up, np.ascontiguousarray(B[:, :m]))
    C = gpu.empty(n, ldc)
    dU, dB = gpu.up(Up), gpu.up(B)
    for _ in range(2):
        gpu.d.trmm_f32(n, m, dU, dB, ldb, C, ldc)
        out = gpu.down(C)
        assert out[:, :m].tobytes() == want.tobytes()
        assert np.isnan(out[:, m:]).all()


@pytest.mark.parametrize("n,m", [(4200, 130), (4096, 256), (2500, 1), (6000, 128)])
def test_trmm_shares_of_the_k_range_sampled_rows(gpu, oracle, n, m):
    Up, B = inputs.uniform(124 + n, tri(n)), inputs.uniform(125 + n, n, m)
    C = gpu.empty(n, m)
    gpu.d.trmm_f32(n, m, gpu.up(Up), gpu.up(B), m, C, m)
    got = gpu.down(C)
    assert np.isfinite(got).all()
    for lo in (0, 63, n // 3, n // 2 - 30, n - 70):
        hi = min(lo + 70, n)
        want, scale = oracle.trmm(n, m, Up, B, rows=(lo, hi))
        assert_within(got[lo:hi], want[lo:hi], scale[lo:hi], "trmm n=%d m=%d rows %d..%d" % (n, m, lo, hi))


@pytest.mark.parametrize("n,m,ldb,ldc", [(1024, 1, 1, 1), (1200, 1, 3, 2), (1024, 32, 32, 32), (1055, 7, 9, 8), (1500, 33, 40, 35),
                                        (2049, 64, 64, 70), (3000, 20, 20, 20)])
def test_trmm_few_columns_streaming_kernel(gpu, oracle, n, m, ldb, ldc):
    """Tall triangle, at most 64 right-hand sides: the kernel that streams U once per 32 columns and adds
    32x32 pieces into a zeroed C.  Whole result against the oracle; padding of C untouched."""
    Up, B = inputs.uniform(126 + n, tri(n)), inputs.uniform(127 + n, n, ldb)
    want, scale = oracle.trmm(n, m, Up, np.ascontiguousarray(B[:, :m]))
    C = gpu.empty(n, ldc)
    gpu.d.trmm_f32(n, m, gpu.up(Up), gpu.up(B), ldb, C, ldc)
    out = gpu.down(C)
    assert_within(out[:, :m], want, scale, "trmm n=%d m=%d" % (n, m))
    assert np.isnan(out[:, m:]).all()


# ------------------------------------------------------ symmetric (SYMV) ----

@pytest.mark.parametrize("n", [1, 2, 3, 5, 16, 17, 63, 64, 65, 130, 257, 512, 1000, 1025, 2050, 4100, 8192])
def test_symv_parity(gpu, oracle, n):
    Up, x = inputs.uniform(170 + n, tri(n)), inputs.uniform(171 + n, n)
    want, scale = oracle.symv(n, Up, x)
    y = gpu.empty(n)
    gpu.d.symv_f32(n, gpu.up(Up), gpu.up(x), y)
    assert_within(gpu.down(y), want, scale, "symv n=%d" % n)


@pytest.mark.parametrize("n", [1, 7, 130, 515, 1500])
def test_symv_integer_inputs_bit_exact_and_repeatable(gpu, oracle, n):
    Up, x = inputs.small_int(180 + n, -3, 3, tri(n)), inputs.small_int(181 + n, -3, 3, n)
    want, _ = oracle.symv(n, Up, x)
    y = gpu.empty(n)
    dU, dx = gpu.up(Up), gpu.up(x)
    for _ in range(2):  # the output is overwritten, not accumulated into, on every call
        gpu.d.symv_f32(n, dU, dx, y)
        assert gpu.down(y).tobytes() == want.tobytes()


# -------------------------------- every product of one packed triangle with a vector ----

@pytest.mark.parametrize("n,ld", [(1, 1), (2, 5), (17, 17), (255, 255), (256, 300), (257, 257), (700, 704)])
def test_pack_unpack_tril_bit_exact(gpu, oracle, n, ld):
    D = inputs.uniform(190 + n, n, ld)
    want = oracle.pack_tril(np.ascontiguousarray(D[:, :n]))
    dP = gpu.empty(tri(n))
    gpu.d.pack_tril_f32(n, gpu.up(D), ld, dP)
    assert gpu.down(dP).tobytes() == want.tobytes()
    dL = gpu.empty(n, ld)
    gpu.d.unpack_tril_f32(n, dP, dL, ld)
    Lo = gpu.down(dL)
    assert Lo[:, :n].tobytes() == oracle.unpack_tril(n, want).tobytes()
    assert np.isnan(Lo[:, n:]).all()


TRIMV = [("trmv_t_f32", False, 1), ("trmv_lower_f32", True, 0), ("trmv_lower_t_f32", True, 1),
         ("symv_lower_f32", True, 2)]


@pytest.mark.parametrize("fn,lower,mode", TRIMV)
@pytest.mark.parametrize("n", [1, 2, 3, 5, 64, 65, 257, 1000, 1025, 2049, 4100])
def test_triangle_vector_products_parity(gpu, oracle, fn, lower, mode, n):
    Tp, x = inputs.uniform(200 + n + mode, tri(n)), inputs.uniform(201 + n, n)
    want, scale = oracle.trimv(n, Tp, x, lower=lower, mode=mode)
    y = gpu.empty(n)
    getattr(gpu.d, fn)(n, gpu.up(Tp), gpu.up(x), y)
    assert_within(gpu.down(y), want, scale, "%s n=%d" % (fn, n))


@pytest.mark.parametrize("fn,lower,mode", TRIMV)
@pytest.mark.parametrize("n", [7, 515, 2300])
def test_triangle_vector_products_integer_inputs_bit_exact(gpu, oracle, fn, lower, mode, n):
    Tp, x = inputs.small_int(210 + n, -3, 3, tri(n)), inputs.small_int(211 + n, -3, 3, n)
    want, _ = oracle.trimv(n, Tp, x, lower=lower, mode=mode)
    y = gpu.empty(n)
    getattr(gpu.d, fn)(n, gpu.up(Tp), gpu.up(x), y)
    assert gpu.down(y).tobytes() == want.tobytes()


# ------------------------------------------------- running example (TTM_UT) ----

@pytest.mark.parametrize("n,Q", [(1, 1), (3, 2), (9, 5), (17, 256), (24, 300), (40, 64)])
def test_pack_unpack_uhc_bit_exact(gpu, oracle, n, Q):
    D = inputs.uniform(140 + n, n, n, Q)
    want = oracle.pack_uhc(D)
    dP = gpu.empty(tri(n) * Q)
    gpu.d.pack_uhc_f32(n, Q, gpu.up(D), dP)
    assert gpu.down(dP).tobytes() == want.tobytes()
    dD = gpu.empty(n, n, Q)
    gpu.d.unpack_uhc_f32(n, Q, dP, dD)
    assert gpu.down(dD).tobytes() == oracle.unpack_uhc(n, n, Q, want).tobytes()


@pytest.mark.parametrize("n,Q,K", [(1, 1, 1), (2, 3, 5), (5, 32, 128), (11, 33, 129), (12, 31, 127), (16, 64, 64),
                                   (23, 100, 40), (30, 7, 300), (40, 260, 130), (64, 96, 256)])
def test_ttm_ut_parity(gpu, oracle, n, Q, K):
    Bp, C = inputs.uniform(150 + n, tri(n) * Q), inputs.normal(151 + n, K, Q)
    want, scale = oracle.ttm_ut(n, Q, K, Bp, C)
    A = gpu.empty(tri(n) * K)
    gpu.d.ttm_ut_f32(n, Q, K, gpu.up(Bp), gpu.up(C), Q, A)
    assert_within(gpu.down(A), want, scale, "ttm_ut n=%d Q=%d K=%d" % (n, Q, K))


def test_ttm_ut_leading_dimension_integer_exactness_and_identity(gpu, oracle):
    n, Q, K, ldc = 21, 45, 70, 52
    Bp = inputs.small_int(160, -3, 3, tri(n) * Q)
    C = inputs.small_int(161, -3, 3, K, ldc)
    want, _ = oracle.ttm_ut(n, Q, K, Bp, np.ascontiguousarray(C[:, :Q]))
    A = gpu.empty(tri(n) * K + 8)
    gpu.d.ttm_ut_f32(n, Q, K, gpu.up(Bp), gpu.up(C), ldc, A)
    out = gpu.down(A)
    assert out[: tri(n) * K].tobytes() == want.tobytes()
    assert np.isnan(out[tri(n) * K:]).all()  # nothing past the packed result is written
    # C = identity copies the packed operand into the packed result
    Bq = inputs.uniform(162, tri(n) * Q)
    A2 = gpu.empty(tri(n) * Q)
    gpu.d.ttm_ut_f32(n, Q, Q, gpu.up(Bq), gpu.up(np.eye(Q, dtype=np.float32)), Q, A2)
    assert gpu.down(A2).tobytes() == Bq.tobytes()


def test_trmm_operand_that_begins_where_a_strided_output_ends(gpu, oracle):
    """A strided matrix ends at the last used element of its last row: an input placed right behind that element,
    inside what would be the unused tail of the output's last row, does not overlap it."""
    n, m, ldc = 40, 24, 64
    U, B = inputs.uniform(301, n * (n + 1) // 2), inputs.uniform(302, n, m)
    used = (n - 1) * ldc + m
    buf = gpu.torch.full((used + n * m,), float("nan"), dtype=gpu.torch.float32, device=gpu.dev)
    buf[used:] = gpu.up(B.ravel())
    gpu.d.trmm_f32(n, m, gpu.up(U), buf[used:], m, buf[:used], ldc)
    want, scale = oracle.trmm(n, m, U, B)
    got = gpu.down(buf)
    rows = np.stack([got[i * ldc: i * ldc + m] for i in range(n)])
    assert_within(rows, want, scale, "trmm into a strided view")
    assert got[used:].tobytes() == B.ravel().tobytes()


# ------------------------------------------------------------------- MTTKRP ----

@pytest.mark.parametrize("n,R", [(1, 1), (2, 32), (5, 3), (31, 32), (33, 32), (64, 32), (70, 17), (100, 32),
                                 (130, 8), (40, 33), (70, 64), (45, 100)])
def test_tet_mttkrp_parity(gpu, oracle, n, R):
    Ap = inputs.uniform(130 + n, tet(n))
    B, C = inputs.normal(131 + n, n, R), inputs.normal(132 + n, n, R)
    want, scale = oracle.tet_mttkrp(n, R, Ap, B, C)
    M = gpu.empty(n, R)
    gpu.d.tet_mttkrp_f32(n, R, gpu.up(Ap), gpu.up(B), R, gpu.up(C), R, M, R)
    assert_within(gpu.down(M), want, scale, "mttkrp n=%d R=%d" % (n, R))


def test_tet_mttkrp_leading_dimensions_and_integer_exactness(gpu, oracle):
    n, R, ldb, ldc, ldm = 75, 20, 24, 32, 21
    Ap = inputs.small_int(140, -2, 2, tet(n))
    B, C = inputs.small_int(141, -2, 2, n, ldb), inputs.small_int(142, -2, 2, n, ldc)
    want, _ = oracle.tet_mttkrp(n, R, Ap, np.ascontiguousarray(B[:, :R]), np.ascontiguousarray(C[:, :R]))
    M = gpu.empty(n, ldm)
    gpu.d.tet_mttkrp_f32(n, R, gpu.up(Ap), gpu.up(B), ldb, gpu.up(C), ldc, M, ldm)
    out = gpu.down(M)
    assert out[:, :R].tobytes() == want.tobytes()
    assert np.isnan(out[:, R:]).all()


def test_tet_mttkrp_wide_factors_block_by_block_exact_on_integers(gpu, oracle):
    """More than 32 columns: every block of 32 is its own launch on shifted factor pointers; the padding
    of M beyond column R stays untouched."""
    n, R, ldb, ldc, ldm = 66, 70, 72, 70, 75
    Ap = inputs.small_int(143, -2, 2, tet(n))
    B, C = inputs.small_int(144, -2, 2, n, ldb), inputs.small_int(145, -2, 2, n, ldc)
    want, _ = oracle.tet_mttkrp(n, R, Ap, np.ascontiguousarray(B[:, :R]), np.ascontiguousarray(C[:, :R]))
    M = gpu.empty(n, ldm)
    gpu.d.tet_mttkrp_f32(n, R, gpu.up(Ap), gpu.up(B), ldb, gpu.up(C), ldc, M, ldm)
    out = gpu.down(M)
    assert out[:, :R].tobytes() == want.tobytes()
    assert np.isnan(out[:, R:]).all()


# ------------------------------------------------------------- degenerate ----

def test_zero_size_calls_succeed_on_device(gpu):
    d, e = gpu.d, gpu.empty(4)
    d.trmv_f32(0, e, e, e)
    d.tet_ttv_f32(0, e, e, e)
    d.band_spmv_f32(0, 16, e, e, e)
    d.trmm_f32(0, 4, e, e, 4, e, 4)
    d.tet_mttkrp_f32(0, 4, e, e, 4, e, 4, e, 4)
    d.pack_triu_f32(0, e, 0, e)
    gpu.torch.cuda.synchronize()
    assert np.isnan(gpu.down(e)).all()


def test_calls_are_stream_ordered(gpu, oracle):
    """Work is enqueued on the stream that is passed in."""
    torch = gpu.torch
    n = 400
    Up, x = inputs.uniform(150, tri(n)), inputs.uniform(151, n)
    want, scale = oracle.trmv(n, Up, x)
    s = torch.cuda.Stream()
    dU, dx, y = gpu.up(Up), gpu.up(x), gpu.empty(n)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        gpu.d.trmv_f32(n, dU, dx, y)
    s.synchronize()
    assert_within(y.cpu().numpy(), want, scale, "trmv on side stream")


# --------------------------------------------------------------------- SYMM ----

@pytest.mark.parametrize("n,m", [(1, 1), (2, 3), (31, 7), (64, 64), (65, 33), (127, 128), (130, 129), (200, 256),
                                 (300, 40), (515, 70), (1024, 128)])
def test_symm_parity(gpu, oracle, n, m):
    Up, B = inputs.uniform(1600 + n, tri(n)), inputs.uniform(1601 + n, n, m)
    want, scale = oracle.symm(n, m, Up, B)
    C = gpu.empty(n, m)
    gpu.d.symm_f32(n, m, gpu.up(Up), gpu.up(B), m, C, m)
    assert_within(gpu.down(C), want, scale, "symm n=%d m=%d" % (n, m))


def test_symm_leading_dimensions_and_integer_exactness(gpu, oracle):
    n, m, ldb, ldc = 330, 37, 45, 41
    Up = inputs.small_int(1610, -3, 3, tri(n))
    B = inputs.small_int(1611, -3, 3, n, ldb)
    want, _ = oracle.symm(n, m, Up, np.ascontiguousarray(B[:, :m]))
    C = gpu.empty(n, ldc)
    gpu.d.symm_f32(n, m, gpu.up(Up), gpu.up(B), ldb, C, ldc)
    got = gpu.down(C)
    assert got[:, :m].tobytes() == want.tobytes()
    assert np.isnan(got[:, m:]).all()


def test_symm_one_column_equals_symv(gpu, oracle):
    n = 700
    Up, x = inputs.small_int(1620, -3, 3, tri(n)), inputs.small_int(1621, -3, 3, n)
    dU, dx, C, y = gpu.up(Up), gpu.up(x), gpu.empty(n, 1), gpu.empty(n)
    gpu.d.symm_f32(n, 1, dU, dx, 1, C, 1)
    gpu.d.symv_f32(n, dU, dx, y)
    assert gpu.down(C).ravel().tobytes() == gpu.down(y).tobytes()
