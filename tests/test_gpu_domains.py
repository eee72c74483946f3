"""GPU parity for the strided-band, sub-triangular and Leslie structures (Section 6.4; Table 2,
SpMV_L): the HIP library through its C ABI against the CPU oracle on the same seeded inputs.

Bars as everywhere: copied values bit-exact; floating outputs within 1e-4 * sum|products| of the
oracle per element; bit-exact on small-integer inputs, where every partial sum is exact in fp32.
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


# ------------------------------------------------------------- strided band ----

@pytest.mark.parametrize("n,w,s,ld", [(1, 1, 1, 1), (9, 1, 3, 12), (300, 1, 1, 300), (300, 1, 64, 300),
                                      (513, 2, 100, 520), (257, 1, 400, 257), (64, 0, 5, 64)])
def test_pack_unpack_sband_bit_exact(gpu, oracle, n, w, s, ld):
    D = inputs.uniform(1200 + n + s, n, ld)
    want = oracle.pack_sband(np.ascontiguousarray(D[:, :n]), w, s)
    dP = gpu.empty((2 * w + 1) * n)
    gpu.d.pack_sband_f32(n, w, s, gpu.up(D), ld, dP)
    assert gpu.down(dP).tobytes() == want.tobytes()
    dU = gpu.empty(n, ld)
    gpu.d.unpack_sband_f32(n, w, s, dP, dU, ld)
    U = gpu.down(dU)
    assert U[:, :n].tobytes() == oracle.unpack_sband(n, w, s, want).tobytes()
    assert np.isnan(U[:, n:]).all()


@pytest.mark.parametrize("n,w,s", [(1, 1, 1), (2, 1, 1), (255, 1, 1), (1000, 1, 7), (4099, 1, 4096), (4099, 1, 5000),
                                   (65536, 1, 1), (65536, 1, 256), (65536, 1, 65536), (3000, 3, 17), (3000, 0, 9),
                                   (777, 16, 40), (900, 70, 3)])
def test_sband_spmv_parity(gpu, oracle, n, w, s):
    D, x = inputs.band_normal(1210 + n + s, n, w), inputs.normal(1211 + n, n)
    want, scale = oracle.sband_spmv(n, w, s, D.ravel(), x)
    y = gpu.empty(n)
    gpu.d.sband_spmv_f32(n, w, s, gpu.up(D.ravel()), gpu.up(x), y)
    assert_within(gpu.down(y), want, scale, "sband n=%d w=%d s=%d" % (n, w, s))


@pytest.mark.parametrize("n,w,s", [(2100, 1, 33), (2100, 2, 600), (500, 1, 1)])
def test_sband_spmv_ignores_padding_and_is_exact_on_integers(gpu, oracle, n, w, s):
    D = inputs.band_normal(1220 + n, n, w, kind="small_int")
    x = inputs.small_int(1221 + n, -3, 3, n)
    want, _ = oracle.sband_spmv(n, w, s, D.ravel(), x)
    i = np.arange(n)
    for d in range(-w, w + 1):  # poison every padding slot
        D[d + w, (i + d * s < 0) | (i + d * s >= n)] = np.nan
    y = gpu.empty(n)
    gpu.d.sband_spmv_f32(n, w, s, gpu.up(D.ravel()), gpu.up(x), y)
    assert gpu.down(y).tobytes() == want.tobytes()


def test_sband_unit_stride_equals_band(gpu):
    n, w = 5000, 4
    D, x = inputs.band_normal(1230, n, w), inputs.normal(1231, n)
    dD, dx, y1, y2 = gpu.up(D.ravel()), gpu.up(x), gpu.empty(n), gpu.empty(n)
    gpu.d.sband_spmv_f32(n, w, 1, dD, dx, y1)
    gpu.d.band_spmv_f32(n, w, dD, dx, y2)
    assert np.allclose(gpu.down(y1), gpu.down(y2), rtol=1e-5, atol=1e-5)


# ----------------------------------------------------------- sub-triangular ----

@pytest.mark.parametrize("N,k,ld", [(1, 0, 1), (1, 1, 1), (40, 0, 40), (40, 13, 48), (300, 300, 300), (700, 257, 704)])
def test_pack_unpack_subtri_bit_exact(gpu, oracle, N, k, ld):
    D = inputs.uniform(1300 + N + k, N, ld)
    want = oracle.pack_subtri(np.ascontiguousarray(D[:, :N]), k)
    dP = gpu.empty(max(tri(k), 1))
    gpu.d.pack_subtri_f32(N, k, gpu.up(D), ld, dP)
    assert gpu.down(dP)[: tri(k)].tobytes() == want.tobytes()
    dU = gpu.empty(N, ld)
    gpu.d.unpack_subtri_f32(N, k, dP, dU, ld)
    U = gpu.down(dU)
    assert U[:, :N].tobytes() == oracle.unpack_subtri(N, k, want).tobytes()
    assert np.isnan(U[:, N:]).all()


@pytest.mark.parametrize("N,k", [(1, 0), (1, 1), (50, 0), (50, 1), (333, 100), (1000, 1000), (2048, 64), (2048, 511),
                                 (4099, 4097), (9000, 8500), (300000, 100)])
def test_subtri_spmv_parity(gpu, oracle, N, k):
    Ap, x = inputs.uniform(1310 + N + k, max(tri(k), 1)), inputs.normal(1311 + N, N)
    want, scale = oracle.subtri_spmv(N, k, Ap[: tri(k)], x)
    y = gpu.empty(N)
    gpu.d.subtri_spmv_f32(N, k, gpu.up(Ap), gpu.up(x), y)
    got = gpu.down(y)
    assert_within(got, want, scale, "subtri N=%d k=%d" % (N, k))
    assert np.all(got[k:] == 0)


def test_subtri_spmv_exact_on_integers(gpu, oracle):
    N, k = 1500, 777
    Ap, x = inputs.small_int(1320, -3, 3, tri(k)), inputs.small_int(1321, -3, 3, N)
    want, _ = oracle.subtri_spmv(N, k, Ap, x)
    y = gpu.empty(N)
    gpu.d.subtri_spmv_f32(N, k, gpu.up(Ap), gpu.up(x), y)
    assert gpu.down(y).tobytes() == want.tobytes()


# ------------------------------------------------------------------- Leslie ----

@pytest.mark.parametrize("n,ld", [(1, 1), (2, 2), (33, 40), (300, 300), (1025, 1030)])
def test_pack_unpack_leslie_bit_exact(gpu, oracle, n, ld):
    D = inputs.uniform(1400 + n, n, ld)
    R, S = oracle.pack_leslie(np.ascontiguousarray(D[:, :n]))
    dR, dS = gpu.empty(n), gpu.empty(max(n - 1, 1))
    gpu.d.pack_leslie_f32(n, gpu.up(D), ld, dR, dS)
    assert gpu.down(dR).tobytes() == R.tobytes()
    assert gpu.down(dS)[: n - 1].tobytes() == S.tobytes()
    dU = gpu.empty(n, ld)
    gpu.d.unpack_leslie_f32(n, dR, dS, dU, ld)
    U = gpu.down(dU)
    assert U[:, :n].tobytes() == oracle.unpack_leslie(n, R, S).tobytes()
    assert np.isnan(U[:, n:]).all()


@pytest.mark.parametrize("n", [1, 2, 3, 255, 256, 257, 1024, 4097, 100000, 1048577, 5000011])
def test_leslie_spmv_parity(gpu, oracle, n):
    R, S, x = inputs.normal(1410 + n, n), inputs.uniform(1411 + n, max(n - 1, 1)), inputs.normal(1412 + n, n)
    want, scale = oracle.leslie_spmv(n, R, S[: n - 1], x)
    y = gpu.empty(n)
    gpu.d.leslie_spmv_f32(n, gpu.up(R), gpu.up(S), gpu.up(x), y)
    got = gpu.down(y)
    assert_within(got, want, scale, "leslie n=%d" % n)
    # every output but the first is one product: exactly rounded
    assert got[1:].tobytes() == want[1:].tobytes()


def test_leslie_spmv_exact_on_integers_and_repeatable_call(gpu, oracle):
    n = 70001
    R, S, x = inputs.small_int(1420, -3, 3, n), inputs.small_int(1421, -3, 3, n - 1), inputs.small_int(1422, -3, 3, n)
    want, _ = oracle.leslie_spmv(n, R, S, x)
    y = gpu.empty(n)
    dR, dS, dx = gpu.up(R), gpu.up(S), gpu.up(x)
    for _ in range(2):  # the second call must not add onto the first call's y(0)
        gpu.d.leslie_spmv_f32(n, dR, dS, dx, y)
        assert gpu.down(y).tobytes() == want.tobytes()


# ------------------------------------------ polynomial-regression tensors ----

@pytest.mark.parametrize("N,d,ld", [(1, 1, 1), (5, 3, 3), (100, 64, 64), (333, 65, 70), (40, 200, 200), (1000, 130, 130),
                                    (20000, 64, 64), (5000, 257, 260), (31, 129, 129)])
def test_pr_a2_parity(gpu, oracle, N, d, ld):
    B = inputs.normal(1800 + N + d, N, ld)
    want, scale = oracle.pr_a2(np.ascontiguousarray(B[:, :d]))
    out = gpu.empty(tri(d))
    gpu.d.pr_a2_f32(N, d, gpu.up(B), ld, out)
    assert_within(gpu.down(out), want, scale, "pr_a2 N=%d d=%d" % (N, d))


@pytest.mark.parametrize("N,d,ld", [(1, 1, 1), (5, 3, 3), (100, 33, 33), (300, 64, 64), (333, 65, 70), (2000, 70, 70),
                                    (40, 130, 130), (600, 129, 129)])
def test_pr_a3_parity(gpu, oracle, N, d, ld):
    B = inputs.normal(1810 + N + d, N, ld)
    want, scale = oracle.pr_a3(np.ascontiguousarray(B[:, :d]))
    out = gpu.empty(tet(d))
    gpu.d.pr_a3_f32(N, d, gpu.up(B), ld, out)
    assert_within(gpu.down(out), want, scale, "pr_a3 N=%d d=%d" % (N, d))


@pytest.mark.parametrize("N,d", [(300, 150), (3000, 40)])  # one share of the samples / several shares with atomics
def test_pr_tensors_exact_on_integers(gpu, oracle, N, d):
    B = inputs.small_int(1820 + N, -2, 2, N, d)
    dB = gpu.up(B)
    w2, _ = oracle.pr_a2(B)
    w3, _ = oracle.pr_a3(B)
    o2, o3 = gpu.empty(tri(d)), gpu.empty(tet(d))
    for _ in range(2):  # a second call must overwrite, not add onto, the first call's result
        gpu.d.pr_a2_f32(N, d, dB, d, o2)
        gpu.d.pr_a3_f32(N, d, dB, d, o3)
        assert gpu.down(o2).tobytes() == w2.tobytes()
        assert gpu.down(o3).tobytes() == w3.tobytes()


def test_pr_tensors_without_samples_are_zero(gpu):
    d = 37
    o2, o3 = gpu.empty(tri(d)), gpu.empty(tet(d))
    gpu.d.pr_a2_f32(0, d, None, d, o2)
    gpu.d.pr_a3_f32(0, d, None, d, o3)
    assert not gpu.down(o2).any() and not gpu.down(o3).any()
