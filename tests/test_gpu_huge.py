"""Packed buffers of more than 2^31 elements (8.7 to 9.2 GB in single precision): every position in the
kernels must be a 64-bit quantity.  Operands are drawn on the device from a seeded generator (they are too
large to draw on the host in reasonable time) and copied to the host once for the oracle, which recomputes
windows of outputs: at the start, where the packed position crosses 2^31, and at the end."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 1e-4


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


def within(got, want, scale, what):
    got, want, scale = (np.asarray(a, dtype=np.float64).ravel() for a in (got, want, scale))
    assert np.isfinite(got).all(), what + ": non-finite"
    bad = np.abs(got - want) > TOL * scale
    assert not bad.any(), "%s: %d of %d outside tolerance" % (what, bad.sum(), bad.size)


def device_uniform(gpu, seed, count):
    g = gpu.torch.Generator(device=gpu.dev)
    g.manual_seed(seed)
    t = gpu.torch.empty(count, dtype=gpu.torch.float32, device=gpu.dev)
    t.uniform_(-1.0, 1.0, generator=g)
    return t


def test_triangle_of_more_than_2_31_elements(gpu, oracle):
    n, m = 66000, 32
    assert tri(n) > 2 ** 31
    dU, dx, dB = device_uniform(gpu, 9600, tri(n)), device_uniform(gpu, 9601, n), device_uniform(gpu, 9602, n * m)
    y, ys, C = gpu.empty(n), gpu.empty(n), gpu.empty(n, m)
    gpu.d.trmv_f32(n, dU, dx, y)
    gpu.d.symv_f32(n, dU, dx, ys)
    gpu.d.trmm_f32(n, m, dU, dB, m, C, m)
    gy, gys, gC = gpu.down(y), gpu.down(ys), gpu.down(C)
    assert np.isfinite(gy).all() and np.isfinite(gys).all() and np.isfinite(gC).all()
    U, x, B = dU.cpu().numpy(), dx.cpu().numpy(), dB.cpu().numpy().reshape(n, m)
    del dU
    cross = next(i for i in range(n) if i * n - i * (i - 1) // 2 >= 2 ** 31)  # first row that starts past 2^31
    for lo in (0, 8190, cross - 20, n // 2, n - 40):
        hi = min(lo + 40, n)
        want, scale = oracle.trmv(n, U, x, rows=(lo, hi))
        within(gy[lo:hi], want[lo:hi], scale[lo:hi], "trmv rows %d..%d" % (lo, hi))
    for lo in (0, cross - 2, n - 4):  # a row of the symmetric product gathers from every packed row above it
        hi = min(lo + 4, n)
        want, scale = oracle.symv(n, U, x, rows=(lo, hi))
        within(gys[lo:hi], want[lo:hi], scale[lo:hi], "symv rows %d..%d" % (lo, hi))
    for lo in (0, cross - 3, n - 6):
        hi = min(lo + 6, n)
        want, scale = oracle.trmm(n, m, U, B, rows=(lo, hi))
        within(gC[lo:hi], want[lo:hi], scale[lo:hi], "trmm rows %d..%d" % (lo, hi))


def test_tetrahedron_of_more_than_2_31_elements(gpu, oracle):
    n = 2400
    assert tet(n) > 2 ** 31
    dA, dv = device_uniform(gpu, 9610, tet(n)), device_uniform(gpu, 9611, n)
    R = 32
    dB, dC = device_uniform(gpu, 9612, n * R), device_uniform(gpu, 9613, n * R)
    M, K = gpu.empty(tri(n)), gpu.empty(n, R)
    gpu.d.tet_ttv_f32(n, dA, dv, M)
    gpu.d.tet_mttkrp_f32(n, R, dA, dB, R, dC, R, K, R)
    gM, gK = gpu.down(M), gpu.down(K)
    assert np.isfinite(gM).all() and np.isfinite(gK).all()
    A, v = dA.cpu().numpy(), dv.cpu().numpy()
    Bf, Cf = dB.cpu().numpy().reshape(n, R), dC.cpu().numpy().reshape(n, R)
    del dA
    cross = next(i for i in range(n) if tet(n) - tet(n - i) >= 2 ** 31)  # first slice that starts past 2^31
    for lo in (0, cross - 1, n - 70):
        hi = min(lo + 2, n) if lo < n - 70 else n
        want, scale = oracle.tet_ttv(n, A, v, rows=(lo, hi))
        a, b = lo * n - lo * (lo - 1) // 2, hi * n - hi * (hi - 1) // 2  # packed rows (i, i..n-1) of slices lo..hi-1
        within(gM[a:b], want[a:b], scale[a:b], "ttv slices %d..%d" % (lo, hi))
        want, scale = oracle.tet_mttkrp(n, R, A, Bf, Cf, rows=(lo, hi))
        within(gK[lo:hi], want[lo:hi], scale[lo:hi], "mttkrp slices %d..%d" % (lo, hi))


def test_band_of_more_than_2_31_elements(gpu, oracle):
    n, w = 1 << 26, 16
    assert (2 * w + 1) * n > 2 ** 31
    dD, dx = device_uniform(gpu, 9620, (2 * w + 1) * n), device_uniform(gpu, 9621, n)
    y = gpu.empty(n)
    gpu.d.band_spmv_f32(n, w, dD, dx, y)
    gy = gpu.down(y)
    assert np.isfinite(gy).all()
    D, x = dD.cpu().numpy(), dx.cpu().numpy()
    del dD
    for lo in (0, n // 2 - 20, n - 40):
        hi = min(lo + 40, n)
        want, scale = oracle.band_spmv(n, w, D, x, rows=(lo, hi))
        within(gy[lo:hi], want[lo:hi], scale[lo:hi], "band rows %d..%d" % (lo, hi))
