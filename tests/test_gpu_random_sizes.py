"""Seeded random sizes through every device entry point, against the oracle: shapes that no
hand-picked case names (odd orders, ragged tiles, widths and strides in odd combinations)."""
import random

import numpy as np
import pytest

from paper_2407_13726_amd import inputs

pytestmark = pytest.mark.gpu


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


@pytest.mark.parametrize("seed0", [11, 12, 13])
def test_random_sizes_match_the_oracle(gpu, oracle, seed0):
    d, up, down = gpu.d, gpu.up, gpu.down
    nan = gpu.empty
    nan64 = lambda *s: gpu.torch.full(s, float("nan"), dtype=gpu.torch.float64, device=gpu.dev)
    fails = []

    def check(name, args, got, want, scale, tol=1e-4):
        got = np.asarray(got, dtype=np.float64).ravel()
        want = np.asarray(want, dtype=np.float64).ravel()
        scale = np.asarray(scale).ravel()
        if not (np.isfinite(got).all() and (np.abs(got - want) <= tol * scale + 1e-300).all()):
            fails.append((name, args))

    rng = random.Random(seed0)
    reps = 6
    seed = 7000 + 1000 * seed0
    for it in range(reps):
        seed += 40
        n = rng.choice([rng.randint(1, 70), rng.randint(70, 700), rng.randint(700, 2600)])
        Up, x = inputs.uniform(seed, tri(n)), inputs.normal(seed+1, n)
        dU, dx = up(Up), up(x)
        y = nan(n); d.trmv_f32(n, dU, dx, y); check("trmv", n, down(y), *oracle.trmv(n, Up, x))
        for name, lower, mode in (("symv", 0, 2), ("trmv_t", 0, 1), ("trmv_lower", 1, 0), ("trmv_lower_t", 1, 1), ("symv_lower", 1, 2)):
            y = nan(n); getattr(d, name + "_f32")(n, dU, dx, y); check(name, n, down(y), *oracle.trimv(n, Up, x, lower=bool(lower), mode=mode))
        N = n + rng.randint(0, 300); xN = inputs.normal(seed+2, N)
        y = nan(N); d.subtri_spmv_f32(N, n, dU, up(xN), y); check("subtri", (N, n), down(y), *oracle.subtri_spmv(N, n, Up, xN))
        U64, x64 = inputs.uniform64(seed+3, tri(n)), inputs.uniform64(seed+4, n)
        y = nan64(n); d.trmv_f64(n, up(U64), up(x64), y); check("trmv_f64", n, down(y), *oracle.trmv_f64(n, U64, x64), tol=1e-12)
        for name, lower, mode in (("symv", 0, 2), ("trmv_t", 0, 1), ("trmv_lower", 1, 0), ("trmv_lower_t", 1, 1), ("symv_lower", 1, 2)):
            y = nan64(n); getattr(d, name + "_f64")(n, up(U64), up(x64), y); check(name + "_f64", n, down(y), *oracle.trimv_f64(n, U64, x64, lower=bool(lower), mode=mode), tol=1e-12)
        xN64 = inputs.uniform64(seed+25, N)
        y = nan64(N); d.subtri_spmv_f64(N, n, up(U64), up(xN64), y); check("subtri_f64", (N, n), down(y), *oracle.subtri_spmv_f64(N, n, U64, xN64), tol=1e-12)
        # matrix right-hand sides
        n2 = rng.choice([rng.randint(1, 100), rng.randint(100, 600)]); m = rng.choice([1, rng.randint(2, 40), rng.randint(40, 300)])
        Up2, B = inputs.uniform(seed+5, tri(n2)), inputs.uniform(seed+6, n2, m)
        C = nan(n2, m); d.trmm_f32(n2, m, up(Up2), up(B), m, C, m); check("trmm", (n2, m), down(C), *oracle.trmm(n2, m, Up2, B))
        C = nan(n2, m); d.symm_f32(n2, m, up(Up2), up(B), m, C, m); check("symm", (n2, m), down(C), *oracle.symm(n2, m, Up2, B))
        U642, B64 = inputs.uniform64(seed+7, tri(n2)), inputs.uniform64(seed+8, n2, m)
        C = nan64(n2, m); d.trmm_f64(n2, m, up(U642), up(B64), m, C, m); check("trmm_f64", (n2, m), down(C), *oracle.trmm_f64(n2, m, U642, B64), tol=1e-12)
        # tall triangles with few or some columns: the streaming kernel, or shares of the k range
        n3 = rng.randint(1024, 3300); m3 = rng.choice([1, rng.randint(2, 64), rng.randint(65, 140)])
        Up3, B3 = inputs.uniform(seed+30, tri(n3)), inputs.uniform(seed+31, n3, m3)
        C = nan(n3, m3); d.trmm_f32(n3, m3, up(Up3), up(B3), m3, C, m3); got3 = down(C)
        if not np.isfinite(got3).all():
            fails.append(("trmm tall: non-finite", (n3, m3)))
        for lo in (0, rng.randint(0, n3 - 20), n3 - 20):
            want, scale = oracle.trmm(n3, m3, Up3, B3, rows=(lo, lo + 20))
            check("trmm tall", (n3, m3, lo), got3[lo:lo+20], want[lo:lo+20], scale[lo:lo+20])
        # band family
        nb = rng.choice([rng.randint(1, 300), rng.randint(300, 20000)]); w = rng.choice([0, 1, 2, 4, 8, 16, rng.randint(0, 64), rng.randint(65, 150)]); s = rng.choice([1, 2, rng.randint(1, max(1, nb)), nb + 5])
        D, xb = inputs.band_normal(seed+9, nb, w), inputs.normal(seed+10, nb)
        y = nan(nb); d.band_spmv_f32(nb, w, up(D.ravel()), up(xb), y); check("band", (nb, w), down(y), *oracle.band_spmv(nb, w, D.ravel(), xb))
        y = nan(nb); d.sband_spmv_f32(nb, w, s, up(D.ravel()), up(xb), y); check("sband", (nb, w, s), down(y), *oracle.sband_spmv(nb, w, s, D.ravel(), xb))
        D64 = inputs.uniform64(seed+11, 2*w+1, nb); xb64 = inputs.uniform64(seed+12, nb)
        y = nan64(nb); d.band_spmv_f64(nb, w, up(D64.ravel()), up(xb64), y); check("band_f64", (nb, w), down(y), *oracle.band_spmv_f64(nb, w, D64.ravel(), xb64), tol=1e-12)
        y = nan64(nb); d.sband_spmv_f64(nb, w, s, up(D64.ravel()), up(xb64), y); check("sband_f64", (nb, w, s), down(y), *oracle.sband_spmv_f64(nb, w, s, D64.ravel(), xb64), tol=1e-12)
        nl = rng.choice([rng.randint(1, 600), rng.randint(600, 300000)])
        R_, S_, xl = inputs.normal(seed+13, nl), inputs.uniform(seed+14, max(nl-1, 1)), inputs.normal(seed+15, nl)
        y = nan(nl); d.leslie_spmv_f32(nl, up(R_), up(S_), up(xl), y); check("leslie", nl, down(y), *oracle.leslie_spmv(nl, R_, S_[:nl-1], xl))
        R64, S64, xl64 = inputs.uniform64(seed+26, nl), inputs.uniform64(seed+27, max(nl-1, 1)), inputs.uniform64(seed+28, nl)
        y = nan64(nl); d.leslie_spmv_f64(nl, up(R64), up(S64), up(xl64), y); check("leslie_f64", nl, down(y), *oracle.leslie_spmv_f64(nl, R64, S64[:nl-1], xl64), tol=1e-12)
        # tetrahedron
        nt = rng.choice([rng.randint(1, 40), rng.randint(40, 150)]); R = rng.choice([1, 5, 16, 31, 32, rng.randint(1, 32), rng.randint(33, 80)])
        Ap, v = inputs.uniform(seed+16, tet(nt)), inputs.normal(seed+17, nt)
        M = nan(tri(nt)); d.tet_ttv_f32(nt, up(Ap), up(v), M); check("ttv", nt, down(M), *oracle.tet_ttv(nt, Ap, v))
        A64, v64 = inputs.uniform64(seed+18, tet(nt)), inputs.uniform64(seed+19, nt)
        M = nan64(tri(nt)); d.tet_ttv_f64(nt, up(A64), up(v64), M); check("ttv_f64", nt, down(M), *oracle.tet_ttv_f64(nt, A64, v64), tol=1e-12)
        Bf, Cf = inputs.normal(seed+20, nt, R), inputs.normal(seed+21, nt, R)
        K = nan(nt, R); d.tet_mttkrp_f32(nt, R, up(Ap), up(Bf), R, up(Cf), R, K, R); check("mttkrp", (nt, R), down(K), *oracle.tet_mttkrp(nt, R, Ap, Bf, Cf))
        # running example
        nq, Q, Kk = rng.randint(1, 40), rng.choice([1, 7, 32, 33, 64, 100]), rng.choice([1, 9, 32, 64, 129, 200])
        Bq, Cq = inputs.uniform(seed+22, tri(nq)*Q), inputs.normal(seed+23, Kk, Q)
        Aq = nan(tri(nq)*Kk); d.ttm_ut_f32(nq, Q, Kk, up(Bq), up(Cq), Q, Aq); check("ttm_ut", (nq, Q, Kk), down(Aq), *oracle.ttm_ut(nq, Q, Kk, Bq, Cq))
        # polynomial regression
        Np, dp = rng.choice([rng.randint(1, 50), rng.randint(50, 3000)]), rng.choice([rng.randint(1, 20), rng.randint(20, 90)])
        Bp = inputs.normal(seed+24, Np, dp)
        o2 = nan(tri(dp)); d.pr_a2_f32(Np, dp, up(Bp), dp, o2); check("pr_a2", (Np, dp), down(o2), *oracle.pr_a2(Bp))
        o3 = nan(tet(dp)); d.pr_a3_f32(Np, dp, up(Bp), dp, o3); check("pr_a3", (Np, dp), down(o3), *oracle.pr_a3(Bp))

    assert not fails, fails
