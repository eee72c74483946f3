"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Every output element of all five configurations is compared with the oracle; for the two
large contractions the oracle's row-window argument spreads its loops over the host's
cores (windows of output rows, one thread each -- the oracle itself is unchanged), once on
the seeded benchmark inputs at the tolerance and once on small-integer inputs, where every
partial sum is exact in fp32 and the result must equal the oracle's bit for bit whatever
the order of summation.  Bars as in test_gpu_parity.py: 1e-4 * sum|products| per element.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2407_13726_amd import inputs
from paper_2407_13726_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-4


def check(got, want, scale, what):
    got, want, scale = (np.asarray(a, dtype=np.float64).ravel() for a in (got, want, scale))
    assert np.isfinite(got).all(), what + ": non-finite output"
    err = np.abs(got - want)
    assert (err <= TOL * scale).all(), "%s: worst err/scale %.3g" % (what, (err / np.maximum(scale, 1e-300)).max())


def by_windows(fn, rows, width):
    """fn(lo, hi) -> (values, scale) with the rows outside [lo, hi) NaN; the windows of `width` rows run on
    up to 16 host threads (the oracle's C loops run outside the interpreter lock) and are merged."""
    cuts = [(lo, min(lo + width, rows)) for lo in range(0, rows, width)]
    threads = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count() or 1))
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda c: fn(*c), cuts))
    want, scale = parts[0]
    for (lo, hi), (w, sc) in zip(cuts[1:], parts[1:]):
        want[lo:hi], scale[lo:hi] = w[lo:hi], sc[lo:hi]
    assert not np.isnan(scale).any()
    return want, scale


def test_c1_trmv_512(gpu, oracle):
    w = wl.trmv_inputs()
    want, scale = oracle.trmv(w["n"], w["Up"], w["x"])
    y = gpu.empty(w["n"])
    gpu.d.trmv_f32(w["n"], gpu.up(w["Up"]), gpu.up(w["x"]), y)
    check(gpu.down(y), want, scale, "C1 trmv")


def test_c2_trmm_16384_every_element(gpu, oracle):
    w = wl.trmm_inputs()
    n, m = w["n"], w["m"]
    C = gpu.empty(n, m)
    gpu.d.trmm_f32(n, m, gpu.up(w["Up"]), gpu.up(w["B"]), m, C, m)
    got = gpu.down(C)
    want, scale = by_windows(lambda lo, hi: oracle.trmm(n, m, w["Up"], w["B"], rows=(lo, hi)), n, 64)
    check(got, want, scale, "C2 trmm")


def test_c2_trmm_16384_small_integers_bit_exact(gpu, oracle):
    n, m = 16384, 256
    Up = inputs.small_int(2001, -2, 2, n * (n + 1) // 2)
    B = inputs.small_int(2002, -2, 2, n, m)
    C = gpu.empty(n, m)
    gpu.d.trmm_f32(n, m, gpu.up(Up), gpu.up(B), m, C, m)
    got = gpu.down(C)
    want, _ = by_windows(lambda lo, hi: oracle.trmm(n, m, Up, B, rows=(lo, hi)), n, 64)
    assert got.tobytes() == want.tobytes(), "rows that differ: %r" % (np.nonzero((got != want).any(axis=1))[0][:10],)


def test_c3_band_4m(gpu, oracle):
    w = wl.band_inputs()
    n, hw = w["n"], w["w"]
    want, scale = oracle.band_spmv(n, hw, w["D"].ravel(), w["x"])
    y = gpu.empty(n)
    gpu.d.band_spmv_f32(n, hw, gpu.up(w["D"].ravel()), gpu.up(w["x"]), y)
    check(gpu.down(y), want, scale, "C3 band")


def test_c4_ttv_512(gpu, oracle):
    w = wl.ttv_inputs()
    n = w["n"]
    want, scale = oracle.tet_ttv(n, w["Ap"], w["v"])
    M = gpu.empty(n * (n + 1) // 2)
    gpu.d.tet_ttv_f32(n, gpu.up(w["Ap"]), gpu.up(w["v"]), M)
    check(gpu.down(M), want, scale, "C4 ttv")


def test_c5_mttkrp_1024_every_element(gpu, oracle):
    w = wl.mttkrp_inputs()
    n, R = w["n"], w["R"]
    M = gpu.empty(n, R)
    gpu.d.tet_mttkrp_f32(n, R, gpu.up(w["Ap"]), gpu.up(w["B"]), R, gpu.up(w["C"]), R, M, R)
    got = gpu.down(M)
    want, scale = by_windows(lambda lo, hi: oracle.tet_mttkrp(n, R, w["Ap"], w["B"], w["C"], rows=(lo, hi)), n, 8)
    check(got, want, scale, "C5 mttkrp")


def test_c5_mttkrp_1024_small_integers_bit_exact(gpu, oracle):
    # |A| <= 1, |B|, |C| <= 2: a slice's sum stays below 2^24 in magnitude, so every partial sum is exact
    n, R = 1024, 32
    Ap = inputs.small_int(5001, -1, 1, n * (n + 1) * (n + 2) // 6)
    B, C = inputs.small_int(5002, -2, 2, n, R), inputs.small_int(5003, -2, 2, n, R)
    M = gpu.empty(n, R)
    gpu.d.tet_mttkrp_f32(n, R, gpu.up(Ap), gpu.up(B), R, gpu.up(C), R, M, R)
    got = gpu.down(M)
    want, _ = by_windows(lambda lo, hi: oracle.tet_mttkrp(n, R, Ap, B, C, rows=(lo, hi)), n, 8)
    assert got.tobytes() == want.tobytes(), "slices that differ: %r" % (np.nonzero((got != want).any(axis=1))[0][:10],)


def test_mttkrp_f64_768_every_element(gpu, oracle):
    """Double-precision MTTKRP at the size bench.py reports beside the step: every slice order up to 768, so every
    shape of block (full, cut by the diagonal, narrow at the left edge, short at the top) occurs many times."""
    n, R = 768, 32
    Ap = inputs.uniform64(5101, n * (n + 1) * (n + 2) // 6)
    B, C = inputs.uniform64(5102, n, R), inputs.uniform64(5103, n, R)
    M = gpu.torch.full((n, R), float("nan"), dtype=gpu.torch.float64, device=gpu.dev)
    gpu.d.tet_mttkrp_f64(n, R, gpu.up(Ap), gpu.up(B), R, gpu.up(C), R, M, R)
    got = gpu.down(M)
    want, scale = by_windows(lambda lo, hi: oracle.tet_mttkrp_f64(n, R, Ap, B, C, rows=(lo, hi)), n, 8)
    got, want, scale = (np.asarray(a, dtype=np.float64).ravel() for a in (got, want, scale))
    assert np.isfinite(got).all()
    err = np.abs(got - want)
    assert (err <= 1e-12 * scale).all(), "worst err/scale %.3g" % (err / np.maximum(scale, 1e-300)).max()


def test_mttkrp_f64_530_small_integers_bit_exact(gpu, oracle):
    n, R = 530, 29
    Ap = inputs.small_int(5111, -3, 3, n * (n + 1) * (n + 2) // 6).astype(np.float64)
    B, C = inputs.small_int(5112, -3, 3, n, R).astype(np.float64), inputs.small_int(5113, -3, 3, n, R).astype(np.float64)
    M = gpu.torch.full((n, R), float("nan"), dtype=gpu.torch.float64, device=gpu.dev)
    gpu.d.tet_mttkrp_f64(n, R, gpu.up(Ap), gpu.up(B), R, gpu.up(C), R, M, R)
    got = gpu.down(M)
    want, _ = by_windows(lambda lo, hi: oracle.tet_mttkrp_f64(n, R, Ap, B, C, rows=(lo, hi)), n, 8)
    assert got.tobytes() == want.tobytes(), "slices that differ: %r" % (np.nonzero((got != want).any(axis=1))[0][:10],)


def test_running_example_ttm_ut_512_sampled_pairs(gpu, oracle):
    """The paper's running example at the size bench.py reports beside the five configurations."""
    w = wl.ttm_ut_inputs()
    n, Q, K = w["n"], w["Q"], w["K"]
    pairs = n * (n + 1) // 2
    A = gpu.empty(pairs * K)
    gpu.d.ttm_ut_f32(n, Q, K, gpu.up(w["Bp"]), gpu.up(w["C"]), Q, A)
    got = gpu.down(A)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(6)
    for p in sorted({0, 1, 63, 64, 65, 511, 512, pairs - 65, pairs - 64, pairs - 2, pairs - 1}
                    | {int(r) for r in rng.integers(0, pairs, 20)}):
        want, scale = oracle.ttm_ut(n, Q, K, w["Bp"], w["C"], rows=(p, p + 1))
        check(got[p * K: (p + 1) * K], want[p * K: (p + 1) * K], scale[p * K: (p + 1) * K], "ttm_ut pair %d" % p)


def test_symv_8192(gpu, oracle):
    """The symmetric product at the size bench.py reports beside the five configurations."""
    w = wl.symv_inputs()
    want, scale = oracle.symv(w["n"], w["Up"], w["x"])
    y = gpu.empty(w["n"])
    gpu.d.symv_f32(w["n"], gpu.up(w["Up"]), gpu.up(w["x"]), y)
    check(gpu.down(y), want, scale, "symv 8192")



def test_symm_16384_sampled_rows(gpu, oracle):
    """The symmetric product with a matrix right-hand side on the TRMM configuration's operands, at
    the size bench.py reports beside the five configurations."""
    w = wl.trmm_inputs()
    n, m = w["n"], w["m"]
    C = gpu.empty(n, m)
    gpu.d.symm_f32(n, m, gpu.up(w["Up"]), gpu.up(w["B"]), m, C, m)
    got = gpu.down(C)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(8)
    rows = sorted({0, 1, 31, 32, 63, 64, 65, 8191, 8192, n - 65, n - 64, n - 33, n - 32, n - 2, n - 1}
                  | {int(r) for r in rng.integers(0, n, 8)})
    for i in rows:
        want, scale = oracle.symm(n, m, w["Up"], w["B"], rows=(i, i + 1))
        check(got[i], want[i], scale[i], "symm row %d" % i)


@pytest.mark.parametrize("which,N,d", [(2, 100000, 1024), (3, 10000, 256)])
def test_pr_tensors_sampled_positions(gpu, oracle, which, N, d):
    """The polynomial-regression tensors at the sizes bench.py reports beside the five configurations
    (Table 1: first dimension 100000 for the second-order tensor, 10000 for the third-order one)."""
    w = wl.pr_inputs(N, d, which)
    count = d * (d + 1) // 2 if which == 2 else d * (d + 1) * (d + 2) // 6
    out = gpu.empty(count)
    (gpu.d.pr_a2_f32 if which == 2 else gpu.d.pr_a3_f32)(N, d, gpu.up(w["B"]), d, out)
    got = gpu.down(out)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(10 + which)
    starts = sorted({0, 1, d - 2, d, count - 3} | {int(r) for r in rng.integers(0, count - 3, 24)})
    fn = oracle.pr_a2 if which == 2 else oracle.pr_a3
    for p in starts:
        want, scale = fn(w["B"], window=(p, p + 3))
        check(got[p:p + 3], want[p:p + 3], scale[p:p + 3], "pr_a%d position %d" % (which, p))


@pytest.mark.parametrize("which,N,d,f64,samples", [(3, 64, 800, False, 24), (3, 24, 2100, False, 5), (3, 24, 2100, True, 3),
                                                  (2, 200, 2100, True, 24)])
def test_pr_tensors_larger_feature_counts_sampled_positions(gpu, oracle, which, N, d, f64, samples):
    """The launch shapes that only larger d selects: four slices per workgroup of the third-order kernel (fp32,
    d > 768), 64 x 128 tiles (d > 2048), 64 x 128 tiles of the second-order kernel in double precision."""
    t = gpu.torch
    B = inputs.normal(5200 + d + which, N, d)
    if f64:
        B = B.astype(np.float64)
    count = d * (d + 1) // 2 if which == 2 else d * (d + 1) * (d + 2) // 6
    out = t.full((count,), float("nan"), dtype=t.float64 if f64 else t.float32, device=gpu.dev)
    fn = {(2, False): gpu.d.pr_a2_f32, (3, False): gpu.d.pr_a3_f32, (2, True): gpu.d.pr_a2_f64, (3, True): gpu.d.pr_a3_f64}[(which, f64)]
    fn(N, d, gpu.up(B), d, out)
    t.cuda.synchronize()
    assert bool(t.isfinite(out).all())
    orc = {(2, False): oracle.pr_a2, (3, False): oracle.pr_a3, (2, True): oracle.pr_a2_f64, (3, True): oracle.pr_a3_f64}[(which, f64)]
    rng = np.random.default_rng(20 + which + d)
    starts = sorted({0, d - 2, count - 3} | {int(r) for r in rng.integers(0, count - 3, samples)})
    tol = 1e-12 if f64 else TOL
    for p in starts:
        want, scale = orc(B, window=(p, p + 3), compact=True)
        got = out[p:p + 3].cpu().numpy().astype(np.float64)
        assert (np.abs(got - want) <= tol * scale).all(), "position %d: %r against %r" % (p, got, want)


def test_trmm_f64_16384_sampled_rows(gpu, oracle):
    """The double-precision TRMM at the shape bench.py reports beside the step (two shares of the k range per
    row-block pair): sampled rows against the long-double oracle, 1e-12 * sum|products|."""
    w = wl.trmm_f64_inputs()
    n, m = w["n"], w["m"]
    t = gpu.torch
    C = t.full((n, m), float("nan"), dtype=t.float64, device=gpu.dev)
    gpu.d.trmm_f64(n, m, gpu.up(w["Up"]), gpu.up(w["B"]), m, C, m)
    got = gpu.down(C)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(3)
    rows = sorted({0, 1, 63, 64, 8191, 8192, n - 65, n - 64, n - 17, n - 16, n - 1} | {int(r) for r in rng.integers(0, n, 8)})
    for i in rows:
        want, scale = oracle.trmm_f64(n, m, w["Up"], w["B"], rows=(i, i + 1))
        err = np.abs(got[i] - want[i])
        assert (err <= 1e-12 * scale[i]).all(), "trmm_f64 row %d: worst err/scale %.3g" % (i, (err / scale[i]).max())
