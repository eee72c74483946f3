"""The entry points only launch kernels (no allocation, no memset, no synchronisation), so a caller can
record them into a HIP graph.  A step of contractions is captured once and replayed several times with
eager work and synchronisations of the program's own in between; every replay must reproduce the eager
result, and a replay after the inputs were overwritten in place must follow the new inputs."""
import numpy as np
import pytest

from paper_2407_13726_amd import inputs

pytestmark = pytest.mark.gpu


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


def test_captured_step_replays_like_eager(gpu, oracle):
    torch, d, up, down = gpu.torch, gpu.d, gpu.up, gpu.down
    n1, n2, m2, n3, w3, n4, n5, R5, ns, nl = 512, 300, 40, 5000, 16, 90, 70, 32, 700, 3000

    def host_inputs(seed):
        si = lambda *shape: inputs.small_int(seed + len(shape) * 7 + shape[0], -2, 2, *shape)
        return {"U1": si(tri(n1)), "x1": si(n1), "U2": si(tri(n2)), "B2": si(n2, m2),
                "D3": inputs.band_normal(seed + 3, n3, w3, kind="small_int"), "x3": si(n3),
                "A4": si(tet(n4)), "v4": si(n4), "A5": si(tet(n5)), "B5": si(n5, R5), "C5": si(n5, R5 + 1)[:, :R5].copy(),
                "Us": si(tri(ns)), "xs": si(ns), "Rl": si(nl), "Sl": si(nl - 1), "xl": si(nl + 1)[:nl].copy()}

    def expected(h):  # integer inputs: exact whatever the summation order
        return {"y1": oracle.trmv(n1, h["U1"], h["x1"])[0], "C2": oracle.trmm(n2, m2, h["U2"], h["B2"])[0],
                "y3": oracle.band_spmv(n3, w3, h["D3"].ravel(), h["x3"])[0], "M4": oracle.tet_ttv(n4, h["A4"], h["v4"])[0],
                "M5": oracle.tet_mttkrp(n5, R5, h["A5"], h["B5"], h["C5"])[0], "ys": oracle.symv(ns, h["Us"], h["xs"])[0],
                "yl": oracle.leslie_spmv(nl, h["Rl"], h["Sl"], h["xl"])[0]}

    h = host_inputs(9000)
    g = {k: up(v.ravel() if k == "D3" else v) for k, v in h.items()}
    o = {"y1": gpu.empty(n1), "C2": gpu.empty(n2, m2), "y3": gpu.empty(n3), "M4": gpu.empty(tri(n4)),
         "M5": gpu.empty(n5, R5), "ys": gpu.empty(ns), "yl": gpu.empty(nl)}

    def step():
        d.trmv_f32(n1, g["U1"], g["x1"], o["y1"])
        d.trmm_f32(n2, m2, g["U2"], g["B2"], m2, o["C2"], m2)
        d.band_spmv_f32(n3, w3, g["D3"], g["x3"], o["y3"])
        d.tet_ttv_f32(n4, g["A4"], g["v4"], o["M4"])
        d.tet_mttkrp_f32(n5, R5, g["A5"], g["B5"], R5, g["C5"], R5, o["M5"], R5)
        d.symv_f32(ns, g["Us"], g["xs"], o["ys"])           # zero kernel + atomics inside
        d.leslie_spmv_f32(nl, g["Rl"], g["Sl"], g["xl"], o["yl"])  # clears y(0), then one atomic per workgroup

    def check(want, what):
        for k, t in o.items():
            assert down(t).tobytes() == want[k].tobytes(), "%s: %s" % (what, k)

    def poison():
        for t in o.values():
            t.fill_(float("nan"))

    want = expected(h)
    step()
    check(want, "eager")

    graph = torch.cuda.CUDAGraph()
    poison()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for r in range(3):
        poison()
        scratch = torch.randn(1 << 16, device=gpu.dev).sum().item()  # eager work and a synchronisation between replays
        assert np.isfinite(scratch)
        graph.replay()
        check(want, "replay %d" % r)

    # new values in the same buffers: the graph holds addresses, not data
    h2 = host_inputs(9100)
    for k, v in h2.items():
        g[k].copy_(up(v.ravel() if k == "D3" else v))
    want2 = expected(h2)
    for r in range(2):
        poison()
        graph.replay()
        check(want2, "replay on new inputs %d" % r)
    poison()
    step()
    check(want2, "eager on new inputs")


def test_captured_matrix_core_products_replay_like_eager(gpu, oracle):
    """The remaining matrix-core entry points, among them the polynomial-regression tensors, whose launch
    shape depends on a run-time occupancy query and whose split launches clear the output with a fill
    kernel before adding into it."""
    torch, d, up, down = gpu.torch, gpu.d, gpu.up, gpu.down
    N, dd, n, m, nq, Q, K = 3000, 40, 200, 24, 20, 32, 64
    B = inputs.small_int(9200, -2, 2, N, dd)
    U, Bm = inputs.small_int(9201, -2, 2, tri(n)), inputs.small_int(9202, -2, 2, n, m)
    Bq, Cq = inputs.small_int(9203, -2, 2, tri(nq) * Q), inputs.small_int(9204, -2, 2, K, Q)
    want = {"a2": oracle.pr_a2(B)[0], "a3": oracle.pr_a3(B)[0], "sy": oracle.symm(n, m, U, Bm)[0],
            "tt": oracle.ttm_ut(nq, Q, K, Bq, Cq)[0]}
    gB, gU, gBm, gBq, gCq = up(B), up(U), up(Bm), up(Bq), up(Cq)
    o = {"a2": gpu.empty(tri(dd)), "a3": gpu.empty(tet(dd)), "sy": gpu.empty(n, m), "tt": gpu.empty(tri(nq) * K)}

    def step():
        d.pr_a2_f32(N, dd, gB, dd, o["a2"])
        d.pr_a3_f32(N, dd, gB, dd, o["a3"])
        d.symm_f32(n, m, gU, gBm, m, o["sy"], m)
        d.ttm_ut_f32(nq, Q, K, gBq, gCq, Q, o["tt"])

    def check(what):
        for k, t in o.items():
            assert down(t).tobytes() == want[k].tobytes(), "%s: %s" % (what, k)

    step()
    check("eager")
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for r in range(3):
        for t in o.values():
            t.fill_(float("nan"))
        assert np.isfinite(torch.randn(1 << 16, device=gpu.dev).sum().item())
        graph.replay()
        check("replay %d" % r)
