"""The library keeps no mutable state of its own: calls issued from several host threads, each on a stream of
its own (all at the default priority), must not disturb one another."""
import threading

import numpy as np
import pytest

from paper_2407_13726_amd import inputs

pytestmark = pytest.mark.gpu


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


def test_concurrent_host_threads_on_their_own_streams(gpu, oracle):
    torch, d, up, down = gpu.torch, gpu.d, gpu.up, gpu.down
    n, m, nt, R, ns, Np, dp = 700, 48, 80, 32, 1500, 4000, 50
    U, B = inputs.small_int(9500, -2, 2, tri(n)), inputs.small_int(9501, -2, 2, n, m)
    A, Bf, Cf = inputs.small_int(9502, -2, 2, tet(nt)), inputs.small_int(9503, -2, 2, nt, R), inputs.small_int(9504, -2, 2, nt, R)
    Us, xs = inputs.small_int(9505, -2, 2, tri(ns)), inputs.small_int(9506, -2, 2, ns)
    Bp = inputs.small_int(9507, -2, 2, Np, dp)
    want = [oracle.trmm(n, m, U, B)[0], oracle.tet_mttkrp(nt, R, A, Bf, Cf)[0], oracle.symv(ns, Us, xs)[0],
            oracle.pr_a3(Bp)[0]]
    gU, gB, gA, gBf, gCf, gUs, gxs, gBp = (up(a) for a in (U, B, A, Bf, Cf, Us, xs, Bp))
    outs = [gpu.empty(n, m), gpu.empty(nt, R), gpu.empty(ns), gpu.empty(tet(dp))]
    calls = [lambda st: d.trmm_f32(n, m, gU, gB, m, outs[0], m, stream=st),
             lambda st: d.tet_mttkrp_f32(nt, R, gA, gBf, R, gCf, R, outs[1], R, stream=st),
             lambda st: d.symv_f32(ns, gUs, gxs, outs[2], stream=st),
             lambda st: d.pr_a3_f32(Np, dp, gBp, dp, outs[3], stream=st)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in calls]
    errors = []

    def worker(q):
        try:
            for _ in range(25):
                calls[q](streams[q])
            streams[q].synchronize()
        except Exception as e:  # reported by the main thread
            errors.append((q, repr(e)))

    threads = [threading.Thread(target=worker, args=(q,)) for q in range(len(calls))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for q, t in enumerate(outs):
        assert down(t).tobytes() == want[q].tobytes(), "call %d" % q
