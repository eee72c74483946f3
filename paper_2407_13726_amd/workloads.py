"""The five benchmark workloads (and the running example measured beside them): sizes, seeds, and
FLOP / byte accounting.

Inputs only (host NumPy arrays from ``inputs``); nothing here computes a
contraction or a packed offset.  Config c, tensor t uses stream seed
``20240713*c + t``.  FLOPs follow the paper's convention (Section 6.2:
structure-aware iterations times the additions and multiplications per
iteration); for MTTKRP the factored evaluation the kernel actually performs is
counted (fewer FLOPs than the three-operand convention) and the paper-convention
figure is reported beside it.  Bytes are the algorithmic minimum: every operand
and result moved once.
"""
from __future__ import annotations

from . import inputs


def _seed(c: int, t: int) -> int:
    return 20240713 * c + t


def _tri(n):
    return n * (n + 1) // 2


def _tet(n):
    return n * (n + 1) * (n + 2) // 6


def trmv_inputs(n: int = 512):
    return {"n": n, "Up": inputs.uniform(_seed(1, 0), _tri(n)), "x": inputs.uniform(_seed(1, 1), n)}


def trmm_inputs(n: int = 16384, m: int = 256):
    return {"n": n, "m": m, "Up": inputs.uniform(_seed(2, 0), _tri(n)), "B": inputs.uniform(_seed(2, 1), n, m)}


def band_inputs(n: int = 4194304, w: int = 16):
    return {"n": n, "w": w, "D": inputs.band_normal(_seed(3, 0), n, w), "x": inputs.normal(_seed(3, 1), n)}


def ttv_inputs(n: int = 512):
    return {"n": n, "Ap": inputs.uniform(_seed(4, 0), _tet(n)), "v": inputs.uniform(_seed(4, 1), n)}


def mttkrp_inputs(n: int = 1024, R: int = 32):
    return {"n": n, "R": R, "Ap": inputs.uniform(_seed(5, 0), _tet(n)),
            "B": inputs.normal(_seed(5, 1), n, R), "C": inputs.normal(_seed(5, 2), n, R)}


def ttm_ut_inputs(n: int = 512, Q: int = 256, K: int = 256):
    """The paper's running example (Fig. 3) at a size whose packed operand (134 MB) and packed result
    (134 MB) leave the caches; stream seeds of "config 6"."""
    return {"n": n, "Q": Q, "K": K, "Bp": inputs.uniform(_seed(6, 0), _tri(n) * Q), "C": inputs.normal(_seed(6, 1), K, Q)}


def symv_inputs(n: int = 8192):
    """A symmetric matrix as its packed upper triangle (134 MB), stream seeds of "config 7"."""
    return {"n": n, "Up": inputs.uniform(_seed(7, 0), _tri(n)), "x": inputs.uniform(_seed(7, 1), n)}


def sband_inputs(n: int = 1 << 24, w: int = 1, s: int = 4096):
    """Section 6.4's strided band (main diagonal and the two diagonals at distance s) at a size that
    leaves the caches (the paper's n = 2^16 is 1 MB and stays in L2); stream seeds of "config 8"."""
    return {"n": n, "w": w, "s": s, "D": inputs.uniform(_seed(8, 0), (2 * w + 1) * n), "x": inputs.uniform(_seed(8, 1), n)}


def subtri_inputs(N: int = 1 << 14, k: int = 1 << 13):
    """Section 6.4's sub-triangular structure at the paper's N = 2^14, triangle size k in the middle
    of the range it sweeps; stream seeds of "config 9"."""
    return {"N": N, "k": k, "Ap": inputs.uniform(_seed(9, 0), _tri(k)), "x": inputs.uniform(_seed(9, 1), N)}


def leslie_inputs(n: int = 1 << 24):
    """Table 2's SpMV_L: first row and sub-diagonal, at a size that leaves the caches (the paper
    notes this kernel does not fit its cache either); stream seeds of "config 10"."""
    return {"n": n, "R": inputs.uniform(_seed(10, 0), n), "S": inputs.uniform(_seed(10, 1), n - 1),
            "x": inputs.uniform(_seed(10, 2), n)}


def pr_inputs(N: int, d: int, which: int):
    """Table 1's polynomial-regression kernels: a dense N x d sample matrix (first dimension 100000 for
    the second-order tensor, 10000 for the third-order one); stream seeds of "config 11" and "config 12"."""
    return {"N": N, "d": d, "B": inputs.normal(_seed(9 + which, 0), N, d)}


def f64_inputs():
    """Double-precision operands (the paper's element type) for the three streaming contractions:
    TRMV n=8192, band SpMV n=2097152 w=16, TTV n=512; stream seeds of "config 13"."""
    n1, n3, w3, n4 = 8192, 1 << 21, 16, 512
    return {"trmv": {"n": n1, "Up": inputs.uniform64(_seed(13, 0), _tri(n1)), "x": inputs.uniform64(_seed(13, 1), n1)},
            "band": {"n": n3, "w": w3, "D": inputs.uniform64(_seed(13, 2), (2 * w3 + 1) * n3),
                     "x": inputs.uniform64(_seed(13, 3), n3)},
            "ttv": {"n": n4, "Ap": inputs.uniform64(_seed(13, 4), _tet(n4)), "v": inputs.uniform64(_seed(13, 5), n4)}}


def domains_f64_inputs():
    """Double-precision operands for the symmetric product (n=8192) and for the strided-band
    (n=2^23, w=1, s=4096), sub-triangular (N=2^14, k=2^13) and Leslie (n=2^23) products; stream
    seeds of "config 15"."""
    ns, nb, sb, Nu, ku, nl = 8192, 1 << 23, 4096, 1 << 14, 1 << 13, 1 << 23
    return {"symv": {"n": ns, "Up": inputs.uniform64(_seed(15, 0), _tri(ns)), "x": inputs.uniform64(_seed(15, 1), ns)},
            "sband": {"n": nb, "w": 1, "s": sb, "D": inputs.uniform64(_seed(15, 2), 3 * nb),
                      "x": inputs.uniform64(_seed(15, 3), nb)},
            "subtri": {"N": Nu, "k": ku, "Ap": inputs.uniform64(_seed(15, 4), _tri(ku)),
                       "x": inputs.uniform64(_seed(15, 5), Nu)},
            "leslie": {"n": nl, "R": inputs.uniform64(_seed(15, 6), nl), "S": inputs.uniform64(_seed(15, 7), nl - 1),
                       "x": inputs.uniform64(_seed(15, 8), nl)}}


def trmm_f64_inputs(n: int = 16384, m: int = 256):
    """The TRMM configuration's shape with double operands; stream seeds of "config 14"."""
    return {"n": n, "m": m, "Up": inputs.uniform64(_seed(14, 0), _tri(n)), "B": inputs.uniform64(_seed(14, 1), n, m)}


def accounting(name: str, **kw) -> dict:
    """Useful FLOPs and algorithmic bytes of one launch."""
    if name.endswith("_f64"):  # same counts, eight bytes per element
        a = dict(accounting(name[:-4], **kw))
        a["bytes"] *= 2
        return a
    if name == "trmv":
        n = kw["n"]
        return {"flops": 2 * _tri(n), "bytes": 4 * (_tri(n) + 2 * n)}
    if name == "trmm":
        n, m = kw["n"], kw["m"]
        return {"flops": 2 * _tri(n) * m, "bytes": 4 * (_tri(n) + 2 * n * m)}
    if name == "band":
        n, w = kw["n"], kw["w"]
        inrange = sum(n - abs(d) for d in range(-w, w + 1) if abs(d) < n)
        return {"flops": 2 * inrange, "bytes": 4 * ((2 * w + 1) * n + 2 * n)}
    if name == "ttv":
        n = kw["n"]
        return {"flops": 2 * _tet(n), "bytes": 4 * (_tet(n) + n + _tri(n))}
    if name == "mttkrp":
        n, R = kw["n"], kw["R"]
        return {"flops": 2 * R * _tet(n) + 2 * R * _tri(n), "flops_paper_convention": 3 * R * _tet(n),
                "bytes": 4 * (_tet(n) + 3 * n * R)}
    if name == "symv":  # every unique element is used twice, the diagonal once
        n = kw["n"]
        return {"flops": 2 * n * n, "bytes": 4 * (_tri(n) + 2 * n)}
    if name == "pr_a2":  # one multiply-add per sample and unique output
        N, d = kw["N"], kw["d"]
        return {"flops": 2 * N * _tri(d), "bytes": 4 * (N * d + _tri(d))}
    if name == "pr_a3":  # factored as the kernel executes it: one scaling per (x, i, j>=i), one multiply-add per unique output
        N, d = kw["N"], kw["d"]
        return {"flops": 2 * N * _tet(d) + N * _tri(d), "flops_paper_convention": 3 * N * _tet(d),
                "bytes": 4 * (N * d + _tet(d))}
    if name == "symm":  # every unique element is used twice per column of B, the diagonal once
        n, m = kw["n"], kw["m"]
        return {"flops": 2 * n * n * m, "bytes": 4 * (_tri(n) + 2 * n * m)}
    if name == "ttm_ut":
        n, Q, K = kw["n"], kw["Q"], kw["K"]
        return {"flops": 2 * _tri(n) * Q * K, "bytes": 4 * (_tri(n) * (Q + K) + K * Q)}
    if name == "sband":  # in-range products only; every slot of every diagonal buffer is streamed
        n, w, st = kw["n"], kw["w"], kw["s"]
        inrange = sum(max(n - abs(d) * st, 0) for d in range(-w, w + 1))
        return {"flops": 2 * inrange, "bytes": 4 * ((2 * w + 1) * n + 2 * n)}
    if name == "subtri":
        N, k = kw["N"], kw["k"]
        return {"flops": 2 * _tri(k), "bytes": 4 * (_tri(k) + k + N)}
    if name == "leslie":
        n = kw["n"]
        return {"flops": 2 * n + (n - 1), "bytes": 4 * (n + (n - 1) + 2 * n)}
    raise ValueError(name)
