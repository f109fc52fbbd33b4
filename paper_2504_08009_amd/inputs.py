"""Seeded synthetic test matrices.

Holds none of the method's arithmetic: it only produces the paper's test distribution (Section 4.1),
    x = (rand - 0.5) * exp(phi * randn),
with rand uniform on (0,1) and randn standard normal, independently per element.  The generator is
counter-based: element (i, j) of matrix `which` is a pure function of (seed, which, i + j*rows), so any
sub-block (a few rows of A, a few columns of B) can be regenerated without the rest.  Values are always
produced on the host with numpy, so that the GPU path and the CPU oracle read identical bits.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _unit(bits):
    """top 53 bits -> double in (0, 1)"""
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def values(seed, which, idx, phi):
    """Values for flat element counters idx (uint64 array)."""
    with np.errstate(over="ignore"):
        base = _mix(np.uint64(seed) * _GOLDEN + np.uint64(which + 1) * _M2)
        c = (idx.astype(np.uint64) * np.uint64(3) + np.uint64(1)) * _GOLDEN + base
        u = _unit(_mix(c))
        u1 = _unit(_mix(c + _GOLDEN))
        u2 = _unit(_mix(c + _GOLDEN + _GOLDEN))
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (u - 0.5) * np.exp(phi * z)


def block(seed, which, rows, cols, phi, row_idx=None, col_idx=None):
    """Sub-block (or all) of the rows x cols matrix `which` (0 = A, 1 = B), column-major order.
    row_idx / col_idx: optional 1-D index arrays."""
    r = np.arange(rows, dtype=np.uint64) if row_idx is None else np.asarray(row_idx, dtype=np.uint64)
    c = np.arange(cols, dtype=np.uint64) if col_idx is None else np.asarray(col_idx, dtype=np.uint64)
    out = np.empty((len(r), len(c)), dtype=np.float64, order="F")
    step = max(1, (1 << 21) // max(1, len(r)))

    def work(c0):
        cc = c[c0:c0 + step]
        idx = r[:, None] + cc[None, :] * np.uint64(rows)
        out[:, c0:c0 + step] = values(seed, which, idx, phi)

    starts = list(range(0, len(c), step))
    if len(starts) > 1:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, starts))
    else:
        for s in starts:
            work(s)
    return out


def gemm_inputs(seed, m, n, k, phi):
    """A (m x k) and B (k x n), column-major float64."""
    return block(seed, 0, m, k, phi), block(seed, 1, k, n, phi)


# The workloads named by the benchmark definition: (m, n, k, phi, moduli counts).
CONFIGS = {
    "c1": dict(m=256, n=256, k=256, phi=0.5, N=[14], seed=250408001),
    "c2": dict(m=1024, n=1024, k=1024, phi=0.5, N=list(range(8, 21)), seed=250408002),
    "c3": dict(m=4096, n=4096, k=4096, phi=1.0, N=[14, 16, 18], seed=250408003),
    "c4": dict(m=16384, n=16384, k=16384, phi=0.5, N=[16], seed=250408004),
    "c5a": dict(m=8192, n=8192, k=1024, phi=4.0, N=[18], seed=250408005),
    "c5b": dict(m=8192, n=8192, k=65536, phi=4.0, N=[18], seed=250408006),
}
