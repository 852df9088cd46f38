"""Shared test helpers: fixture parsing, tolerance check, dense scatter, a Python Philox."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_blocks(name):
    """Parse a golden text file made of [header] blocks of whitespace-separated numbers."""
    blocks, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                blocks[cur] = []
            else:
                blocks[cur].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def close(a, r, rtol):
    """Element passes if |a-r| <= rtol*|r| + rtol*rms(r)  (rms guards cancellation near 0).
    Returns (ok, worst ratio of error to allowance)."""
    a = np.asarray(a, np.float64)
    r = np.asarray(r, np.float64)
    rms = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
    allow = rtol * np.abs(r) + rtol * rms
    err = np.abs(a - r)
    bad = err > allow
    worst = float(np.max(err / np.maximum(allow, 1e-300))) if r.size else 0.0
    return (not bad.any()) and np.isfinite(a).all(), worst


def assert_close(a, r, rtol, what=""):
    ok, worst = close(a, r, rtol)
    assert ok, "%s: worst error/allowance = %.3g at rtol %g" % (what, worst, rtol)


def scatter_dense(idx, W, d):
    """Dense [m, d] float64 matrix holding W at the positions idx names."""
    m, k = idx.shape
    Wd = np.zeros((m, d), np.float64)
    Wd[np.arange(m)[:, None], idx] = W.astype(np.float64)
    return Wd


# Philox-4x32-10 written with Python integers, independent of the C oracle and of the kernels.
M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def py_philox(ctr, key):
    c0, c1, c2, c3 = ctr
    k0, k1 = key
    for _ in range(10):
        p0, p1 = M0 * c0, M1 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & MASK, (p0 >> 32) ^ c3 ^ k1, p0 & MASK
        k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
    return c0, c1, c2, c3


def py_draw(seed, epoch, j, t, a, d):
    w = py_philox((j, t, a, epoch & MASK), (seed & MASK, ((seed >> 32) ^ (epoch >> 32)) & MASK))
    return (w[0] * d) >> 32
