"""Seeded synthetic inputs shaped like the paper's workloads.

This module only produces inputs (random connectivity, weights, activations, target
lists, schedules).  It holds none of the layer's arithmetic and is the one module that
both the CPU oracle's tests and the HIP path's tests / benchmark draw from.  The public
extreme-classification datasets the paper trains on are not available offline; these
generators reproduce their shapes only (label counts, positives per instance, width of
the penultimate layer), with Zipf label popularity standing in for the long tail.

Every stream is ``numpy.random.Generator(PCG64(1000 * config_index + stream))`` with
streams 0 idx, 1 W, 2 x, 3 targets, 4 redistribution seed.
"""
from collections import namedtuple

import numpy as np

Config = namedtuple(
    "Config",
    "name index m d k b storage positives zipf_a steps fraction period n_x_batches")

# storage: "f32" or "bf16" (x and W stored as bfloat16; everything else float32).
# period: redistribution after every `period`-th step (Tiny: once, after its single step).
CONFIGS = {
    "tiny": Config("tiny", 0, 1024, 64, 8, 16, "f32", 3, None, 1, 0.10, 1, 4),
    "medium": Config("medium", 1, 30938, 1024, 32, 128, "f32", 19, 1.1, 100, 0.10, 10, 4),
    "large": Config("large", 2, 500000, 32768, 32, 256, "f32", 5, 1.1, 100, 0.05, 10, 4),
    "large_wide": Config("large_wide", 3, 670000, 32768, 64, 512, "bf16", 5, 1.1, 100, 0.05, 10, 4),
    "stress": Config("stress", 4, 3000000, 65536, 32, 1024, "f32", 36, 1.05, 50, 0.20, 1, 2),
}

STREAM_IDX, STREAM_W, STREAM_X, STREAM_TARGETS, STREAM_REDIST = range(5)

ADAM = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def custom(m, d, k, b, storage="f32", positives=3, zipf_a=None, index=9, fraction=0.1, name="custom"):
    """A config of arbitrary shape (used by parity tests for ragged / edge sizes)."""
    return Config(name, index, m, d, k, b, storage, positives, zipf_a, 1, fraction, 1, 2)


def rng(cfg, stream, sub=0):
    return np.random.Generator(np.random.PCG64([1000 * cfg.index + stream, sub]))


def f32_to_bf16_bits(a):
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_bits_to_f32(a):
    return (a.astype(np.uint32) << 16).view(np.float32)


def store(a, storage):
    """Put a float32 array in the config's storage type."""
    a = np.ascontiguousarray(a, np.float32)
    return f32_to_bf16_bits(a) if storage == "bf16" else a


def as_f32(a):
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def gen_idx(cfg):
    """k distinct uniform-random columns per row (int32 [m,k]); rows with a repeat are redrawn."""
    r = rng(cfg, STREAM_IDX)
    idx = r.integers(0, cfg.d, size=(cfg.m, cfg.k), dtype=np.int32)
    while True:
        s = np.sort(idx, axis=1)
        bad = np.nonzero((s[:, 1:] == s[:, :-1]).any(axis=1))[0]
        if bad.size == 0:
            return idx
        if cfg.k * 2 > cfg.d:  # dense rows: a permutation prefix is cheaper than rejection
            for j in bad:
                idx[j] = r.permutation(cfg.d)[:cfg.k]
        else:
            idx[bad] = r.integers(0, cfg.d, size=(bad.size, cfg.k), dtype=np.int32)


def gen_W(cfg):
    """W ~ N(0, 1/k) in the config's storage type."""
    w = rng(cfg, STREAM_W).standard_normal((cfg.m, cfg.k), dtype=np.float32)
    w *= np.float32(1.0 / np.sqrt(cfg.k))
    return store(w, cfg.storage)


def gen_x(cfg, batch=0):
    """x = max(0, N(0,1)): about half the entries are exact zeros."""
    x = rng(cfg, STREAM_X, batch).standard_normal((cfg.b, cfg.d), dtype=np.float32)
    np.maximum(x, 0, out=x)
    return store(x, cfg.storage)


def gen_g(cfg, batch=0):
    """A dense upstream gradient of BCE-like magnitude (for testing the backward calls alone)."""
    g = rng(cfg, STREAM_TARGETS, 1000 + batch).standard_normal((cfg.b, cfg.m), dtype=np.float32)
    g *= np.float32(1.0 / cfg.b)
    return g


def _label_sampler(cfg):
    """Returns f(rng, n) -> n label ids drawn with the config's popularity law."""
    if cfg.zipf_a is None:
        return lambda r, n: r.integers(0, cfg.m, size=n, dtype=np.int64)
    ranks = np.arange(1, cfg.m + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-cfg.zipf_a))
    cdf /= cdf[-1]
    perm = rng(cfg, STREAM_TARGETS, 999).permutation(cfg.m)  # head labels are not contiguous ids

    def draw(r, n):
        pos = np.searchsorted(cdf, r.random(n), side="right")
        return perm[np.minimum(pos, cfg.m - 1)]
    return draw


def gen_targets(cfg, batch=0):
    """CSR target lists: `positives` distinct labels per instance.  (tgt_off int64, tgt_lab int32)."""
    r = rng(cfg, STREAM_TARGETS, batch)
    draw = _label_sampler(cfg)
    p = cfg.positives
    lab = np.empty((cfg.b, p), np.int64)
    for i in range(cfg.b):
        got = []
        seen = set()
        while len(got) < p:
            for c in draw(r, p - len(got)):
                c = int(c)
                if c not in seen:
                    seen.add(c)
                    got.append(c)
        lab[i] = got
    off = np.arange(cfg.b + 1, dtype=np.int64) * p
    return off, lab.reshape(-1).astype(np.int32)


def redistribution_seed(cfg):
    return int(rng(cfg, STREAM_REDIST).integers(0, 2 ** 63 - 1))


def is_redistribution_step(cfg, step):
    """step is 1-based; True if a redistribution follows that step."""
    return step % cfg.period == 0
