"""CPU oracle of the uniformly-sparse output layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``usl_oracle.c`` (plain loops, double accumulation).  Nothing in
the product package imports this module; tests, the smoke check and the benchmark's
``cpu_baseline`` leg do.  It imports nothing from the HIP package either.

Arrays are numpy, C-contiguous: ``idx[m,k]`` int32, ``W[m,k]`` float32 (or uint16 holding
bfloat16 bit patterns), ``x[b,d]`` likewise, ``out/g[b,m]`` float32, targets as CSR
(``tgt_off[b+1]`` int64, ``tgt_lab[nnz]`` int32).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "usl_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_sanitized():
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (gcc), as a second library.
    A process that loads it needs the sanitizer runtime preloaded; tests/test_oracle_sanitized.py does that
    in a child process and points USL_ORACLE_LIB at the result."""
    out = os.path.join(_HERE, "liboracle_san.so")
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer", "-shared", "-fPIC", "-o", out, _SRC, "-lm"])
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(os.environ.get("USL_ORACLE_LIB") or build())
        _lib.orc_redistribute.restype = ctypes.c_int64
        _lib.orc_count_bad_rows.restype = ctypes.c_int64
        _lib.orc_draw_column.restype = ctypes.c_int32
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _storage(a):
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("x / W must be float32 or uint16 (bfloat16 bits), got %s" % a.dtype)


def _chk(a, dtype=None):
    assert a.flags["C_CONTIGUOUS"], "array must be C-contiguous"
    if dtype is not None:
        assert a.dtype == dtype, (a.dtype, dtype)
    return a


def num_threads():
    return int(lib().orc_num_threads())


def forward(x, idx, W):
    """Algorithm 1: out[i,j] = sum_t W[j,t] * x[i, idx[j,t]]."""
    _chk(x), _chk(idx, np.int32), _chk(W)
    st = _storage(x)
    assert _storage(W) == st
    b, d = x.shape
    m, k = idx.shape
    out = np.empty((b, m), np.float32)
    lib().orc_forward(_p(x), _p(idx), _p(W), _p(out), ctypes.c_int64(m), ctypes.c_int32(d),
                      ctypes.c_int32(k), ctypes.c_int32(b), ctypes.c_int(st))
    return out


def backward_weight(g, x, idx):
    """Algorithm 3: grad_W[j,t] = sum_i g[i,j] * x[i, idx[j,t]]."""
    _chk(g, np.float32), _chk(x), _chk(idx, np.int32)
    b, d = x.shape
    m, k = idx.shape
    assert g.shape == (b, m)
    gw = np.empty((m, k), np.float32)
    lib().orc_backward_weight(_p(g), _p(x), _p(idx), _p(gw), ctypes.c_int64(m), ctypes.c_int32(d),
                              ctypes.c_int32(k), ctypes.c_int32(b), ctypes.c_int(_storage(x)))
    return gw


def backward_input(g, idx, W, d):
    """Algorithm 2: grad_x[i,c] = sum_{(j,t): idx[j,t]=c} W[j,t] * g[i,j]."""
    _chk(g, np.float32), _chk(idx, np.int32), _chk(W)
    b, m = g.shape
    k = idx.shape[1]
    assert idx.shape[0] == m
    gx = np.empty((b, d), np.float32)
    lib().orc_backward_input(_p(g), _p(idx), _p(W), _p(gx), ctypes.c_int64(m), ctypes.c_int32(d),
                             ctypes.c_int32(k), ctypes.c_int32(b), ctypes.c_int(_storage(W)))
    return gx


def bce_loss_grad(out, tgt_off, tgt_lab, scale):
    """Sparse-target BCE summed over labels; returns (loss as python float (double), g)."""
    _chk(out, np.float32), _chk(tgt_off, np.int64), _chk(tgt_lab, np.int32)
    b, m = out.shape
    g = np.empty_like(out)
    loss = ctypes.c_double(0.0)
    lib().orc_bce_loss_grad(_p(out), _p(tgt_off), _p(tgt_lab), ctypes.c_float(scale), _p(g),
                            ctypes.byref(loss), ctypes.c_int64(m), ctypes.c_int32(b))
    return loss.value, g


def sqh_loss_grad(out, tgt_off, tgt_lab, scale):
    """Sparse-target squared hinge summed over labels; returns (loss (double), g)."""
    _chk(out, np.float32), _chk(tgt_off, np.int64), _chk(tgt_lab, np.int32)
    b, m = out.shape
    g = np.empty_like(out)
    loss = ctypes.c_double(0.0)
    lib().orc_sqh_loss_grad(_p(out), _p(tgt_off), _p(tgt_lab), ctypes.c_float(scale), _p(g),
                            ctypes.byref(loss), ctypes.c_int64(m), ctypes.c_int32(b))
    return loss.value, g


def forward_rows(x, idx, W, rows):
    """Scores of the labels listed in rows only (Section 6, outlook: a label subset is a slicing of
    the [m][k] arrays): out_rows[i][q] = sum_t W[rows[q]][t] * x[i][idx[rows[q]][t]]."""
    return forward(x, np.ascontiguousarray(idx[rows]), np.ascontiguousarray(W[rows]))


def backward_weight_rows(g_rows, x, idx, rows):
    """grad_W of the listed labels: [len(rows)][k]."""
    return backward_weight(g_rows, x, np.ascontiguousarray(idx[rows]))


def backward_input_rows(g_rows, idx, W, rows, d):
    """grad_x contributed by the listed labels only."""
    return backward_input(g_rows, np.ascontiguousarray(idx[rows]), np.ascontiguousarray(W[rows]), d)


def topk(out, kk):
    """The kk best labels of every row, best first (ties: smaller label); returns (labels, scores)."""
    _chk(out, np.float32)
    b, m = out.shape
    assert 1 <= kk <= m
    lab = np.empty((b, kk), np.int32)
    val = np.empty((b, kk), np.float32)
    lib().orc_topk(_p(out), ctypes.c_int64(m), ctypes.c_int32(b), ctypes.c_int32(kk), _p(lab), _p(val))
    return lab, val


def precision_hits(top_lab, tgt_off, tgt_lab):
    """hits[r] = number of instances whose rank-r prediction is a target; P@k = hits[:k].sum()/(k*b)."""
    _chk(top_lab, np.int32), _chk(tgt_off, np.int64), _chk(tgt_lab, np.int32)
    b, kk = top_lab.shape
    hits = np.zeros(kk, np.int64)
    lib().orc_precision_hits(_p(top_lab), _p(tgt_off), _p(tgt_lab), ctypes.c_int32(b), ctypes.c_int32(kk),
                             _p(hits))
    return hits


def adam_step(W, grad_W, m1, m2, t, lr, beta1, beta2, eps):
    """In-place Adam on W, m1, m2.  For bfloat16 W returns the unrounded float32 values."""
    _chk(W), _chk(grad_W, np.float32), _chk(m1, np.float32), _chk(m2, np.float32)
    st = _storage(W)
    wf = np.empty(W.shape, np.float32) if st == 1 else None
    lib().orc_adam_step(_p(W), _p(grad_W), _p(m1), _p(m2), ctypes.c_int64(W.size),
                        ctypes.c_int64(t), ctypes.c_float(lr), ctypes.c_float(beta1),
                        ctypes.c_float(beta2), ctypes.c_float(eps), ctypes.c_int(st),
                        _p(wf) if wf is not None else None)
    return wf


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*ctr)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return tuple(int(v) for v in o)


def draw_column(seed, epoch, j, t, a, d):
    return int(lib().orc_draw_column(ctypes.c_uint64(seed), ctypes.c_uint64(epoch),
                                     ctypes.c_uint32(j), ctypes.c_uint32(t), ctypes.c_uint32(a),
                                     ctypes.c_int32(d)))


def init_indices(m, d, k, seed):
    """k distinct uniform columns per row."""
    idx = np.empty((m, k), np.int32)
    lib().orc_init_indices(_p(idx), ctypes.c_int64(m), ctypes.c_int32(d), ctypes.c_int32(k),
                           ctypes.c_uint64(seed))
    return idx


def redistribute(idx, W, m1, m2, d, fraction, seed, epoch):
    """In-place prune (global smallest |W|) + random regrow.  Returns (n, flags[m,k] uint8)."""
    _chk(idx, np.int32), _chk(W), _chk(m1, np.float32), _chk(m2, np.float32)
    m, k = idx.shape
    flags = np.zeros((m, k), np.uint8)
    n = lib().orc_redistribute(_p(idx), _p(W), _p(m1), _p(m2), ctypes.c_int64(m),
                               ctypes.c_int32(d), ctypes.c_int32(k), ctypes.c_double(fraction),
                               ctypes.c_uint64(seed), ctypes.c_uint64(epoch),
                               ctypes.c_int(_storage(W)), _p(flags))
    if n < 0:
        raise ValueError("m*k does not fit 32 bits")
    return int(n), flags


def redistribute_rows(idx, W, m1, m2, d, per_row, seed, epoch):
    """In-place per-row prune (the per_row smallest |W| of every row) + random regrow.  Returns flags[m,k]."""
    _chk(idx, np.int32), _chk(W), _chk(m1, np.float32), _chk(m2, np.float32)
    m, k = idx.shape
    assert 0 <= per_row <= k
    flags = np.zeros((m, k), np.uint8)
    lib().orc_redistribute_rows(_p(idx), _p(W), _p(m1), _p(m2), ctypes.c_int64(m), ctypes.c_int32(d),
                                ctypes.c_int32(k), ctypes.c_int32(per_row), ctypes.c_uint64(seed),
                                ctypes.c_uint64(epoch), ctypes.c_int(_storage(W)), _p(flags))
    return flags


def count_bad_rows(idx, d):
    _chk(idx, np.int32)
    m, k = idx.shape
    return int(lib().orc_count_bad_rows(_p(idx), ctypes.c_int64(m), ctypes.c_int32(d),
                                        ctypes.c_int32(k)))
