"""Pins of the CPU oracle to things other than itself: the paper's worked example, dense
brute force through numpy/torch library routines, closed forms and invariants.  No GPU."""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import (GOLDEN, assert_close, py_draw, py_philox, read_blocks, scatter_dense)


# ---------------------------------------------------------------- worked example, Fig. 1(c)
def fig1c():
    blk = read_blocks("fig1c_uniform_format.txt")
    dense = blk["dense feature x label"]            # [4 features, 5 labels]
    idx = np.ascontiguousarray(blk["indices s x m"].T.astype(np.int32))      # -> [m, k]
    W = np.ascontiguousarray(blk["weights s x m"].T.astype(np.float32))
    return dense, idx, W


def test_fig1c_forward_recovers_dense_matrix(orc):
    dense, idx, W = fig1c()
    x = np.eye(4, dtype=np.float32)                 # instance i is the unit vector e_i
    out = orc.forward(x, idx, W)                    # out[i, j] must be dense[i, j]
    np.testing.assert_array_equal(out, dense.astype(np.float32))
    assert orc.count_bad_rows(idx, 4) == 0


def test_fig1c_backward_products(orc):
    dense, idx, W = fig1c()
    g = np.arange(10, dtype=np.float32).reshape(2, 5) - 3
    x = np.array([[1, 2, 3, 4], [0, -1, .5, 2]], np.float32)
    gx = orc.backward_input(g, idx, W, 4)
    assert_close(gx, g.astype(np.float64) @ dense.T.astype(np.float32).astype(np.float64), 1e-6, "grad_x")
    gw = orc.backward_weight(g, x, idx)
    full = g.T.astype(np.float64) @ x.astype(np.float64)          # [m, d]
    assert_close(gw, np.take_along_axis(full, idx.astype(np.int64), 1), 1e-6, "grad_W")


# ---------------------------------------------------------------- dense brute force
@pytest.mark.parametrize("m,d,k,b", [(1024, 64, 8, 16), (257, 33, 33, 5), (90, 700, 17, 3), (7, 5, 1, 2)])
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_products_equal_dense_matmul(orc, m, d, k, b, storage):
    cfg = wl.custom(m, d, k, b, storage=storage)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    Wd = scatter_dense(idx, wl.as_f32(W), d)
    x64, g64 = wl.as_f32(x).astype(np.float64), g.astype(np.float64)
    assert_close(orc.forward(x, idx, W), x64 @ Wd.T, 1e-6, "forward")
    assert_close(orc.backward_input(g, idx, W, d), g64 @ Wd, 1e-6, "backward_input")
    full = g64.T @ x64
    assert_close(orc.backward_weight(g, x, idx), np.take_along_axis(full, idx.astype(np.int64), 1),
                 1e-6, "backward_weight")


def test_adjoint_identities(orc):
    """<g, fwd(x)> = <bwd_input(g), x> = <grad_W, W> ties the three products together."""
    cfg = wl.custom(3000, 512, 32, 12)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    a = np.vdot(g.astype(np.float64), orc.forward(x, idx, W).astype(np.float64))
    b_ = np.vdot(orc.backward_input(g, idx, W, cfg.d).astype(np.float64), x.astype(np.float64))
    c = np.vdot(orc.backward_weight(g, x, idx).astype(np.float64), W.astype(np.float64))
    assert abs(a - b_) <= 1e-5 * abs(a) and abs(a - c) <= 1e-5 * abs(a)


# ---------------------------------------------------------------- BCE
def dense_targets(off, lab, b, m):
    y = np.zeros((b, m), np.float64)
    for i in range(b):
        y[i, lab[off[i]:off[i + 1]]] = 1.0
    return y


def test_bce_matches_torch_library_routine(orc):
    cfg = wl.custom(777, 64, 8, 9, positives=4)
    out = (wl.rng(cfg, 7).standard_normal((cfg.b, cfg.m)) * 3).astype(np.float32)
    off, lab = wl.gen_targets(cfg)
    y = dense_targets(off, lab, cfg.b, cfg.m)
    scale = float(np.float32(1.0 / cfg.b))       # the call takes scale as a float32
    loss, g = orc.bce_loss_grad(out, off, lab, scale)
    z = torch.tensor(out, dtype=torch.float64, requires_grad=True)
    ref = scale * torch.nn.functional.binary_cross_entropy_with_logits(z, torch.tensor(y), reduction="sum")
    ref.backward()
    assert abs(loss - ref.item()) <= 1e-12 * abs(ref.item())
    assert_close(g, z.grad.numpy(), 1e-6, "g")


def test_bce_closed_forms_and_edge_cases(orc):
    m, b = 6, 3
    out = np.zeros((b, m), np.float32)
    out[1] = [40, -40, 40, -40, 100, -100]
    out[2] = [1, -1, 2, -2, .5, -.5]
    # instance 0: positives {1} ; instance 1: {0, 1}; instance 2: none.  Label 1 repeated for instance 0.
    off = np.array([0, 3, 5, 5], np.int64)
    lab = np.array([1, 1, 1, 0, 1], np.int32)
    scale = 0.5
    loss, g = orc.bce_loss_grad(out, off, lab, scale)
    assert np.isfinite(g).all() and np.isfinite(loss)
    # z = 0: l = ln 2 whatever y, g = scale * (1/2 - y); a repeated target counts once
    np.testing.assert_allclose(g[0], scale * (0.5 - np.array([0, 1, 0, 0, 0, 0])), rtol=0, atol=1e-7)
    # saturated scores: g -> scale * (1 - y) for z >> 0 and -scale * y for z << 0
    np.testing.assert_allclose(g[1], scale * np.array([0, -1, 1, 0, 1, 0]), rtol=0, atol=1e-7)
    z2 = out[2].astype(np.float64)
    expect = 6 * np.log(2) + (0 + 40 + 40 + 0 + 100 + 0) + np.sum(np.log1p(np.exp(-np.abs(out[1].astype(np.float64))))) \
        + np.sum(np.log1p(np.exp(z2)))
    # instance 1: l(40,1)=~0, l(-40,1)=40, l(40,0)=40, l(-40,0)=~0, l(100,0)=100, l(-100,0)=~0
    assert abs(loss - scale * expect) < 1e-9
    # sum_j g = scale * (sum sigmoid - #positives)
    sig = 1 / (1 + np.exp(-z2))
    assert abs(g[2].astype(np.float64).sum() - scale * sig.sum()) < 1e-6
    # in place (g aliases out) gives the same numbers
    import oracle, ctypes
    o2 = out.copy()
    l2 = ctypes.c_double()
    oracle.lib().orc_bce_loss_grad(o2.ctypes.data_as(ctypes.c_void_p), off.ctypes.data_as(ctypes.c_void_p),
                                   lab.ctypes.data_as(ctypes.c_void_p), ctypes.c_float(scale),
                                   o2.ctypes.data_as(ctypes.c_void_p), ctypes.byref(l2),
                                   ctypes.c_int64(m), ctypes.c_int32(b))
    np.testing.assert_array_equal(o2, g)
    assert l2.value == loss


def test_bce_gradient_is_derivative_of_loss(orc):
    cfg = wl.custom(40, 8, 2, 3, positives=2)
    out = wl.rng(cfg, 7).standard_normal((cfg.b, cfg.m)).astype(np.float32)
    off, lab = wl.gen_targets(cfg)
    _, g = orc.bce_loss_grad(out, off, lab, 0.25)
    h = 2.0 ** -6      # exactly representable step keeps the float32 scores exact
    for (i, j) in [(0, 0), (1, int(lab[off[1]])), (2, 39), (0, int(lab[0]))]:
        op, om = out.copy(), out.copy()
        op[i, j] += h
        om[i, j] -= h
        lp, _ = orc.bce_loss_grad(op, off, lab, 0.25)
        lm, _ = orc.bce_loss_grad(om, off, lab, 0.25)
        assert abs((lp - lm) / (2 * h) - g[i, j]) < 2e-5


# ---------------------------------------------------------------- squared hinge
def test_sqh_closed_forms(orc):
    """Section 3.3: l = max(0, 1 - y z)^2, gradient -2 y max(0, 1 - y z), zero iff y z >= 1."""
    out = np.array([[2.0, 1.0, 0.5, 0.0, -0.5, -1.0, -3.0],
                    [2.0, 1.0, 0.5, 0.0, -0.5, -1.0, -3.0]], np.float32)
    off = np.array([0, 7, 7], np.int64)          # instance 0: every label positive; instance 1: none
    lab = np.arange(7, dtype=np.int32)
    loss, g = orc.sqh_loss_grad(out, off, lab, 0.5)
    z = out[0].astype(np.float64)
    pos = np.maximum(0, 1 - z)                    # y = +1
    neg = np.maximum(0, 1 + z)                    # y = -1
    np.testing.assert_allclose(g[0], 0.5 * -2 * pos, rtol=1e-7)
    np.testing.assert_allclose(g[1], 0.5 * 2 * neg, rtol=1e-7)
    assert abs(loss - 0.5 * ((pos ** 2).sum() + (neg ** 2).sum())) < 1e-12
    assert (g[0][:2] == 0).all() and (g[1][5:] == 0).all()      # exact zeros at margin >= 1
    assert g[0][2] != 0 and g[1][4] != 0


def test_sqh_matches_torch_autograd(orc):
    cfg = wl.custom(500, 64, 8, 6, positives=5)
    out = (wl.rng(cfg, 7).standard_normal((cfg.b, cfg.m)) * 1.5).astype(np.float32)
    off, lab = wl.gen_targets(cfg)
    y = 2 * dense_targets(off, lab, cfg.b, cfg.m) - 1
    scale = float(np.float32(1.0 / cfg.b))
    loss, g = orc.sqh_loss_grad(out, off, lab, scale)
    z = torch.tensor(out, dtype=torch.float64, requires_grad=True)
    ref = scale * (torch.clamp(1 - torch.tensor(y) * z, min=0) ** 2).sum()
    ref.backward()
    assert abs(loss - ref.item()) <= 1e-12 * abs(ref.item())
    assert_close(g, z.grad.numpy(), 1e-6, "g")
    assert ((g == 0) == (y * out.astype(np.float64) >= 1)).all()


# ---------------------------------------------------------------- Adam
def test_adam_matches_torch_optimizer(orc):
    r = np.random.default_rng(5)
    n = 1000
    W0 = r.standard_normal(n).astype(np.float32)
    W, m1, m2 = W0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    hp = dict(lr=float(np.float32(1e-3)), betas=(float(np.float32(0.9)), float(np.float32(0.999))),
              eps=float(np.float32(1e-8)))
    opt = torch.optim.Adam([p], **hp)
    for t in range(1, 8):
        gw = (r.standard_normal(n) * 10.0 ** r.integers(-6, 2, n)).astype(np.float32)
        orc.adam_step(W, gw, m1, m2, t, 1e-3, 0.9, 0.999, 1e-8)
        p.grad = torch.tensor(gw, dtype=torch.float64)
        opt.step()
        # the oracle rounds its state to float32 every step, torch keeps double: 1e-6 is ample
        assert_close(W, p.detach().numpy(), 1e-6, "W at step %d" % t)
        st = opt.state[p]
        assert_close(m1, st["exp_avg"].numpy(), 1e-6, "m1")
        assert_close(m2, st["exp_avg_sq"].numpy(), 1e-6, "m2")


def test_adam_closed_forms(orc):
    gw = np.array([0.5, -2.0, 1e-3, 0.0, 3e4], np.float32)
    W = np.ones(5, np.float32)
    m1, m2 = np.zeros(5, np.float32), np.zeros(5, np.float32)
    lr, eps, T = 1e-2, 1e-8, 5
    for t in range(1, T + 1):
        # constant gradient: m1/c1 = gw and m2/c2 = gw^2 at every step, so each step moves
        # W by -lr * gw / (|gw| + eps)
        orc.adam_step(W, gw, m1, m2, t, lr, 0.9, 0.999, eps)
        expect = 1.0 - t * np.float32(lr).astype(np.float64) * gw / (np.abs(gw) + np.float32(eps).astype(np.float64))
        np.testing.assert_allclose(W, expect, rtol=3e-7 * t)
    assert W[3] == 1.0 and m1[3] == 0 and m2[3] == 0          # zero gradient leaves W alone


def test_adam_bf16_storage_rounds_to_nearest_even(orc):
    r = np.random.default_rng(6)
    n = 4096
    Wf = r.standard_normal(n).astype(np.float32)
    Wb = wl.f32_to_bf16_bits(Wf)
    W32 = wl.bf16_bits_to_f32(Wb).copy()
    gw = r.standard_normal(n).astype(np.float32)
    m1a, m2a, m1b, m2b = (np.zeros(n, np.float32) for _ in range(4))
    pre = orc.adam_step(Wb, gw, m1a, m2a, 1, 1e-3, 0.9, 0.999, 1e-8)
    orc.adam_step(W32, gw, m1b, m2b, 1, 1e-3, 0.9, 0.999, 1e-8)
    np.testing.assert_array_equal(pre, W32)          # same arithmetic on the widened value
    # nearest: |bf16 - f32| <= half a bf16 ulp of the result
    back = wl.bf16_bits_to_f32(Wb).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(back))) - 7)
    assert (np.abs(back - W32) <= ulp / 2).all()
    # ties go to the even mantissa.  With eps = 0 and t = 1 the step is exactly -lr*sign(g), so
    # lr = 2^-8 and g = -1 land 1.0 and 1+2^-7 exactly halfway between two bfloat16 values.
    tb = np.array([0x3F80, 0x3F81], np.uint16)
    gneg = np.full(2, -1.0, np.float32)
    pre = orc.adam_step(tb, gneg, np.zeros(2, np.float32), np.zeros(2, np.float32), 1, 2.0 ** -8, 0.9, 0.999, 0.0)
    assert pre.tolist() == [1 + 2.0 ** -8, 1 + 2.0 ** -7 + 2.0 ** -8]
    assert tb.tolist() == [0x3F80, 0x3F82]


# ---------------------------------------------------------------- random numbers
def test_philox_known_answers(orc):
    with open(GOLDEN + "/philox4x32_10_kat.txt") as fh:
        rows = [l.split() for l in fh if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(h, 16) for h in row]
        assert orc.philox4x32_10(v[0:4], v[4:6]) == tuple(v[6:10])
        assert py_philox(v[0:4], v[4:6]) == tuple(v[6:10])


def test_draw_matches_python_integers(orc):
    r = np.random.default_rng(1)
    for _ in range(300):
        seed, epoch = int(r.integers(0, 2 ** 63)) * 2 + 1, int(r.integers(0, 2 ** 63)) * 2
        j, t, a = int(r.integers(0, 2 ** 31)), int(r.integers(0, 64)), int(r.integers(0, 9))
        d = int(r.integers(1, 2 ** 17))
        c = orc.draw_column(seed, epoch, j, t, a, d)
        assert c == py_draw(seed, epoch, j, t, a, d) and 0 <= c < d


# ---------------------------------------------------------------- connectivity
def py_regrow(idx_row, empty, j, d, seed, epoch):
    """Second implementation of the refill rule, on Python integers."""
    row, empty = list(idx_row), list(empty)
    for t in range(len(row)):
        if not empty[t]:
            continue
        a = 0
        while True:
            c = py_draw(seed, epoch, j, t, a, d)
            a += 1
            if all(empty[u] or row[u] != c for u in range(len(row))):
                row[t], empty[t] = c, False
                break
    return row


@pytest.mark.parametrize("m,d,k", [(64, 64, 8), (30, 9, 9), (50, 40, 33), (5, 3, 1)])
def test_init_indices(orc, m, d, k):
    seed = 0x1234567890ABCDEF
    idx = orc.init_indices(m, d, k, seed)
    assert orc.count_bad_rows(idx, d) == 0
    assert idx.min() >= 0 and idx.max() < d
    assert all(len(set(r)) == k for r in idx.tolist())
    for j in range(m):
        assert idx[j].tolist() == py_regrow([0] * k, [True] * k, j, d, seed, 2 ** 64 - 1)
    np.testing.assert_array_equal(idx, orc.init_indices(m, d, k, seed))
    assert (idx != orc.init_indices(m, d, k, seed + 1)).any()


def test_count_bad_rows_sees_planted_faults(orc):
    idx = orc.init_indices(20, 50, 6, 3)
    a = idx.copy(); a[3, 5] = a[3, 0]
    b = idx.copy(); b[7, 2] = 50
    c = idx.copy(); c[9, 0] = -1
    assert [orc.count_bad_rows(v, 50) for v in (idx, a, b, c)] == [0, 1, 1, 1]


def brute_prune_set(W, n):
    if W.dtype == np.uint16:
        mag = (W.reshape(-1) & 0x7FFF).astype(np.int64)
    else:
        mag = (W.reshape(-1).view(np.uint32) & 0x7FFFFFFF).astype(np.int64)
    order = np.lexsort((np.arange(mag.size), mag))     # by magnitude bits, then flat slot
    flags = np.zeros(mag.size, np.uint8)
    flags[order[:n]] = 1
    return flags.reshape(W.shape)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("m,d,k,frac", [(1024, 64, 8, 0.10), (200, 40, 32, 0.33), (64, 9, 8, 0.9), (33, 70, 5, 0.05)])
def test_redistribute_against_brute_force(orc, m, d, k, frac, storage):
    cfg = wl.custom(m, d, k, 1, storage=storage)
    idx0, W0 = wl.gen_idx(cfg), wl.gen_W(cfg)
    Wf = wl.as_f32(W0).copy()
    # plant ties, signed zeros and a NaN so the ordering rules are exercised
    flat = Wf.reshape(-1)
    flat[5], flat[11], flat[17] = 0.0, -0.0, np.float32("nan")
    flat[100:140] = np.float32(0.015625) * np.where(np.arange(40) % 2, 1, -1)
    W0 = wl.store(Wf, storage)
    m1_0 = np.full((m, k), 0.25, np.float32)
    m2_0 = np.full((m, k), 0.5, np.float32)
    idx, W, m1, m2 = idx0.copy(), W0.copy(), m1_0.copy(), m2_0.copy()
    seed, epoch = 99, 4
    n, flags = orc.redistribute(idx, W, m1, m2, d, frac, seed, epoch)
    assert n == int(np.floor(frac * m * k)) == int(flags.sum())
    np.testing.assert_array_equal(flags, brute_prune_set(W0, n))
    assert flags.reshape(-1)[17] == 0                       # NaN has the largest key: kept
    keep = flags == 0
    for new, old in ((idx, idx0), (W, W0), (m1, m1_0), (m2, m2_0)):   # survivors bit-identical
        np.testing.assert_array_equal(new[keep].view(np.uint8), old[keep].view(np.uint8))
    assert (W[flags == 1].view(np.uint8) == 0).all()        # regrown value is +0
    assert (m1[flags == 1] == 0).all() and (m2[flags == 1] == 0).all()
    assert orc.count_bad_rows(idx, d) == 0                  # fan-in k, in range, no repeats
    for j in range(m):                                      # refill rule, second implementation
        assert idx[j].tolist() == py_regrow(idx0[j].tolist(), flags[j].astype(bool).tolist(), j, d, seed, epoch)
    # same (seed, epoch) reproduces; another epoch rewires differently
    idx_b, W_b = idx0.copy(), W0.copy()
    orc.redistribute(idx_b, W_b, m1_0.copy(), m2_0.copy(), d, frac, seed, epoch)
    np.testing.assert_array_equal(idx_b, idx)
    idx_c = idx0.copy()
    orc.redistribute(idx_c, W0.copy(), m1_0.copy(), m2_0.copy(), d, frac, seed, epoch + 1)
    assert (idx_c != idx).any()


def test_redistribute_fraction_zero_and_one(orc):
    cfg = wl.custom(100, 50, 8, 1)
    idx0, W0 = wl.gen_idx(cfg), wl.gen_W(cfg)
    m1_0, m2_0 = np.ones((100, 8), np.float32), np.ones((100, 8), np.float32)
    idx, W, m1, m2 = idx0.copy(), W0.copy(), m1_0.copy(), m2_0.copy()
    n, flags = orc.redistribute(idx, W, m1, m2, 50, 0.0, 1, 0)
    assert n == 0 and flags.sum() == 0
    for new, old in ((idx, idx0), (W, W0), (m1, m1_0), (m2, m2_0)):
        np.testing.assert_array_equal(new, old)
    n, flags = orc.redistribute(idx, W, m1, m2, 50, 0.00124, 1, 0)   # floor(0.00124*800) = 0
    assert n == 0
    n, flags = orc.redistribute(idx, W, m1, m2, 50, 1.0, 1, 0)
    assert n == 800 and flags.all() and (W == 0).all() and orc.count_bad_rows(idx, 50) == 0


def test_regrown_columns_are_uniform_over_structural_zeros(orc):
    """Chi-square over d of the columns drawn in many redistributions, and survivors never re-drawn
    into the same row."""
    m, d, k = 512, 64, 8
    cfg = wl.custom(m, d, k, 1)
    idx, W = wl.gen_idx(cfg), wl.gen_W(cfg)
    m1, m2 = np.zeros((m, k), np.float32), np.zeros((m, k), np.float32)
    counts = np.zeros(d)
    r = np.random.default_rng(0)
    for epoch in range(60):
        before = idx.copy()
        W[:] = r.standard_normal((m, k)).astype(np.float32)
        n, flags = orc.redistribute(idx, W, m1, m2, d, 0.25, 7, epoch)
        new = idx[flags == 1]
        counts += np.bincount(new, minlength=d)
        assert orc.count_bad_rows(idx, d) == 0
    total = counts.sum()
    chi2 = ((counts - total / d) ** 2 / (total / d)).sum()
    # 63 degrees of freedom: mean 63, sd 11.2; 130 is beyond 6 sd
    assert chi2 < 130, chi2


# ---------------------------------------------------------------- prediction and P@k (Section 2)

def _read_patk_example():
    rows = {"scores": [], "targets": [], "top": [], "hits": [], "patk": []}
    with open(os.path.join(GOLDEN, "precision_at_k_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key].append(vals)
    return rows


def test_topk_and_precision_worked_example(orc):
    ex = _read_patk_example()
    scores = np.array(ex["scores"], np.float32)
    off = np.zeros(len(ex["targets"]) + 1, np.int64)
    off[1:] = np.cumsum([len(t) for t in ex["targets"]])
    lab = np.array([int(v) for t in ex["targets"] for v in t], np.int32)
    top, val = orc.topk(scores, 3)
    assert top.tolist() == [[int(v) for v in r] for r in ex["top"]]
    assert np.array_equal(val, np.take_along_axis(scores, top.astype(np.int64), 1))
    hits = orc.precision_hits(top, off, lab)
    assert hits.tolist() == [int(v) for v in ex["hits"][0]]
    patk = [hits[:k].sum() / (k * 3) for k in (1, 2, 3)]
    assert np.allclose(patk, [float(v) for v in ex["patk"][0]], rtol=0, atol=1e-15)


def test_topk_matches_stable_sort_with_ties(orc):
    # small integer scores force many ties; a stable sort of the negated scores lists equal scores by label
    g = np.random.default_rng(5)
    scores = g.integers(-4, 5, size=(7, 300)).astype(np.float32)
    scores[scores == 0] *= g.choice([-1.0, 1.0], size=(scores == 0).sum()).astype(np.float32)  # mix -0 / +0
    top, val = orc.topk(scores, 17)
    ref = np.argsort(-scores.astype(np.float64), axis=1, kind="stable")[:, :17]
    assert np.array_equal(top, ref.astype(np.int32))
    assert np.array_equal(val.view(np.uint32), np.take_along_axis(scores, ref, 1).view(np.uint32))


def test_topk_closed_forms(orc):
    m = 1000
    j = np.arange(m, dtype=np.float32)
    # a peak at label c: the order is c, c-1, c+1, c-2, ... (the left neighbour first: smaller label)
    c = 400
    top, _ = orc.topk((-np.abs(j - c))[None, :].copy(), 5)
    assert top[0].tolist() == [400, 399, 401, 398, 402]
    # kk = m returns a permutation sorted by score; an increasing row reverses
    top, val = orc.topk(j[None, :].copy(), m)
    assert top[0].tolist() == list(range(m - 1, -1, -1))
    # infinities are ordinary scores
    z = np.zeros((1, 8), np.float32); z[0, 3] = np.inf; z[0, 5] = -np.inf
    top, _ = orc.topk(z, 8)
    assert top[0].tolist() == [3, 0, 1, 2, 4, 6, 7, 5]


def test_precision_hits_closed_forms(orc):
    # a predictor that lists an instance's own targets first scores min(k, n_targets)/k
    b, m, kk = 6, 50, 5
    g = np.random.default_rng(9)
    counts = [0, 1, 2, 3, 5, 8]
    off = np.zeros(b + 1, np.int64); off[1:] = np.cumsum(counts)
    lab = np.concatenate([g.choice(m, n, replace=False) for n in counts]).astype(np.int32)
    top = np.empty((b, kk), np.int32)
    for i in range(b):
        own = lab[off[i]:off[i + 1]].tolist()
        rest = [q for q in range(m) if q not in own]
        top[i] = (own + rest)[:kk]
    hits = orc.precision_hits(top, off, lab)
    assert hits.tolist() == [sum(1 for n in counts if n > r) for r in range(kk)]
    # repeats in the target list count once; predictions that are no targets count nothing
    off2 = np.array([0, 3], np.int64); lab2 = np.array([7, 7, 7], np.int32)
    assert orc.precision_hits(np.array([[7, 8, 9]], np.int32), off2, lab2).tolist() == [1, 0, 0]


# ---------------------------------------------------------------- label subsets (Section 6, outlook)

def test_label_subset_products_are_slices_of_the_full_products(orc):
    cfg = wl.custom(300, 90, 8, 6, index=71)
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    r = wl.rng(cfg, 3)
    rows = r.choice(cfg.m, size=57, replace=True).astype(np.int64)          # with repeats, unsorted
    # forward: the listed columns of the full score matrix, bit for bit
    full = orc.forward(x, idx, W)
    np.testing.assert_array_equal(orc.forward_rows(x, idx, W, rows), full[:, rows])
    # backward: the same as the full backward calls on a gradient that is zero off the listed labels
    rows_u = np.unique(rows)
    g_rows = r.standard_normal((cfg.b, len(rows_u))).astype(np.float32)
    g_full = np.zeros((cfg.b, cfg.m), np.float32)
    g_full[:, rows_u] = g_rows
    np.testing.assert_array_equal(orc.backward_weight_rows(g_rows, x, idx, rows_u),
                                  orc.backward_weight(g_full, x, idx)[rows_u])
    np.testing.assert_array_equal(orc.backward_input_rows(g_rows, idx, W, rows_u, cfg.d),
                                  orc.backward_input(g_full, idx, W, cfg.d))
    # and against the dense matrix the format stands for (numpy matmul in float64)
    dense = scatter_dense(idx, W, cfg.d)                                     # [m][d]
    ref = x.astype(np.float64) @ dense[rows].T
    assert_close(orc.forward_rows(x, idx, W, rows), ref, 1e-6, "subset scores vs dense")


# ---------------------------------------------------------------- per-row variant of the redistribution

@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("m,d,k,per_row", [(300, 64, 8, 1), (200, 40, 32, 10), (64, 9, 8, 8), (33, 70, 5, 2)])
def test_redistribute_rows_against_brute_force(orc, m, d, k, per_row, storage):
    cfg = wl.custom(m, d, k, 1, storage=storage, index=81)
    idx0, W0 = wl.gen_idx(cfg), wl.gen_W(cfg)
    Wf = wl.as_f32(W0).copy()
    Wf[3, :] = np.float32(0.5) * np.where(np.arange(k) % 2, 1, -1)      # a row of equal magnitudes: slots 0.. go
    Wf[4, 0], Wf[4, 1] = 0.0, -0.0                                      # signed zeros tie, slot order decides
    Wf[5, 2] = np.float32("nan")                                        # largest key: goes last
    W0 = wl.store(Wf, storage)
    m1_0 = np.full((m, k), 0.25, np.float32)
    m2_0 = np.full((m, k), 0.5, np.float32)
    idx, W, m1, m2 = idx0.copy(), W0.copy(), m1_0.copy(), m2_0.copy()
    seed, epoch = 123, 9
    flags = orc.redistribute_rows(idx, W, m1, m2, d, per_row, seed, epoch)
    # second implementation of the prune rule: numpy lexsort per row
    mag = (W0 & 0x7FFF).astype(np.int64) if W0.dtype == np.uint16 else (W0.view(np.uint32) & 0x7FFFFFFF).astype(np.int64)
    ref = np.zeros((m, k), np.uint8)
    for j in range(m):
        order = np.lexsort((np.arange(k), mag[j]))
        ref[j, order[:per_row]] = 1
    np.testing.assert_array_equal(flags, ref)
    assert (flags.sum(axis=1) == per_row).all()
    assert flags[3, :per_row].all() and (per_row == k or not flags[5, 2])
    keep = flags == 0
    for new, old in ((idx, idx0), (W, W0), (m1, m1_0), (m2, m2_0)):
        np.testing.assert_array_equal(new[keep].view(np.uint8), old[keep].view(np.uint8))
    assert (W[flags == 1].view(np.uint8) == 0).all()
    assert (m1[flags == 1] == 0).all() and (m2[flags == 1] == 0).all()
    assert orc.count_bad_rows(idx, d) == 0
    for j in range(m):                                      # refill rule, second implementation
        assert idx[j].tolist() == py_regrow(idx0[j].tolist(), flags[j].astype(bool).tolist(), j, d, seed, epoch)


def test_redistribute_rows_zero_and_all(orc):
    cfg = wl.custom(50, 30, 8, 1)
    idx0, W0 = wl.gen_idx(cfg), wl.gen_W(cfg)
    idx, W = idx0.copy(), W0.copy()
    m1, m2 = np.ones((50, 8), np.float32), np.ones((50, 8), np.float32)
    assert orc.redistribute_rows(idx, W, m1, m2, 30, 0, 1, 0).sum() == 0
    np.testing.assert_array_equal(idx, idx0); np.testing.assert_array_equal(W, W0)
    assert orc.redistribute_rows(idx, W, m1, m2, 30, 8, 7, 3).all()
    # every slot empty: the same as the initial connectivity rule under that (seed, epoch)
    ref = idx0.copy()
    for j in range(50):
        ref[j] = py_regrow(idx0[j].tolist(), [True] * 8, j, 30, 7, 3)
    np.testing.assert_array_equal(idx, ref)
