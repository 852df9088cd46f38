"""The input gradient (Algorithm 2) in its register-list form -- lists of each (window of 32768 labels, 2048
features) in registers, rows of g staged through LDS -- against the oracle, element by element (1e-4, as for the
other form).  The form applies where 32768 * k == 32 * d; USL_TUNE_BWI=lds switches it on below the size at which
the library would choose it by itself."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu

# (m, d, k, b, storage)
SHAPES = [
    (70000, 2048, 2, 5, "f32"),       # three windows of 23336 labels, the last one short with a ragged end of 16-byte pieces
    (32772, 2048, 2, 3, "f32"),       # two windows of 16388 and 16384 labels
    (100000, 8192, 8, 37, "f32"),     # four feature blocks
    (40000, 32768, 32, 3, "f32"),     # the headline's d and k
    (40000, 32768, 32, 3, "bf16"),
    (66000, 65536, 64, 2, "bf16"),    # d of two histogram chunks
    (70000, 2048, 2, 300, "f32"),     # three passes over the batch (128 + 128 + 44 instances: USL_TUNE_BWI_ROWS below)
    (20, 2048, 2, 1, "f32"),          # fewer labels than LDS banks, most lists empty, one instance
    (131072, 4096, 4, 2, "bf16"),     # exactly four full windows
    (50000, 2048, 8, 3, "f32"),       # k/d = 1/256: windows of 8192 labels at most
    (30000, 2048, 32, 2, "f32"),      # k/d = 1/64: windows of 2048 labels, the shortest the form takes
    (99996, 4096, 6, 3, "bf16"),      # a window size that is no power of two (21844 labels at most), k no power of two
    (65540, 6144, 12, 2, "f32"),      # three feature blocks
]


@pytest.fixture()
def lds_form(monkeypatch):
    monkeypatch.setenv("USL_TUNE_BWI", "lds")


@pytest.mark.parametrize("m,d,k,b,storage", SHAPES)
def test_backward_input_register_lists(orc, lds_form, m, d, k, b, storage, monkeypatch):
    import gpu_util as gu
    monkeypatch.setenv("USL_TUNE_BWI_ROWS", "128")
    from paper_2306_03725_amd import usl
    cfg = wl.custom(m, d, k, b, storage=storage, positives=3, index=200 + SHAPES.index((m, d, k, b, storage)))
    print("bwi lds", m, d, k, b, storage, flush=True)
    idx, W, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_g(cfg)
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_g = gu.dev(idx), gu.dev(W), gu.dev(g)
    gx = gu.empty((b, d)).fill_(float("nan"))
    L.backward_input(d_g, d_idx, d_W, gx, b)
    ref = orc.backward_input(g, idx, W, d)
    assert_close(gu.host(gx), ref, 1e-4, "grad_x")
    # a second call reuses the lists; a smaller batch leaves the other rows alone
    gx.fill_(float("nan"))
    nb = max(1, b // 2)
    L.backward_input(d_g, d_idx, d_W, gx, nb)
    got = gu.host(gx)
    assert_close(got[:nb], ref[:nb], 1e-4, "grad_x, second call")
    assert np.isnan(got[nb:]).all()
    np.testing.assert_array_equal(gu.host(d_idx), idx)
    L.check()
    L.close()


@pytest.mark.parametrize("pattern", ["uniform", "two_features"])
def test_an_infinite_gradient_stays_in_its_own_features(orc, lds_form, pattern):
    """One entry of g is +inf: exactly the features its label is connected to become infinite (or NaN where a weight
    is zero or another infinity cancels), every other feature is finite and right.  The empty places of the register
    lists and of the overflow lists must not multiply it by their zero weight."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    m, d, k, b = 40000, 2048, 2, 2
    cfg = wl.custom(m, d, k, b, positives=3, index=236)
    idx, W, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_g(cfg)
    if pattern == "two_features":
        idx[:, 0], idx[:, 1] = 7, 2040
    j_inf = 0      # label 0 is what an empty place would read if it read a real label
    g[1, j_inf] = np.inf
    W[j_inf, :] = np.abs(W[j_inf, :]) + 0.5
    L = usl.Layer(m, d, k, b)
    gx = gu.empty((b, d)).fill_(float("nan"))
    L.backward_input(gu.dev(g), gu.dev(idx), gu.dev(W), gx, b)
    got = gu.host(gx)
    g_fin = g.copy()
    g_fin[1, j_inf] = 0.0
    ref = orc.backward_input(g_fin, idx, W, d)
    touched = np.zeros(d, bool)
    touched[idx[j_inf]] = True
    assert np.isposinf(got[1, touched]).all()
    assert np.isfinite(got[1, ~touched]).all() and np.isfinite(got[0]).all()
    rest = got.copy()
    rest[1, touched] = ref[1, touched]
    assert_close(rest, ref, 1e-4, "grad_x away from the infinite entry")
    L.close()


def test_buffers_that_are_not_16_byte_aligned(orc, lds_form):
    """g or grad_x at an address that is not a multiple of 16: the other form does the work."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    m, d, k, b = 70000, 2048, 2, 3
    cfg = wl.custom(m, d, k, b, positives=3, index=235)
    idx, W, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_g(cfg)
    ref = orc.backward_input(g, idx, W, d)
    L = usl.Layer(m, d, k, b)
    d_idx, d_W = gu.dev(idx), gu.dev(W)
    g_store, gx_store = gu.empty((b * m + 1,)), gu.empty((b * d + 1,)).fill_(float("nan"))
    g_off = g_store[1:].view(b, m)
    g_off.copy_(torch.from_numpy(g))
    gx_off = gx_store[1:].view(b, d)
    assert g_off.data_ptr() % 16 == 4 and gx_off.data_ptr() % 16 == 4
    gx = gu.empty((b, d))
    L.backward_input(g_off, d_idx, d_W, gx, b)
    assert_close(gu.host(gx), ref, 1e-4, "grad_x, g off by 4 bytes")
    L.backward_input(gu.dev(g), d_idx, d_W, gx_off, b)
    assert_close(gu.host(gx_off), ref, 1e-4, "grad_x off by 4 bytes")
    L.close()


@pytest.mark.parametrize("pattern", ["two_features", "half_skewed"])
def test_lists_longer_than_the_registers(orc, lds_form, pattern):
    """Connectivity far from uniform: lists that do not fit a lane's registers go through the overflow list (its
    part held in LDS and the part read from memory)."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    m, d, k, b = 40000, 2048, 2, 3
    cfg = wl.custom(m, d, k, b, positives=3, index=230)
    idx, W, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_g(cfg)
    if pattern == "two_features":
        idx[:, 0], idx[:, 1] = 7, 2040
    else:                      # every second label into a handful of features, the rest uniform
        idx[::2, 0] = (np.arange(0, m, 2) % 5) * 400 + 3
        idx[::2, 1] = (np.arange(0, m, 2) % 5) * 400 + 4
    L = usl.Layer(m, d, k, b)
    gx = gu.empty((b, d)).fill_(float("nan"))
    L.backward_input(gu.dev(g), gu.dev(idx), gu.dev(W), gx, b)
    assert_close(gu.host(gx), orc.backward_input(g, idx, W, d), 1e-4, "grad_x")
    L.close()


def test_changed_idx_is_noticed(orc, lds_form):
    """Contents of idx replaced at the same address without usl_invalidate: NaN and USL_ESTALE, then right again."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    m, d, k, b = 70000, 2048, 2, 4
    cfg = wl.custom(m, d, k, b, positives=3, index=240)
    idx1, W, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_g(cfg)
    idx2 = wl.gen_idx(wl.custom(m, d, k, b, index=241))
    L = usl.Layer(m, d, k, b)
    d_idx, d_W, d_g, gx = gu.dev(idx1), gu.dev(W), gu.dev(g), gu.empty((b, d))
    L.backward_input(d_g, d_idx, d_W, gx, b)
    assert_close(gu.host(gx), orc.backward_input(g, idx1, W, d), 1e-4, "grad_x, first idx")
    d_idx.copy_(torch.from_numpy(idx2))
    rc = usl._lib.usl_backward_input(L._h, d_g.data_ptr(), d_idx.data_ptr(), d_W.data_ptr(), gx.data_ptr(), b)
    assert rc == usl.USL_OK
    assert torch.isnan(gx).all()
    with pytest.raises(usl.UslError) as e:
        L.check()
    assert e.value.status == usl.USL_ESTALE
    rc = usl._lib.usl_backward_input(L._h, d_g.data_ptr(), d_idx.data_ptr(), d_W.data_ptr(), gx.data_ptr(), b)
    assert rc == usl.USL_OK
    assert_close(gu.host(gx), orc.backward_input(g, idx2, W, d), 1e-4, "grad_x after the check invalidated the lists")
    L.check()
    L.close()


# the last three: a layer large enough for the kernels of the large layers (float32, k = 32, one row of x per stage);
# targets with an empty instance, a label listed twice and a dense instance
# both = "on": the kernel that computes the weight gradient from the same gathers (lists of half the length)
@pytest.mark.parametrize("both", ["off", "on"])
@pytest.mark.parametrize("loss_kind,storage,easy,shape", [
    (0, "f32", False, (70000, 2048, 2, 9)), (1, "bf16", False, (70000, 2048, 2, 9)), (1, "f32", True, (70000, 2048, 2, 9)),
    (0, "f32", False, (270000, 32768, 32, 5)), (1, "f32", False, (270000, 32768, 32, 5)), (1, "f32", True, (270000, 32768, 32, 5)),
    (0, "bf16", False, (100000, 8192, 8, 37)), (0, "f32", False, (20, 2048, 2, 1))])
def test_train_step_with_register_lists(orc, lds_form, loss_kind, storage, easy, shape, both, monkeypatch):
    """The fused step where the input gradient takes this form: loss row-major, then the products."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    if easy:
        monkeypatch.setenv("USL_TUNE_SPARSE", "always")
    monkeypatch.setenv("USL_TUNE_BOTH", both)
    m, d, k, b = shape
    cfg = wl.custom(m, d, k, b, storage=storage, positives=min(3, m), index=250 + loss_kind)
    print("train_step lds", shape, loss_kind, storage, easy, both, flush=True)
    hp = wl.ADAM
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    if easy:
        W = wl.store(-np.abs(wl.as_f32(W)) * 8.0 - 0.5, storage)
    off, lab = wl.gen_targets(cfg)
    if m == 270000:
        lists = [list(lab[off[i]:off[i + 1]]) for i in range(b)]
        lists[0] = []
        lists[1] = lists[1] + lists[1][:2] + [m - 1, 0, m - 1]
        lists[2] = list(range(0, m, 1000))
        off = np.cumsum([0] + [len(l) for l in lists]).astype(np.int64)
        lab = np.array([v for l in lists for v in l], np.int32)
    r = wl.rng(cfg, 5)
    m1 = (r.standard_normal((m, k)) * 1e-3).astype(np.float32)
    m2 = (r.random((m, k)) * 1e-6).astype(np.float32)
    scale, t = float(np.float32(1.0 / b)), 2
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x, d_m1, d_m2 = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(m1), gu.dev(m2)
    g, gW, gx, loss = gu.empty((b, m)), gu.empty((m, k)), gu.empty((b, d)).fill_(float("nan")), gu.empty((1,))
    L.train_step(d_x, d_idx, d_W, d_m1, d_m2, gu.dev(off), gu.dev(lab), loss_kind, scale, t,
                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], g, gW, gx, loss, b)
    out = orc.forward(x, idx, W)
    ref_loss, ref_g = (orc.bce_loss_grad if loss_kind == 0 else orc.sqh_loss_grad)(out, off, lab, scale)
    got_g = gu.host(g)
    assert_close(got_g, ref_g, 1e-5, "g")
    assert abs(float(loss.item()) - ref_loss) <= 1e-5 * abs(ref_loss)
    got_gW = gu.host(gW)
    assert_close(got_gW, orc.backward_weight(got_g, x, idx), 1e-5, "grad_W")
    assert_close(gu.host(gx), orc.backward_input(got_g, idx, W, d), 1e-4, "grad_x")
    m1r, m2r, W2 = m1.copy(), m2.copy(), W.copy()
    orc.adam_step(W2, got_gW, m1r, m2r, t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"])
    assert_close(gu.host(d_m1), m1r, 1e-4, "m1")
    assert_close(gu.host(d_m2), m2r, 1e-4, "m2")
    L.check()
    L.close()


@pytest.mark.parametrize("pattern", ["two_features", "half_skewed"])
def test_both_products_with_lists_longer_than_the_registers(orc, lds_form, pattern, monkeypatch):
    """The step whose backward products share one pass of gathers, on connectivity far from uniform: the weight
    gradients of overflow entries are summed in LDS and, beyond what LDS holds, in memory."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    monkeypatch.setenv("USL_TUNE_BOTH", "on")
    m, d, k, b = 40000, 2048, 2, 3
    cfg = wl.custom(m, d, k, b, positives=3, index=260)
    hp = wl.ADAM
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    if pattern == "two_features":
        idx[:, 0], idx[:, 1] = 7, 2040
    else:
        idx[::2, 0] = (np.arange(0, m, 2) % 5) * 400 + 3
        idx[::2, 1] = (np.arange(0, m, 2) % 5) * 400 + 4
    off, lab = wl.gen_targets(cfg)
    m1, m2 = np.zeros((m, k), np.float32), np.zeros((m, k), np.float32)
    scale = float(np.float32(1.0 / b))
    L = usl.Layer(m, d, k, b)
    g, gW, gx, loss = gu.empty((b, m)), gu.empty((m, k)).fill_(float("nan")), gu.empty((b, d)).fill_(float("nan")), gu.empty((1,))
    L.train_step(gu.dev(x), gu.dev(idx), gu.dev(W), gu.dev(m1), gu.dev(m2), gu.dev(off), gu.dev(lab), 0, scale, 1,
                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], g, gW, gx, loss, b)
    got_g = gu.host(g)
    assert_close(gu.host(gW), orc.backward_weight(got_g, x, idx), 1e-5, "grad_W")
    assert_close(gu.host(gx), orc.backward_input(got_g, idx, W, d), 1e-4, "grad_x")
    L.close()
