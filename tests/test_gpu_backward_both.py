"""usl_backward: both gradients of the backward pass (Algorithms 2 and 3) from one call, against the oracle's two
products, element by element (1e-5 for grad_W, 1e-4 for grad_x: the tolerances of the separate calls).  Where
16 * d / k lies between 2048 and 16384 the call can take its one-pass form (lists of a window's connections in
registers with a weight-gradient sum per connection, two rows of g in LDS at a time); USL_TUNE_BOTH=on switches it on
below the size at which the library would choose it by itself, =off keeps the two separate kernels."""
import numpy as np
import pytest

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu

# (m, d, k, b, storage)
SHAPES = [
    (70000, 2048, 2, 5, "f32"),       # five windows of 14000 labels, an odd batch: a pass of four instances, then one of one
    (40000, 32768, 32, 3, "f32"),     # the headline's d and k
    (40000, 32768, 32, 4, "bf16"),
    (100000, 8192, 8, 37, "f32"),     # four feature blocks
    (20, 2048, 2, 1, "f32"),          # fewer labels than LDS banks, most lists empty, one instance
    (50000, 2048, 8, 2, "f32"),       # k/d = 1/256: windows of 4096 labels at most
    (99996, 4096, 6, 3, "bf16"),      # a window size that is no power of two, k no power of two
    (66000, 65536, 64, 2, "bf16"),    # d of two histogram chunks
    (65540, 6144, 12, 6, "f32"),      # three feature blocks, a last window with a ragged end
    (70000, 2048, 2, 301, "f32"),     # three passes over the batch (128 + 128 + 45 instances: USL_TUNE_BWI_ROWS below), the weight
                                      # gradient of a later pass added to the earlier ones
]


def run_and_compare(orc, L, gu, cfg, idx, W, x, g, b, nb):
    m, d, k = cfg.m, cfg.d, cfg.k
    d_idx, d_W, d_x, d_g = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(g)
    gW, gx = gu.empty((m, k)).fill_(float("nan")), gu.empty((b, d)).fill_(float("nan"))
    L.backward(d_g, d_x, d_idx, d_W, gW, gx, b)
    assert_close(gu.host(gW), orc.backward_weight(g, x, idx), 1e-5, "grad_W")
    ref_x = orc.backward_input(g, idx, W, d)
    assert_close(gu.host(gx), ref_x, 1e-4, "grad_x")
    # a second call reuses the lists; a smaller batch leaves the other rows of grad_x alone
    gW.fill_(float("nan")); gx.fill_(float("nan"))
    L.backward(d_g, d_x, d_idx, d_W, gW, gx, nb)
    assert_close(gu.host(gW), orc.backward_weight(g[:nb], x[:nb], idx), 1e-5, "grad_W, second call")
    got = gu.host(gx)
    assert_close(got[:nb], ref_x[:nb], 1e-4, "grad_x, second call")
    assert np.isnan(got[nb:]).all()
    np.testing.assert_array_equal(gu.host(d_idx), idx)
    np.testing.assert_array_equal(gu.host(d_g), g)
    L.check()


@pytest.mark.parametrize("both", ["on", "off"])
@pytest.mark.parametrize("m,d,k,b,storage", SHAPES)
def test_backward_both_products(orc, m, d, k, b, storage, both, monkeypatch):
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    monkeypatch.setenv("USL_TUNE_BOTH", both)
    monkeypatch.setenv("USL_TUNE_BWI_ROWS", "128")
    cfg = wl.custom(m, d, k, b, storage=storage, positives=3, index=300 + SHAPES.index((m, d, k, b, storage)))
    print("backward", m, d, k, b, storage, both, flush=True)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    L = usl.Layer(m, d, k, b, storage)
    run_and_compare(orc, L, gu, cfg, idx, W, x, g, b, max(1, b // 2))
    L.close()


@pytest.mark.parametrize("pattern", ["two_features", "half_skewed", "one_block"])
def test_backward_with_lists_longer_than_the_registers(orc, pattern, monkeypatch):
    """Connectivity far from uniform: the weight gradients of the entries that do not fit the registers are summed in
    LDS and, beyond what LDS holds, in memory; with all connections in one of two feature blocks a workgroup has more
    of them (about 64000) than LDS holds places for at the end, and brings them into slot order piece by piece."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    monkeypatch.setenv("USL_TUNE_BOTH", "on")
    m, d, k, b = (60000, 2048, 2, 4) if pattern != "one_block" else (40000, 4096, 4, 4)
    cfg = wl.custom(m, d, k, b, positives=3, index=330)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    if pattern == "two_features":
        idx[:, 0], idx[:, 1] = 7, 2040
    elif pattern == "one_block":
        idx[:] = (idx[:, :1] % 2048 + np.arange(k, dtype=np.int32) * 511) % 2048   # distinct within a row
    else:
        idx[::2, 0] = (np.arange(0, m, 2) % 5) * 400 + 3
        idx[::2, 1] = (np.arange(0, m, 2) % 5) * 400 + 4
    L = usl.Layer(m, d, k, b)
    run_and_compare(orc, L, gu, cfg, idx, W, x, g, b, 3)
    L.close()


def test_backward_of_a_gradient_that_is_almost_all_zeros(orc, monkeypatch):
    """The gradient of a trained layer under the squared hinge loss (Section 3.3): after a few calls the context expects
    it and lists the nonzeros first; every call, before and after, gives both products."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    monkeypatch.setenv("USL_TUNE_BOTH", "on")
    m, d, k, b = 70000, 2048, 2, 6
    cfg = wl.custom(m, d, k, b, positives=3, index=340)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    rng = np.random.default_rng(341)
    g = (g * (rng.random(g.shape) < 0.002)).astype(np.float32)
    L = usl.Layer(m, d, k, b)
    d_idx, d_W, d_x, d_g = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(g)
    ref_W, ref_x = orc.backward_weight(g, x, idx), orc.backward_input(g, idx, W, d)
    for call in range(5):
        gW, gx = gu.empty((m, k)).fill_(float("nan")), gu.empty((b, d)).fill_(float("nan"))
        L.backward(d_g, d_x, d_idx, d_W, gW, gx, b)
        assert_close(gu.host(gW), ref_W, 1e-5, "grad_W, call %d" % call)
        assert_close(gu.host(gx), ref_x, 1e-4, "grad_x, call %d" % call)
    # ... and a dense gradient afterwards
    g2 = wl.gen_g(cfg)
    d_g2 = gu.dev(g2)
    gW, gx = gu.empty((m, k)).fill_(float("nan")), gu.empty((b, d)).fill_(float("nan"))
    L.backward(d_g2, d_x, d_idx, d_W, gW, gx, b)
    assert_close(gu.host(gW), orc.backward_weight(g2, x, idx), 1e-5, "grad_W, dense again")
    assert_close(gu.host(gx), orc.backward_input(g2, idx, W, d), 1e-4, "grad_x, dense again")
    L.check()
    L.close()


def test_changed_idx_is_noticed_before_the_weights_move(orc, monkeypatch):
    """Contents of idx replaced at the same address without usl_invalidate (past the binding, which would notice): the
    lists of the one-pass form are stale.  Both gradients come back as NaN, usl_train_step leaves W, m1 and m2 as they
    were (a step from a wrong gradient could not be taken back), usl_check says USL_ESTALE; the next call is right."""
    import torch
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    monkeypatch.setenv("USL_TUNE_BOTH", "on")
    m, d, k, b = 70000, 2048, 2, 4
    cfg = wl.custom(m, d, k, b, positives=3, index=350)
    hp = wl.ADAM
    idx1, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    idx2 = wl.gen_idx(wl.custom(m, d, k, b, index=351))
    off, lab = wl.gen_targets(cfg)
    L = usl.Layer(m, d, k, b)
    d_idx, d_W, d_x, d_g = gu.dev(idx1), gu.dev(W), gu.dev(x), gu.dev(g)
    gW, gx = gu.empty((m, k)), gu.empty((b, d))
    p = lambda t: t.data_ptr()
    L.backward(d_g, d_x, d_idx, d_W, gW, gx, b)
    assert_close(gu.host(gW), orc.backward_weight(g, x, idx1), 1e-5, "grad_W, first idx")
    d_idx.copy_(torch.from_numpy(idx2))
    assert usl._lib.usl_backward(L._h, p(d_g), p(d_x), p(d_idx), p(d_W), p(gW), p(gx), b) == usl.USL_OK
    assert torch.isnan(gW).all() and torch.isnan(gx).all()
    # the whole step on the stale lists
    d_m1, d_m2 = gu.dev(np.zeros((m, k), np.float32)), gu.dev(np.zeros((m, k), np.float32))
    d_off, d_lab, loss, out = gu.dev(off), gu.dev(lab), gu.empty((1,)), gu.empty((b, m))
    gW.zero_(); gx.zero_()
    scale = float(np.float32(1.0 / b))
    step = lambda: usl._lib.usl_train_step(L._h, p(d_x), p(d_idx), p(d_W), p(d_m1), p(d_m2), p(d_off), p(d_lab), 0, scale, 1,
                                           hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], p(out), p(gW), p(gx), p(loss), b)
    assert step() == usl.USL_OK
    assert torch.isnan(gW).all() and torch.isnan(gx).all()
    np.testing.assert_array_equal(gu.host(d_W), W)
    assert not gu.host(d_m1).any() and not gu.host(d_m2).any()
    with pytest.raises(usl.UslError) as e:
        L.check()
    assert e.value.status == usl.USL_ESTALE
    # the check invalidated the lists: the same call is right now
    assert step() == usl.USL_OK
    got_g = gu.host(out)
    assert_close(gu.host(gW), orc.backward_weight(got_g, x, idx2), 1e-5, "grad_W after the check")
    assert_close(gu.host(gx), orc.backward_input(got_g, idx2, W, d), 1e-4, "grad_x after the check")
    assert (gu.host(d_W) != W).any()
    L.check()
    L.close()
