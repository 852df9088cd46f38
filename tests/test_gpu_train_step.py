"""The fused training step (usl_train_step) against the oracle's chain forward -> loss -> backward-weight
-> backward-input -> Adam on the same inputs, with the tolerances of the separate calls."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu

# (m, d, k, b, storage, loss_kind, with_grad_x, easy_negatives)
CASES = [
    (1024, 64, 8, 16, "f32", 0, True, False),
    (3001, 1000, 32, 37, "f32", 1, True, False),       # m % 4 != 0: scalar loss path; ragged tile of instances
    (3000, 1000, 32, 70, "bf16", 0, True, False),
    (30938, 1024, 32, 128, "f32", 1, True, True),      # squared hinge with nearly all gradients zero
    (500, 200, 5, 7, "f32", 0, True, False),
    (270001, 2048, 32, 9, "f32", 0, True, False),
    (270000, 2048, 32, 33, "f32", 1, False, False),    # no input gradient
    (2000, 40000, 16, 3, "bf16", 1, True, False),
    (400001, 4096, 32, 5, "f32", 1, True, True),       # large layer, squared hinge, easy negatives: the lists of nonzeros
    (400000, 4096, 64, 3, "bf16", 1, True, True),
    (400000, 70000, 16, 2, "f32", 1, True, True),      # ... with an input row wider than one LDS slice
    (270000, 32768, 32, 4, "f32", 0, False, False),    # no input gradient, large float32 layer with one row of x per stage
    (270001, 20000, 32, 3, "f32", 1, False, False),    # ... with m % 4 != 0 and a ragged last block of labels
]


@pytest.mark.parametrize("m,d,k,b,storage,loss_kind,with_gx,easy", CASES)
def test_train_step(orc, m, d, k, b, storage, loss_kind, with_gx, easy, monkeypatch):
    import gpu_util as gu
    if easy:      # try the lists of nonzero gradients at once (left alone the library waits for two sparse steps in a row)
        monkeypatch.setenv("USL_TUNE_SPARSE", "always")
    from paper_2306_03725_amd import usl
    cfg = wl.custom(m, d, k, b, storage=storage, positives=min(3, m), index=60 + CASES.index((m, d, k, b, storage, loss_kind, with_gx, easy)))
    print("train_step", m, d, k, b, storage, loss_kind, with_gx, easy, flush=True)
    hp = wl.ADAM
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    if easy:      # all weights negative and large on non-negative activations: scores far below -1
        W = wl.store(-np.abs(wl.as_f32(W)) * 8.0 - 0.5, storage)
    off, lab = wl.gen_targets(cfg)
    if m == 3001 or m == 3000:   # an instance without positives, repeated ids, a very dense instance
        lists = [list(lab[off[i]:off[i + 1]]) for i in range(b)]
        lists[0] = []
        lists[1] = lists[1] + lists[1][:2]
        lists[2] = list(range(0, m, 3))
        lists[b - 1] = [m - 1, 0]
        off = np.cumsum([0] + [len(l) for l in lists]).astype(np.int64)
        lab = np.array([v for l in lists for v in l], np.int32)
    r = wl.rng(cfg, 5)
    m1 = (r.standard_normal((m, k)) * 1e-3).astype(np.float32)
    m2 = (r.random((m, k)) * 1e-6).astype(np.float32)
    scale = float(np.float32(1.0 / b))
    t = 3
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x, d_m1, d_m2 = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(m1), gu.dev(m2)
    g = gu.empty((b, m)).fill_(float("nan"))
    gW = gu.empty((m, k)).fill_(float("nan"))
    gx = gu.empty((b, d)).fill_(float("nan")) if with_gx else None
    loss = gu.empty((1,))
    L.train_step(d_x, d_idx, d_W, d_m1, d_m2, gu.dev(off), gu.dev(lab), loss_kind, scale, t,
                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], g, gW, gx, loss, b)
    # the oracle's chain; every stage is handed the GPU's input of that stage (teacher forcing)
    out = orc.forward(x, idx, W)
    ref_loss, ref_g = (orc.bce_loss_grad if loss_kind == 0 else orc.sqh_loss_grad)(out, off, lab, scale)
    got_g = gu.host(g)
    assert_close(got_g, ref_g, 1e-5, "g")
    assert abs(float(loss.item()) - ref_loss) <= 1e-5 * abs(ref_loss)
    if easy:
        assert (ref_g == 0).mean() > 0.99
    got_gW = gu.host(gW)
    assert_close(got_gW, orc.backward_weight(got_g, x, idx), 1e-5, "grad_W")
    if with_gx:
        assert_close(gu.host(gx), orc.backward_input(got_g, idx, W, d), 1e-4, "grad_x")
    W2, m1r, m2r = W.copy(), m1.copy(), m2.copy()
    wf = orc.adam_step(W2, got_gW, m1r, m2r, t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"])
    assert_close(gu.host(d_m1), m1r, 1e-4, "m1")
    assert_close(gu.host(d_m2), m2r, 1e-4, "m2")
    if storage == "f32":
        assert_close(gu.host(d_W), W2, 1e-4, "W")
    else:
        got = wl.as_f32(gu.host(d_W)).astype(np.float64)
        pre = wf
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(pre), 1e-30))) - 7)
        rms = float(np.sqrt(np.mean(pre.astype(np.float64) ** 2)))
        assert (np.abs(got - pre) <= 0.5 * ulp * (1 + 1e-3) + 1e-4 * np.abs(pre) + 1e-4 * rms).all()
    # the separate calls on the same inputs give the same gradient, bit for bit, where no order is free
    L2 = usl.Layer(m, d, k, b, storage)
    out2 = gu.empty((b, m))
    L2.forward(d_x, d_idx, gu.dev(W), out2, b)
    (L2.bce_loss_grad if loss_kind == 0 else L2.sqh_loss_grad)(out2, gu.dev(off), gu.dev(lab), scale, out2, loss, b)
    np.testing.assert_array_equal(gu.host(out2), got_g)
