"""Seeded sweep over irregular shapes: every product, the fused step and a redistribution, HIP path (through
the C ABI) against the CPU oracle.  The shapes are drawn to straddle the kernels' tile sizes (32 / 64 / 256 /
512 / 2048 labels, 16-byte row alignment, the fan-ins with register-resident kernels and those without)."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu


def draw_shapes(n, seed=2306):
    r = np.random.default_rng(seed)
    shapes = []
    for q in range(n):
        k = int(r.choice([1, 3, 8, 8, 16, 16, 32, 32, 32, 33, 64, 64]))
        d = int(max(k, r.choice([k, 40, 257, 1000, 1024, 4099, 16384, 20000, 33000])))
        m = int(r.choice([1, 31, 33, 255, 513, 2047, 2049, 5000, 70001]))
        b = int(r.choice([1, 2, 31, 32, 33, 65]))
        if m * k * b > 40e6:          # keep the oracle at a second or two per case
            b = max(1, int(40e6 // (m * k)))
        storage = "bf16" if q % 3 == 2 else "f32"
        shapes.append((m, d, k, b, storage))
    return shapes


SHAPES = draw_shapes(24) + [
    # enough labels for the register-resident kernels (several labels per lane), irregular everything else
    (300001, 257, 32, 2, "f32"), (262145, 33000, 16, 1, "f32"), (270003, 20000, 8, 3, "bf16"),
    (280000, 64, 64, 2, "bf16"), (263000, 16384, 32, 2, "bf16"), (290001, 9000, 64, 1, "f32"),
    # rows gathered in two slices: the slice-aware slot order with every register-resident fan-in
    (600, 40000, 64, 3, "f32"), (270001, 65536, 8, 1, "f32"), (5000, 50001, 16, 2, "f32"), (264000, 33000, 32, 2, "f32"),
]


@pytest.mark.parametrize("m,d,k,b,storage", SHAPES)
def test_random_shape(orc, m, d, k, b, storage):
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    cfg = wl.custom(m, d, k, b, storage=storage, positives=min(2, m), index=100 + SHAPES.index((m, d, k, b, storage)))
    print("shape", m, d, k, b, storage, flush=True)
    hp = wl.ADAM
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    off, lab = wl.gen_targets(cfg)
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x, d_g = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(g)
    out, gW, gx = gu.empty((b, m)).fill_(float("nan")), gu.empty((m, k)).fill_(float("nan")), gu.empty((b, d)).fill_(float("nan"))
    L.forward(d_x, d_idx, d_W, out, b)
    L.backward_weight(d_g, d_x, d_idx, gW, b)
    L.backward_input(d_g, d_idx, d_W, gx, b)
    assert_close(gu.host(out), orc.forward(x, idx, W), 1e-5, "out")
    assert_close(gu.host(gW), orc.backward_weight(g, x, idx), 1e-5, "grad_W")
    ref_gx = orc.backward_input(g, idx, W, d)
    assert_close(gu.host(gx), ref_gx, 1e-4, "grad_x")
    # both backward products from one call
    gW.fill_(float("nan")); gx.fill_(float("nan"))
    L.backward(d_g, d_x, d_idx, d_W, gW, gx, b)
    assert_close(gu.host(gW), orc.backward_weight(g, x, idx), 1e-5, "grad_W (one call)")
    assert_close(gu.host(gx), ref_gx, 1e-4, "grad_x (one call)")
    # redistribution of a third of the layer, then the fused step on the new connectivity
    r = wl.rng(cfg, 4)
    m1 = (r.standard_normal((m, k)) * 1e-3).astype(np.float32)
    m2 = (r.random((m, k)) * 1e-6).astype(np.float32)
    d_m1, d_m2 = gu.dev(m1), gu.dev(m2)
    n = L.redistribute(d_idx, d_W, d_m1, d_m2, 0.34, 99, 1)
    n_ref, _ = orc.redistribute(idx, W, m1, m2, d, 0.34, 99, 1)
    assert n == n_ref
    np.testing.assert_array_equal(gu.host(d_idx), idx)
    np.testing.assert_array_equal(gu.host(d_W).view(np.uint8), W.view(np.uint8))
    scale = float(np.float32(1.0 / b))
    loss = gu.empty((1,))
    loss_kind = (m + k) % 2
    L.train_step(d_x, d_idx, d_W, d_m1, d_m2, gu.dev(off), gu.dev(lab), loss_kind, scale, 1,
                 hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], out, gW, gx, loss, b)
    ref_out = orc.forward(x, idx, W)
    ref_loss, ref_g = (orc.bce_loss_grad if loss_kind == 0 else orc.sqh_loss_grad)(ref_out, off, lab, scale)
    got_g = gu.host(out)
    assert_close(got_g, ref_g, 1e-5, "g (fused)")
    assert abs(float(loss.item()) - ref_loss) <= 1e-5 * abs(ref_loss) + 1e-12
    got_gW = gu.host(gW)
    assert_close(got_gW, orc.backward_weight(got_g, x, idx), 1e-5, "grad_W (fused)")
    assert_close(gu.host(gx), orc.backward_input(got_g, idx, W, d), 1e-4, "grad_x (fused)")
    pre = orc.adam_step(W, got_gW, m1, m2, 1, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"])
    assert_close(gu.host(d_m1), m1, 1e-4, "m1 (fused)")
    assert_close(gu.host(d_m2), m2, 1e-4, "m2 (fused)")
    if storage == "f32":
        assert_close(gu.host(d_W), W, 1e-4, "W (fused)")
    else:
        got = wl.bf16_bits_to_f32(gu.host(d_W)).astype(np.float64)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(pre), 1e-30))) - 7)
        rms = float(np.sqrt(np.mean(pre.astype(np.float64) ** 2)))
        assert (np.abs(got - pre) <= 0.5 * ulp * (1 + 1e-3) + 1e-4 * np.abs(pre) + 1e-4 * rms).all()
    L.close()


@pytest.mark.parametrize("m,d,k,b,storage", [(3001, 1000, 32, 37, "f32"), (790001, 256, 32, 3, "f32"), (2500, 4096, 64, 6, "bf16"),
                                             (300001, 33000, 32, 2, "f32"), (1024, 64, 8, 16, "f32")])
def test_repeated_calls_are_bit_identical(m, d, k, b, storage):
    """Forward, the losses and backward-weight (a split batch leaves partial gradients that are added in a
    fixed order) fix the order of every sum: repeated calls on the same inputs must agree bit for bit.  A data
    race between wavefronts shows up here."""
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    cfg = wl.custom(m, d, k, b, storage=storage, positives=min(3, m), index=140)
    idx, W, x, g = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg), wl.gen_g(cfg)
    off, lab = wl.gen_targets(cfg)
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x, d_g, d_off, d_lab = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(g), gu.dev(off), gu.dev(lab)
    ref = None
    for rep in range(6):
        out, gW, g2, loss = gu.empty((b, m)), gu.empty((m, k)), gu.empty((b, m)), gu.empty((1,))
        if rep % 2:      # perturb the timing between repetitions
            torch.empty(1 << 22, device="cuda").normal_()
        L.forward(d_x, d_idx, d_W, out, b)
        L.sqh_loss_grad(out, d_off, d_lab, 0.5, g2, loss, b)
        L.backward_weight(d_g, d_x, d_idx, gW, b)
        got = (gu.host(out).view(np.uint32), gu.host(g2).view(np.uint32), float(loss.item()))
        gw_bits = gu.host(gW).view(np.uint32)
        if ref is None:
            ref, ref_gw = got, gw_bits
        else:
            np.testing.assert_array_equal(got[0], ref[0])
            np.testing.assert_array_equal(got[1], ref[1])
            assert got[2] == ref[2]
            np.testing.assert_array_equal(gw_bits, ref_gw)
