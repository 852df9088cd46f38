"""The allocation-free variant of the BCE loss call (static device scratch) against the allocating one:
same g bit for bit, same loss bit for bit (same kernels, same fixed order of the additions), on two calls in
a row, the second with a smaller input; and against the oracle to the loss tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu


def test_bce_noalloc_matches_the_allocating_call(orc):
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    m, d, k, max_b = 30938, 1024, 32, 24
    L = usl.Layer(m, d, k, max_b)
    for b, index in ((24, 51), (7, 52)):          # the second call is smaller: stale slots must not be read
        cfg = wl.custom(m, d, k, b, positives=5, zipf_a=1.1, index=index)
        print("noalloc case", m, b, flush=True)
        r = wl.rng(cfg, 7)
        out = (r.standard_normal((b, m)) * 3).astype(np.float32)
        off, lab = wl.gen_targets(cfg)
        scale = float(np.float32(1.0 / b))
        d_out, d_off, d_lab = gu.dev(out), gu.dev(off), gu.dev(lab)
        g_ref, loss_ref = gu.empty((b, m)), gu.empty((1,))
        L.bce_loss_grad(d_out, d_off, d_lab, scale, g_ref, loss_ref, b)
        g, loss = gu.empty((b, m)).fill_(float("nan")), gu.empty((1,)).fill_(float("nan"))
        L.bce_loss_grad_noalloc(d_out, d_off, d_lab, scale, g, loss, b)
        torch.cuda.synchronize()
        assert torch.equal(g, g_ref)
        assert gu.host(loss).view(np.uint32)[0] == gu.host(loss_ref).view(np.uint32)[0]
        ref_loss, ref_g = orc.bce_loss_grad(out, off, lab, scale)
        assert_close(gu.host(g), ref_g, 1e-5, "g")
        assert abs(float(loss.item()) - ref_loss) <= 1e-5 * abs(ref_loss)
    # beyond the static array: refused on the host, nothing launched
    big = usl.Layer(3_000_000, 64, 8, 1024)
    with pytest.raises(usl.UslError) as e:
        big.bce_loss_grad_noalloc(4096, 4096, 4096, 1.0, 4096, 4096, 1024)
    assert e.value.status == usl.USL_ESHAPE
    big.close()
    L.close()
