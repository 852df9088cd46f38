"""Label-subset products (Section 6, outlook: a subset of labels is a slicing of the [m][k] arrays):
HIP path through the C ABI against the CPU oracle, same tolerances as the full products."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_close

pytestmark = pytest.mark.gpu

# (m, d, k, b, n_rows, storage)
CASES = [
    (1024, 64, 8, 16, 100, "f32"),
    (3001, 1000, 32, 37, 3001, "f32"),        # every label once, permuted
    (30938, 1024, 32, 24, 5000, "f32"),
    (30938, 1024, 32, 24, 1, "bf16"),
    (500, 200, 5, 7, 77, "f32"),              # generic-k kernels
    (300000, 2048, 32, 9, 280000, "f32"),     # subset large enough for the register-resident blocks
    (2000, 40000, 16, 3, 333, "bf16"),        # rows wider than the LDS budget
]


@pytest.mark.parametrize("m,d,k,b,n,storage", CASES)
def test_label_subset_products(orc, m, d, k, b, n, storage):
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    cfg = wl.custom(m, d, k, b, storage=storage, positives=1, index=40 + CASES.index((m, d, k, b, n, storage)))
    print("subset", m, d, k, b, n, storage, flush=True)
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    r = wl.rng(cfg, 9)
    rows = r.permutation(m)[:n] if n == m else r.choice(m, size=n, replace=True)
    rows = rows.astype(np.int32)
    g_rows = (r.standard_normal((b, n)) * 0.01).astype(np.float32)
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x, d_rows, d_g = gu.dev(idx), gu.dev(W), gu.dev(x), gu.dev(rows), gu.dev(g_rows)
    out = gu.empty((b, n)).fill_(float("nan"))
    gW = gu.empty((n, k)).fill_(float("nan"))
    gx = gu.empty((b, d)).fill_(float("nan"))
    L.forward_rows(d_x, d_idx, d_W, d_rows, n, out, b)
    L.backward_weight_rows(d_g, d_x, d_idx, d_rows, n, gW, b)
    L.backward_input_rows(d_g, d_idx, d_W, d_rows, n, gx, b)
    rows64 = rows.astype(np.int64)
    assert_close(gu.host(out), orc.forward_rows(x, idx, W, rows64), 1e-5, "out_rows")
    assert_close(gu.host(gW), orc.backward_weight_rows(g_rows, x, idx, rows64), 1e-5, "grad_W_rows")
    assert_close(gu.host(gx), orc.backward_input_rows(g_rows, idx, W, rows64, d), 1e-4, "grad_x")
    # the full-width calls of the same context are untouched by the subset calls in between
    full = gu.empty((b, m))
    L.forward(d_x, d_idx, d_W, full, b)
    if n <= 5000:
        sub = gu.host(full)[:, rows64]
        assert_close(gu.host(out), sub, 1e-5, "subset vs columns of the full product")
    # a second subset of another size through the same context
    n2 = max(1, n // 3)
    rows2 = np.ascontiguousarray(rows[:n2])
    out2 = gu.empty((b, n2))
    L.forward_rows(d_x, d_idx, d_W, gu.dev(rows2), n2, out2, b)
    assert_close(gu.host(out2), orc.forward_rows(x, idx, W, rows2.astype(np.int64)), 1e-5, "out_rows, second size")


def test_label_subset_argument_errors():
    import gpu_util as gu
    from paper_2306_03725_amd import usl
    L = usl.Layer(100, 10, 2, 4)
    t = gu.empty((400,))
    rows = gu.empty((4,), torch.int32).zero_()
    with pytest.raises(usl.UslError) as e:
        L.forward_rows(t, rows, t, rows, 0, t, 4)
    assert e.value.status == 1
    with pytest.raises(usl.UslError) as e:
        L.forward_rows(t, rows, t, rows, 4, t, 5)
    assert e.value.status == 2
