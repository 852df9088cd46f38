"""Prediction (Section 2): top-k labels of the score rows and the precision-at-k hit counts, HIP path
(through the C ABI) against the CPU oracle.  Integer and index work: bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def usl():
    from paper_2306_03725_amd import usl as u
    assert torch.cuda.is_available()
    return u


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


def run_topk(usl, gu, orc, scores, kk):
    b, m = scores.shape
    L = usl.Layer(m, 1, 1, b)
    lab = gu.empty((b, kk), torch.int32).fill_(-7)
    val = gu.empty((b, kk)).fill_(float("nan"))
    L.topk(gu.dev(scores), b, kk, lab, val)
    ref_lab, ref_val = orc.topk(scores, kk)
    np.testing.assert_array_equal(gu.host(lab), ref_lab)
    np.testing.assert_array_equal(gu.host(val).view(np.uint32), ref_val.view(np.uint32))
    return lab, ref_lab


# (m, b, kk): one segment; a ragged second segment; exactly one / one more than a segment; kk == m;
# several segments with the largest kk
TOPK_CASES = [(1024, 16, 5), (30938, 7, 3), (16384, 3, 1), (16385, 3, 32), (5, 4, 5), (1, 2, 1),
              (100000, 5, 32), (40, 3, 32)]


@pytest.mark.parametrize("m,b,kk", TOPK_CASES)
def test_topk_random_scores(usl, gu, orc, m, b, kk):
    print("topk", m, b, kk, flush=True)
    r = np.random.default_rng([m, b, kk])
    scores = (r.standard_normal((b, m)) * 3).astype(np.float32)
    run_topk(usl, gu, orc, scores, kk)


@pytest.mark.parametrize("m,b,kk", [(3000, 6, 17), (50000, 4, 32), (16390, 2, 8)])
def test_topk_ties_zeros_infinities(usl, gu, orc, m, b, kk):
    """Few distinct values: the order inside a tie is by label; -0 and +0 tie; infinities are scores."""
    r = np.random.default_rng([m, kk, 3])
    scores = r.integers(-2, 3, size=(b, m)).astype(np.float32)
    zeros = scores == 0
    scores[zeros] *= r.choice([-1.0, 1.0], size=int(zeros.sum())).astype(np.float32)
    scores[0, r.integers(0, m, 3)] = np.inf
    scores[1, :] = -np.inf                       # a whole row of equal scores: labels 0..kk-1
    scores[2 % b, m - 1] = 100.0                 # the very last label wins
    if b > 3:
        scores[3] = -0.0                         # all zeros of one sign ...
        scores[3, 1::2] = 0.0                    # ... and the other: still one tie
    run_topk(usl, gu, orc, scores, kk)


def test_topk_all_in_one_lane(usl, gu, orc):
    """The kk best scores all sit in labels that one lane of the workgroup reads (stride 256)."""
    m, b, kk = 40000, 2, 32
    scores = np.random.default_rng(4).standard_normal((b, m)).astype(np.float32)
    scores[0, 5::256][:60] += 50.0
    scores[1, 16384 + 255::256][:40] += 50.0
    run_topk(usl, gu, orc, scores, kk)


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_precision_hits(usl, gu, orc, name):
    cfg = wl.CONFIGS[name]
    m, b, kk = cfg.m, cfg.b, 5
    off, lab = wl.gen_targets(cfg)
    r = wl.rng(cfg, 31)
    scores = r.standard_normal((b, m)).astype(np.float32)
    for i in range(b):                            # lift some of every instance's targets into the top
        t = lab[off[i]:off[i + 1]]
        scores[i, t[: 1 + i % 3]] += 6.0
    top, ref_top = run_topk(usl, gu, orc, scores, kk)
    L = usl.Layer(m, cfg.d, cfg.k, b)
    hits = gu.empty((kk,), torch.int64).fill_(-1)
    L.precision_hits(top, gu.dev(off), gu.dev(lab), b, kk, hits)
    ref = orc.precision_hits(ref_top, off, lab)
    np.testing.assert_array_equal(gu.host(hits), ref)
    assert ref.sum() > 0
    L.precision_hits(top, gu.dev(off), gu.dev(lab), b, kk, hits)      # overwritten, not accumulated
    np.testing.assert_array_equal(gu.host(hits), ref)


def test_topk_argument_errors(usl, gu):
    L = usl.Layer(100, 10, 2, 4)
    out = gu.empty((4, 100)).zero_()
    lab, val = gu.empty((4, 40), torch.int32), gu.empty((4, 40))
    for kk, status in ((0, 1), (33, 2), (101, 2)):
        with pytest.raises(usl.UslError) as e:
            L.topk(out, 4, kk, lab, val)
        assert e.value.status == status
    with pytest.raises(usl.UslError):
        L.topk(out, 5, 3, lab, val)              # batch beyond max_b


@pytest.mark.parametrize("m,d,k,b,kk,storage", [(1024, 64, 8, 16, 5, "f32"), (30938, 1024, 32, 70, 3, "f32"),
                                                (3001, 1000, 32, 37, 32, "bf16"), (270001, 2048, 32, 33, 5, "f32"),
                                                (500, 203, 5, 65, 1, "f32")])
def test_predict_is_forward_then_topk(usl, gu, orc, m, d, k, b, kk, storage):
    """usl_predict (scores through library scratch) against the oracle's top-k of the scores the forward call
    writes, and those scores against the oracle's."""
    _predict_case(usl, gu, orc, m, d, k, b, kk, storage)


def test_predict_in_chunks(usl, gu, orc, monkeypatch):
    """A scratch cap of 70 rows: 150 instances go through as 70 + 70 + 10; a cap below 64 rows means 64."""
    m = 30938
    monkeypatch.setenv("USL_TUNE_PREDICT_BYTES", str(70 * m * 4))
    _predict_case(usl, gu, orc, m, 1024, 32, 150, 5, "f32")
    monkeypatch.setenv("USL_TUNE_PREDICT_BYTES", str(3 * m * 4))
    _predict_case(usl, gu, orc, m, 1024, 32, 130, 2, "f32")


def _predict_case(usl, gu, orc, m, d, k, b, kk, storage):
    from helpers import assert_close
    cfg = wl.custom(m, d, k, b, storage=storage, positives=1, index=150)
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    L = usl.Layer(m, d, k, b, storage)
    d_idx, d_W, d_x = gu.dev(idx), gu.dev(W), gu.dev(x)
    lab, val = gu.empty((b, kk), torch.int32).fill_(-1), gu.empty((b, kk)).fill_(float("nan"))
    L.predict(d_x, d_idx, d_W, b, kk, lab, val)
    out = gu.empty((b, m))
    L.forward(d_x, d_idx, d_W, out, b)
    scores = gu.host(out)
    assert_close(scores, orc.forward(x, idx, W), 1e-5, "scores")
    ref_lab, ref_val = orc.topk(scores, kk)
    np.testing.assert_array_equal(gu.host(lab), ref_lab)
    np.testing.assert_array_equal(gu.host(val).view(np.uint32), ref_val.view(np.uint32))
