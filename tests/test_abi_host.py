"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and turns bad arguments into status codes before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def usl():
    lib = os.path.join(ROOT, "paper_2306_03725_amd", "libusl.so")
    if not os.path.exists(lib):
        from paper_2306_03725_amd import build
        build.build(force=True)
    from paper_2306_03725_amd import usl as u
    return u


def header_symbols():
    text = open(os.path.join(ROOT, "include", "usl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(usl_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(usl):
    names = header_symbols()
    assert len(names) >= 15
    lib = ctypes.CDLL(usl.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(usl.SYMBOLS) == names
    assert "gfx950" in usl.version()


def test_create_rejects_bad_shapes(usl):
    bad = [dict(m=0, d=4, k=2, max_b=1), dict(m=4, d=0, k=1, max_b=1), dict(m=4, d=4, k=0, max_b=1),
           dict(m=4, d=4, k=2, max_b=0)]
    for kw in bad:
        with pytest.raises(usl.UslError) as e:
            usl.Layer(**kw)
        assert e.value.status == usl.USL_EINVAL
    for kw in [dict(m=4, d=4, k=5, max_b=1), dict(m=2 ** 31, d=8, k=1, max_b=1),
               dict(m=2 ** 27, d=64, k=32, max_b=1), dict(m=4, d=2 ** 24 + 1, k=1, max_b=1),
               dict(m=4, d=4, k=2, max_b=65536)]:
        with pytest.raises(usl.UslError) as e:
            usl.Layer(**kw)
        assert e.value.status == usl.USL_ESHAPE
    with pytest.raises(usl.UslError) as e:
        usl.Layer(4, 4, 2, 1, storage=7)
    assert e.value.status == usl.USL_EINVAL
    h = ctypes.c_void_p()
    assert usl._lib.usl_create(None, 4, 4, 2, 1, 0, None) == usl.USL_EINVAL
    assert usl._lib.usl_destroy(None) == usl.USL_OK


def test_calls_check_arguments_before_launching(usl):
    L = usl.Layer(64, 16, 4, 8)
    p = 4096    # never dereferenced: every call below must fail on the host
    cases = [
        (lambda: L.forward(None, p, p, p, 1), usl.USL_EINVAL),
        (lambda: L.forward(p, p, p, None, 1), usl.USL_EINVAL),
        (lambda: L.forward(p, p, p, p, 0), usl.USL_EINVAL),
        (lambda: L.forward(p, p, p, p, 9), usl.USL_ESHAPE),
        (lambda: L.backward_weight(p, p, None, p, 1), usl.USL_EINVAL),
        (lambda: L.backward_input(p, p, p, p, -1), usl.USL_EINVAL),
        (lambda: L.bce_loss_grad(p, p, p, float("nan"), p, p, 1), usl.USL_EINVAL),
        (lambda: L.bce_loss_grad(p, p, p, 1.0, p, None, 1), usl.USL_EINVAL),
        (lambda: L.adam_step(p, p, p, p, 0, 1e-3, 0.9, 0.999, 1e-8), usl.USL_EINVAL),
        (lambda: L.adam_step(p, p, p, p, 1, 1e-3, 1.0, 0.999, 1e-8), usl.USL_EINVAL),
        (lambda: L.adam_step(p, p, p, p, 1, 1e-3, 0.9, 0.999, -1.0), usl.USL_EINVAL),
        (lambda: L.redistribute(p, p, p, p, 1.5, 1, 0), usl.USL_EINVAL),
        (lambda: L.redistribute(p, p, p, p, -0.1, 1, 0), usl.USL_EINVAL),
        (lambda: L.redistribute(p, p, p, p, float("nan"), 1, 0), usl.USL_EINVAL),
        (lambda: L.redistribute(p, p, p, p, 0.5, 1, 2 ** 64 - 1), usl.USL_EINVAL),
        (lambda: L.redistribute(None, p, p, p, 0.5, 1, 0), usl.USL_EINVAL),
        (lambda: L.init_indices(None, 1), usl.USL_EINVAL),
    ]
    for call, status in cases:
        with pytest.raises(usl.UslError) as e:
            call()
        assert e.value.status == status, str(e.value)
        assert str(e.value)
    # fraction 0 (and any fraction that rounds to no slot) returns before touching anything
    assert L.redistribute(p, p, p, p, 0.0, 1, 0) == 0
    assert L.redistribute(p, p, p, p, 1.0 / 1024, 1, 0) == 0
    L.invalidate()
    L.close()


def test_valid_call_without_a_gpu_reports_hip_error(usl):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    L = usl.Layer(64, 16, 4, 8)
    with pytest.raises(usl.UslError) as e:
        L.forward(4096, 4096, 4096, 4096, 1)
    assert e.value.status == usl.USL_EHIP


def test_product_package_does_not_touch_the_oracle():
    """No file of the product package imports, loads or names the oracle."""
    pkg = os.path.join(ROOT, "paper_2306_03725_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "oracle" not in text.lower(), os.path.join(base, f)


def test_build_check_of_the_untracked_warm_up_load():
    """The build refuses a compile in which the register that receives k_bwi_lds's warm-up load (issued from inline
    assembly, unknown to the compiler's wait bookkeeping) is touched anywhere else inside the loop."""
    from paper_2306_03725_amd import build
    good = """_ZN1_9k_bwi_ldsIfEEvPKf:
; %bb.0:
	v_mov_b32_e32 v7, 0
.LBB0_1:                                ; =>This Loop Header: Depth=1
	s_waitcnt vmcnt(0)
	s_barrier
; %bb.2:                                ;   in Loop: Header=BB0_1 Depth=1
	;;#ASMSTART
	global_load_dword v7, v3, s[4:5]
	;;#ASMEND
.LBB0_3:                                ;   Parent Loop BB0_1 Depth=1
                                        ; =>  This Inner Loop Header: Depth=2
	ds_read_b32 v8, v9
	s_cbranch_scc1 .LBB0_3
; %bb.4:                                ;   in Loop: Header=BB0_1 Depth=1
	s_cbranch_scc1 .LBB0_1
; %bb.5:
	v_mov_b32_e32 v7, 0
	s_endpgm
.Lfunc_end0:
""".splitlines()
    assert build.scan_listing_for_untracked_load(good) == 1
    for bad_line, where in (("\tv_mov_b32_e32 v12, v7", "ds_read_b32 v8, v9"), ("\tscratch_store_dwordx2 off, v[6:7], off", "s_barrier")):
        bad = list(good)
        bad.insert(next(i for i, l in enumerate(bad) if where in l), bad_line)
        with pytest.raises(RuntimeError, match="v7"):
            build.scan_listing_for_untracked_load(bad)
    spilled = list(good)
    at = next(i for i, l in enumerate(spilled) if "ds_read_b32 v8, v9" in l)
    spilled[at:at] = ["\tscratch_load_dword v20, off, off", "\tscratch_load_dword v21, off, off offset:4"]
    with pytest.raises(RuntimeError, match="register reloads"):
        build.scan_listing_for_untracked_load(spilled)
    with pytest.raises(RuntimeError, match="no warm-up load"):
        build.scan_listing_for_untracked_load([l for l in good if "global_load_dword" not in l])
    # the kernel for both products issues its warm-up loads from a loop over lines, inside the loop over the passes
    # (full addresses, no scalar base): the loop over the passes is the one that is searched
    nested = """_ZN1_10k_both_ldsIfEEvPKf:
; %bb.0:
	v_mov_b32_e32 v5, 0
.LBB1_1:                                ; =>This Loop Header: Depth=1
                                        ;     Child Loop BB1_3 Depth 2
	s_waitcnt vmcnt(0)
	s_barrier
; %bb.2:                                ;   in Loop: Header=BB1_1 Depth=1
	v_mov_b32_e32 v6, v0
.LBB1_3:                                ;   Parent Loop BB1_1 Depth=1
                                        ; =>  This Inner Loop Header: Depth=2
	v_cmp_le_i32_e32 vcc, s71, v6
; %bb.4:                                ;   in Loop: Header=BB1_3 Depth=2
	;;#ASMSTART
	global_load_dword v5, v[12:13], off
	;;#ASMEND
	s_cbranch_execnz .LBB1_3
; %bb.5:                                ;   in Loop: Header=BB1_1 Depth=1
	ds_read_b32 v8, v9
	s_cbranch_scc1 .LBB1_1
; %bb.6:
	s_endpgm
.Lfunc_end1:
""".splitlines()
    assert build.scan_listing_for_untracked_load(nested) == 1
    bad = list(nested)
    bad.insert(next(i for i, l in enumerate(bad) if "ds_read_b32 v8, v9" in l), "\tv_add_u32_e32 v5, v5, v9")
    with pytest.raises(RuntimeError, match="v5"):
        build.scan_listing_for_untracked_load(bad)
