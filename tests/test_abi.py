"""The C-ABI library loads, exports every symbol the header declares, and rejects
bad shapes on the host before touching a device (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2505_23317_amd import cfdetr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cfdetr.h")).read()
    return sorted(set(re.findall(r"CFDETR_API[^;(]*?\b(cfdetr_\w+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = _declared()
    for must in ("cfdetr_coarse_encode", "cfdetr_select_fine", "cfdetr_fine_encode",
                 "cfdetr_multilevel_batch", "cfdetr_create", "cfdetr_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = cfdetr.load_library()
    names = _declared()
    assert sorted(names) == sorted(cfdetr.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def _good_cfg():
    c = cfdetr.CfdetrConfig()
    c.n_levels = 2
    c.patch[0], c.patch[1], c.patch[2] = 32, 16, 0
    c.img_h = c.img_w = 128
    c.d_model, c.n_heads, c.n_layers, c.d_ffn = 64, 2, 1, 128
    c.max_batch, c.max_tokens_total = 1, 64
    c.image_dtype, c.act_dtype, c.ln_eps = cfdetr.CFDETR_FP32, cfdetr.CFDETR_BF16, 1e-5
    return c


@pytest.mark.parametrize("field,value", [
    ("n_levels", 4), ("n_levels", 0), ("img_h", 100), ("d_model", 60), ("n_heads", 3),
    ("n_heads", 4), ("d_ffn", 100), ("n_layers", 0), ("max_batch", 65), ("max_batch", 0),
    ("max_tokens_total", 15),
])
def test_create_rejects_bad_shapes_on_the_host(field, value):
    lib = cfdetr.load_library()
    c = _good_cfg()
    setattr(c, field, value)
    w = cfdetr.CfdetrWeights()
    out = ctypes.c_void_p(1234)
    st = lib.cfdetr_create(ctypes.byref(c), ctypes.byref(w), ctypes.byref(out))
    assert st == cfdetr.CFDETR_ESHAPE
    assert out.value is None


def test_create_rejects_bad_patch_chain_and_null_arguments():
    lib = cfdetr.load_library()
    w = cfdetr.CfdetrWeights()
    out = ctypes.c_void_p()
    c = _good_cfg()
    c.patch[1] = 8
    assert lib.cfdetr_create(ctypes.byref(c), ctypes.byref(w), ctypes.byref(out)) == cfdetr.CFDETR_ESHAPE
    c = _good_cfg()
    c.patch[0], c.patch[1] = 48, 24
    c.img_h = c.img_w = 96
    assert lib.cfdetr_create(ctypes.byref(c), ctypes.byref(w), ctypes.byref(out)) == cfdetr.CFDETR_ESHAPE
    c = _good_cfg()
    assert lib.cfdetr_create(None, ctypes.byref(w), ctypes.byref(out)) == cfdetr.CFDETR_EINVAL
    # good shape but null weight pointers: rejected before any device work
    assert lib.cfdetr_create(ctypes.byref(c), ctypes.byref(w), ctypes.byref(out)) == cfdetr.CFDETR_EINVAL
    c.act_dtype = 7
    assert lib.cfdetr_create(ctypes.byref(c), ctypes.byref(w), ctypes.byref(out)) == cfdetr.CFDETR_EINVAL


def test_null_context_is_rejected_everywhere():
    lib = cfdetr.load_library()
    assert lib.cfdetr_coarse_encode(None, None, 1, None, None, None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_select_fine(None, None, None, None, 1, None, None, None, None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_fine_encode(None, None, 1, None, None, None, None, None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_multilevel_batch(None, None, 1, None, None, None, None, None, None, None,
                                       None, None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_sync_status(None, None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_profile_begin(None) == cfdetr.CFDETR_EINVAL
    assert lib.cfdetr_workspace_bytes(None) == 0
    lib.cfdetr_destroy(None)
