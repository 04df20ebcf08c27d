"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before touching the GPU (none of these calls launches work)."""
import ctypes
import os
import re

import pytest

import paper_2309_06626_amd.binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparse_conv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(n for n in names if n.startswith(("sparse_conv", "sparse_mask", "dense_conv", "sc_"))))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert {"sparse_conv_plan", "sparse_conv_run", "dense_conv_run", "sparse_conv_workspace_bytes",
            "sparse_mask_generate", "sparse_mask_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = B.lib()
    seen = set()
    for s in range(8):
        msg = L.sc_status_string(s).decode()
        assert msg and msg not in seen
        seen.add(msg)


def good():
    return B.make_desc(2, 16, 8, 8, 16, sparsity=0.5)


def test_output_shape_and_workspace():
    d = good()
    assert B.sparse_conv_output_shape(d) == (8, 8, 128)
    assert B.sparse_conv_workspace_bytes(d) >= 128 * 4 + 128 + 16 * 144 * 2
    d = B.make_desc(1, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3)
    assert B.sparse_conv_output_shape(d) == (112, 112, 112 * 112)
    d = B.make_desc(1, 4, 9, 7, 4, 3, 2, 2, 1, 0, 1, 2, 1)
    assert B.sparse_conv_output_shape(d) == ((9 - 4 - 1) // 2 + 1, (7 + 2 - 1 - 1) // 1 + 1,
                                             ((9 - 4 - 1) // 2 + 1) * ((7 + 2 - 1 - 1) + 1))


@pytest.mark.parametrize("field,value,status", [
    ("n", 0, B.SC_ERR_BAD_SHAPE), ("c_in", -1, B.SC_ERR_BAD_SHAPE), ("kh", 0, B.SC_ERR_BAD_SHAPE),
    ("stride_w", 0, B.SC_ERR_BAD_SHAPE), ("pad_h", -1, B.SC_ERR_BAD_SHAPE), ("dil_w", 0, B.SC_ERR_BAD_SHAPE),
    ("kh", 64, B.SC_ERR_BAD_SHAPE),            # window larger than the padded input: empty output
    ("groups", 2, B.SC_ERR_UNSUPPORTED), ("dtype", 9, B.SC_ERR_UNSUPPORTED), ("layout", 5, B.SC_ERR_UNSUPPORTED),
    ("mask_mode", 3, B.SC_ERR_UNSUPPORTED), ("out_mode", 2, B.SC_ERR_UNSUPPORTED),
    ("sparsity", 1.0, B.SC_ERR_BAD_SHAPE), ("sparsity", float("nan"), B.SC_ERR_BAD_SHAPE),
    ("n", 1 << 22, B.SC_ERR_BAD_SHAPE),        # 32-bit element offsets would overflow
])
def test_descriptor_validation(field, value, status):
    d = good()
    setattr(d, field, value)
    n = ctypes.c_size_t()
    assert B.lib().sparse_conv_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == status
    out = ctypes.c_void_p(123)
    # plan validates the descriptor before looking at any pointer or calling HIP
    assert B.lib().sparse_conv_plan(ctypes.byref(d), 256, 256, 256, 1 << 30, None, ctypes.byref(out)) == status
    assert out.value is None


def test_null_and_alignment_errors_come_before_any_gpu_work():
    L = B.lib()
    d = good()
    n = ctypes.c_size_t()
    assert L.sparse_conv_workspace_bytes(None, ctypes.byref(n)) == B.SC_ERR_NULL
    assert L.sparse_conv_workspace_bytes(ctypes.byref(d), None) == B.SC_ERR_NULL
    assert L.sparse_conv_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == B.SC_OK
    out = ctypes.c_void_p()
    assert L.sparse_conv_plan(ctypes.byref(d), None, 256, 256, n.value, None, ctypes.byref(out)) == B.SC_ERR_NULL
    assert L.sparse_conv_plan(ctypes.byref(d), 256, None, 256, n.value, None, ctypes.byref(out)) == B.SC_ERR_NULL
    assert L.sparse_conv_plan(ctypes.byref(d), 256, 256, None, n.value, None, ctypes.byref(out)) == B.SC_ERR_NULL
    assert L.sparse_conv_plan(ctypes.byref(d), 256, 256, 256, n.value, None, None) == B.SC_ERR_NULL
    assert L.sparse_conv_plan(ctypes.byref(d), 256, 256, 256, n.value - 1, None, ctypes.byref(out)) == B.SC_ERR_WORKSPACE
    assert L.sparse_conv_plan(ctypes.byref(d), 256, 256, 512 + 64, n.value, None, ctypes.byref(out)) == B.SC_ERR_ALIGN
    assert L.sparse_conv_plan(ctypes.byref(d), 256, 256 + 4, 512, n.value, None, ctypes.byref(out)) == B.SC_ERR_ALIGN
    assert L.sparse_conv_run(None, 256, 256, 256, None) == B.SC_ERR_NULL
    assert L.dense_conv_run(None, 256, 256, 256, None) == B.SC_ERR_NULL
    assert L.sparse_conv_plan_info(None, None, None, None, None, None) == B.SC_ERR_NULL
    assert L.sc_add_relu(None, 256, 256, B.SC_BF16, 10, None) == B.SC_ERR_NULL
    assert L.sc_add_relu(256, 256, 256, 7, 10, None) == B.SC_ERR_UNSUPPORTED
    assert L.sc_add(256, None, 256, B.SC_BF16, 10, None) == B.SC_ERR_NULL
    assert L.sc_add(256, 256, 256, 7, 10, None) == B.SC_ERR_UNSUPPORTED
    assert L.sc_add(256, 256, 256, B.SC_F16, -1, None) == B.SC_ERR_BAD_SHAPE
    assert L.sc_maxpool2d_nhwc(256, 256, B.SC_BF16, 1, 4, 4, 8, 3, 2, 2, None) == B.SC_ERR_BAD_SHAPE
    L.sparse_conv_plan_destroy(None)  # harmless


def test_missing_library_is_a_loud_error(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.lib()


def test_mask_generator_rejects_bad_arguments_before_any_gpu_work():
    L = B.lib()
    size = ctypes.c_size_t(123)
    assert L.sparse_mask_workspace_bytes(7, 5, ctypes.byref(size)) == B.SC_OK and size.value >= 7 * 5 * 8 and size.value % 8 == 0
    assert L.sparse_mask_workspace_bytes(7, 5, None) == B.SC_ERR_NULL
    assert L.sparse_mask_workspace_bytes(0, 5, ctypes.byref(size)) == B.SC_ERR_BAD_SHAPE and size.value == 0
    assert L.sparse_mask_workspace_bytes(1 << 14, 1 << 14, ctypes.byref(size)) == B.SC_ERR_BAD_SHAPE
    fake = 0x1000   # never dereferenced: every check below fails on the host
    gen = L.sparse_mask_generate
    assert gen(None, 8, 8, 4, 4, 0.5, fake, fake, 1 << 20, None) == B.SC_ERR_NULL
    assert gen(fake, 8, 8, 4, 4, 0.5, None, fake, 1 << 20, None) == B.SC_ERR_NULL
    assert gen(fake, 8, 8, 4, 4, 0.5, fake, None, 1 << 20, None) == B.SC_ERR_NULL
    assert gen(fake, 8, 8, 9, 4, 0.5, fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE      # layer larger than the input
    assert gen(fake, 8, 8, 4, 0, 0.5, fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE
    assert gen(fake, 0, 8, 4, 4, 0.5, fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE
    assert gen(fake, 8, 8, 4, 4, -0.1, fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE
    assert gen(fake, 8, 8, 4, 4, 1.5, fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE
    assert gen(fake, 8, 8, 4, 4, float("nan"), fake, fake, 1 << 20, None) == B.SC_ERR_BAD_SHAPE
    assert gen(fake, 8, 8, 4, 4, 0.5, fake, fake, 4 * 4 * 8 - 1, None) == B.SC_ERR_WORKSPACE
    assert gen(fake, 8, 8, 4, 4, 0.5, fake, fake + 4, 1 << 20, None) == B.SC_ERR_ALIGN


def test_grouped_layers_other_than_depthwise_are_refused():
    L = B.lib()
    size = ctypes.c_size_t()
    for kw in (dict(c_in=16, c_out=16, groups=4), dict(c_in=16, c_out=32, groups=16), dict(c_in=16, c_out=16, groups=16, layout=B.SC_NCHW)):
        d = B.make_desc(1, kw["c_in"], 8, 8, kw["c_out"], groups=kw["groups"], layout=kw.get("layout", B.SC_NHWC))
        assert L.sparse_conv_workspace_bytes(ctypes.byref(d), ctypes.byref(size)) == B.SC_ERR_UNSUPPORTED
    d = B.make_desc(1, 16, 8, 8, 16, groups=16)
    assert L.sparse_conv_workspace_bytes(ctypes.byref(d), ctypes.byref(size)) == B.SC_OK


def test_plan_refresh_calls_reject_null_arguments():
    L = B.lib()
    fake = 0x1000
    assert L.sparse_conv_plan_set_mask(None, fake, None) == B.SC_ERR_NULL
    assert L.sparse_conv_plan_set_filters(None, fake, None) == B.SC_ERR_NULL
