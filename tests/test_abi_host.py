"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host logic (descriptors, output-size rule, validation, error codes) behaves as documented.
No compute call reaches a launch here: every one is rejected by validation first."""
import ctypes
import os
import re

import pytest

from paper_1910_00078_amd import cvx

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "cvx.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cvx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    L = cvx.lib()
    for n in names:
        assert hasattr(L, n), "libcvx.so does not export %s" % n
    assert sorted(cvx.EXPORTS) == names


def test_status_strings():
    assert cvx.cvx_status_string(0) == "CVX_OK"
    assert cvx.cvx_status_string(4) == "CVX_ERR_UNSUPPORTED"
    assert cvx.cvx_status_string(99) == "CVX_ERR_UNKNOWN"


def _desc(dtype, shape):
    t = cvx.cvx_tensor_desc_create()
    cvx.cvx_tensor_desc_set_4d(t, dtype, *shape)
    return t


def _conv(pad=(0, 0), stride=(1, 1), dil=(1, 1), groups=1):
    c = cvx.cvx_conv_desc_create()
    cvx.cvx_conv_desc_set_2d(c, *pad, *stride, *dil)
    cvx.cvx_conv_desc_set_group_count(c, groups)
    return c


def test_descriptor_roundtrip():
    t = _desc(cvx.CVX_BF16, (32, 64, 56, 56))
    assert cvx.cvx_tensor_desc_get_4d(t) == (cvx.CVX_BF16, 32, 64, 56, 56)
    c = _conv((3, 2), (2, 1), (1, 4), 2)
    assert cvx.cvx_conv_desc_get_2d(c) == (3, 2, 2, 1, 1, 4, 2)
    fresh = cvx.cvx_conv_desc_create()
    assert cvx.cvx_conv_desc_get_2d(fresh) == (0, 0, 1, 1, 1, 1, 1)
    for d in (c, fresh):
        cvx.cvx_conv_desc_destroy(d)
    cvx.cvx_tensor_desc_destroy(t)


@pytest.mark.parametrize("x,w,pad,stride,dil,want", [
    ((1, 8, 8, 8), (8, 8, 3, 3), (1, 1), (1, 1), (1, 1), (1, 8, 8, 8)),
    ((32, 64, 56, 56), (64, 64, 3, 3), (1, 1), (1, 1), (1, 1), (32, 64, 56, 56)),
    ((64, 256, 56, 56), (64, 256, 1, 1), (0, 0), (1, 1), (1, 1), (64, 64, 56, 56)),
    ((64, 3, 224, 224), (64, 3, 7, 7), (3, 3), (2, 2), (1, 1), (64, 64, 112, 112)),   # 111.5 -> floor
    ((128, 256, 28, 28), (256, 256, 3, 3), (1, 1), (2, 2), (1, 1), (128, 256, 14, 14)),  # 13.5 -> floor
    ((1, 1, 5, 5), (1, 1, 3, 3), (0, 0), (1, 1), (2, 2), (1, 1, 1, 1)),
    ((2, 3, 9, 7), (4, 3, 2, 3), (0, 2), (3, 2), (2, 1), (2, 4, 3, 5)),
])
def test_output_dim_rule(x, w, pad, stride, dil, want):
    """Floor rule; the two stride-2 cases are the ones where the stride does not divide the span."""
    xd, wd, c = _desc(cvx.CVX_F32, x), _desc(cvx.CVX_F32, w), _conv(pad, stride, dil)
    assert cvx.cvx_conv_fwd_output_dim(c, xd, wd) == want


def _expect(status, fn, *a):
    with pytest.raises(cvx.CvxError) as e:
        fn(*a)
    assert e.value.status == status, str(e.value)


def test_descriptor_validation():
    t = cvx.cvx_tensor_desc_create()
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_tensor_desc_set_4d, t, 9, 1, 1, 1, 1)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_tensor_desc_set_4d, t, cvx.CVX_F32, 0, 1, 1, 1)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_tensor_desc_set_4d, t, cvx.CVX_F32, 1, -1, 1, 1)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_tensor_desc_set_4d, t, cvx.CVX_F32, 65536, 32768, 1, 1)  # 2^31 elements
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_tensor_desc_get_4d, t)       # never set
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_tensor_desc_set_4d, None, cvx.CVX_F32, 1, 1, 1, 1)
    c = cvx.cvx_conv_desc_create()
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_desc_set_2d, c, -1, 0, 1, 1, 1, 1)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_desc_set_2d, c, 0, 0, 0, 1, 1, 1)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_desc_set_2d, c, 0, 0, 1, 1, 1, 0)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_desc_set_group_count, c, 0)
    assert cvx.cvx_conv_desc_get_2d(c) == (0, 0, 1, 1, 1, 1, 1)        # failed sets change nothing


def test_output_dim_errors():
    xd, c = _desc(cvx.CVX_F32, (1, 4, 6, 6)), _conv()
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_conv_fwd_output_dim, c, xd, _desc(cvx.CVX_F32, (2, 3, 3, 3)))
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_fwd_output_dim, c, xd, _desc(cvx.CVX_F32, (2, 4, 7, 7)))
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_fwd_output_dim, _conv(dil=(3, 3)), xd, _desc(cvx.CVX_F32, (2, 4, 3, 3)))
    g2 = _conv(groups=2)
    assert cvx.cvx_conv_fwd_output_dim(g2, xd, _desc(cvx.CVX_F32, (6, 2, 3, 3))) == (1, 6, 4, 4)
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_conv_fwd_output_dim, g2, xd, _desc(cvx.CVX_F32, (5, 2, 3, 3)))
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_conv_fwd_output_dim, g2, xd, _desc(cvx.CVX_F32, (6, 4, 3, 3)))


def test_compute_calls_reject_bad_arguments_before_launching():
    """Fake (never dereferenced) device addresses: each call must fail in validation."""
    h = cvx.cvx_create(0)
    xd, wd = _desc(cvx.CVX_BF16, (2, 8, 6, 6)), _desc(cvx.CVX_BF16, (4, 8, 3, 3))
    c = _conv((1, 1))
    yd = _desc(cvx.CVX_BF16, (2, 4, 6, 6))
    bd = _desc(cvx.CVX_BF16, (1, 4, 1, 1))
    X, Wt, Y, B = 0x10000, 0x20000, 0x30000, 0x40000
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd, None, xd, X, wd, Wt, c, yd, Y)
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd, h, xd, None, wd, Wt, c, yd, Y)
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd, h, xd, X, wd, Wt, c, yd, None)
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd, h, xd, X, None, Wt, c, yd, Y)
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_conv_fwd, h, xd, X, wd, Wt, c, _desc(cvx.CVX_BF16, (2, 4, 5, 6)), Y)
    _expect(cvx.CVX_ERR_UNSUPPORTED, cvx.cvx_conv_fwd, h, xd, X, wd, Wt, c, _desc(cvx.CVX_F16, (2, 4, 6, 6)), Y)
    _expect(cvx.CVX_ERR_UNSUPPORTED, cvx.cvx_conv_fwd, h, xd, X, _desc(cvx.CVX_F32, (4, 8, 3, 3)), Wt, c, yd, Y)
    _expect(cvx.CVX_ERR_ALIGNMENT, cvx.cvx_conv_fwd, h, xd, X + 1, wd, Wt, c, yd, Y)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_fwd, h, xd, X, wd, Wt, c, yd, X + 64)      # y overlaps x
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_fwd_fused, h, xd, X, wd, Wt, c, bd, B, 17, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_conv_fwd_fused, h, xd, X, wd, Wt, c,
            _desc(cvx.CVX_BF16, (1, 5, 1, 1)), B, cvx.CVX_ACT_RELU, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_UNSUPPORTED, cvx.cvx_conv_fwd_fused, h, xd, X, wd, Wt, c,
            _desc(cvx.CVX_F16, (1, 4, 1, 1)), B, cvx.CVX_ACT_RELU, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd_fused, h, xd, X, wd, Wt, c, None, B, cvx.CVX_ACT_RELU, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_NULL, cvx.cvx_conv_fwd_fused_bn, h, xd, X, wd, Wt, c, bd, B, None, B, B, B, 1e-5,
            cvx.CVX_ACT_RELU, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_conv_fwd_fused_bn, h, xd, X, wd, Wt, c, bd, B, B, B, B, B, -1.0,
            cvx.CVX_ACT_RELU, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_SHAPE_MISMATCH, cvx.cvx_bias_add, h, _desc(cvx.CVX_BF16, (1, 3, 1, 1)), B, yd, Y)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_activation_fwd, h, 42, 0.0, yd, Y)
    _expect(cvx.CVX_ERR_BAD_PARAM, cvx.cvx_set_kernel_policy, h, 5)
    assert "policy" in cvx.cvx_last_error()
    cvx.cvx_destroy(h)


def test_stream_roundtrip_and_query():
    h = cvx.cvx_create(0)
    assert cvx.cvx_get_stream(h) == 0
    cvx.cvx_set_stream(h, 0x1234)
    assert cvx.cvx_get_stream(h) == 0x1234
    cvx.cvx_destroy(h)
    xd, wd = _desc(cvx.CVX_F32, (1, 8, 8, 8)), _desc(cvx.CVX_F32, (8, 8, 3, 3))
    name, ws = cvx.cvx_conv_fwd_query(xd, wd, _conv((1, 1)), _desc(cvx.CVX_F32, (1, 8, 8, 8)))
    assert ws == 0 and name


def test_kernel_choice_is_host_logic_and_follows_the_shape():
    """cvx_conv_fwd_query needs no GPU: the choice of kernel family is a pure function of the
    descriptors.  The benchmark layers and a few neighbours land where they were built to."""
    import workloads as wl
    code = {wl.F32: cvx.CVX_F32, wl.F16: cvx.CVX_F16, wl.BF16: cvx.CVX_BF16}

    def family(w):
        plan = cvx.ConvPlan(code[w.dtype], (w.N, w.C, w.H, w.W), (w.K, w.C // w.groups, w.R, w.S),
                            w.pad, w.stride, w.dil, w.groups)
        try:
            return plan.kernel_name()
        finally:
            plan.close()

    want = {"c1": "direct_", "c2": "igemm_", "c3a": "pointwise_", "c3b": "pointwise_", "c4": "stem_stream_",
            "c5a": "igemm_", "c5b": "igemm_"}
    for name, prefix in want.items():
        assert family(wl.WORKLOADS[name]).startswith(prefix), name
    v = wl.small_variant
    assert family(v(wl.WORKLOADS["c4"], K=96)).startswith("stem_256x64")            # K > 64: the general stem kernel
    assert family(v(wl.WORKLOADS["c3a"], stride=(2, 2))).startswith("igemm_")        # strided 1x1 is not pointwise
    assert family(v(wl.WORKLOADS["c3a"], H=7, W=7)).startswith("igemm_")             # 49 pixels: not a multiple of 8
    assert family(v(wl.WORKLOADS["c2"], C=128, K=128, groups=4)).startswith("igemm_")
    assert family(v(wl.WORKLOADS["c2"], C=64, K=64, groups=64)).startswith("direct_")  # depthwise
    assert family(v(wl.WORKLOADS["c2"], dtype=wl.F32)).startswith("tiled_f32_")         # fp32 of a real size: the fp32 MFMA kernel
    assert family(v(wl.WORKLOADS["c4"], dtype=wl.F32)).startswith("tiled_f32_")         # any filter size


def test_kernel_search_is_cheap_on_the_host():
    """The problem -> kernel search (cvx_conv_fwd_query runs all of it, uncached, on every call)
    stays in the microseconds for the benchmark layers and for the shapes that used to make it long
    (tiny images, where many tile shapes compete).  Compute calls do not even pay this: a handle
    keeps the plan of the problems it has seen."""
    import time
    import workloads as wl
    code = {wl.F32: cvx.CVX_F32, wl.F16: cvx.CVX_F16, wl.BF16: cvx.CVX_BF16}
    cases = [wl.WORKLOADS[n] for n in ("c1", "c2", "c3a", "c3b", "c4", "c5a", "c5b")]
    cases.append(wl.small_variant(wl.WORKLOADS["c5a"], N=4096, H=1, W=1))
    cases.append(wl.small_variant(wl.WORKLOADS["c5a"], N=4096, H=2, W=2))
    for w in cases:
        plan = cvx.ConvPlan(code[w.dtype], (w.N, w.C, w.H, w.W), (w.K, w.C // w.groups, w.R, w.S),
                            w.pad, w.stride, w.dil, w.groups)
        L, buf, ws = cvx.lib(), ctypes.create_string_buffer(128), ctypes.c_ulonglong()
        n = 2000
        t0 = time.perf_counter()
        for _ in range(n):
            L.cvx_conv_fwd_query(plan.xd, plan.wd, plan.cd, plan.yd, buf, 128, ctypes.byref(ws))
        us = (time.perf_counter() - t0) / n * 1e6
        plan.close()
        # ctypes itself costs about a microsecond per call; the bound leaves room for a slow CI host
        assert us < 25.0, "%s: %.1f us per uncached kernel search" % (w.name, us)


def test_out_params_untouched_on_failure():
    L = cvx.lib()
    h = ctypes.c_void_p(0xdead)
    n = ctypes.c_int(-7)
    xd, wd = _desc(cvx.CVX_F32, (1, 4, 6, 6)), _desc(cvx.CVX_F32, (2, 3, 3, 3))
    st = L.cvx_conv_fwd_output_dim(_conv(), xd, wd, ctypes.byref(n), ctypes.byref(n), ctypes.byref(n), ctypes.byref(n))
    assert st == cvx.CVX_ERR_SHAPE_MISMATCH and n.value == -7
    assert L.cvx_create(None, None) == cvx.CVX_ERR_NULL and h.value == 0xdead
