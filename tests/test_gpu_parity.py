"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU oracle on the same
seeded inputs, element by element.  Tolerances: fp32 relative L2 <= 1e-5; fp16/bf16 every element
within 1e-2*|ref| + 1e-3*rms(ref)."""
import os
import sys

import numpy as np
import pytest

import workloads as wl
from paper_1910_00078_amd import cvx

from parity import run_gpu, run_oracle, tolerance_ok, to_device, to_host_f64, DT_CODE

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def check_case(w, *, policy=0, seed=wl.BASE_SEED, **kw):
    say("case %s dtype=%s N=%d C=%d H=%d W=%d K=%d R=%d S=%d pad=%s stride=%s dil=%s g=%d policy=%d %s"
        % (w.name, w.dtype, w.N, w.C, w.H, w.W, w.K, w.R, w.S, w.pad, w.stride, w.dil, w.groups, policy, kw))
    x, wt, b = wl.make_inputs(w, seed)
    got, name = run_gpu(w, x, wt, b, policy=policy, **kw)
    okw = {k: v for k, v in kw.items() if k not in ("bias_f32", "pin", "offsets")}
    ref = run_oracle(w, x, wt, b, **okw)
    assert got.shape == ref.shape
    ok, msg = tolerance_ok(got, ref, w.dtype)
    assert ok, "%s via %s: %s" % (w.name, name, msg)
    return name


# ---- the benchmark configurations at full size, in the launch configuration the bench times ----
@pytest.mark.parametrize("name", ["c1", "c2", "c3a", "c3b", "c4", "c5a", "c5b"])
def test_full_size_configs(name):
    check_case(wl.WORKLOADS[name])


def test_full_size_configs_run_the_kernels_built_for_them():
    """At full size, the launch itself reports the kernel."""
    want = {"c1": "direct_f32", "c2": "igemm_512x64_c16_3x3", "c3a": "pointwise_256x64_c32_r5",
            "c3b": "pointwise_128x256_c32_r6", "c4": "stem_stream_512x64_k11", "c5a": "igemm_256x64_c32_3x3",
            "c5b": "igemm_256x128_c16_3x3"}
    for name, kernel in want.items():
        assert check_case(wl.WORKLOADS[name]) == kernel, name


@pytest.mark.parametrize("which", ["x", "w", "y"])
@pytest.mark.parametrize("base", ["c2", "c3a", "c4", "c1"])
def test_buffers_that_are_only_element_aligned(base, which):
    """A base pointer one element off a 16-byte boundary is not an error: the generic kernel serves
    the call (the fast kernels want 16-byte-aligned x, w and y)."""
    w = wl.WORKLOADS[base]
    if base != "c1":
        w = wl.small_variant(w, N=2, H=min(w.H, 30), W=min(w.W, 30))
    off = tuple(1 if which == n else 0 for n in "xwy")
    name = check_case(w, offsets=off)
    assert name.startswith("direct_"), name


@pytest.mark.parametrize("which", ["x", "w", "y"])
def test_fp32_buffers_that_are_only_element_aligned(which):
    """fp32 data one element off a 16-byte boundary stays on the matrix-instruction kernel, which then
    stages its chunks element by element instead of in 16-byte pieces."""
    w = wl.small_variant(wl.WORKLOADS["c2"], N=2, H=28, W=28, C=24, K=40, dtype=wl.F32)
    off = tuple(1 if which == n else 0 for n in "xwy")
    assert check_case(w, offsets=off).startswith("tiled_f32_")
    assert check_case(w).startswith("tiled_f32_")


def test_tensors_over_two_gibibytes_take_the_generic_kernel():
    """x and y of 2.15 GB each (the fast kernels index bytes in 32 bits and decline): every output is
    written, and 4000 sampled outputs -- the four corners of the last plane and the last elements among
    them -- agree with the oracle computed point by point."""
    import torch
    from oracle import conv_oracle
    N, C, H, W, K = 1, 8, 11600, 11600, 8
    w = wl.small_variant(wl.WORKLOADS["c2"], name="over_2gib", N=N, C=C, H=H, W=W, K=K)
    say("case %s: N=%d C=%d H=%d W=%d K=%d" % (w.name, N, C, H, W, K))
    rng = np.random.default_rng(5)
    block = wl.to_storage(rng.uniform(0, 1, 1 << 22).astype(np.float32), wl.BF16)
    x = np.resize(block, N * C * H * W).reshape(N, C, H, W)          # a seeded 4M-element block, repeated
    wt = wl.to_storage(rng.normal(0, np.sqrt(2 / (C * 9)), (K, C, 3, 3)).astype(np.float32), wl.BF16)
    b = wl.to_storage(rng.uniform(-0.1, 0.1, K).astype(np.float32), wl.BF16)
    dx, dw, db = to_device(x, wl.BF16), to_device(wt, wl.BF16), to_device(b, wl.BF16)
    y = torch.full((N, K, H, W), float("nan"), dtype=dx.dtype, device="cuda")
    info = {}
    cvx.conv_fwd_fused(dx, dw, db, pad=w.pad, stride=w.stride, dil=w.dil, act=cvx.CVX_ACT_RELU, out=y, info=info)
    torch.cuda.synchronize()
    assert info["kernel"].startswith("direct_"), info["kernel"]
    assert not torch.isnan(y).any().item()
    idx = np.stack([np.zeros(4000, np.int64), rng.integers(0, K, 4000), rng.integers(0, H, 4000), rng.integers(0, W, 4000)], 1).astype(np.int32)
    idx[:8] = [[0, 0, 0, 0], [0, K - 1, H - 1, W - 1], [0, K - 1, H - 1, 0], [0, K - 1, 0, W - 1], [0, 0, H - 1, W - 1],
               [0, 3, H // 2, W // 2], [0, K - 1, H - 2, W - 2], [0, K - 1, H - 1, W - 3]]
    ref = conv_oracle.conv_fwd_points(wl.to_f64(x, wl.BF16), wl.to_f64(wt, wl.BF16), wl.to_f64(b, wl.BF16), idx,
                                      pad=w.pad, stride=w.stride, dil=w.dil, act=1)
    bits = y.view(torch.int16)[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy().view(np.uint16)
    got = wl.to_f64(bits, wl.BF16)
    rms = float(np.sqrt(np.mean(ref * ref)))
    bad = np.abs(got - ref) > 1e-2 * np.abs(ref) + 1e-3 * rms
    assert not bad.any(), "%d of %d sampled outputs outside tolerance" % (int(bad.sum()), len(ref))


@pytest.mark.parametrize("name", ["c1", "c2", "c4"])
def test_full_size_configs_generic_kernel(name):
    w = wl.WORKLOADS[name]
    if name != "c1":
        w = wl.small_variant(w, N=2)
    check_case(w, policy=1)


# ---- reduced shapes that still span several tiles and ragged tails ----
def _v(base, **kw):
    return wl.small_variant(wl.WORKLOADS[base], **kw)


SMALL = [
    _v("c2", name="c2_n3", N=3),
    _v("c2", name="c2_ragged", N=2, C=24, K=40, H=19, W=23),
    _v("c2", name="c2_f16", N=2, dtype=wl.F16),
    _v("c2", name="c2_f32", N=1, C=16, K=24, H=20, W=20, dtype=wl.F32),
    # fp32 on the tiled fp32-MFMA kernel: full-width row tiles, ragged channels / filters / widths, stride and
    # dilation, groups, many small images per tile, and a long reduction (C*R*S = 4608) for the 1e-5 bound
    _v("c2", name="f32_c2_like", N=2, dtype=wl.F32),
    _v("c2", name="f32_ragged", N=3, C=20, K=40, H=19, W=23, dtype=wl.F32),
    _v("c5b", name="f32_stride2", N=2, C=32, K=48, dtype=wl.F32),
    _v("c2", name="f32_dil2_pad2", N=2, C=16, K=32, H=24, W=22, pad=(2, 2), dil=(2, 2), dtype=wl.F32),
    _v("c2", name="f32_groups4", N=2, C=64, K=64, H=28, W=28, groups=4, dtype=wl.F32),
    _v("c5a", name="f32_small_images", N=16, C=32, K=32, dtype=wl.F32),
    _v("c5a", name="f32_long_reduction", N=4, C=512, K=64, dtype=wl.F32),
    _v("c3a", name="f32_1x1", N=2, C=64, K=96, H=28, W=28, dtype=wl.F32),
    _v("c4", name="f32_7x7_stem", N=2, C=3, H=64, W=64, K=48, dtype=wl.F32),
    _v("c2", name="f32_5x5", N=2, C=16, K=32, H=20, W=20, R=5, S=5, pad=(2, 2), dtype=wl.F32),
    _v("c2", name="f32_rect_2x3_stride", N=2, C=24, K=24, H=30, W=31, R=2, S=3, pad=(0, 2), stride=(2, 1), dil=(1, 2), dtype=wl.F32),
    _v("c3a", name="c3a_n2", N=2),
    _v("c3b", name="c3b_n2", N=2),
    _v("c3a", name="1x1_ragged", N=3, C=40, K=24, H=13, W=11),
    # pointwise kernel: spans that straddle images, ragged K, each tile shape, both 16-bit types
    _v("c3a", name="pw_k64_straddle", N=5, C=64, K=64, H=12, W=10),
    _v("c3a", name="pw_k70_two_kblocks", N=3, C=96, K=70, H=20, W=18),
    _v("c3b", name="pw_k200_c32", N=7, C=32, K=200, H=8, W=8),
    _v("c3b", name="pw_k128", N=2, C=128, K=128, H=28, W=28),
    _v("c3a", name="pw_one_chunk", N=1, C=32, K=8, H=2, W=4),
    _v("c3b", name="pw_f16_c512", N=2, C=512, K=96, H=14, W=12, dtype=wl.F16),
    _v("c3a", name="1x1_stride2", N=2, C=64, K=32, H=15, W=14, stride=(2, 2)),
    # 3x3 unit-stride shapes: image widths 7..64, many small images per tile, ragged K, fp16,
    # vertical padding / dilation other than 1
    _v("c2", name="s1_w7_straddle", N=11, C=32, K=64, H=7, W=7),
    _v("c2", name="s1_w14_k70", N=3, C=48, K=70, H=14, W=14),
    _v("c2", name="s1_w28_f16", N=2, C=32, K=32, H=28, W=28, dtype=wl.F16),
    _v("c2", name="s1_w64_h5", N=3, C=16, K=16, H=5, W=64),
    _v("c2", name="s1_w10_h3_pad0h", N=2, C=16, K=24, H=9, W=10, pad=(0, 1)),
    _v("c2", name="s1_w20_dilh2", N=2, C=32, K=40, H=11, W=20, pad=(2, 1), dil=(2, 1)),
    _v("c2", name="s1_w9_padh3", N=1, C=16, K=8, H=4, W=9, pad=(3, 1)),
    # whole-image tiles staged as runs of y (planes that are not a multiple of 16 bytes): pixel-by-pixel
    # staging (odd planes) and four-pixel staging, ragged filter blocks, a last tile with fewer images,
    # groups (runs that start at any alignment), both 16-bit types
    _v("c2", name="runs_5x5_k40_groups2", N=13, C=32, K=40, H=5, W=5, groups=2),
    _v("c2", name="runs_6x6_k72", N=9, C=16, K=72, H=6, W=6),
    _v("c2", name="runs_9x11_k33_f16", N=5, C=24, K=33, H=9, W=11, dtype=wl.F16),
    _v("c2", name="runs_10x10_k130", N=3, C=16, K=130, H=10, W=10),
    _v("c4", name="c4_n2", N=2),
    _v("c4", name="c4_ragged", N=2, H=61, W=45, K=24),
    _v("c4", name="c4_bf16", N=1, H=64, W=64, dtype=wl.BF16),
    _v("c4", name="stem_k96_c4", N=2, C=4, H=50, W=66, K=96),
    _v("c4", name="stem_c1_5x3_pad0", N=2, C=1, H=33, W=40, K=16, R=5, S=3, pad=(0, 0), stride=(1, 2)),
    _v("c4", name="stem_3x8_stride4", N=1, C=2, H=20, W=70, K=8, R=3, S=8, pad=(1, 5), stride=(3, 4)),
    _v("c4", name="stem_narrow", N=3, C=3, H=9, W=9, K=5),
    _v("c5a", name="c5a_small", N=6, C=64, K=96),
    _v("c5b", name="c5b_small", N=3, C=64, K=48),
    _v("c5b", name="c5b_k256_wide_filter_tile", N=3, C=32),
    _v("c5b", name="c5b_k200_ragged_filter_tile", N=2, C=48, K=200),
    _v("c5b", name="c5b_odd", N=2, C=32, K=32, H=27, W=25),
    _v("c2", name="dil2", N=2, C=32, K=32, H=20, W=18, pad=(2, 2), dil=(2, 2)),
    _v("c2", name="rect_filter", N=2, C=16, K=16, H=17, W=21, R=3, S=5, pad=(1, 2)),
    _v("c2", name="asym", N=2, C=8, K=8, H=16, W=30, R=2, S=3, pad=(0, 2), stride=(2, 1), dil=(1, 2)),
    _v("c2", name="big_pad", N=1, C=8, K=8, H=5, W=6, pad=(4, 5)),
    _v("c2", name="5x5", N=2, C=16, K=32, H=14, W=14, R=5, S=5, pad=(2, 2)),
    _v("c2", name="groups4", N=2, C=32, K=64, H=14, W=14, groups=4),
    # grouped convolution on the MFMA path: 8 or more channels per group
    _v("c2", name="groups4_c128_k128", N=3, C=128, K=128, H=14, W=14, groups=4),
    _v("c2", name="groups2_k96_ragged", N=2, C=64, K=96, H=19, W=17, groups=2),
    _v("c3a", name="groups4_1x1", N=2, C=64, K=64, H=12, W=12, groups=4),
    _v("c5b", name="groups8_stride2_f16", N=2, C=128, K=64, H=15, W=15, groups=8, dtype=wl.F16),
    _v("c2", name="groups3_c40_odd", N=2, C=120, K=24, H=9, W=11, groups=3),
    _v("c2", name="depthwise", N=2, C=32, K=32, H=14, W=14, groups=32),
    _v("c1", name="c1_tiny_1x1img", H=1, W=1, pad=(1, 1)),
    _v("c1", name="c1_C1K1", C=1, K=1),
    _v("c2", name="c_not_mult8", N=2, C=20, K=12, H=9, W=9),
    _v("c2", name="c3_k5", N=2, C=3, K=5, H=12, W=12),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_reduced_shapes(w):
    check_case(w)


@pytest.mark.parametrize("w", SMALL[::3], ids=lambda w: w.name)
def test_reduced_shapes_generic_kernel(w):
    check_case(w, policy=1)


PINNED = [
    # name, variant, workload: the eight-wave implicit-GEMM kernels are chosen on their own only for the
    # full-size layers; pinned, their two producer loops (the fixed-load-count one for blocks in the
    # interior of the tensor, the general one at its edges and for ragged shapes) and the skipping of
    # empty pixel tiles are exercised on small tensors too
    ("p512_c64_k64", "igemm_512x64_c16_3x3", wl.small_variant(wl.WORKLOADS["c2"], N=3, H=40, W=40)),
    ("p512_no_pad", "igemm_512x64_c16_3x3", wl.small_variant(wl.WORKLOADS["c2"], N=3, H=40, W=40, pad=(0, 0))),
    ("p512_odd_stages", "igemm_512x64_c16_3x3", wl.small_variant(wl.WORKLOADS["c2"], N=3, H=28, W=28, C=48)),
    ("p512_ragged_filters", "igemm_512x64_c16_3x3", wl.small_variant(wl.WORKLOADS["c2"], N=5, H=28, W=28, K=48)),
    ("p512_whole_images", "igemm_512x64_c16_3x3", wl.small_variant(wl.WORKLOADS["c5a"], N=16, C=64, K=64)),
    ("p256x128_stride2", "igemm_256x128_c16_3x3", wl.small_variant(wl.WORKLOADS["c5b"], N=3, C=64, K=128)),
    ("p256x128_ragged_filters", "igemm_256x128_c16_3x3", wl.small_variant(wl.WORKLOADS["c5b"], N=3, C=32, K=200)),
    ("p256x128_whole_images", "igemm_256x128_c16_3x3", wl.small_variant(wl.WORKLOADS["c5a"], N=9, C=128, K=128)),
]


@pytest.mark.parametrize("case", PINNED, ids=lambda c: c[0])
def test_pinned_eight_wave_variants(case):
    variant, w = case[1], case[2]
    PT = 512 if "512x64" in variant else 128 if "128x128" in variant else 256
    Ho = (w.H + 2 * w.pad[0] - w.dil[0] * (w.R - 1) - 1) // w.stride[0] + 1
    Wo = (w.W + 2 * w.pad[1] - w.dil[1] * (w.S - 1) - 1) // w.stride[1] + 1
    nb, th = (min(w.N, PT // (Ho * Wo)), Ho) if Ho * Wo <= PT else (1, PT // Wo)
    if len(case) > 3:
        nb, th = case[3]                      # the largest tile does not fit this variant's LDS
    say("case %s pinned to %s NB=%d TH=%d: N=%d C=%d H=%d W=%d K=%d pad=%s stride=%s" % (case[0], variant, nb, th, w.N, w.C, w.H, w.W, w.K, w.pad, w.stride))
    x, wt, b = wl.make_inputs(w)
    got, name = run_gpu(w, x, wt, b, pin="%s,%d,%d" % (variant, nb, th))
    assert name == variant
    ok, msg = tolerance_ok(got, run_oracle(w, x, wt, b), w.dtype)
    assert ok, msg


@pytest.mark.parametrize("variant", ["tiled_f32_256x64_c8_3x3", "tiled_f32_128x64_c8_3x3", "tiled_f32_256x64_c8", "tiled_f32_128x64_c8", "tiled_f32_128x32_c8", "tiled_f32_128x32_c2"])
def test_pinned_fp32_variants(variant):
    for w in (wl.small_variant(wl.WORKLOADS["c2"], N=2, C=24, K=72, H=20, W=20, dtype=wl.F32),
              wl.small_variant(wl.WORKLOADS["c5a"], N=5, C=16, K=16, dtype=wl.F32)):
        say("case pinned %s: N=%d C=%d H=%d W=%d K=%d" % (variant, w.N, w.C, w.H, w.W, w.K))
        x, wt, b = wl.make_inputs(w)
        got, name = run_gpu(w, x, wt, b, pin=variant)
        assert name == variant
        ok, msg = tolerance_ok(got, run_oracle(w, x, wt, b), w.dtype)
        assert ok, msg


def test_kernel_families_serve_the_shapes_they_were_built_for():
    want = {"c2": "igemm_", "c3a": "pointwise_", "c3b": "pointwise_", "c4": "stem_", "c5a": "igemm_", "c5b": "igemm_",
            "c1": "direct_"}
    for name, prefix in want.items():
        w = wl.WORKLOADS[name]
        plan = cvx.ConvPlan(DT_CODE[w.dtype], (w.N, w.C, w.H, w.W), (w.K, w.C // w.groups, w.R, w.S),
                            w.pad, w.stride, w.dil, w.groups)
        got = plan.kernel_name()
        plan.close()
        assert got.startswith(prefix), "%s is served by %s" % (name, got)
    f32 = cvx.ConvPlan(DT_CODE[wl.F32], (32, 64, 56, 56), (64, 64, 3, 3), (1, 1), (1, 1), (1, 1))
    got = f32.kernel_name()
    f32.close()
    assert got.startswith("tiled_f32_"), "fp32 3x3 is served by %s" % got
    grouped = cvx.ConvPlan(DT_CODE[wl.BF16], (2, 128, 14, 14), (128, 32, 3, 3), (1, 1), (1, 1), (1, 1), 4)
    got = grouped.kernel_name()
    grouped.close()
    assert got.startswith("igemm_"), "grouped 3x3 is served by %s" % got


# ---- epilogue variants ----
@pytest.mark.parametrize("act,alpha", [(cvx.CVX_ACT_IDENTITY, 0.0), (cvx.CVX_ACT_RELU, 0.0),
                                        (cvx.CVX_ACT_LEAKY_RELU, 0.1), (cvx.CVX_ACT_TANH, 0.0),
                                        (cvx.CVX_ACT_LOGISTIC, 0.0)])
@pytest.mark.parametrize("base", ["c2", "c1", "c4", "c3a", "c2_f32"])
def test_activations(base, act, alpha):
    w = wl.WORKLOADS[base[:2]] if base == "c2_f32" else wl.WORKLOADS[base]
    if base == "c2_f32":
        w = wl.small_variant(w, N=2, H=30, W=30, dtype=wl.F32)
    elif base != "c1":
        w = wl.small_variant(w, N=2, H=min(w.H, 40), W=min(w.W, 40))
    check_case(w, act=act, alpha=alpha)


@pytest.mark.parametrize("base", ["c2", "c3a", "c1"])
def test_no_bias_and_fp32_bias(base):
    w = wl.WORKLOADS[base]
    if base != "c1":
        w = wl.small_variant(w, N=2)
    check_case(w, use_bias=False, act=cvx.CVX_ACT_IDENTITY)
    check_case(w, bias_f32=True)


@pytest.mark.parametrize("base", ["c2", "c3b", "c1", "c2_f32"])
def test_batchnorm_epilogue(base):
    w = wl.WORKLOADS[base[:2]] if base == "c2_f32" else wl.WORKLOADS[base]
    if base == "c2_f32":
        w = wl.small_variant(w, N=2, H=30, W=30, dtype=wl.F32)
    elif base != "c1":
        w = wl.small_variant(w, N=2)
    rng = np.random.default_rng(5)
    bn = (rng.uniform(0.5, 1.5, w.K), rng.uniform(-0.5, 0.5, w.K), rng.uniform(-0.3, 0.3, w.K),
          rng.uniform(0.5, 2.0, w.K))
    bn = tuple(t.astype(np.float32).astype(np.float64) for t in bn)
    check_case(w, bn=bn, eps=1e-3)


@pytest.mark.parametrize("shape", [dict(N=6, C=32, K=80, H=7, W=7), dict(N=2, C=16, K=24, H=14, W=14)], ids=["7x7", "14x14"])
def test_every_epilogue_on_tiles_staged_as_runs(shape):
    w = wl.small_variant(wl.WORKLOADS["c2"], **shape)
    rng = np.random.default_rng(9)
    bn = (rng.uniform(0.5, 1.5, w.K), rng.uniform(-0.5, 0.5, w.K), rng.uniform(-0.3, 0.3, w.K), rng.uniform(0.5, 2.0, w.K))
    bn = tuple(t.astype(np.float32).astype(np.float64) for t in bn)
    for act, alpha in [(cvx.CVX_ACT_IDENTITY, 0.0), (cvx.CVX_ACT_RELU, 0.0), (cvx.CVX_ACT_LEAKY_RELU, 0.1), (cvx.CVX_ACT_TANH, 0.0)]:
        check_case(w, act=act, alpha=alpha)
    check_case(w, bn=bn, eps=1e-3)
    check_case(w, bn=bn, eps=1e-3, act=cvx.CVX_ACT_LOGISTIC)
    check_case(w, use_bias=False, act=cvx.CVX_ACT_IDENTITY)


def test_plain_conv_fwd_and_unfused_operators_agree_with_fused():
    """conv_fwd, then bias_add, then activation as three launches (the unfused route of Sec. V)
    lands within one output rounding per step of the fused call, and both within tolerance."""
    import torch
    w = wl.small_variant(wl.WORKLOADS["c2"], N=2)
    x, wt, b = wl.make_inputs(w)
    dx, dw, db = to_device(x, w.dtype), to_device(wt, w.dtype), to_device(b, w.dtype)
    plan = cvx.ConvPlan(DT_CODE[w.dtype], tuple(dx.shape), tuple(dw.shape), w.pad, w.stride, w.dil)
    y = torch.full(plan.y_shape, float("nan"), dtype=dx.dtype, device="cuda")
    plan.run_plain(dx.data_ptr(), dw.data_ptr(), y.data_ptr())
    torch.cuda.synchronize()
    ref_plain = run_oracle(w, x, wt, b, act=0, use_bias=False)
    ok, msg = tolerance_ok(to_host_f64(y, w.dtype), ref_plain, w.dtype)
    assert ok, msg
    cvx.cvx_bias_add(plan.h, plan.bd, db.data_ptr(), plan.yd, y.data_ptr())
    cvx.cvx_activation_fwd(plan.h, cvx.CVX_ACT_RELU, 0.0, plan.yd, y.data_ptr())
    torch.cuda.synchronize()
    ref = run_oracle(w, x, wt, b, act=1)
    ok, msg = tolerance_ok(to_host_f64(y, w.dtype), ref, w.dtype)
    assert ok, msg
    plan.close()


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("shape,offset", [((2, 5, 4, 8), 0), ((3, 7, 3, 5), 0), ((2, 4, 6, 8), 1), ((1, 3, 1, 1), 0)])
def test_unfused_bias_add_and_activation_elementwise(dtype, shape, offset):
    """cvx_bias_add / cvx_activation_fwd on their own against y + b[k] and act(y) in fp64: vector
    path (aligned, HW a multiple of the vector), scalar path (HW not a multiple, or a base pointer
    that is only element-aligned) and the tail past the last whole vector."""
    import torch
    n, k, h, w_ = shape
    rng = np.random.default_rng(11)
    tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[dtype]
    count = n * k * h * w_
    buf = torch.from_numpy(rng.uniform(-2, 2, count + offset).astype(np.float32)).to(tdt).cuda()
    y = buf[offset:]                                      # offset 1: only element-aligned
    bias = torch.from_numpy(rng.uniform(-1, 1, k).astype(np.float32)).to(tdt).cuda()
    y0 = y.double().cpu().numpy().reshape(shape)
    b0 = bias.double().cpu().numpy()
    hdl = cvx.cvx_create(torch.cuda.current_stream().cuda_stream)
    yd, bd = cvx.cvx_tensor_desc_create(), cvx.cvx_tensor_desc_create()
    cvx.cvx_tensor_desc_set_4d(yd, DT_CODE[dtype], n, k, h, w_)
    cvx.cvx_tensor_desc_set_4d(bd, DT_CODE[dtype], 1, k, 1, 1)
    tol = {wl.F32: 1e-6, wl.F16: 2e-3, wl.BF16: 1.6e-2}[dtype]
    cvx.cvx_bias_add(hdl, bd, bias.data_ptr(), yd, y.data_ptr())
    torch.cuda.synchronize()
    want = y0 + b0[None, :, None, None]
    got = y.double().cpu().numpy().reshape(shape)
    assert np.all(np.abs(got - want) <= tol * (1 + np.abs(want))), "bias_add"
    for act, alpha in [(cvx.CVX_ACT_RELU, 0.0), (cvx.CVX_ACT_LEAKY_RELU, 0.25), (cvx.CVX_ACT_TANH, 0.0)]:
        before = y.double().cpu().numpy().reshape(shape)
        cvx.cvx_activation_fwd(hdl, act, alpha, yd, y.data_ptr())
        torch.cuda.synchronize()
        want = {cvx.CVX_ACT_RELU: np.maximum(before, 0), cvx.CVX_ACT_LEAKY_RELU: np.where(before > 0, before, alpha * before),
                cvx.CVX_ACT_TANH: np.tanh(before)}[act]
        got = y.double().cpu().numpy().reshape(shape)
        assert np.all(np.abs(got - want) <= tol * (1 + np.abs(want))), "activation %d" % act
    cvx.cvx_tensor_desc_destroy(yd)
    cvx.cvx_tensor_desc_destroy(bd)
    cvx.cvx_destroy(hdl)


def test_repeated_runs_are_bit_identical():
    import torch
    for name in ("c2", "c3a", "c4", "c5b"):
        w = wl.small_variant(wl.WORKLOADS[name], N=2)
        x, wt, b = wl.make_inputs(w)
        dx, dw, db = to_device(x, w.dtype), to_device(wt, w.dtype), to_device(b, w.dtype)
        outs = [cvx.conv_fwd_fused(dx, dw, db, pad=w.pad, stride=w.stride, dil=w.dil) for _ in range(3)]
        torch.cuda.synchronize()
        for o in outs[1:]:
            assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16)), name


def test_non_default_stream_and_reused_plan():
    import torch
    w = wl.small_variant(wl.WORKLOADS["c2"], N=2)
    x, wt, b = wl.make_inputs(w)
    dx, dw, db = to_device(x, w.dtype), to_device(wt, w.dtype), to_device(b, w.dtype)
    ref = run_oracle(w, x, wt, b, act=1)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        plan = cvx.ConvPlan(DT_CODE[w.dtype], tuple(dx.shape), tuple(dw.shape), w.pad, w.stride, w.dil,
                            stream=s.cuda_stream)
        y = torch.full(plan.y_shape, float("nan"), dtype=dx.dtype, device="cuda")
        for _ in range(3):
            plan.run(dx.data_ptr(), dw.data_ptr(), db.data_ptr(), y.data_ptr())
        s.synchronize()
        plan.close()
    ok, msg = tolerance_ok(to_host_f64(y, w.dtype), ref, w.dtype)
    assert ok, msg


def test_compute_errors_are_reported_not_launched():
    import torch
    x = torch.zeros((1, 8, 6, 6), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((4, 8, 3, 3), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cvx.CvxError) as e:
        cvx.conv_fwd_fused(x, wt, torch.zeros(5, dtype=torch.bfloat16, device="cuda"), pad=1)
    assert e.value.status == cvx.CVX_ERR_SHAPE_MISMATCH
    with pytest.raises(cvx.CvxError) as e:
        cvx.conv_fwd_fused(x, wt, None, pad=0, dil=4)
    assert e.value.status == cvx.CVX_ERR_BAD_PARAM
    with pytest.raises(ValueError):
        cvx.conv_fwd_fused(x.cpu(), wt.cpu())
