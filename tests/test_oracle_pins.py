"""Pins for the fp64 CPU oracle: every check here is against something other than the oracle
itself -- hand-worked numbers (tests/golden/hand_worked_conv.json), closed forms, algebraic
identities, numpy / scipy library routines the special cases reduce to, and an im2col brute force
whose indices are derived differently (scatter by input pixel instead of gather by output pixel).
A dropped term, a sign or index error, a transposed filter or a flipped filter fails at least one.
"""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.signal import correlate2d

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_conv.json")
ACTS = {"identity": 0, "relu": 1, "leaky": 2, "tanh": 3, "logistic": 4}


def _cases():
    with open(GOLD) as f:
        return json.load(f)["cases"]


def _run_case(conv_fwd, case):
    bn = case.get("bn")
    if bn is not None:
        bn = tuple(np.array(bn[k], float) for k in ("scale", "shift", "mean", "var"))
    return conv_fwd(np.array(case["x"], float), np.array(case["w"], float),
                    None if case["bias"] is None else np.array(case["bias"], float),
                    pad=tuple(case["pad"]), stride=tuple(case["stride"]), dil=tuple(case["dil"]),
                    act=ACTS[case["act"]], alpha=case.get("alpha", 0.0), bn=bn, eps=case.get("eps", 0.0))


def _case_ok(y, case):
    """Exact equality unless the case carries a tolerance (inputs such as ln 2 that are themselves
    rounded); the expected values are the file's, worked by hand."""
    want = np.array(case["y"], float)
    if y.shape != want.shape:
        return False
    if "tol" in case:
        return bool(np.all(np.abs(y - want) <= case["tol"]))
    return bool(np.array_equal(y, want))


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_hand_worked_examples(oracle, case):
    y = _run_case(oracle.conv_fwd, case)
    assert _case_ok(y, case), (case["name"], y)


# Mistakes planted in a COPY of the oracle's source (compiled on the CPU into a temporary library):
# each must be caught by at least one hand-worked case, which shows that the cases pin the line
# they are meant to pin.  (original text, replacement, cases expected to notice)
PLANTED = [
    ("sqrt(var + eps)", "(var + eps)", {"G_bias_batchnorm", "H_batchnorm_per_channel"}),
    ("sqrt(var + eps)", "(sqrt(var) + eps)", {"G_bias_batchnorm", "H_batchnorm_per_channel"}),
    ("(v - mean)", "(v + mean)", {"G_bias_batchnorm", "H_batchnorm_per_channel"}),
    ("gamma = bn[k], beta = bn[K + k]", "gamma = bn[K + k], beta = bn[k]", {"G_bias_batchnorm"}),
    ("mean = bn[2 * K + k], var = bn[3 * K + k]", "mean = bn[3 * K + k], var = bn[2 * K + k]", {"G_bias_batchnorm"}),
    ("mean = bn[2 * K + k]", "mean = bn[2 * K]", {"H_batchnorm_per_channel"}),
    ("double v = acc + (b ? b[k] : 0.0);", "double v = acc;", {"G_bias_batchnorm", "D_bias_relu"}),
    ("v = gamma * (v - mean) / sqrt(var + eps) + beta;\n    }\n    return apply_act(v, act, alpha);",
     "v = gamma * (apply_act(v, act, alpha) - mean) / sqrt(var + eps) + beta; return v;\n    }\n    return apply_act(v, act, alpha);",
     {"G2_bias_batchnorm_relu"}),
    ("case ACT_LEAKY_RELU: return v > 0.0 ? v : alpha * v;", "case ACT_LEAKY_RELU: return v > 0.0 ? v : 0.0;", {"I_leaky_relu"}),
    ("case ACT_LEAKY_RELU: return v > 0.0 ? v : alpha * v;", "case ACT_LEAKY_RELU: return v > 0.0 ? alpha * v : v;", {"I_leaky_relu"}),
    ("return tanh(v);", "return 1.0 / (1.0 + exp(-v));", {"J_tanh_closed_forms"}),
    ("return tanh(v);", "return tanh(0.5 * v);", {"J_tanh_closed_forms"}),
    ("return 1.0 / (1.0 + exp(-v));", "return 1.0 / (1.0 + exp(v));", {"K_logistic_closed_forms"}),
    ("return 1.0 / (1.0 + exp(-v));", "return tanh(v);", {"K_logistic_closed_forms"}),
    ("p * stride_h - pad_h + r * dil_h", "p * stride_h - pad_h + (R - 1 - r) * dil_h", {"A_valid"}),
    ("q * stride_w - pad_w + s * dil_w", "q * stride_w + pad_w + s * dil_w", {"B_pad1"}),
]


@pytest.mark.parametrize("old,new,catchers", PLANTED, ids=[str(i) for i in range(len(PLANTED))])
def test_planted_mistakes_are_caught(oracle, tmp_path, old, new, catchers):
    import ctypes
    import subprocess
    from oracle import conv_oracle as mod
    src = open(os.path.join(os.path.dirname(mod.__file__), "conv_oracle.c")).read()
    assert src.count(old) == 1, "the oracle line this mistake is planted in has changed: %r" % old
    bad_c, bad_so = tmp_path / "bad.c", tmp_path / "libbad.so"
    bad_c.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", str(bad_so), str(bad_c), "-lm"])
    good_lib = mod._lib
    try:
        mod._lib = None
        real_cdll = ctypes.CDLL
        # load the perturbed library through the module's own marshalling code
        mod.ctypes.CDLL = lambda path, *a, **k: real_cdll(str(bad_so), *a, **k)
        try:
            mod._load()
        finally:
            mod.ctypes.CDLL = real_cdll
        failed = {c["name"] for c in _cases() if not _case_ok(_run_case(mod.conv_fwd, c), c)}
    finally:
        mod._lib = good_lib
    assert catchers <= failed, "planted %r -> %r: cases that noticed: %s" % (old, new, sorted(failed))
    for c in _cases():                                   # and the real oracle still passes them all
        assert _case_ok(_run_case(oracle.conv_fwd, c), c)


def test_cross_correlation_not_flipped(oracle):
    """The asymmetric 3x3 example: true (flipped) convolution would give 56, not 4."""
    c = _cases()[0]
    y = oracle.conv_fwd(np.array(c["x"], float), np.array(c["w"], float))
    assert y[0, 0, 0, 0] == 4.0 and y[0, 0, 0, 0] != 56.0


# ------------------------------------------------------------------------------------------
# independent brute force: scatter formulation (loop over INPUT pixels and taps, add into the
# output the tap reaches), the reverse of the oracle's gather.
# ------------------------------------------------------------------------------------------
def scatter_conv(x, w, pad, stride, dil, groups=1):
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    ph, pw = pad
    sh, sw = stride
    dh, dw = dil
    Ho = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
    y = np.zeros((N, K, Ho, Wo))
    Kg = K // groups
    for h in range(H):
        for r in range(R):
            top = h + ph - r * dh            # = p * sh
            if top < 0 or top % sh:
                continue
            p = top // sh
            if p >= Ho:
                continue
            for wv in range(W):
                for s in range(S):
                    left = wv + pw - s * dw
                    if left < 0 or left % sw:
                        continue
                    q = left // sw
                    if q >= Wo:
                        continue
                    for g in range(groups):
                        xs = x[:, g * Cg:(g + 1) * Cg, h, wv]            # N x Cg
                        ws = w[g * Kg:(g + 1) * Kg, :, r, s]             # Kg x Cg
                        y[:, g * Kg:(g + 1) * Kg, p, q] += xs @ ws.T
    return y


def im2col_conv(x, w, pad, stride, dil):
    """Patch matrix (C*R*S) x (Ho*Wo) built from a zero-padded copy, then one matrix product
    (the im2col route of Sec. IV-A)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    ph, pw = pad
    sh, sw = stride
    dh, dw = dil
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw))
    xp[:, :, ph:ph + H, pw:pw + W] = x
    Ho = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
    cols = np.empty((N, C, R, S, Ho, Wo))
    for r in range(R):
        for s in range(S):
            cols[:, :, r, s] = xp[:, :, r * dh: r * dh + (Ho - 1) * sh + 1: sh,
                                  s * dw: s * dw + (Wo - 1) * sw + 1: sw]
    cols = cols.reshape(N, C * R * S, Ho * Wo)
    return (w.reshape(K, -1) @ cols).reshape(N, K, Ho, Wo)


GRID = [
    # N, C, H, W, K, R, S, pad, stride, dil
    (2, 3, 7, 9, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 2, 8, 6, 3, 1, 1, (0, 0), (1, 1), (1, 1)),
    (1, 2, 9, 8, 3, 1, 1, (0, 0), (2, 3), (1, 1)),
    (2, 3, 11, 10, 2, 7, 7, (3, 3), (2, 2), (1, 1)),
    (1, 4, 9, 12, 5, 3, 5, (2, 0), (1, 2), (1, 1)),
    (1, 2, 10, 9, 2, 2, 3, (0, 3), (3, 1), (2, 1)),
    (2, 1, 12, 13, 3, 3, 2, (2, 1), (2, 3), (3, 2)),
    (1, 3, 6, 6, 2, 5, 5, (3, 2), (1, 1), (1, 1)),
    (1, 2, 13, 7, 2, 3, 3, (0, 0), (3, 3), (2, 3)),
    (3, 5, 5, 4, 6, 3, 3, (1, 2), (2, 1), (1, 1)),
]


@pytest.mark.parametrize("cfg", GRID, ids=lambda c: "x".join(map(str, c[:7])))
def test_brute_force_scatter_and_im2col(oracle, cfg):
    N, C, H, W, K, R, S, pad, stride, dil = cfg
    rng = np.random.default_rng(hash(cfg) % (2 ** 32))
    x = rng.integers(-4, 5, size=(N, C, H, W)).astype(float)     # small integers: exact in fp64
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(float)
    y = oracle.conv_fwd(x, w, pad=pad, stride=stride, dil=dil)
    assert np.array_equal(y, scatter_conv(x, w, pad, stride, dil))
    assert np.array_equal(y, im2col_conv(x, w, pad, stride, dil))


def test_random_parameter_sweep_against_im2col(oracle):
    rng = np.random.default_rng(20191000)
    for _ in range(60):
        R, S = rng.integers(1, 6, size=2)
        dil = tuple(int(v) for v in rng.integers(1, 4, size=2))
        pad = tuple(int(v) for v in rng.integers(0, 4, size=2))
        stride = tuple(int(v) for v in rng.integers(1, 4, size=2))
        H = int(dil[0] * (R - 1) + 1 + rng.integers(0, 6))
        W = int(dil[1] * (S - 1) + 1 + rng.integers(0, 6))
        N, C, K = (int(v) for v in rng.integers(1, 4, size=3))
        x = rng.integers(-4, 5, size=(N, C, H, W)).astype(float)
        w = rng.integers(-3, 4, size=(K, C, int(R), int(S))).astype(float)
        y = oracle.conv_fwd(x, w, pad=pad, stride=stride, dil=dil)
        assert np.array_equal(y, im2col_conv(x, w, pad, stride, dil)), (N, C, H, W, K, R, S, pad, stride, dil)


# ------------------------------------------------------------------------------------------
# closed forms and identities
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("r0,s0", list(itertools.product(range(3), range(3))))
def test_delta_filter_is_a_shifted_copy(oracle, r0, s0):
    rng = np.random.default_rng(7)
    N, C, H, W, K = 2, 3, 6, 5, 4
    x = rng.standard_normal((N, C, H, W))
    w = np.zeros((K, C, 3, 3))
    c0 = 1
    for k in range(K):
        w[k, (c0 + k) % C, r0, s0] = 1.0
    y = oracle.conv_fwd(x, w, pad=1)
    xz = np.zeros((N, C, H + 2, W + 2))
    xz[:, :, 1:-1, 1:-1] = x
    for k in range(K):
        want = xz[:, (c0 + k) % C, r0:r0 + H, s0:s0 + W]       # y[p,q] = x[p + r0 - 1, q + s0 - 1]
        assert np.array_equal(y[:, k], want)


def test_all_ones_3x3_counts_taps(oracle):
    C = 5
    y = oracle.conv_fwd(np.ones((1, C, 6, 7)), np.ones((2, C, 3, 3)), pad=1)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[:, :, 0, 1:-1] == 6 * C) and np.all(y[:, :, 1:-1, 0] == 6 * C)
    assert np.all(y[:, :, -1, 1:-1] == 6 * C) and np.all(y[:, :, 1:-1, -1] == 6 * C)
    for p, q in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[:, :, p, q] == 4 * C)


def test_all_ones_7x7_stride2_counts_taps(oracle):
    """7x7, pad 3, stride 2 on a 16x16 image of ones: y[p,q] = C * rows_in(p) * cols_in(q), where
    rows_in(p) counts taps r with 0 <= 2p-3+r < 16."""
    C, H = 3, 16
    y = oracle.conv_fwd(np.ones((1, C, H, H)), np.ones((1, C, 7, 7)), pad=3, stride=2)
    assert y.shape == (1, 1, 8, 8)
    # by hand: p=0 covers rows -3..3 -> 4 inside; p=1: -1..5 -> 6; p=2..6: all 7; p=7: 11..17 -> 5
    cnt = [4, 6, 7, 7, 7, 7, 7, 5]
    assert np.array_equal(y[0, 0], C * np.outer(cnt, cnt))


def test_constant_input_no_padding(oracle):
    rng = np.random.default_rng(3)
    w = rng.integers(-5, 6, size=(4, 3, 3, 2)).astype(float)
    b = np.array([1.0, -2.0, 0.5, 7.0])
    y = oracle.conv_fwd(np.full((2, 3, 8, 7), 2.5), w, b)
    for k in range(4):
        assert np.all(y[:, k] == 2.5 * w[k].sum() + b[k])


def test_linearity_in_x_and_w(oracle):
    rng = np.random.default_rng(11)
    x1, x2 = rng.standard_normal((2, 2, 3, 9, 8))
    w1, w2 = rng.standard_normal((2, 4, 3, 3, 3))
    kw = dict(pad=(1, 2), stride=(2, 1), dil=(1, 2))
    a, b = 0.75, -1.5
    lhs = oracle.conv_fwd(a * x1 + b * x2, w1, **kw)
    rhs = a * oracle.conv_fwd(x1, w1, **kw) + b * oracle.conv_fwd(x2, w1, **kw)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    lhs = oracle.conv_fwd(x1, a * w1 + b * w2, **kw)
    rhs = a * oracle.conv_fwd(x1, w1, **kw) + b * oracle.conv_fwd(x1, w2, **kw)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_1x1_is_a_matrix_product(oracle):
    rng = np.random.default_rng(5)
    N, C, H, W, K = 3, 7, 5, 6, 4
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C, 1, 1))
    y = oracle.conv_fwd(x, w)
    want = np.matmul(w.reshape(K, C), x.reshape(N, C, H * W)).reshape(N, K, H, W)
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)
    ys = oracle.conv_fwd(x, w, stride=(2, 3))
    xs = x[:, :, ::2, ::3]
    want = np.matmul(w.reshape(K, C), xs.reshape(N, C, -1)).reshape(N, K, *xs.shape[2:])
    np.testing.assert_allclose(ys, want, rtol=1e-13, atol=1e-13)


def test_stride_is_subsampling_of_stride_one(oracle):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 3, 11, 12))
    w = rng.standard_normal((2, 3, 3, 5))
    full = oracle.conv_fwd(x, w, pad=(1, 2))
    sub = oracle.conv_fwd(x, w, pad=(1, 2), stride=(3, 2))
    assert np.array_equal(sub, full[:, :, ::3, ::2])


def test_dilation_equals_zero_stuffed_filter(oracle):
    rng = np.random.default_rng(13)
    x = rng.standard_normal((1, 2, 12, 13))
    w = rng.standard_normal((3, 2, 3, 2))
    dh, dw = 2, 3
    wz = np.zeros((3, 2, dh * 2 + 1, dw * 1 + 1))
    wz[:, :, ::dh, ::dw] = w
    a = oracle.conv_fwd(x, w, pad=(2, 1), stride=(1, 2), dil=(dh, dw))
    b = oracle.conv_fwd(x, wz, pad=(2, 1), stride=(1, 2))
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_scipy_correlate2d_third_opinion(oracle):
    rng = np.random.default_rng(17)
    N, C, H, W, K, R, S = 2, 3, 9, 7, 2, 3, 4
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C, R, S))
    y = oracle.conv_fwd(x, w, pad=(1, 2))
    for n in range(N):
        for k in range(K):
            want = sum(correlate2d(np.pad(x[n, c], ((1, 1), (2, 2))), w[k, c], mode="valid")
                       for c in range(C))
            np.testing.assert_allclose(y[n, k], want, rtol=1e-12, atol=1e-12)


def test_batch_and_filter_independence(oracle):
    rng = np.random.default_rng(19)
    x = rng.standard_normal((4, 3, 6, 6))
    w = rng.standard_normal((5, 3, 3, 3))
    b = rng.standard_normal(5)
    y = oracle.conv_fwd(x, w, b, pad=1, act=1)
    pn, pk = rng.permutation(4), rng.permutation(5)
    yp = oracle.conv_fwd(x[pn], w[pk], b[pk], pad=1, act=1)
    assert np.array_equal(yp, y[pn][:, pk])
    assert np.array_equal(oracle.conv_fwd(x[1:2], w[2:3], b[2:3], pad=1, act=1), y[1:2, 2:3])


def test_bias_and_activations(oracle):
    rng = np.random.default_rng(23)
    x = rng.standard_normal((2, 3, 6, 5))
    w = rng.standard_normal((4, 3, 3, 3))
    b = rng.standard_normal(4)
    plain = oracle.conv_fwd(x, w, pad=1)
    withb = oracle.conv_fwd(x, w, b, pad=1)
    np.testing.assert_allclose(withb - plain, np.broadcast_to(b[None, :, None, None], plain.shape),
                               rtol=0, atol=1e-13)
    assert np.array_equal(oracle.conv_fwd(x, w, b, pad=1, act=1), np.maximum(withb, 0.0))
    leaky = oracle.conv_fwd(x, w, b, pad=1, act=2, alpha=0.125)
    assert np.array_equal(leaky, np.where(withb > 0, withb, 0.125 * withb))
    np.testing.assert_allclose(oracle.conv_fwd(x, w, b, pad=1, act=3), np.tanh(withb), rtol=1e-14)
    from scipy.special import expit
    np.testing.assert_allclose(oracle.conv_fwd(x, w, b, pad=1, act=4), expit(withb), rtol=1e-13)
    assert (withb < 0).any() and (withb > 0).any()


def test_groups_are_block_diagonal(oracle):
    """Grouped convolution (Sec. IV-A): each group of filters sees only its slice of channels and
    the results are stacked; groups=1 is the ordinary convolution; groups=C is depthwise."""
    rng = np.random.default_rng(29)
    N, C, K, G = 2, 6, 4, 2
    x = rng.standard_normal((N, C, 7, 6))
    w = rng.standard_normal((K, C // G, 3, 3))
    y = oracle.conv_fwd(x, w, pad=1, stride=(2, 1), groups=G)
    parts = [oracle.conv_fwd(x[:, g * 3:(g + 1) * 3], w[g * 2:(g + 1) * 2], pad=1, stride=(2, 1))
             for g in range(G)]
    assert np.array_equal(y, np.concatenate(parts, axis=1))
    wfull = np.zeros((K, C, 3, 3))                      # same thing as a dense block-diagonal filter
    for k in range(K):
        g = k // (K // G)
        wfull[k, g * 3:(g + 1) * 3] = w[k]
    np.testing.assert_allclose(y, oracle.conv_fwd(x, wfull, pad=1, stride=(2, 1)), atol=1e-13)
    assert np.array_equal(y, scatter_conv(x, w, (1, 1), (2, 1), (1, 1), groups=G)) or \
        np.allclose(y, scatter_conv(x, w, (1, 1), (2, 1), (1, 1), groups=G), atol=1e-12)
    wd = rng.standard_normal((C, 1, 3, 3))              # depthwise: groups == C
    yd = oracle.conv_fwd(x, wd, pad=1, groups=C)
    for c in range(C):
        want = correlate2d(np.pad(x[0, c], 1), wd[c, 0], mode="valid")
        np.testing.assert_allclose(yd[0, c], want, atol=1e-12)


def test_batchnorm_epilogue(oracle):
    """Conv + bias + spatial batch-norm (inference) + activation, Table I first row with the
    per-channel transform of Sec. IV-B: gamma*(v-mean)/sqrt(var+eps)+beta."""
    rng = np.random.default_rng(31)
    x = rng.standard_normal((2, 3, 5, 5))
    w = rng.standard_normal((4, 3, 3, 3))
    b = rng.standard_normal(4)
    gamma, beta, mean = rng.standard_normal((3, 4))
    var = rng.uniform(0.5, 2.0, 4)
    eps = 1e-3
    pre = oracle.conv_fwd(x, w, b, pad=1)
    want = gamma[None, :, None, None] * (pre - mean[None, :, None, None]) / \
        np.sqrt(var + eps)[None, :, None, None] + beta[None, :, None, None]
    got = oracle.conv_fwd(x, w, b, pad=1, bn=(gamma, beta, mean, var), eps=eps)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    got = oracle.conv_fwd(x, w, b, pad=1, bn=(gamma, beta, mean, var), eps=eps, act=1)
    np.testing.assert_allclose(got, np.maximum(want, 0), rtol=1e-13, atol=1e-13)
    # identity statistics leave the convolution unchanged
    one, zero = np.ones(4), np.zeros(4)
    same = oracle.conv_fwd(x, w, b, pad=1, bn=(one, zero, zero, one), eps=0.0)
    np.testing.assert_allclose(same, pre, rtol=1e-15, atol=0)


def test_points_agree_with_full_and_with_brute_force(oracle):
    rng = np.random.default_rng(37)
    x = rng.integers(-4, 5, size=(3, 4, 9, 8)).astype(float)
    w = rng.integers(-3, 4, size=(5, 4, 3, 3)).astype(float)
    b = rng.integers(-3, 4, size=5).astype(float)
    kw = dict(pad=(1, 1), stride=(2, 1), dil=(1, 2))
    want = np.maximum(scatter_conv(x, w, (1, 1), (2, 1), (1, 2)) + b[None, :, None, None], 0)
    idx = np.array([(n, k, p, q) for n in range(3) for k in range(5)
                    for p in range(want.shape[2]) for q in range(want.shape[3])][::7], np.int32)
    got = oracle.conv_fwd_points(x, w, b, idx, act=1, **kw)
    assert np.array_equal(got, want[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])
    with pytest.raises(ValueError):
        oracle.conv_fwd_points(x, w, b, np.array([[0, 0, 99, 0]], np.int32), **kw)


def test_output_extent_rule(oracle):
    assert oracle.out_extent(224, 7, 3, 2, 1) == 112      # (224+6-7)/2 = 111.5 -> floor -> +1
    assert oracle.out_extent(28, 3, 1, 2, 1) == 14
    assert oracle.out_extent(56, 3, 1, 1, 1) == 56
    assert oracle.out_extent(5, 3, 0, 1, 2) == 1
    assert oracle.out_extent(4, 3, 0, 1, 2) == 0          # dilated filter does not fit
    assert oracle.out_extent(7, 1, 0, 3, 1) == 3
    with pytest.raises(ValueError):
        oracle.conv_fwd(np.ones((1, 1, 4, 4)), np.ones((1, 1, 3, 3)), dil=2)


def test_rejects_bad_parameters(oracle):
    x, w = np.ones((1, 2, 4, 4)), np.ones((2, 2, 3, 3))
    with pytest.raises(ValueError):
        oracle.conv_fwd(x, w, stride=0)
    with pytest.raises(ValueError):
        oracle.conv_fwd(x, w, pad=-1)
    with pytest.raises(ValueError):
        oracle.conv_fwd(x, np.ones((2, 3, 3, 3)))
    with pytest.raises(ValueError):
        oracle.conv_fwd(x, np.ones((3, 1, 3, 3)), groups=2)
