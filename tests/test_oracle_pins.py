"""Pins for the CPU oracle: each layer is checked against something other than itself --
brute force on tiny tensors, closed forms, exact identities the paper states (Lemma 2, Eq. (12)),
special cases that reduce to a numpy routine.  No GPU, no HIP library."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


# ------------------------------------------------------------------ independent brute force
def brute_conv(x, w, b, sh, sw, ph, pw):
    """Definition of the layer written as pure-Python loops over an explicitly zero-padded input."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw))
    xp[:, :, ph:ph + H, pw:pw + W] = x
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    y = np.zeros((N, K, P, Q))
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        win = xp[n, :, p * sh:p * sh + R, q * sw:q * sw + S]
        y[n, k, p, q] = math.fsum((win * w[k]).ravel().tolist() + [b[k]])
    return y


def brute_maxpool(x, k, s, pad, out):
    N, C, H, W = x.shape
    y = np.full((N, C, out[0], out[1]), np.nan)
    for n, c, p, q in itertools.product(range(N), range(C), range(out[0]), range(out[1])):
        vals = [x[n, c, i, j]
                for i in range(p * s - pad, p * s - pad + k) if 0 <= i < H
                for j in range(q * s - pad, q * s - pad + k) if 0 <= j < W]
        y[n, c, p, q] = max(vals)       # raises on an empty window: every window must touch the input
    return y


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("shape", [
    # N, C, H, W, K, R, S, sh, sw, ph, pw   (non-square, asymmetric: catches swapped axes)
    (2, 3, 7, 9, 4, 3, 3, 1, 1, 1, 1),
    (1, 2, 9, 6, 3, 5, 5, 1, 1, 2, 2),
    (2, 3, 11, 8, 2, 3, 3, 2, 2, 1, 1),
    (1, 4, 8, 10, 3, 3, 2, 2, 1, 0, 1),
    (1, 2, 13, 12, 2, 7, 7, 4, 4, 3, 3),
    (1, 1, 12, 15, 2, 11, 11, 4, 4, 0, 0),
])
def test_conv_brute_force(shape):
    N, C, H, W, K, R, S, sh, sw, ph, pw = shape
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C, R, S))
    b = rng.standard_normal(K)
    y = oracle.conv2d(x, w, b, (sh, sw), (ph, pw))
    ref = brute_conv(x, w, b, sh, sw, ph, pw)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_conv_1x1_is_per_pixel_matvec():
    x = rng.standard_normal((2, 5, 4, 3))
    w = rng.standard_normal((6, 5, 1, 1))
    b = rng.standard_normal(6)
    y = oracle.conv2d(x, w, b)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x) + b[None, :, None, None]
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)


def test_conv_1x1_equals_centre_only_5x5_bit_exact():
    x = rng.standard_normal((2, 6, 9, 7))
    w1 = rng.standard_normal((4, 6, 1, 1))
    b = rng.standard_normal(4)
    w5 = np.zeros((4, 6, 5, 5))
    w5[:, :, 2, 2] = w1[:, :, 0, 0]
    assert np.array_equal(oracle.conv2d(x, w1, b), oracle.conv2d(x, w5, b, 1, 2))


def test_conv_single_tap_shifts_input_without_flip():
    """A filter with one tap at (r0, s0) copies x shifted by (r0-pad, s0-pad): cross-correlation.
    A flipped kernel or swapped r/s would shift the other way."""
    x = rng.standard_normal((1, 3, 6, 8))
    for r0, s0 in [(0, 0), (0, 2), (2, 1), (1, 1)]:
        w = np.zeros((3, 3, 3, 3))
        for c in range(3):
            w[c, c, r0, s0] = 1.0
        y = oracle.conv2d(x, w, None, 1, 1)
        xp = np.zeros((1, 3, 8, 10))
        xp[:, :, 1:7, 1:9] = x
        assert np.array_equal(y, xp[:, :, r0:r0 + 6, s0:s0 + 8])


def test_conv_stacking_identity_eq12_bit_exact():
    """Eq. (12): two same-kernel branches on one input, concatenated == one conv with stacked
    filters and biases."""
    x = rng.standard_normal((2, 5, 7, 7))
    wl, wr = rng.standard_normal((3, 5, 3, 3)), rng.standard_normal((4, 5, 3, 3))
    bl, br = rng.standard_normal(3), rng.standard_normal(4)
    sep = oracle.concat([oracle.conv2d(x, wl, bl, 1, 1), oracle.conv2d(x, wr, br, 1, 1)])
    one = oracle.conv2d(x, np.concatenate([wl, wr]), np.concatenate([bl, br]), 1, 1)
    assert np.array_equal(sep, one)


@pytest.mark.parametrize("stride", [2, 3, 4])
def test_strided_conv_is_subsampled_stride1(stride):
    """The streamline rule (Sec. 3.1, pooling layer) multiplies strides: a stride-s conv is the
    stride-1 conv sampled at every s-th position."""
    x = rng.standard_normal((1, 3, 13, 17))
    w = rng.standard_normal((2, 3, 3, 3))
    b = rng.standard_normal(2)
    full = oracle.conv2d(x, w, b, 1, 1)
    sub = oracle.conv2d(x, w, b, stride, 1)
    assert np.array_equal(sub, full[:, :, ::stride, ::stride])


def test_conv_relu_flag_and_linearity():
    x = rng.standard_normal((1, 2, 5, 5))
    w = rng.standard_normal((3, 2, 3, 3))
    b = rng.standard_normal(3)
    y = oracle.conv2d(x, w, b, 1, 1)
    assert np.array_equal(oracle.conv2d(x, w, b, 1, 1, relu=True), np.maximum(y, 0))
    np.testing.assert_allclose(oracle.conv2d(2 * x, w, None, 1, 1), 2 * (y - b[None, :, None, None]), atol=1e-12)


# ------------------------------------------------------------------ max-pool / ReLU / concat
@pytest.mark.parametrize("h,k,s,pad,expect", [
    (56, 3, 2, 0, 28), (112, 3, 2, 0, 56), (28, 3, 2, 0, 14), (14, 3, 2, 0, 7),   # GoogLeNet chain
    (55, 3, 2, 0, 27), (27, 3, 2, 0, 13),                                         # AlexNet chain
    (28, 3, 1, 1, 28), (7, 3, 1, 1, 7),                                           # inception pool branch
    (5, 2, 2, 1, 3), (4, 2, 2, 1, 3), (6, 3, 3, 1, 3), (3, 3, 2, 1, 2),           # padding rule
])
def test_pool_output_size(h, k, s, pad, expect):
    assert oracle.pool_out_size(h, k, s, pad) == expect
    # every window of the stated size touches the input
    assert (expect - 1) * s - pad < h


@pytest.mark.parametrize("N,C,H,W,k,s,pad", [
    (2, 3, 8, 7, 3, 2, 0), (1, 2, 7, 9, 3, 2, 0), (1, 2, 6, 5, 3, 1, 1), (1, 1, 5, 5, 2, 2, 1),
    (1, 2, 9, 9, 3, 3, 1),
])
def test_maxpool_brute_force_negative_inputs(N, C, H, W, k, s, pad):
    x = -np.abs(rng.standard_normal((N, C, H, W))) - 0.5     # all negative: zero padding would win
    y = oracle.maxpool(x, k, s, pad)
    ref = brute_maxpool(x, k, s, pad, y.shape[2:])
    assert np.array_equal(y, ref)
    assert (y < 0).all()


def test_maxpool_special_cases():
    x = rng.standard_normal((2, 3, 6, 7))
    assert np.array_equal(oracle.maxpool(x, 1, 1, 0), x)
    assert np.array_equal(oracle.maxpool(np.full((1, 2, 9, 9), -3.25), 3, 2, 0), np.full((1, 2, 4, 4), -3.25))
    # a stride-1 3x3 pad-1 pool equals scipy-free sliding maximum over the zero-free padded input
    xp = np.full((2, 3, 8, 9), -np.inf)
    xp[:, :, 1:7, 1:8] = x
    win = np.lib.stride_tricks.sliding_window_view(xp, (3, 3), axis=(2, 3))
    assert np.array_equal(oracle.maxpool(x, 3, 1, 1), win.max(axis=(-1, -2)))


def test_relu_and_concat_exact():
    x = rng.standard_normal((2, 3, 4, 5))
    assert np.array_equal(oracle.relu(x), np.where(x > 0, x, 0.0))
    a, b, c = x, rng.standard_normal((2, 1, 4, 5)), rng.standard_normal((2, 4, 4, 5))
    y = oracle.concat([a, b, c])
    assert y.shape == (2, 8, 4, 5)
    assert np.array_equal(y[:, :3], a) and np.array_equal(y[:, 3:4], b) and np.array_equal(y[:, 4:], c)


# ------------------------------------------------------------------ LRN
def lrn_scalar(x, n, alpha, beta, k):
    """Closed form b = a / (k + alpha/n * sum a^2)^beta evaluated one element at a time."""
    N, C, H, W = x.shape
    y = np.empty_like(x)
    lo = n // 2
    for i, c, h, w in itertools.product(range(N), range(C), range(H), range(W)):
        window = [x[i, cc, h, w] for cc in range(c - lo, c - lo + n) if 0 <= cc < C]
        y[i, c, h, w] = x[i, c, h, w] / (k + alpha / n * math.fsum(v * v for v in window)) ** beta
    return y


@pytest.mark.parametrize("n,alpha,beta,k", [(5, 1e-4, 0.75, 1.0), (3, 0.5, 0.5, 2.0), (5, 2.0, 0.75, 1.0), (1, 0.3, 0.75, 1.0)])
def test_lrn_closed_form(n, alpha, beta, k):
    x = rng.standard_normal((2, 7, 3, 4)) * 3
    np.testing.assert_allclose(oracle.lrn(x, n, alpha, beta, k), lrn_scalar(x, n, alpha, beta, k), rtol=1e-14)


def test_lrn_special_cases():
    a = 1.7
    x = np.full((1, 8, 2, 2), a)
    y = oracle.lrn(x, 5, 0.9, 0.75, 1.0)
    for c, cnt in [(0, 3), (1, 4), (2, 5), (5, 5), (6, 4), (7, 3)]:      # window clipped at the channel edges
        np.testing.assert_allclose(y[0, c], a / (1.0 + 0.9 / 5 * cnt * a * a) ** 0.75, rtol=1e-14)
    x = rng.standard_normal((1, 6, 3, 3))
    np.testing.assert_allclose(oracle.lrn(x, 5, 0.0, 0.75, 2.0), x / 2.0 ** 0.75, rtol=1e-14)   # alpha = 0
    np.testing.assert_allclose(oracle.lrn(x, 5, 0.7, 0.0, 2.0), x, rtol=1e-14)                  # beta = 0
    np.testing.assert_allclose(oracle.lrn(x, 1, 0.7, 0.75, 1.0), x / (1 + 0.7 * x * x) ** 0.75, rtol=1e-14)
    # odd symmetry and channel-reversal symmetry of a centred window
    np.testing.assert_allclose(oracle.lrn(-x), -oracle.lrn(x), rtol=1e-15)
    np.testing.assert_allclose(oracle.lrn(x[:, ::-1], 5, 0.9)[:, ::-1], oracle.lrn(x, 5, 0.9), rtol=1e-14)


# ------------------------------------------------------------------ BN, Lemma 2
def test_bn_definition_and_lemma2_fold():
    N, C, K = 2, 4, 5
    x = rng.standard_normal((N, C, 6, 6))
    w, b = rng.standard_normal((K, C, 3, 3)), rng.standard_normal(K)
    gamma, beta = rng.uniform(0.5, 1.5, K), rng.standard_normal(K)
    mean, var = rng.standard_normal(K), rng.uniform(0.5, 1.5, K)
    eps = 1e-5
    y = oracle.conv2d(x, w, b, 1, 1)
    ybn = oracle.bn(y, gamma, beta, mean, var, eps)
    ref = gamma[None, :, None, None] * (y - mean[None, :, None, None]) / np.sqrt(var + eps)[None, :, None, None] \
        + beta[None, :, None, None]
    np.testing.assert_allclose(ybn, ref, rtol=1e-14, atol=1e-14)
    # Lemma 2 / Eq. (9): conv -> BN -> Scale == one conv with W~ = eta W, B~ = eta B + beta - eta mu
    wf, bf = oracle.fold_bn(w, b, gamma, beta, mean, var, eps)
    eta = gamma / np.sqrt(var + eps)
    np.testing.assert_allclose(wf, eta[:, None, None, None] * w, rtol=1e-15)
    np.testing.assert_allclose(bf, eta * b + beta - eta * mean, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(oracle.conv2d(x, wf, bf, 1, 1), ybn, rtol=0, atol=1e-12)
    # gamma=1, beta=0, mean=0, var=1-eps: the fold is the identity
    one, zero = np.ones(K), np.zeros(K)
    wi, bi = oracle.fold_bn(w, b, one, zero, zero, one - eps, eps)
    np.testing.assert_allclose(wi, w, rtol=1e-15)
    np.testing.assert_allclose(bi, b, rtol=1e-15)


def test_bottleneck_fold_matches_original_in_fp64():
    layers = workloads.CONFIGS[4]["original"]
    params = workloads.make_params(4)
    x = workloads.make_input(4, 1)[:, :, :12, :12]
    y0 = oracle.forward(layers, params, x)
    y1 = oracle.forward(layers, params, x, fold=True)
    assert y0.shape == (1, 256, 12, 12)
    np.testing.assert_allclose(y1, y0, rtol=0, atol=1e-11)
    assert (y0 >= 0).all() and (y0 > 0).any()


def _bn_of(q, y, eps):
    return oracle.bn(y, q["gamma"], q["beta"], q["mean"], q["var"], eps)


def _manual_bottleneck(x, q, project, eps, fold, rnd):
    """Sec. 4.2's bottleneck written out call by call from the single-layer oracle functions: main path 1x1 -> 3x3
    (pad 1) -> 1x1, each followed by BN(+Scale), a ReLU after the first two; shortcut = x, or conv1x1 + BN of x on a
    projection block; output = ReLU(main + shortcut).  q: the block's parameter dicts in workload order (conv a, bn a,
    conv b, bn b, conv c, bn c[, conv p, bn p]).  fold: each conv+BN pair as the one conv of Lemma 2.
    rnd: applied to every tensor a layer leaves in memory -- in the original form after each conv, BN and the
    final add (ReLU of a rounded value is exact); in the folded form the only layers left are the tensor layers,
    each with what was merged into it (its ReLU; for the last one the shortcut sum and its ReLU), so there is one
    rounding per conv."""
    def unit(inp, i, pad, relu_after, last_with=None):
        cq, bq = q[i], q[i + 1]
        if fold:
            wf, bf = oracle.fold_bn(cq["w"], cq["b"], bq["gamma"], bq["beta"], bq["mean"], bq["var"], eps)
            y = oracle.conv2d(inp, wf, bf, 1, pad)
            if last_with is not None:
                return rnd(oracle.add_relu(y, last_with))
            return rnd(oracle.relu(y) if relu_after else y)
        y = rnd(oracle.conv2d(inp, cq["w"], cq["b"], 1, pad))
        y = rnd(_bn_of(bq, y, eps))
        if last_with is not None:
            return rnd(oracle.add_relu(y, last_with))
        return oracle.relu(y) if relu_after else y
    a = unit(x, 0, 0, True)
    b = unit(a, 2, 1, True)
    sc = unit(x, 6, 0, False) if project else x
    return unit(b, 4, 0, False, last_with=sc)


@pytest.mark.parametrize("project", [True, False])
@pytest.mark.parametrize("fold", [False, True])
@pytest.mark.parametrize("mirror", [False, True])
def test_bottleneck_against_manual_chain(project, fold, mirror):
    # an asymmetric block (mid != in != out unless identity) so that swapped operands or a wrong shortcut show
    cin, mid, out = (10, 6, 14) if project else (14, 6, 14)
    layers = [workloads.bottleneck(mid, out, project)]
    q = []
    workloads._walk(np.random.default_rng(77), layers, cin, "bf16" if mirror else "f32", q)
    x = np.abs(rng.standard_normal((2, cin, 5, 6)))
    if mirror:
        x = oracle.round_bf16(x)
    rnd = oracle.round_bf16 if mirror else (lambda a: a)
    want = _manual_bottleneck(x, q, project, workloads.BN_EPS, fold, rnd)
    got = oracle.forward(layers, q, x, mirror_bf16=mirror, fold=fold)
    assert got.shape == (2, out, 5, 6)
    assert np.array_equal(got, want)
    # the chain is sensitive to what it pins: dropping the middle ReLU or taking the shortcut from the wrong tensor changes it
    assert (want > 0).any() and (want == 0).any()
    if mirror:
        exact = oracle.forward(layers, q, x, fold=fold)
        assert not np.array_equal(got, exact) and np.abs(got - exact).max() < 0.1 * np.abs(exact).max()
        assert np.array_equal(oracle.round_bf16(got), got)          # what is stored is representable


def test_mirrored_forward_rounds_after_every_stored_layer():
    """bf16 storage rule: every tensor a layer writes is rounded once (nearest even); arithmetic inside a layer is exact
    fp64.  Pinned on a conv -> ReLU -> LRN -> pool -> conv -> ReLU -> avgpool -> fc -> softmax chain written out by hand."""
    R = oracle.round_bf16
    layers = [workloads.conv(6, 3, 1, 1), ("relu", {}), workloads.lrn(), workloads.maxpool(3, 2),
              workloads.conv(5, 1), ("relu", {}), ("avgpool", {"k": 3}), ("fc", {"out": 4}), ("softmax", {})]
    q = []
    workloads._walk(np.random.default_rng(5), layers, 3, "bf16", q)
    x = R(rng.standard_normal((2, 3, 6, 6)))
    trace = []
    got = oracle.forward(layers, q, x, mirror_bf16=True, trace=trace)
    steps = []
    t = R(oracle.conv2d(x, q[0]["w"], q[0]["b"], 1, 1)); steps.append(t)
    t = oracle.relu(t); steps.append(t)                  # exact on rounded values
    t = R(oracle.lrn(t, 5, 1e-4, 0.75, 1.0)); steps.append(t)
    t = oracle.maxpool(t, 3, 2, 0); steps.append(t)      # a selection: exact
    t = R(oracle.conv2d(t, q[1]["w"], q[1]["b"], 1, 0)); steps.append(t)
    t = oracle.relu(t); steps.append(t)
    t = R(oracle.avgpool(t, 3)); steps.append(t)
    logits = R(oracle.fc(t, q[2]["w"], q[2]["b"])); steps.append(logits)
    want = oracle.softmax(logits); steps.append(want)    # probabilities stay fp32 in the library: not rounded to bf16
    assert np.array_equal(got, want)
    assert len(trace) == len(steps)
    for (kind, out), ref in zip(trace, steps):           # every stored tensor, not only the last
        assert np.array_equal(out, ref), kind
    # moving or dropping a rounding is visible at this size
    unrounded = oracle.forward(layers, q, x)
    assert not np.array_equal(unrounded, want)
    t2 = oracle.relu(oracle.conv2d(x, q[0]["w"], q[0]["b"], 1, 1))       # first rounding dropped
    t2 = R(oracle.lrn(t2, 5, 1e-4, 0.75, 1.0))
    assert not np.array_equal(t2, trace[2][1])


# ------------------------------------------------------------------ tail layers, bf16 rounding
def test_avgpool_fc_softmax():
    x = rng.standard_normal((2, 3, 7, 7))
    np.testing.assert_allclose(oracle.avgpool(x, 7)[:, :, 0, 0], x.mean(axis=(2, 3)), rtol=1e-13)
    np.testing.assert_allclose(oracle.avgpool(x, 3, 2)[0, 1, 1, 2], x[0, 1, 2:5, 4:7].mean(), rtol=1e-13)
    w, b = rng.standard_normal((5, 3 * 49)), rng.standard_normal(5)
    z = oracle.fc(x, w, b)
    np.testing.assert_allclose(z, x.reshape(2, -1) @ w.T + b, rtol=1e-12, atol=1e-12)
    p = oracle.softmax(z)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(p[:, 1] / p[:, 3], np.exp(z[:, 1] - z[:, 3]), rtol=1e-12)
    np.testing.assert_allclose(oracle.softmax(z + 1000.0), p, rtol=1e-10)      # shift invariance, no overflow


def test_add_relu():
    a, b = rng.standard_normal(100), rng.standard_normal(100)
    assert np.array_equal(oracle.add_relu(a, b), np.maximum(a + b, 0.0))


def test_round_bf16():
    # hand-checked values: 8 significant bits, ties to even
    cases = {1.0: 1.0, 1.0 + 2 ** -8: 1.0, 1.0 + 3 * 2 ** -8: 1.0 + 2 ** -6, 1.0 + 2 ** -7: 1.0 + 2 ** -7,
             1.0 + 2 ** -8 + 2 ** -20: 1.0 + 2 ** -7, -3.0 - 2 ** -7: -3.0, 0.0: 0.0, 2.0 ** -130: 2.0 ** -130,
             255.5: 256.0, 254.5: 254.0}
    for v, r in cases.items():
        assert oracle.round_bf16(np.array([v]))[0] == r, v
    # subnormals of the format (spacing 2^-133 below 2^-126), its largest finite value, and the tie above it
    big = (2.0 - 2.0 ** -7) * 2.0 ** 127
    edge = {2.0 ** -133: 2.0 ** -133, 2.0 ** -134: 0.0, 3 * 2.0 ** -134: 2.0 ** -132, 2.0 ** -134 * 1.01: 2.0 ** -133,
            5 * 2.0 ** -134: 2.0 ** -132, 2.0 ** -126 - 2.0 ** -134: 2.0 ** -126, 2.0 ** -127 + 2.0 ** -133: 2.0 ** -127 + 2.0 ** -133,
            big: big, big + 2.0 ** 118: big, (2.0 - 2.0 ** -8) * 2.0 ** 127: np.inf, -(2.0 - 2.0 ** -8) * 2.0 ** 127: -np.inf,
            big + 2.0 ** 119 - 2.0 ** 90: big, np.inf: np.inf}
    for v, r in edge.items():
        assert oracle.round_bf16(np.array([v]))[0] == r, v
    assert np.isnan(oracle.round_bf16(np.array([np.nan]))[0])
    assert np.signbit(oracle.round_bf16(np.array([-2.0 ** -134]))[0]) or oracle.round_bf16(np.array([-2.0 ** -134]))[0] == 0.0
    # against the bit-level rule of the storage format on random fp32 values
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000))).astype(np.float32)
    assert np.array_equal(oracle.round_bf16(x).astype(np.float32), workloads.round_to_bf16(x))
    y = oracle.round_bf16(x)
    assert np.array_equal(oracle.round_bf16(y), y)                              # idempotent
    assert ((y.astype(np.float32).view(np.uint32) & 0xFFFF) == 0).all()         # bf16-representable


# ------------------------------------------------------------------ structure of the workloads
def test_googlenet_parameter_count_matches_table6_storage():
    with open(os.path.join(GOLDEN, "googlenet_storage.txt")) as f:
        mb = float([l for l in f if not l.startswith("#")][0])
    params = workloads.make_params(5)
    count = sum(q["w"].size + q["b"].size for q in params)
    assert len(params) == 58                     # 57 convolutions + the classifier
    assert abs(count * 4 / 2 ** 20 - mb) < 0.03   # 26.70 MiB vs the table's 26.72


def test_inception_3a_widths_and_paper_variant():
    rows = {}
    with open(os.path.join(GOLDEN, "inception_3a_paper_slim.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                name, a, b = line.split()
                rows[name] = (int(a), int(b))
    _, c1, c3r, c3, c5r, c5, cp = workloads.INCEPTION_WIDTHS["3a"]
    assert (c5, c3r, c3) == (rows["5x5"][0], rows["3x3_reduce"][0], rows["3x3"][0])
    assert c1 + c3 + c5 + cp == rows["concat"][0]
    # the printed 196 cannot keep the concatenated width; 192 = 128 + 64 does
    assert rows["3x3"][1] + rows["5x5"][1] != rows["concat"][1]
    var = workloads.inception_3a_paper_variant()[1]["branches"]
    assert var[0][0][1]["k"] == rows["3x3_reduce"][1] and var[1][2][1]["k"] == rows["5x5"][1]
    assert var[0][2][1]["k"] + var[1][2][1]["k"] == rows["concat"][1]


def test_googlenet_shape_chain_and_slim_boundaries():
    """Spatial 224 -> 112 -> 56 -> 28 -> 14 -> 7 -> 1 and widths 256 ... 1024; the slim net has the
    same tensor shape at every block boundary (rule 2 of Sec. 3.3)."""
    x = workloads.make_input(5, 1)
    shapes = {}
    for form in ("original", "slim"):
        tr = []
        y = oracle.forward(workloads.CONFIGS[5][form], workloads.make_params(5, form), x, trace=tr)
        shapes[form] = [t.shape for kind, t in tr if kind in ("inception", "avgpool", "fc", "softmax")]
        np.testing.assert_allclose(y.sum(axis=1), 1.0, rtol=1e-12)
        if form == "original":
            assert tr[0][1].shape == (1, 64, 112, 112) and tr[2][1].shape == (1, 64, 56, 56)
            assert tr[9][1].shape == (1, 192, 28, 28)
        else:
            assert tr[0][1].shape == (1, 64, 56, 56) and tr[5][1].shape == (1, 192, 28, 28)
    widths = [s[1] for s in shapes["original"][:9]]
    assert widths == [256, 480, 512, 512, 512, 528, 832, 832, 1024]
    assert [s[2] for s in shapes["original"][:9]] == [28, 28, 14, 14, 14, 14, 14, 7, 7]
    assert shapes["original"] == shapes["slim"]
    assert shapes["original"][-1] == (1, 1000)


def test_config_shapes():
    # config 1: both forms end at 192 x 28 x 28
    x = workloads.make_input(1)
    for form in ("original", "slim"):
        y = oracle.forward(workloads.CONFIGS[1][form], workloads.make_params(1, form), x)
        assert y.shape == (1, 192, 28, 28)
    # config 2: 256 x 28 x 28 both ways (small spatial crop keeps it fast; widths are what matters)
    x = workloads.make_input(2, 1)[:, :, :9, :9]
    for form in ("original", "slim"):
        y = oracle.forward(workloads.CONFIGS[2][form], workloads.make_params(2, form), x)
        assert y.shape == (1, 256, 9, 9)
    # config 3: original 256 x 13 x 13; the slim chain lands on 14 x 14 (stride rule, floor)
    x = workloads.make_input(3, 1)
    y = oracle.forward(workloads.CONFIGS[3]["original"], workloads.make_params(3), x)
    assert y.shape == (1, 256, 13, 13)
    y = oracle.forward(workloads.CONFIGS[3]["slim"], workloads.make_params(3, "slim"), x)
    assert y.shape == (1, 256, 14, 14)


def test_inception_composition_against_manual_chain():
    layers = workloads.CONFIGS[2]["original"]
    params = workloads.make_params(2)
    x = workloads.make_input(2, 1)[:, :, :7, :7].astype(np.float64)
    y = oracle.forward(layers, params, x)
    c = lambda i, inp, pad=0: np.maximum(oracle.conv2d(inp, params[i]["w"], params[i]["b"], 1, pad), 0)
    b1 = c(0, x)
    b2 = c(2, c(1, x), 1)
    b3 = c(4, c(3, x), 2)
    b4 = c(5, oracle.maxpool(x, 3, 1, 1))
    assert np.array_equal(y, np.concatenate([b1, b2, b3, b4], axis=1))


def test_input_prefix_property_and_distributions():
    a, b = workloads.make_input(2, 1), workloads.make_input(2, 3)
    assert np.array_equal(a, b[:1])
    assert (b >= 0).all()
    x1 = workloads.make_input(1)
    assert x1.shape == (1, 64, 56, 56) and x1.min() >= 0 and x1.max() < 1
    w = workloads.make_params(1)[0]["w"]
    assert abs(w.std() - math.sqrt(2 / 576)) < 2e-3
    x4 = workloads.make_input(4, 1)
    assert ((x4.view(np.uint32) & 0xFFFF) == 0).all()      # bf16-representable


def test_table4_fixture_is_consistent():
    rows = {}
    with open(os.path.join(GOLDEN, "table4_layer_ms.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                name, a, b = line.split()
                rows[name] = (float(a), float(b))
    tot = rows.pop("Total")
    assert 0 <= tot[0] - sum(v[0] for v in rows.values()) < 2.0
    assert 0 <= tot[1] - sum(v[1] for v in rows.values()) < 2.0
    assert abs(tot[0] / tot[1] - 3.09) < 0.01


# ---- layer-wise regression of a slim layer (Sec. 3.1: the optimisation goal below Eq. (4), Lemma 1) ------------
def _loss(x, w, b, y, stride, pad):
    f = oracle.conv2d(x, w, b, stride, pad, relu=True)
    return oracle.regression_loss_grad(f, y)[0]


def test_regression_gradients_match_finite_differences():
    """The gradient is what the loss does under a small change of one parameter: central differences of L
    itself (which only needs the forward pass, pinned above) against dw, db for every bias and a spread of
    weights; strides, padding and a non-square filter so that a transposed index or a dropped padding
    term shows."""
    rng = np.random.default_rng(42)
    for (N, C, H, W, K, R, S, stride, pad) in [(2, 3, 7, 6, 4, 3, 2, 2, 1), (1, 2, 5, 5, 3, 3, 3, 1, 1), (2, 2, 6, 8, 2, 1, 1, 1, 0),
                                                (1, 1, 9, 7, 2, 5, 3, (2, 1), (2, 0))]:
        x = rng.standard_normal((N, C, H, W))
        w = rng.standard_normal((K, C, R, S)) * 0.4
        b = rng.standard_normal(K) * 0.2
        f = oracle.conv2d(x, w, b, stride, pad, relu=True)
        y = np.abs(rng.standard_normal(f.shape))
        loss, dz = oracle.regression_loss_grad(f, y)
        assert loss == pytest.approx(((f - y) ** 2).sum(), rel=1e-14)
        dw, db = oracle.conv2d_bwd_params(x, dz, R, S, stride, pad)
        h = 1e-6
        for k in range(K):
            bp, bm = b.copy(), b.copy()
            bp[k] += h
            bm[k] -= h
            fd = (_loss(x, w, bp, y, stride, pad) - _loss(x, w, bm, y, stride, pad)) / (2 * h)
            assert fd == pytest.approx(db[k], rel=1e-5, abs=1e-7)
        for _ in range(12):
            idx = tuple(int(rng.integers(0, n)) for n in w.shape)
            wp, wm = w.copy(), w.copy()
            wp[idx] += h
            wm[idx] -= h
            fd = (_loss(x, wp, b, y, stride, pad) - _loss(x, wm, b, y, stride, pad)) / (2 * h)
            assert fd == pytest.approx(dw[idx], rel=1e-5, abs=1e-7)


def test_conv_param_gradient_of_1x1_is_a_matrix_product():
    """For a 1x1 convolution z = W X per image, so dW = sum_n dZ_n X_n^T and db = row sums of dZ: numpy's matmul."""
    rng = np.random.default_rng(43)
    x = rng.standard_normal((3, 5, 4, 6))
    dz = rng.standard_normal((3, 7, 4, 6))
    dw, db = oracle.conv2d_bwd_params(x, dz, 1, 1, 1, 0)
    ref = sum(dz[n].reshape(7, -1) @ x[n].reshape(5, -1).T for n in range(3))
    np.testing.assert_allclose(dw[:, :, 0, 0], ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, dz.sum(axis=(0, 2, 3)), rtol=1e-12)
    # linear in dz, and a strided / padded case against brute force over the definition
    dz2 = rng.standard_normal(dz.shape)
    dw2, db2 = oracle.conv2d_bwd_params(x, dz + 2 * dz2, 1, 1, 1, 0)
    dwb, dbb = oracle.conv2d_bwd_params(x, dz2, 1, 1, 1, 0)
    np.testing.assert_allclose(dw2, dw + 2 * dwb, rtol=1e-12, atol=1e-12)
    x = rng.standard_normal((2, 2, 5, 4))
    P, Q = oracle.conv_out_size(5, 3, 2, 1), oracle.conv_out_size(4, 2, 1, 0)
    dz = rng.standard_normal((2, 3, P, Q))
    dw, _ = oracle.conv2d_bwd_params(x, dz, 3, 2, (2, 1), (1, 0))
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (0, 0)))
    for k in range(3):
        for c in range(2):
            for r in range(3):
                for s in range(2):
                    want = sum(dz[n, k, p, q] * xp[n, c, p * 2 + r, q + s] for n in range(2) for p in range(P) for q in range(Q))
                    assert dw[k, c, r, s] == pytest.approx(want, rel=1e-12, abs=1e-12)


def test_regression_has_zero_gradient_at_the_generating_layer_and_descends():
    """If the target is the output of a layer of the same shape, that layer's parameters have zero loss and zero
    gradient; from a perturbed start, gradient steps with a small rate lower the loss every time."""
    rng = np.random.default_rng(44)
    x = rng.standard_normal((4, 3, 8, 8))
    w_star = rng.standard_normal((5, 3, 3, 3)) * 0.3
    b_star = rng.standard_normal(5) * 0.1
    y = oracle.conv2d(x, w_star, b_star, 2, 1, relu=True)
    loss, dz = oracle.regression_loss_grad(y, y)
    assert loss == 0.0 and not dz.any()
    w, b = w_star + rng.standard_normal(w_star.shape) * 0.1, b_star + 0.05
    losses = []
    for _ in range(25):
        loss, w, b = oracle.regression_step(x, w, b, y, 2, 1, lr=2e-3)
        losses.append(loss)
    assert all(b_ < a_ for a_, b_ in zip(losses, losses[1:]))
    assert losses[-1] < 0.2 * losses[0]
