"""Pins of the oracle's average-pooling layer against things that are not the oracle: the layer is affine
(Section 2: exact transformer), so it must agree with a convolution carrying the same weights, with the dense layer
it folds into, with closed forms, a second implementation and sampled points.  No GPU needed."""
import numpy as np
import pytest

import workloads as wl
from helpers import FLOAT32_ORDERS, affine_matrix, ball_box, forward, forward_float32, np_deeppoly, sample_box
from oracle import OracleNet


def make_oracle(net, **opts):
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    if opts:
        o.set_options(**opts)
    return o


def analysed_layers(net):
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    return [i for i, L in enumerate(net.layers, start=1)
            if L["type"] == "relu" or i in feeds or i == len(net.layers)]


def lenet_like(seed=0):
    """conv-ReLU, 2x2 average, conv-ReLU, overlapping 3x3 stride-2 average with padding, dense-ReLU, dense."""
    return wl.pool_net("tiny_lenet", (2, 10, 10), [("conv", 3, 3, 1, 1), ("pool", 2, 2, 0), ("conv", 4, 2, 1, 0),
                                                   ("pool", 3, 2, 1)], [8], n_out=3, seed=seed)


def as_convolutions(net):
    """The same network with every pooling layer replaced by a convolution whose filter has 1/(k*k) on the channel
    diagonal (exact in float32 only when k*k is a power of two)."""
    out = wl.Net(net.name + "_conv", net.input_shape)
    for L in net.layers:
        if L["type"] == "avgpool":
            c = net.shape_of(L["src"])[0]
            k = L["kernel"]
            W = np.zeros((c, c, k, k), np.float32)
            for d in range(c):
                W[d, d] = np.float32(1.0 / (k * k))
            out.conv(L["src"], W, np.zeros(c, np.float32), L["stride"], L["pad"])
        else:
            out.layers.append(dict(L))
    return out


def test_hand_computed_average():
    """One 2x2 average over a 1x2x2 box: the mean of the lower ends and the mean of the upper ends (values exact in
    binary); a second, overlapping 2x2 stride-1 average with padding 1 divides by 4 also at the border."""
    net = wl.Net("hand", (1, 2, 2))
    net.avgpool(0, 2)
    o = make_oracle(net)
    lo0 = np.array([0.25, 0.5, -1.0, 2.0])
    hi0 = np.array([0.75, 0.5, 1.0, 4.0])
    o.analyze_box(lo0, hi0)
    lo, hi = o.get_bounds(1)
    assert lo.tolist() == [0.4375] and hi.tolist() == [1.5625]
    net = wl.Net("hand_pad", (1, 2, 2))
    net.avgpool(0, 2, 1, 1)
    o = make_oracle(net)
    o.analyze_box(lo0, hi0)
    lo, hi = o.get_bounds(1)
    # output 3x3; corner (0,0) sees only input (0,0); centre sees all four; edge (0,1) sees inputs (0,0),(0,1)
    assert lo.reshape(3, 3)[0, 0] == 0.0625 and hi.reshape(3, 3)[0, 0] == 0.1875
    assert lo.reshape(3, 3)[1, 1] == 0.4375 and hi.reshape(3, 3)[1, 1] == 1.5625
    assert lo.reshape(3, 3)[0, 1] == 0.1875 and hi.reshape(3, 3)[0, 1] == 0.3125
    assert lo.reshape(3, 3)[2, 0] == -0.25 and hi.reshape(3, 3)[2, 0] == 0.25


def test_power_of_two_average_equals_diagonal_convolution():
    net = wl.pool_net("p2", (2, 8, 8), [("conv", 3, 3, 1, 1), ("pool", 2, 2, 0), ("conv", 4, 3, 1, 1), ("pool", 2, 1, 1)],
                      [8], n_out=3, seed=3)
    ref = as_convolutions(net)
    c = np.random.default_rng(0).random(net.n_in).astype(np.float32)
    a, b = make_oracle(net), make_oracle(ref)
    a.analyze(c, 0.03)
    b.analyze(c, 0.03)
    for l in analysed_layers(net):
        (alo, ahi), (blo, bhi) = a.get_bounds(l), b.get_bounds(l)
        np.testing.assert_allclose(alo, blo, rtol=0, atol=1e-13)
        np.testing.assert_allclose(ahi, bhi, rtol=0, atol=1e-13)
    assert np.array_equal(a.certify(1)[1] > 0, b.certify(1)[1] > 0)
    np.testing.assert_allclose(a.certify(1)[1], b.certify(1)[1], rtol=0, atol=1e-12)


def test_global_average_head_equals_the_folded_dense_head():
    """A residual net whose head is global average pooling + dense against the same net with the two folded into one
    dense layer (4x4 positions: the folded weights are exact)."""
    kw = dict(input_shape=(2, 8, 8), channels=(3, 4), blocks=(2, 1), n_out=3, seed=5)
    folded, pooled = wl.resnet("f", **kw), wl.resnet("p", pool_head=True, **kw)
    assert pooled.layers[-2]["type"] == "avgpool" and pooled.shape_of(pooled.out_layer - 1) == (4, 1, 1)
    c = np.random.default_rng(1).random(folded.n_in).astype(np.float32)
    a, b = make_oracle(pooled), make_oracle(folded)
    a.analyze(c, 0.02)
    b.analyze(c, 0.02)
    (alo, ahi), (blo, bhi) = a.get_bounds(pooled.out_layer), b.get_bounds(folded.out_layer)
    np.testing.assert_allclose(alo, blo, rtol=0, atol=1e-12)
    np.testing.assert_allclose(ahi, bhi, rtol=0, atol=1e-12)
    np.testing.assert_allclose(a.certify(0)[1], b.certify(0)[1], rtol=0, atol=1e-12)


@pytest.mark.parametrize("cand", [0, 1])
def test_second_implementation_agrees(cand):
    """3x3 windows: 1/9 is not a binary fraction, so the comparison is with the NumPy DeepPoly on the exact matrix."""
    net = lenet_like(2)
    c = np.random.default_rng(3).random(net.n_in).astype(np.float32)
    lo0, hi0 = ball_box(c, 0.04)
    o = make_oracle(net, candidates=cand)
    o.analyze(c, 0.04)
    ref = np_deeppoly(net, lo0, hi0, candidates=cand)
    for l in analysed_layers(net):
        lo, hi = o.get_bounds(l)
        np.testing.assert_allclose(lo, ref[l][0], rtol=0, atol=1e-10)
        np.testing.assert_allclose(hi, ref[l][1], rtol=0, atol=1e-10)
        assert np.all(lo <= ref[l][0] + 1e-12) and np.all(hi >= ref[l][1] - 1e-12)


def test_eps_zero_and_samples():
    net = lenet_like(1)
    c = np.random.default_rng(5).random(net.n_in).astype(np.float32)
    o = make_oracle(net)
    o.analyze(c, 0.0)
    vals = forward(net, c[None].astype(np.float64))
    for l in analysed_layers(net):
        lo, hi = o.get_bounds(l)
        assert np.all(lo <= vals[l][0] + 1e-13) and np.all(hi >= vals[l][0] - 1e-13)    # the forward pass rounds too
        assert np.max(hi - lo) < 1e-12
    o.analyze(c, 0.05)
    lo0, hi0 = ball_box(c, 0.05)
    X = sample_box(lo0, hi0, 4000, np.random.default_rng(6))
    vals = forward(net, X)
    for l in analysed_layers(net):
        lo, hi = o.get_bounds(l)
        assert np.all(vals[l] >= lo[None] - 1e-12) and np.all(vals[l] <= hi[None] + 1e-12)
        assert np.all(np.isfinite(lo)) and np.all(np.isfinite(hi))


def test_requested_bounds_of_a_pooling_layer_are_the_exact_affine_image():
    """Rows of a pooling layer itself: after a stable (all-active) ReLU the whole prefix is affine, so the bounds are
    the exact interval image of the composed matrix."""
    rng = np.random.default_rng(9)
    net = wl.Net("stable", (2, 6, 6))
    W = rng.standard_normal((3, 2, 3, 3)).astype(np.float32) * np.float32(0.1)
    b = np.full(3, 5.0, np.float32)                       # keeps every neuron positive on [0,1]^n
    p = net.avgpool(net.relu(net.conv(0, W, b, 1, 1)), 3, 2, 1)
    net.dense(p, rng.standard_normal((2, net.n_neurons(p))).astype(np.float32), np.zeros(2, np.float32))
    o = make_oracle(net)
    o.request_bounds(p)
    c = rng.random(net.n_in).astype(np.float32)
    o.analyze(c, 0.1)
    lo0, hi0 = ball_box(c, 0.1)
    A1, b1 = affine_matrix(net, 1)
    A3, _ = affine_matrix(net, 3)
    M, v = A3 @ A1, A3 @ b1
    Mp, Mn = np.maximum(M, 0), np.minimum(M, 0)
    lo, hi = o.get_bounds(p)
    np.testing.assert_allclose(lo, Mp @ lo0 + Mn @ hi0 + v, rtol=0, atol=1e-12)
    np.testing.assert_allclose(hi, Mp @ hi0 + Mn @ lo0 + v, rtol=0, atol=1e-12)


def test_early_termination_interval_image_and_soundness():
    net = lenet_like(4)
    c = np.random.default_rng(7).random(net.n_in).astype(np.float32)
    full = make_oracle(net)
    full.analyze(c, 0.03)
    o = make_oracle(net)
    o.set_early_termination(True)
    o.analyze(c, 0.03)
    lo0, hi0 = ball_box(c, 0.03)
    X = sample_box(lo0, hi0, 2000, np.random.default_rng(8))
    vals = forward(net, X)
    for l in range(1, net.out_layer + 1):
        if net.layers[l - 1]["type"] == "avgpool":       # interval image: window means of the predecessor's intervals
            ilo, ihi = o.get_interval_image(l)
            plo, phi = o.get_bounds(net.layers[l - 1]["src"])
            A, _ = affine_matrix(net, l)
            np.testing.assert_allclose(ilo, A @ plo, rtol=0, atol=1e-13)
            np.testing.assert_allclose(ihi, A @ phi, rtol=0, atol=1e-13)
            assert np.all(vals[l] >= ilo[None] - 1e-12) and np.all(vals[l] <= ihi[None] + 1e-12)
    for l in analysed_layers(net):
        lo, hi = o.get_bounds(l)
        flo, fhi = full.get_bounds(l)
        assert np.all(vals[l] >= lo[None] - 1e-12) and np.all(vals[l] <= hi[None] + 1e-12)
        assert np.all(lo <= flo + 1e-9) and np.all(hi >= fhi - 1e-9)      # never tighter than the full analysis


def test_float_inference_error_of_an_average_and_containment():
    """eta of an averaging neuron is gamma(K+1) * mean|x| + (K+1) * 2^-149 with K = window size, evaluated on the
    predecessor's bounds; every float32 evaluation (any order; division or multiplication by the rounded reciprocal)
    stays inside the bounds, and some evaluation leaves the bounds of the plain analysis of a long average."""
    u = 2.0 ** -24
    net = lenet_like(6)
    c = np.random.default_rng(11).random(net.n_in).astype(np.float32)
    o = make_oracle(net)
    for l, L in enumerate(net.layers, start=1):       # eta of a layer is evaluated on its predecessor's bounds
        if L["type"] == "avgpool":
            o.request_bounds(l)
    o.set_float_inference(True)
    o.analyze(c, 0.02)
    for l in range(1, net.out_layer + 1):
        L = net.layers[l - 1]
        if L["type"] != "avgpool":
            continue
        K = L["kernel"] ** 2
        plo, phi = o.get_bounds(L["src"])
        A, _ = affine_matrix(net, l)
        want = (K + 1) * u / (1 - (K + 1) * u) * (A @ np.maximum(np.abs(plo), np.abs(phi))) + (K + 1) * 2.0 ** -149
        eta = o.get_inference_error(l)
        assert np.all(eta >= want * (1 - 1e-12)) and np.all(eta <= want * (1 + 1e-9) + 1e-300)
    rng = np.random.default_rng(12)
    lo0, hi0 = ball_box(c, 0.02)
    for trial in range(30):
        x = np.clip((lo0 + (hi0 - lo0) * rng.random(net.n_in)).astype(np.float32), lo0.astype(np.float32), hi0.astype(np.float32))
        x = np.minimum(np.maximum(x.astype(np.float64), lo0), hi0).astype(np.float32)
        if np.any(x.astype(np.float64) < lo0) or np.any(x.astype(np.float64) > hi0):
            continue
        vals = forward_float32(net, x, FLOAT32_ORDERS[trial % len(FLOAT32_ORDERS)], rng)
        for l in analysed_layers(net):
            lo, hi = o.get_bounds(l)
            assert np.all(vals[l].astype(np.float64) >= lo) and np.all(vals[l].astype(np.float64) <= hi), (trial, l)


def test_float_inference_matters_for_a_point_box_average():
    """A point box through one 3x3 average: the plain analysis gives the exact mean (to float64 rounding); a float32
    evaluation differs from it, and the float-inference bounds contain every such evaluation."""
    net = wl.Net("avg_point", (1, 3, 3))
    net.avgpool(0, 3)
    x = np.array([0.1, 0.7, 0.3, 0.9, 0.2, 0.6, 0.8, 0.4, 0.5], np.float32) + np.float32(1e-3)
    plain = make_oracle(net)
    plain.analyze_box(x.astype(np.float64), x.astype(np.float64))
    plo, phi = plain.get_bounds(1)
    exact = float(np.sum(x.astype(np.float64)) / 9.0)
    assert plo[0] <= exact <= phi[0] and phi[0] - plo[0] < 1e-15
    o = make_oracle(net)
    o.set_float_inference(True)
    o.analyze_box(x.astype(np.float64), x.astype(np.float64))
    lo, hi = o.get_bounds(1)
    assert hi[0] - lo[0] < 2 * 10.5 * 2.0 ** -24 * exact
    rng = np.random.default_rng(0)
    outside = 0
    for trial in range(60):
        v = float(forward_float32(net, x, FLOAT32_ORDERS[trial % len(FLOAT32_ORDERS)], rng)[1][0])
        assert lo[0] <= v <= hi[0]
        outside += not (plo[0] <= v <= phi[0])
    assert outside > 0


def test_rectangular_window_stride_and_padding():
    """kh != kw, stride_h != stride_w, pad_h != pad_w: against the NumPy DeepPoly on the exact matrix and sampled points
    (a transposed stride or padding changes which inputs a window holds)."""
    rng = np.random.default_rng(21)
    net = wl.Net("rect_pool", (2, 7, 9))
    W = (rng.standard_normal((3, 2, 2, 3)) * 0.4).astype(np.float32)
    net.layers.append(dict(type="conv", src=0, W=W, b=(rng.standard_normal(3) * 0.1).astype(np.float32), stride=(1, 2), pad=(1, 0),
                           shape=(3, 8, 4)))
    net.layers.append(dict(type="relu", src=1, shape=(3, 8, 4)))
    net.layers.append(dict(type="avgpool", src=2, kernel=(3, 2), stride=(2, 1), pad=(1, 0), shape=(3, 4, 3)))
    net.layers.append(dict(type="relu", src=3, shape=(3, 4, 3)))
    net.layers.append(dict(type="avgpool", src=4, kernel=(2, 3), stride=(1, 2), pad=(0, 2), shape=(3, 3, 3)))
    Wd = (rng.standard_normal((4, 27)) * 0.3).astype(np.float32)
    net.dense(5, Wd, np.zeros(4, np.float32))
    c = rng.random(net.n_in).astype(np.float32)
    o = make_oracle(net)
    o.request_bounds(5)
    o.analyze(c, 0.05)
    lo0, hi0 = ball_box(c, 0.05)
    ref = np_deeppoly(net, lo0, hi0)
    vals = forward(net, sample_box(lo0, hi0, 3000, np.random.default_rng(22)))
    for l in (1, 2, 3, 4, 6):
        lo, hi = o.get_bounds(l)
        assert np.all(vals[l] >= lo[None] - 1e-12) and np.all(vals[l] <= hi[None] + 1e-12)
        if l != 6:          # (the NumPy version takes no candidate over layer 5, which is bounded here)
            np.testing.assert_allclose(lo, ref[l][0], rtol=0, atol=1e-10)
            np.testing.assert_allclose(hi, ref[l][1], rtol=0, atol=1e-10)
    assert np.all(o.get_bounds(6)[0] >= ref[6][0] - 1e-10) and np.all(o.get_bounds(6)[1] <= ref[6][1] + 1e-10)


def test_one_ninth_is_enclosed_in_exact_rationals():
    """A 3x3 window that holds a single input (the corner of a padded 1x1 image): the output is x/9, and 1/9 is no
    binary fraction.  For x = 1, -1 and 3 the bounds must enclose the rational value and be at most a few ulps apart on
    each side (a weight rounded the wrong way for one of the signs leaves the rational value outside)."""
    from fractions import Fraction
    net = wl.Net("ninth", (1, 1, 1))
    net.avgpool(0, 3, 1, 2)                  # output 3x3, every window holds the one pixel
    W = np.array([[1, -1, 0, 0, 0, 0, 0, 0, 0]], np.float32)
    for x in (1.0, -1.0, 3.0):
        o = make_oracle(net)
        o.analyze_box(np.array([x]), np.array([x]))
        lo, hi = o.get_bounds(1)
        exact = Fraction(x) / 9
        for a, b in zip(lo, hi):
            assert Fraction(float(a)) <= exact <= Fraction(float(b))
            assert b - a <= 4 * np.spacing(abs(x) / 9)
    # ... and through a later layer, with coefficients of both signs over the pooled neurons
    net.dense(1, W, np.zeros(1, np.float32))
    o = make_oracle(net)
    o.analyze_box(np.array([1.0]), np.array([1.0]))
    lo, hi = o.get_bounds(2)
    assert lo[0] <= 0.0 <= hi[0] and hi[0] - lo[0] <= 4 * np.spacing(1 / 9)
    assert hi[0] > 0.0 and lo[0] < 0.0       # 1/9 - 1/9 with outward-rounded ends is a proper interval around 0
