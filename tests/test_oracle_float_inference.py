"""Pins of the oracle's float32-inference mode (paper Section 4.1, last paragraph: the analysis also has to cover
the rounding of the inference itself, whatever the order of its sums).

What fixes the mode from outside the oracle:
  * the classical error bound of a float32 sum of products, retyped here with exact rational arithmetic;
  * float32 evaluations of the networks in several summation orders (NumPy float32, written here), which the
    bounds must contain - and which the bounds of the real-valued analysis do NOT contain on a point box;
  * a hand-made neuron whose float32 value differs from the exact one by a known amount.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from helpers import FLOAT32_ORDERS, ball_box, forward, forward_float32
from oracle import OracleNet

U = Fraction(1, 2 ** 24)


def build(net, float_inference=True, early=False, request=()):
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    for lid in request:
        o.request_bounds(lid)
    o.set_float_inference(float_inference)
    if early:
        o.set_early_termination(True)
    return o


def gamma(k):
    return k * U / (1 - k * U)


def bounded_layers(net):
    out = []
    for i, L in enumerate(net.layers, start=1):
        feeds_relu = any(M["type"] == "relu" and M["src"] == i for M in net.layers)
        if L["type"] == "relu" or feeds_relu or i == net.out_layer:
            out.append(i)
    return out


def tiny_fc(seed=0):
    return wl.fc_net("tiny_fc", [12, 10, 8], n_in=9, n_out=4, seed=seed)


def tiny_conv(seed=0):
    return wl.conv_net("tiny_conv", (2, 6, 6), [(3, 3, 1, 1), (4, 3, 2, 1)], [10], n_out=3, seed=seed)


def tiny_resnet(seed=0):
    return wl.resnet("tiny_res", (2, 6, 6), channels=(3, 4), blocks=(1, 1), n_out=3, seed=seed)


NETS = [tiny_fc, tiny_conv, tiny_resnet]


def test_single_neuron_error_constant_is_the_classical_bound():
    # one dense neuron of K = 3 inputs on a point box: eta = gamma(K+1)*(sum|w||x| + |b|) + (K+1)*2^-149, and the
    # bounds are the exact value -/+ eta
    W = np.array([[0.75, -1.5, 0.3125]], np.float32)
    b = np.array([-0.625], np.float32)
    x = np.array([0.5, 0.25, 0.875], np.float32)
    net = wl.Net("one", (3, 1, 1))
    net.dense(0, W, b)
    o = build(net)
    o.set_box(x.astype(np.float64), x.astype(np.float64))
    o.analyze()
    mag = sum(abs(Fraction(float(w))) * abs(Fraction(float(v))) for w, v in zip(W[0], x)) + abs(Fraction(float(b[0])))
    eta = gamma(4) * mag + 4 * Fraction(1, 2 ** 149)
    exact = sum(Fraction(float(w)) * Fraction(float(v)) for w, v in zip(W[0], x)) + Fraction(float(b[0]))
    got = o.get_inference_error(1)[0]
    assert Fraction(got) >= eta and Fraction(got) <= eta * (1 + Fraction(1, 2 ** 40))
    lo, hi = o.get_bounds(1)
    assert Fraction(lo[0]) <= exact - eta and Fraction(hi[0]) >= exact + eta
    assert Fraction(hi[0]) - Fraction(lo[0]) <= 2 * eta * (1 + Fraction(1, 2 ** 30))


def test_bias_term_of_the_error_constant():
    # w*x = 2^-25 vanishes next to b = 1 in float32 (the exact value 1 + 2^-25 lies below the midpoint 1 + 2^-24):
    # the float32 neuron is 1.  An error constant without the |b| term (2*u*2^-25) would not reach down to it.
    W = np.array([[1.0]], np.float32)
    b = np.array([1.0], np.float32)
    x = np.array([2.0 ** -25], np.float32)
    net = wl.Net("bias", (1, 1, 1))
    net.dense(0, W, b)
    assert np.float32(np.float32(W[0, 0] * x[0]) + b[0]) == np.float32(1.0)
    o = build(net)
    o.set_box(x.astype(np.float64), x.astype(np.float64))
    o.analyze()
    lo, hi = o.get_bounds(1)
    assert lo[0] <= 1.0 < 1.0 + 2.0 ** -25 <= hi[0]
    off = build(net, float_inference=False)
    off.set_box(x.astype(np.float64), x.astype(np.float64))
    off.analyze()
    lo0, hi0 = off.get_bounds(1)
    assert lo0[0] > 1.0            # the real-valued analysis excludes the float32 result


def test_mode_off_is_the_plain_analysis_and_on_contains_it():
    for maker in NETS:
        net = maker()
        lo0, hi0 = ball_box(net.center(0), 0.01)
        plain = OracleNet(*net.input_shape)
        wl.build_into(net, plain)
        plain.set_box(lo0, hi0)
        plain.analyze()
        off = build(net, float_inference=False)
        off.set_box(lo0, hi0)
        off.analyze()
        on = build(net)
        on.set_box(lo0, hi0)
        on.analyze()
        for lid in bounded_layers(net):
            a, b = plain.get_bounds(lid)
            c, d = off.get_bounds(lid)
            assert np.array_equal(a, c) and np.array_equal(b, d)
            e, f = on.get_bounds(lid)
            assert np.all(e <= a) and np.all(f >= b)
            # ... and not by much: the error constants are of the order fan-in * 2^-24 of the activations
            scale = 1.0 + max(np.abs(a).max(), np.abs(b).max())
            assert (a - e).max() <= 1e-3 * scale and (f - b).max() <= 1e-3 * scale
            assert (f - b).max() > 0 or net.layers[lid - 1]["type"] == "relu"


@pytest.mark.parametrize("maker", NETS)
@pytest.mark.parametrize("eps", [0.0, 0.02])
def test_float32_evaluations_in_any_order_are_contained(maker, eps):
    rng = np.random.default_rng(7)
    escaped_plain = 0
    for seed in range(3):
        net = maker(seed)
        center = net.center(seed)
        lo0, hi0 = ball_box(center, eps)
        on = build(net)
        on.set_box(lo0, hi0)
        on.analyze()
        off = build(net, float_inference=False)
        off.set_box(lo0, hi0)
        off.analyze()
        layers = bounded_layers(net) + [i for i, L in enumerate(net.layers, start=1) if L["type"] == "add"]
        pts = [center] if eps == 0.0 else [center] + [
            np.clip(center.astype(np.float64) + eps * 0.999 * rng.choice([-1.0, 1.0], center.size), lo0, hi0).astype(np.float32)
            for _ in range(4)]
        for x in pts:
            assert np.all(x >= lo0) and np.all(x <= hi0)
            for order in FLOAT32_ORDERS:
                vals = forward_float32(net, x, order, rng)
                for lid in set(layers):
                    lo, hi = on.get_bounds(lid)
                    v = vals[lid].astype(np.float64)
                    assert np.all(v >= lo) and np.all(v <= hi), (net.name, seed, order, lid)
                    if lid in bounded_layers(net):
                        a, b = off.get_bounds(lid)
                        escaped_plain += int(np.any(v < a) or np.any(v > b))
    if eps == 0.0:
        # on a point box the real-valued analysis is exact up to float64 rounding, and float32 results fall outside it
        assert escaped_plain > 0


def test_sum_layer_interval_is_the_rounded_sum():
    # a residual sum in float32 is one rounded addition: on a point box its interval must contain that float32 value,
    # and be no wider than the exact sum's interval moved outward by 2^-24 relative
    net = tiny_resnet(3)
    x = net.center(1)
    rng = np.random.default_rng(0)
    on = build(net)
    on.set_box(x.astype(np.float64), x.astype(np.float64))
    on.analyze()
    vals = forward_float32(net, x, "forward", rng)
    exact = forward(net, x[None, :].astype(np.float64))
    for lid, L in enumerate(net.layers, start=1):
        if L["type"] != "add":
            continue
        lo, hi = on.get_bounds(lid)
        v = vals[lid].astype(np.float64)
        assert np.all(lo <= v) and np.all(v <= hi)
        eta = on.get_inference_error(lid)
        assert np.all(eta >= 2.0 ** -24 * np.maximum(np.abs(lo), np.abs(hi)) * (1 - 1e-12))
        assert np.all(eta <= 2.0 ** -24 * np.maximum(np.abs(lo), np.abs(hi)) * (1 + 1e-12))
        # the real-valued sum of the real-valued network is inside as well
        assert np.all(lo <= exact[lid][0]) and np.all(exact[lid][0] <= hi)


@pytest.mark.parametrize("maker", NETS)
def test_with_early_termination(maker):
    rng = np.random.default_rng(11)
    net = maker(2)
    center = net.center(0)
    eps = 0.003
    lo0, hi0 = ball_box(center, eps)
    on = build(net, early=True)
    on.set_box(lo0, hi0)
    on.analyze()
    full = build(net)
    full.set_box(lo0, hi0)
    full.analyze()
    pts = [center] + [np.clip(center.astype(np.float64) + eps * 0.999 * rng.choice([-1.0, 1.0], center.size), lo0, hi0).astype(np.float32)
                      for _ in range(3)]
    for lid in bounded_layers(net):
        lo, hi = on.get_bounds(lid)
        flo, fhi = full.get_bounds(lid)
        if net.layers[lid - 1]["type"] != "relu":
            ilo, ihi = on.get_interval_image(lid)
            assert np.all(ilo <= lo) and np.all(hi <= ihi)
        # stopped neurons keep looser bounds with the same sign; the others match the full analysis
        assert np.all(lo <= flo + 1e-9 * (1 + np.abs(flo))) and np.all(hi >= fhi - 1e-9 * (1 + np.abs(fhi)))
        for x in pts:
            for order in ("forward", "random", "descending"):
                v = forward_float32(net, x, order, rng)[lid].astype(np.float64)
                assert np.all(v >= lo) and np.all(v <= hi), (net.name, order, lid)


def test_certification_margins_cover_float32_outputs():
    rng = np.random.default_rng(5)
    net = tiny_fc(4)
    center = net.center(2)
    eps = 0.002
    lo0, hi0 = ball_box(center, eps)
    on = build(net)
    on.set_box(lo0, hi0)
    on.analyze()
    y = forward_float32(net, center, "forward", rng)[net.out_layer]
    label = int(np.argmax(y))
    _, margins = on.certify(label)
    others = [j for j in range(y.size) if j != label]
    for _ in range(5):
        x = np.clip(center.astype(np.float64) + eps * 0.999 * rng.choice([-1.0, 1.0], center.size), lo0, hi0).astype(np.float32)
        for order in FLOAT32_ORDERS:
            out = forward_float32(net, x, order, rng)[net.out_layer].astype(np.float64)
            assert np.all(out[label] - out[others] >= margins)


def rounded_sum_net():
    """x -> add(E relu(D x), x) -> first component, with D = 2^-25 * identity and E = identity.  At x = (1, 1) every
    affine neuron is exact in float32 (one non-zero product, zero bias), the residual sum 1 + 2^-25 is not: it rounds
    to 1."""
    net = wl.Net("rounded_sum", (2, 1, 1))
    d = net.dense(0, np.array([[2.0 ** -25, 0.0], [0.0, 2.0 ** -25]], np.float32), np.zeros(2, np.float32))
    r = net.relu(d)
    e = net.dense(r, np.eye(2, dtype=np.float32), np.zeros(2, np.float32))
    s = net.add(e, 0)
    net.dense(s, np.array([[1.0, 0.0]], np.float32), np.zeros(1, np.float32))
    return net, s


def test_rounded_sum_hand_example():
    net, s = rounded_sum_net()
    x = np.array([1.0, 1.0], np.float32)
    vals = forward_float32(net, x, "forward", np.random.default_rng(0))
    assert vals[s][0] == np.float32(1.0) and vals[net.out_layer][0] == np.float32(1.0)
    exact = 1.0 + 2.0 ** -25
    on = build(net)
    on.set_box(x.astype(np.float64), x.astype(np.float64))
    on.analyze()
    # the sum layer's own interval: the exact sum moved outward by one float32 rounding (and the summands' tiny errors)
    lo, hi = on.get_bounds(s)
    assert lo[0] <= 1.0 and hi[0] >= exact
    assert lo[0] >= exact - 2.0 ** -24 * exact * (1 + 1e-6) and hi[0] <= exact + 2.0 ** -24 * exact * (1 + 1e-6)
    # an expression substituted THROUGH the sum layer is charged the same rounding
    ylo, yhi = on.get_bounds(net.out_layer)
    assert ylo[0] <= 1.0 and yhi[0] >= exact
    # (one rounding of the sum, gamma(3) for the output neuron of two inputs: 4 * 2^-24 relative in all)
    assert ylo[0] >= exact - 4.001 * 2.0 ** -24 * exact and yhi[0] <= exact + 4.001 * 2.0 ** -24 * exact
    # ... on top of the output neuron's own error: both constants (each pinned above) add up along the path, so the
    # bound may not be tighter than their sum allows
    eta_s, eta_y = on.get_inference_error(s)[0], on.get_inference_error(net.out_layer)[0]
    assert ylo[0] <= exact - (eta_y + eta_s) * (1 - 1e-9) and yhi[0] >= exact + (eta_y + eta_s) * (1 - 1e-9)
    # the real-valued analysis excludes the float32 result
    off = build(net, float_inference=False, request=[s])
    off.set_box(x.astype(np.float64), x.astype(np.float64))
    off.analyze()
    assert off.get_bounds(s)[0][0] > 1.0 and off.get_bounds(net.out_layer)[0][0] > 1.0
