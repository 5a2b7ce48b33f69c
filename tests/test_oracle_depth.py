"""Pins of the oracle's handling of interval-coefficient WIDTHS on deep networks, and of the rounding direction of
interval x scalar products, against things that are not the oracle.  No GPU needed.

Section 4.1 of the paper keeps every coefficient of an expression as an interval to the end of the
back-substitution.  The oracle's default instead re-centres the interval coefficients before each substitution and
pays their width, times the largest magnitude of the neuron, into the constant.  Which of the two is "the value
DeepPoly defines" on a deep network is settled here by a third party: the matrix-form NumPy DeepPoly of
helpers.py (round to nearest float64, no intervals at all), given the same lower-line choices."""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from helpers import np_deeppoly
from oracle import OracleNet


def make_oracle(net):
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    return o


def analysed_layers(net):
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    return [i for i, L in enumerate(net.layers, start=1)
            if L["type"] == "relu" or i in feeds or i == len(net.layers)]


def deep_fc():
    return wl.fc_net("deep_fc", [64] * 24, n_in=16, n_out=4, seed=2), 0.01


def deep_resnet():
    net = wl.scaled_resnet(8, 16)        # depth and topology of the 34-layer residual configuration, channels / 8
    return net, net.eps


@pytest.mark.parametrize("maker", [deep_fc, deep_resnet])
def test_deep_networks_recentred_oracle_is_deeppoly_and_the_literal_scheme_is_the_outlier(maker):
    net, eps = maker()
    c = np.random.default_rng(3).random(net.n_in).astype(np.float32)
    a = make_oracle(net)
    a.analyze(c, eps)
    lam = {i: a.get_relaxation(i)[2] for i, L in enumerate(net.layers, start=1) if L["type"] == "relu"}
    lo0, hi0 = a.get_bounds(0)
    ref = np_deeppoly(net, lo0, hi0, lam_override=lam)
    # (1) every interval of every analysed layer of the default (re-centred) oracle is the plain float64 DeepPoly
    # value to 1e-9, and contains it up to rounding noise: outward rounding and the width slack cost nothing visible
    n_unstable = 0
    for lid in analysed_layers(net):
        (l, u), (rl, ru) = a.get_bounds(lid), ref[lid]
        assert np.max(np.abs(l - rl) / (1 + np.abs(rl))) < 1e-9, lid
        assert np.max(np.abs(u - ru) / (1 + np.abs(ru))) < 1e-9, lid
        assert np.all(l <= rl + 1e-11 * (1 + np.abs(rl))) and np.all(u >= ru - 1e-11 * (1 + np.abs(ru))), lid
        n_unstable += int(np.sum((l < 0) & (u > 0)))
    assert n_unstable > 50                   # (counted on the inputs of the ReLU layers: ReLU outputs never have l < 0)
    # (2) the literal scheme, given the very same intervals of all earlier layers (hence the same relaxations), is
    # never tighter than that value and drifts away from it with depth
    b = make_oracle(net)
    b.set_collapse(False)
    b.set_ball(c, eps)
    drift = []
    for lid in range(1, b.num_layers):
        if net.layers[lid - 1]["type"] == "relu":
            b.analyze_layer(lid)
            continue
        if lid not in analysed_layers(net):
            continue
        la, ua = a.get_bounds(lid)
        lb, ub = b.bound_rows(lid, np.arange(la.size, dtype=np.int32))
        rl, ru = ref[lid]
        assert np.all(lb <= rl + 1e-11 * (1 + np.abs(rl))) and np.all(ub >= ru - 1e-11 * (1 + np.abs(ru))), lid
        drift.append(max(np.max((rl - lb) / (1 + np.abs(rl))), np.max((ub - ru) / (1 + np.abs(ru)))))
        b.set_bounds(lid, la, ua)
    assert drift[0] < 1e-12                  # the first layers agree to rounding noise
    assert max(drift[-4:]) > 1e-4, drift[-4:]   # at the deep end the literal widths are 5 orders above the 1e-9 agreement


def _exact_affine_chain(Ws, bs, x):
    v = [Fraction(float(t)) for t in x]
    for W, b in zip(Ws, bs):
        v = [sum(Fraction(float(W[i, j])) * v[j] for j in range(W.shape[1])) + Fraction(float(b[i]))
             for i in range(W.shape[0])]
    return v


@pytest.mark.parametrize("collapse", [True, False])
def test_interval_coefficient_times_scalar_of_either_sign_is_rounded_outward(collapse):
    """Chains of four dense layers without ReLU on a point box: the coefficients of the last layer's rows are
    intervals after the second product (the product of two float32 values is still exact in float64, that of three
    is not) and are then multiplied by weights of both signs.  The exact output is a rational number; the oracle's interval must contain it and be only a few units
    in the last place wide.  A wrong end or a wrong rounding direction in the product of an interval with a
    negative (or a positive) scalar puts the exact value outside in some of the trials."""
    rng = np.random.default_rng(11)
    special = np.array([-1 / 3, -1 / 7, 1 / 3, 1 / 7, -1 / 11, 1 / 13], np.float32)
    n_strict = 0
    for trial in range(120):
        # network x -> W1 -> W2 -> W3 -> W4.  A row of the last layer starts as a row of W4 (points), becomes W4*W3
        # (still points), W4*W3*W2 (intervals) and is then multiplied by the entries of W1: all negative in the first
        # half of the trials
        W1 = rng.choice(special, (3, 3))
        if trial < 60:
            W1 = -np.abs(W1)
        net_W = [W1.astype(np.float32), rng.choice(special, (3, 3)), rng.choice(special, (3, 3)), rng.choice(special, (2, 3))]
        bs = [rng.choice(special, W.shape[0]).astype(np.float32) for W in net_W]
        o = OracleNet(3, 1, 1)
        src = 0
        for W, b in zip(net_W, bs):
            src = o.add_dense(src, W, b)
        o.set_collapse(collapse)
        x = rng.choice(np.array([1 / 3, 1 / 5, 1 / 7, 0.3], np.float64), 3)
        o.analyze_box(x, x)
        lo, hi = o.get_bounds(src)
        exact = _exact_affine_chain(net_W, bs, x)
        mag = np.abs(x)
        for W in net_W:
            mag = np.abs(W.astype(np.float64)) @ mag + 1
        for i in range(len(exact)):
            assert Fraction(float(lo[i])) <= exact[i] <= Fraction(float(hi[i])), (trial, i, lo[i], float(exact[i]), hi[i])
            assert hi[i] - lo[i] <= 64 * 2.0 ** -53 * mag[i], (trial, i)
            n_strict += hi[i] > lo[i]
    assert n_strict > 100           # the rounding is visible: the ends differ although the box is a point


@pytest.mark.parametrize("collapse", [True, False])
def test_scalar_chain_isolates_the_rounding_of_one_product(collapse):
    """x -> w1*x -> w2*(.) -> w3*(.) -> w4*(.) with one neuron per layer, zero biases and the point box x = 1: the
    row of the last layer is w4 (a point), then w4*w3 (still a point: two float32 values multiply exactly in
    float64), then w4*w3*w2 (an interval one unit in the last place wide, since that product is not representable),
    then that interval times w1 < 0; every other operation (products with 1, sums with 0) is exact.
    So the reported interval is exactly what `interval x negative scalar` returns: it must contain the rational
    w4*w3*w2*w1 and be at most a few units in the last place wide.  Swapped ends, inward rounding or a lost width all
    show here because no other outward rounding can hide them."""
    w1s = np.array([-(1 - 2.0 ** -24), -1 / 3, -1 / 7, -0.3, -1 / 11, -(1 + 2.0 ** -23)], np.float32)
    others = np.array([1 / 3, 1 / 7, -1 / 3, 0.3, 1 / 11, -1 / 13, 0.7], np.float32)
    one = np.ones(1)
    widths = []
    w4 = np.float32(1 / 7)
    for w1 in w1s:
        for w2 in others:
            for w3 in others:
                o = OracleNet(1, 1, 1)
                src = 0
                for w in (w1, w2, w3, w4):
                    src = o.add_dense(src, np.array([[w]], np.float32), None)
                o.set_collapse(collapse)
                o.analyze_box(one, one)
                lo, hi = o.get_bounds(src)
                exact = Fraction(float(w1)) * Fraction(float(w2)) * Fraction(float(w3)) * Fraction(float(w4))
                assert Fraction(float(lo[0])) <= exact <= Fraction(float(hi[0])), (w1, w2, w3, lo[0], float(exact), hi[0])
                ulp = np.spacing(abs(float(exact)))
                assert hi[0] - lo[0] <= 6 * ulp, (w1, w2, w3)     # one ulp of width times |w1| <= 2, and one rounding per end
                widths.append((hi[0] - lo[0]) / ulp)
    assert np.mean(np.array(widths) > 0) > 0.9      # the products are not representable: the ends differ
