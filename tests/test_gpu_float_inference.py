"""GPU parity of the float32-inference mode (paper Section 4.1, last paragraph): the library's bounds against the
oracle's in the same mode, and against float32 evaluations of the networks in several summation orders."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import FLOAT32_ORDERS, ball_box, forward_float32
from parity import (analysed_layers, compare_all, compare_layer, float_inference_layers, make_gpu, make_oracle,
                    oracle_with_gpu_ties)
from test_gpu_parity import mid_resnet, odd_fc, pad0_conv, quad_fc, rect_conv, tiny_conv, tiny_fc, tiny_resnet
from test_oracle_float_inference import rounded_sum_net

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def pair(net, center, eps, early=False):
    g = make_gpu(net)
    g.set_float_inference(True)
    if early:
        g.set_early_termination(True)
    g.analyze(center, eps)
    o = make_oracle(net)
    o.set_float_inference(True)
    oracle_with_gpu_ties(net, o, g, center, eps, extra_layers=float_inference_layers(net))
    return g, o


def all_bounded(net):
    return sorted(set(analysed_layers(net)) | set(float_inference_layers(net)))


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (odd_fc, 0.05), (quad_fc, 0.03), (tiny_conv, 0.05), (pad0_conv, 0.03),
                                       (tiny_resnet, 0.02), (mid_resnet, 0.01), (rect_conv, 0.04)])
def test_small_networks_match_the_oracle_in_the_same_mode(maker, eps):
    net = maker(1)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    g, o = pair(net, c, eps)
    for lid in all_bounded(net):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = g.get_bounds_f64(lid)
        compare_layer(glo, ghi, olo, ohi, f"{net.name} layer {lid}")
    # the mode only ever widens
    plain = make_gpu(net)
    plain.analyze(c, eps)
    for lid in analysed_layers(net):
        a, b = plain.get_bounds_f64(lid)
        glo, ghi = g.get_bounds_f64(lid)
        assert np.all(glo <= a) and np.all(ghi >= b)


@pytest.mark.parametrize("maker", [tiny_fc, quad_fc, tiny_conv, pad0_conv, tiny_resnet, mid_resnet, rect_conv])
@pytest.mark.parametrize("early", [False, True])
def test_point_box_widths_and_float32_orders(maker, early):
    """On a point box the intervals are nothing but accumulated inference error (plus the library's own float64 and
    storage slack): float32 evaluations in every order lie inside, the real-valued analysis does not contain them, and
    the widths agree with the oracle's."""
    net = maker(2)
    rng = np.random.default_rng(9)
    c = rng.random(net.n_in).astype(np.float32)
    g, o = pair(net, c, 0.0, early=early)
    plain = make_gpu(net)
    plain.analyze(c, 0.0)
    escaped = 0
    for order in FLOAT32_ORDERS:
        vals = forward_float32(net, c, order, rng)
        for lid in all_bounded(net):
            glo, ghi = g.get_bounds_f64(lid)
            v = vals[lid].astype(np.float64)
            assert np.all(v >= glo) and np.all(v <= ghi), (net.name, order, lid)
            if lid in analysed_layers(net):
                a, b = plain.get_bounds_f64(lid)
                escaped += int(np.any(v < a) or np.any(v > b))
    assert escaped > 0
    if not early:
        for lid in all_bounded(net):
            if net.layers[lid - 1]["type"] == "relu":
                continue
            olo, ohi = o.get_bounds(lid)
            glo, ghi = g.get_bounds_f64(lid)
            wo, wg = ohi - olo, ghi - glo
            assert np.all(wg >= wo * (1 - 1e-6))
            # the library adds its float32 coefficient storage slack (about 2^-24 per coefficient and layer) on top
            assert np.all(wg <= 3.0 * wo + 1e-30), (net.name, lid, float(np.max(wg / wo)))


def test_rounded_sum_hand_example():
    net, s = rounded_sum_net()
    x = np.array([1.0, 1.0], np.float32)
    g = make_gpu(net)
    g.set_float_inference(True)
    g.analyze(x, 0.0)
    exact = 1.0 + 2.0 ** -25
    lo, hi = g.get_bounds_f64(s)
    assert lo[0] <= 1.0 and hi[0] >= exact
    # (the library stores the coefficient 1 + 2^-25 over x_0 as the float32 1.0 and charges one 2^-24 for it)
    assert lo[0] >= exact - 2.6 * 2.0 ** -24 * exact
    ylo, yhi = g.get_bounds_f64(net.out_layer)
    assert ylo[0] <= 1.0 and yhi[0] >= exact
    assert ylo[0] >= exact - 5.6 * 2.0 ** -24 * exact
    o = make_oracle(net)
    o.set_float_inference(True)
    o.set_box(x.astype(np.float64), x.astype(np.float64))
    o.analyze()
    for lid in (s, net.out_layer):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = g.get_bounds_f64(lid)
        assert np.all(glo <= olo) and np.all(ghi >= ohi)
        assert np.all(ghi - glo <= 3.0 * (ohi - olo))


def test_batched_equals_single_and_certify():
    net = wl.config(0)
    centers = np.stack([net.center(j) for j in range(3)])
    g = make_gpu(net)
    g.set_float_inference(True)
    g.analyze_batch(centers, net.eps)
    batched = {l: [g.get_bounds_f64(l, b) for b in range(3)] for l in analysed_layers(net)}
    labels = np.array([1, 2, 3], np.int32)
    _, mb = g.certify_batch(labels)
    o = make_oracle(net)
    o.set_float_inference(True)
    for b in range(3):
        g.analyze(centers[b], net.eps)
        for l in analysed_layers(net):
            lo, hi = g.get_bounds_f64(l)
            assert np.array_equal(lo, batched[l][b][0]) and np.array_equal(hi, batched[l][b][1])
        _, m1 = g.certify(int(labels[b]))
        assert np.array_equal(m1, mb[b])
        oracle_with_gpu_ties(net, o, g, centers[b], net.eps)
        compare_all(net, g, o, what=f"fc6x100 input {b}")
        _, mo = o.certify(int(labels[b]))
        compare_layer(m1, m1, mo, m1, f"fc6x100 input {b} margins")
        # the float32 outputs respect the margins
        rng = np.random.default_rng(b)
        lo0, hi0 = ball_box(centers[b], net.eps)
        others = [j for j in range(10) if j != labels[b]]
        for order in ("forward", "random", "pairwise"):
            x = np.clip(centers[b].astype(np.float64) + net.eps * 0.999 * rng.choice([-1.0, 1.0], net.n_in), lo0, hi0).astype(np.float32)
            y = forward_float32(net, x, order, rng)[net.out_layer].astype(np.float64)
            assert np.all(y[labels[b]] - y[others] >= m1.astype(np.float64))


def test_switching_the_mode_off_restores_the_plain_bounds():
    net = tiny_resnet(1)
    c = np.random.default_rng(3).random(net.n_in).astype(np.float32)
    ref = make_gpu(net)
    ref.analyze(c, 0.02)
    g = make_gpu(net)
    g.set_float_inference(True)
    g.analyze(c, 0.02)
    g.set_float_inference(False)
    g.analyze(c, 0.02)
    for lid in analysed_layers(net):
        a, b = ref.get_bounds_f64(lid)
        lo, hi = g.get_bounds_f64(lid)
        assert np.array_equal(a, lo) and np.array_equal(b, hi)
