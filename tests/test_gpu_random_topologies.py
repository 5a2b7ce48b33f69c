"""GPU parity on randomly drawn small topologies: convolutions with random kernel sizes, strides and paddings
(rectangular too), residual blocks with identity and strided 1x1 shortcuts, dense layers with and without a ReLU
in between, odd channel counts.  Every interval is compared with the oracle's and with sampled outputs, with and
without early termination.  Seeds are fixed: a failing case is reproducible by its seed."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box, forward_float32
from parity import (analysed_layers, check_samples_inside, compare_all, compare_layer, float_inference_layers, make_gpu,
                    make_oracle, oracle_with_gpu_ties)
from test_gpu_early_term import check_early

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def random_net(seed: int) -> wl.Net:
    rng = np.random.default_rng(seed)
    C, H, W = int(rng.integers(1, 5)), int(rng.integers(5, 14)), int(rng.integers(5, 14))
    net = wl.Net(f"random_{seed}", (C, H, W))

    def conv(src, co, kh, kw, sh, sw, ph, pw, scale=1.0):
        ci, h, w = net.shape_of(src)
        Wt = (rng.standard_normal((co, ci, kh, kw)) * np.sqrt(2.0 / (ci * kh * kw)) * scale).astype(np.float32)
        b = (rng.standard_normal(co) * 0.1).astype(np.float32)
        ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
        net.layers.append(dict(type="conv", src=src, W=Wt, b=b, stride=(sh, sw), pad=(ph, pw), shape=(co, ho, wo)))
        return len(net.layers)

    def dense(src, n_out):
        n_in = net.n_neurons(src)
        Wt = (rng.standard_normal((n_out, n_in)) * np.sqrt(2.0 / n_in)).astype(np.float32)
        b = (rng.standard_normal(n_out) * 0.1).astype(np.float32)
        return net.dense(src, Wt, b)

    cur = 0
    for _ in range(int(rng.integers(1, 4))):
        c, h, w = net.shape_of(cur)
        if min(h, w) < 3:
            break
        kind = rng.integers(0, 3)
        if kind < 2:                       # plain convolution + ReLU
            kh, kw = int(rng.integers(1, min(4, h) + 1)), int(rng.integers(1, min(4, w) + 1))
            sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
            ph, pw = int(rng.integers(0, kh)), int(rng.integers(0, kw))
            cur = net.relu(conv(cur, int(rng.integers(1, 10)), kh, kw, sh, sw, ph, pw))
        else:                              # residual block: conv-relu-conv + shortcut, sum, ReLU
            s = int(rng.integers(1, 3))
            co = c if s == 1 and rng.random() < 0.5 else int(rng.integers(1, 9))
            a = net.relu(conv(cur, co, 3, 3, s, s, 1, 1))
            a = conv(a, co, 3, 3, 1, 1, 1, 1, scale=0.3)
            sc = cur if (s == 1 and co == c) else conv(cur, co, 1, 1, s, s, 0, 0)
            cur = net.relu(net.add(a, sc))
    for _ in range(int(rng.integers(0, 3))):
        cur = dense(cur, int(rng.integers(3, 40)))
        if rng.random() < 0.8:             # sometimes two dense layers with nothing in between
            cur = net.relu(cur)
    dense(cur, int(rng.integers(2, 7)))
    net.eps = float(rng.choice([0.002, 0.01, 0.04]))
    return net


@pytest.mark.parametrize("seed", range(40))
def test_random_topology(seed):
    net = random_net(seed)
    c = np.random.default_rng(10_000 + seed).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, net.eps)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, c, net.eps)
    compare_all(net, g, o, what=net.name)
    lo0, hi0 = ball_box(c, net.eps)
    check_samples_inside(net, g, lo0, hi0, 300, np.random.default_rng(seed), what=net.name)
    g.set_early_termination(True)
    g.analyze(c, net.eps)
    check_early(net, g, c, net.eps, what=net.name + " early", samples=100, seed=seed)


@pytest.mark.parametrize("seed", range(0, 40, 2))
def test_random_topology_float_inference(seed):
    """Section 4.1, rounding of the inference: same comparison in float32-inference mode, plus float32 evaluations of
    the network in several summation orders at corners of the box."""
    net = random_net(seed)
    rng = np.random.default_rng(20_000 + seed)
    c = np.random.default_rng(10_000 + seed).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_float_inference(True)
    if seed % 4 == 2:
        g.set_early_termination(True)
    g.analyze(c, net.eps)
    layers = sorted(set(analysed_layers(net)) | set(float_inference_layers(net)))
    if seed % 4 == 0:
        o = make_oracle(net)
        o.set_float_inference(True)
        oracle_with_gpu_ties(net, o, g, c, net.eps, extra_layers=float_inference_layers(net))
        for lid in layers:
            olo, ohi = o.get_bounds(lid)
            glo, ghi = g.get_bounds_f64(lid)
            compare_layer(glo, ghi, olo, ohi, f"{net.name} layer {lid}")
    lo0, hi0 = ball_box(c, net.eps)
    for k in range(3):
        x = c if k == 0 else np.clip(c.astype(np.float64) + net.eps * 0.999 * rng.choice([-1.0, 1.0], c.size), lo0, hi0).astype(np.float32)
        for order in ("forward", "random", "descending", "pairwise"):
            vals = forward_float32(net, x, order, rng)
            for lid in layers:
                glo, ghi = g.get_bounds_f64(lid)
                v = vals[lid].astype(np.float64)
                assert np.all(v >= glo) and np.all(v <= ghi), (net.name, order, lid)
