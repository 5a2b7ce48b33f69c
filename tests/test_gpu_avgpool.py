"""GPU parity of the average-pooling layer (an affine layer without a stored filter; Section 2, affine transformer):
the HIP library against the oracle on LeNet-like networks, a residual net with a pooling head and a pooled shortcut,
and randomly drawn topologies; plain, with early termination, in float32-inference mode, batched and chunked."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box, forward, forward_float32
from parity import (STRICT_CONTAIN_TOL, analysed_layers, check_samples_inside, compare_all, compare_layer,
                    float_inference_layers, make_gpu, make_oracle, oracle_with_gpu_relaxation, oracle_with_gpu_ties)
from test_gpu_early_term import check_early

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def lenet_like(seed=0):
    """conv-ReLU, 2x2 average, conv-ReLU, overlapping 3x3 stride-2 average with padding, dense-ReLU, dense."""
    return wl.pool_net("tiny_lenet", (2, 10, 10), [("conv", 3, 3, 1, 1), ("pool", 2, 2, 0), ("conv", 4, 2, 1, 0),
                                                   ("pool", 3, 2, 1)], [8], n_out=3, seed=seed)


def lenet5(seed=0):
    """The classic shape: 1x28x28, conv5-ReLU-pool2-conv5-ReLU-pool2, dense 120, 84, 10 (6 and 16 channels: one vector
    path with 4-channel groups, one without)."""
    return wl.pool_net("lenet5", (1, 28, 28), [("conv", 6, 5, 1, 2), ("pool", 2, 2, 0), ("conv", 16, 5, 1, 0), ("pool", 2, 2, 0)],
                       [120, 84], n_out=10, seed=seed)


def pooled_resnet(seed=0):
    """Residual net whose head is global average pooling + dense, as a layer of its own."""
    return wl.resnet("pool_res", (3, 16, 16), channels=(8, 16), blocks=(2, 2), n_out=10, seed=seed, pool_head=True)


def pooled_shortcut(seed=0):
    """A down-sampling block whose shortcut is a 2x2 average followed by a 1x1 convolution (the two branches reach the
    block's input with the same accumulated stride and different windows), then a pooling layer that feeds a ReLU."""
    rng = np.random.default_rng(seed)
    net = wl.Net("pool_shortcut", (3, 12, 12))

    def cv(src, co, k, scale=1.0):
        ci = net.shape_of(src)[0]
        return ((rng.standard_normal((co, ci, k, k)) * np.sqrt(2.0 / (ci * k * k)) * scale).astype(np.float32),
                (rng.standard_normal(co) * 0.1).astype(np.float32))
    x = net.relu(net.conv(0, *cv(0, 6, 3), 1, 1))
    h = net.relu(net.conv(x, *cv(x, 8, 3), 2, 1))
    h = net.conv(h, *cv(h, 8, 3, 0.3), 1, 1)
    sp = net.avgpool(x, 2)
    sc = net.conv(sp, *cv(sp, 8, 1), 1, 0)
    y = net.relu(net.add(h, sc))
    z = net.relu(net.avgpool(y, 3, 1, 1))                 # a pooling layer whose own rows are bounded and may stop early
    W = (rng.standard_normal((5, net.n_neurons(z))) * 0.1).astype(np.float32)
    net.dense(z, W, np.zeros(5, np.float32))
    return net


def run_pair(net, c, eps):
    g = make_gpu(net)
    g.analyze(c, eps)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, c, eps)
    return g, o


@pytest.mark.parametrize("maker,eps", [(lenet_like, 0.03), (lenet5, 0.01), (pooled_resnet, 0.01), (pooled_shortcut, 0.01)])
def test_pooled_networks_match_oracle_and_contain_samples(maker, eps):
    net = maker(1)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    g, o = run_pair(net, c, eps)
    worst = compare_all(net, g, o, what=net.name)
    lo0, hi0 = ball_box(c, eps)
    check_samples_inside(net, g, lo0, hi0, 5_000, rng, what=net.name)
    n_uns = sum(int(np.sum((o.get_bounds(l)[0] < 0) & (o.get_bounds(l)[1] > 0))) for l in analysed_layers(net))
    assert n_uns > 0
    print(net.name, "worst looseness / allowed =", worst)
    oracle_with_gpu_relaxation(net, o, g, c, eps)
    compare_all(net, g, o, what=net.name + " (GPU slopes)", contain_tol=STRICT_CONTAIN_TOL)
    # certification rows cross the pooling layers too
    y = forward(net, c[None].astype(np.float64))[net.out_layer][0]
    label = int(np.argmax(y))
    ok_g, m_g = g.certify(label)
    ok_o, m_o = o.certify(label)
    assert np.all(m_g <= m_o + STRICT_CONTAIN_TOL * (1 + np.abs(m_o))) and np.all(m_o - m_g <= 1e-3 * (1 + np.abs(m_o)))


def test_pooling_head_equals_folded_head():
    """Global average + dense against the same network with the two folded into one dense layer (8x8 positions: the
    folded float32 weights are exact): the same function, so the same bounds up to the rounding slack."""
    kw = dict(input_shape=(3, 16, 16), channels=(8, 16), blocks=(2, 2), n_out=10, seed=3)
    folded, pooled = wl.resnet("f", **kw), wl.resnet("p", pool_head=True, **kw)
    c = np.random.default_rng(2).random(folded.n_in).astype(np.float32)
    a, b = make_gpu(pooled), make_gpu(folded)
    a.analyze(c, 0.01)
    b.analyze(c, 0.01)
    (alo, ahi), (blo, bhi) = a.get_bounds_f64(pooled.out_layer), b.get_bounds_f64(folded.out_layer)
    tol = 1e-6 * (1 + np.maximum(np.abs(blo), np.abs(bhi)))
    assert np.all(np.abs(alo - blo) <= tol) and np.all(np.abs(ahi - bhi) <= tol)


@pytest.mark.parametrize("maker,eps", [(lenet_like, 0.03), (lenet5, 0.01), (pooled_shortcut, 0.01)])
def test_pooled_networks_early_termination(maker, eps):
    net = maker(2)
    c = np.random.default_rng(6).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze(c, eps)
    check_early(net, g, c, eps, what=net.name + " early", samples=500, seed=1)


@pytest.mark.parametrize("maker,eps", [(lenet_like, 0.03), (lenet5, 0.005), (pooled_resnet, 0.005), (pooled_shortcut, 0.01)])
@pytest.mark.parametrize("early", [False, True])
def test_pooled_networks_float_inference(maker, eps, early):
    net = maker(3)
    rng = np.random.default_rng(7)
    c = rng.random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_float_inference(True)
    g.set_early_termination(early)
    g.analyze(c, eps)
    layers = sorted(set(analysed_layers(net)) | set(float_inference_layers(net)))
    if not early:
        o = make_oracle(net)
        o.set_float_inference(True)
        oracle_with_gpu_ties(net, o, g, c, eps, extra_layers=float_inference_layers(net))
        for lid in layers:
            olo, ohi = o.get_bounds(lid)
            glo, ghi = g.get_bounds_f64(lid)
            compare_layer(glo, ghi, olo, ohi, f"{net.name} layer {lid}")
    lo0, hi0 = ball_box(c, eps)
    for k in range(3):
        x = c if k == 0 else np.clip(c.astype(np.float64) + eps * 0.999 * rng.choice([-1.0, 1.0], c.size), lo0, hi0).astype(np.float32)
        for order in ("forward", "random", "descending", "pairwise"):
            vals = forward_float32(net, x, order, rng)
            for lid in layers:
                glo, ghi = g.get_bounds_f64(lid)
                v = vals[lid].astype(np.float64)
                assert np.all(v >= glo) and np.all(v <= ghi), (net.name, order, lid)


def test_batched_and_chunked_are_bitwise_equal():
    net = lenet5(4)
    g = make_gpu(net)
    centers = np.stack([np.random.default_rng(30 + j).random(net.n_in).astype(np.float32) for j in range(3)])
    g.analyze_batch(centers, 0.01)
    batched = {l: [g.get_bounds_f64(l, b) for b in range(3)] for l in analysed_layers(net)}
    for b in range(3):
        g.analyze(centers[b], 0.01)
        for l in analysed_layers(net):
            lo, hi = g.get_bounds_f64(l)
            assert np.array_equal(lo, batched[l][b][0]) and np.array_equal(hi, batched[l][b][1]), (b, l)
    mn, full = g.workspace_size(1)
    small = torch.empty(mn * 53 + 4096, dtype=torch.uint8, device="cuda")      # 53 rows at a time
    assert small.numel() < full
    g.set_workspace(small)
    g.analyze(centers[2], 0.01)
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l)
        assert np.array_equal(lo, batched[l][2][0]) and np.array_equal(hi, batched[l][2][1]), l


def random_pool_net(seed: int) -> wl.Net:
    """Convolutions (+ReLU) and average poolings with random rectangular windows, strides and paddings in random order:
    pooling after a ReLU, after a convolution, after another pooling, before a ReLU; odd channel counts."""
    rng = np.random.default_rng(seed)
    C, H, W = int(rng.integers(1, 6)), int(rng.integers(6, 15)), int(rng.integers(6, 15))
    net = wl.Net(f"random_pool_{seed}", (C, H, W))
    cur = 0
    n_pool = 0
    for step in range(int(rng.integers(2, 6))):
        c, h, w = net.shape_of(cur)
        if min(h, w) < 2:
            break
        kh, kw = int(rng.integers(1, min(4, h) + 1)), int(rng.integers(1, min(4, w) + 1))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, kh)), int(rng.integers(0, kw))
        ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
        if rng.random() < 0.5 or (step == 1 and n_pool == 0):
            if kh * kw == 1:
                kh = 2 if h >= 2 else 1
                kw = 2 if w >= 2 and kh == 1 else kw
                ph, pw = min(ph, kh - 1), min(pw, kw - 1)
                ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
            net.layers.append(dict(type="avgpool", src=cur, kernel=(kh, kw), stride=(sh, sw), pad=(ph, pw), shape=(c, ho, wo)))
            cur = len(net.layers)
            n_pool += 1
            if rng.random() < 0.3:
                cur = net.relu(cur)
        else:
            co = int(rng.integers(1, 10))
            Wt = (rng.standard_normal((co, c, kh, kw)) * np.sqrt(2.0 / (c * kh * kw))).astype(np.float32)
            b = (rng.standard_normal(co) * 0.1).astype(np.float32)
            net.layers.append(dict(type="conv", src=cur, W=Wt, b=b, stride=(sh, sw), pad=(ph, pw), shape=(co, ho, wo)))
            cur = len(net.layers)
            if rng.random() < 0.8:
                cur = net.relu(cur)
    for _ in range(int(rng.integers(0, 2))):
        n_in = net.n_neurons(cur)
        Wt = (rng.standard_normal((int(rng.integers(3, 30)), n_in)) * np.sqrt(2.0 / n_in)).astype(np.float32)
        cur = net.relu(net.dense(cur, Wt, (rng.standard_normal(Wt.shape[0]) * 0.1).astype(np.float32)))
    if rng.random() < 0.7 or net.layers[cur - 1]["type"] == "relu":
        n_in = net.n_neurons(cur)
        Wt = (rng.standard_normal((int(rng.integers(2, 7)), n_in)) * np.sqrt(2.0 / n_in)).astype(np.float32)
        net.dense(cur, Wt, (rng.standard_normal(Wt.shape[0]) * 0.1).astype(np.float32))
    net.eps = float(rng.choice([0.002, 0.01, 0.04]))
    return net


@pytest.mark.parametrize("seed", range(30))
def test_random_pooled_topology(seed):
    net = random_pool_net(seed)
    assert any(L["type"] == "avgpool" for L in net.layers)
    rng = np.random.default_rng(20_000 + seed)
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
    # float32-inference mode: against the oracle, and float32 evaluations at corners
    g.set_early_termination(seed % 3 == 0)
    g.set_float_inference(True)
    g.analyze(c, net.eps)
    layers = sorted(set(analysed_layers(net)) | set(float_inference_layers(net)))
    if seed % 3 != 0:
        o = make_oracle(net)
        o.set_float_inference(True)
        oracle_with_gpu_ties(net, o, g, c, net.eps, extra_layers=float_inference_layers(net))
        for lid in layers:
            olo, ohi = o.get_bounds(lid)
            glo, ghi = g.get_bounds_f64(lid)
            compare_layer(glo, ghi, olo, ohi, f"{net.name} layer {lid} (float inference)")
    for k in range(2):
        x = c if k == 0 else np.clip(c.astype(np.float64) + net.eps * 0.999 * rng.choice([-1.0, 1.0], c.size), lo0, hi0).astype(np.float32)
        for order in ("forward", "random", "pairwise"):
            vals = forward_float32(net, x, order, rng)
            for lid in layers:
                glo, ghi = g.get_bounds_f64(lid)
                v = vals[lid].astype(np.float64)
                assert np.all(v >= glo) and np.all(v <= ghi), (net.name, order, lid)


def test_pooling_as_the_last_layer_certify_forms_and_point_box():
    """A network that ENDS in a pooling layer: certification rows and linear forms start on the pooled outputs, and a
    point box (eps = 0) gives the forward value."""
    rng = np.random.default_rng(3)
    net = wl.Net("pool_last", (3, 8, 8))
    W = (rng.standard_normal((5, 3, 3, 3)) * 0.3).astype(np.float32)
    x = net.relu(net.conv(0, W, (rng.standard_normal(5) * 0.1).astype(np.float32), 1, 1))
    net.avgpool(x, 8)                                            # global average: 5 outputs
    c = rng.random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    o = make_oracle(net)
    g.analyze(c, 0.02)
    oracle_with_gpu_ties(net, o, g, c, 0.02)
    compare_all(net, g, o, what=net.name)
    y = forward(net, c[None].astype(np.float64))[net.out_layer][0]
    label = int(np.argmax(y))
    (ok_g, m_g), (ok_o, m_o) = g.certify(label), o.certify(label)
    assert np.all(m_g <= m_o + 1e-6 * (1 + np.abs(m_o))) and np.all(m_o - m_g <= 1e-3 * (1 + np.abs(m_o)))
    coef = rng.standard_normal((4, 5)).astype(np.float32)
    off = rng.standard_normal(4).astype(np.float32)
    lb = g.bound_outputs(coef, off).astype(np.float64).reshape(-1)
    ref = o.bound_outputs(coef.astype(np.float64), off.astype(np.float64))
    assert np.all(lb <= ref + 2e-6 * (1 + np.abs(ref))) and np.all(ref - lb <= 1e-3 * (1 + np.abs(ref)))
    g.analyze(c, 0.0)
    lo, hi = g.get_bounds_f64(net.out_layer)
    assert np.all(lo <= y + 1e-12) and np.all(hi >= y - 1e-12) and np.max(hi - lo) < 1e-5
    g.set_coefficient_storage(64)
    g.analyze(c, 0.0)
    lo, hi = g.get_bounds_f64(net.out_layer)
    assert np.all(lo <= y + 1e-12) and np.all(hi >= y - 1e-12) and np.max(hi - lo) < 1e-12
