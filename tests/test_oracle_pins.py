"""Pins of the CPU oracle against things that are NOT the oracle: closed forms, special cases,
hand-computed values, equivalent formulations, brute force.  No GPU needed."""
import json
import math
import os

import numpy as np
import pytest

import workloads as wl
from helpers import affine_matrix, ball_box, forward, np_deeppoly, sample_box
from oracle import OracleNet

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def make_oracle(net, **opts):
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    if opts:
        o.set_options(**opts)
    return o


def tiny_fc(seed=0, widths=(6, 6), n_in=4, n_out=3):
    return wl.fc_net("tiny_fc", list(widths), n_in=n_in, n_out=n_out, seed=seed)


def tiny_conv(seed=0):
    return wl.conv_net("tiny_conv", (2, 6, 6), [(3, 3, 1, 1), (4, 4, 2, 1)], [8], n_out=3, seed=seed)


def tiny_resnet(seed=0):
    return wl.resnet("tiny_res", (2, 8, 8), channels=(3, 4), blocks=(2, 1), n_out=3, seed=seed)


def analysed_layers(net):
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    return [i for i, L in enumerate(net.layers, start=1)
            if L["type"] == "relu" or i in feeds or i == len(net.layers)]


# ------------------------------------------------------------------------------------------------
def test_first_affine_layer_closed_form():
    """l = W+ L0 + W- U0 + b, u = W+ U0 + W- L0 + b (exactly rounded sums via math.fsum)."""
    net = wl.config(0)
    o = make_oracle(net)
    c = net.center(0)
    o.analyze(c, net.eps)
    lo0, hi0 = ball_box(c, net.eps)
    blo, bhi = o.get_bounds(0)
    assert np.all(blo <= lo0) and np.all(bhi >= hi0)
    assert np.max(np.abs(blo - lo0)) < 1e-15 and np.max(np.abs(bhi - hi0)) < 1e-15
    W = net.layers[0]["W"].astype(np.float64)
    b = net.layers[0]["b"].astype(np.float64)
    lo, hi = o.get_bounds(1)
    for i in range(W.shape[0]):
        wp, wn = np.maximum(W[i], 0), np.minimum(W[i], 0)
        l_exact = math.fsum(list(wp * lo0) + list(wn * hi0) + [b[i]])
        u_exact = math.fsum(list(wp * hi0) + list(wn * lo0) + [b[i]])
        assert lo[i] <= l_exact + 1e-15 and l_exact - lo[i] < 1e-12
        assert hi[i] >= u_exact - 1e-15 and hi[i] - u_exact < 1e-12


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv, tiny_resnet])
def test_eps_zero_collapses_to_forward_pass(maker):
    net = maker(3)
    o = make_oracle(net)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    o.analyze(c, 0.0)
    vals = forward(net, c[None, :].astype(np.float64))
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        v = vals[lid][0]
        assert np.all(lo <= v + 1e-13) and np.all(hi >= v - 1e-13)
        assert np.max(hi - lo) < 1e-11, (lid, np.max(hi - lo))


def _shift_biases(net, shift):
    """Make every hidden affine layer strongly positive (all ReLUs active) or negative (all dead)."""
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    feeds |= {L[k] for L in net.layers if L["type"] == "add" for k in ("a", "b")}
    for i, L in enumerate(net.layers, start=1):
        if i in feeds and L["type"] in ("dense", "conv", "avgpool"):
            L["W"] = (L["W"] * np.float32(0.02)).astype(np.float32)
            L["b"] = (L["b"] + np.float32(shift)).astype(np.float32)


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv, tiny_resnet])
def test_all_stable_network_is_exact_affine_image(maker):
    """With every ReLU stably active DeepPoly is exact on each layer, so the bounds are the interval
    image of the composed affine map, A+ L0 + A- U0 + c.  A is obtained from forward passes of basis
    vectors, not from the oracle."""
    net = maker(11)
    _shift_biases(net, 5.0)
    o = make_oracle(net)
    rng = np.random.default_rng(2)
    c = rng.random(net.n_in).astype(np.float32)
    eps = 0.05
    o.analyze(c, eps)
    lo0, hi0 = ball_box(c, eps)
    mid = 0.5 * (lo0 + hi0)
    n = net.n_in
    base = forward(net, mid[None, :])
    pert = forward(net, mid[None, :] + np.eye(n))
    for lid in analysed_layers(net):
        if net.layers[lid - 1]["type"] == "relu":
            src_lo, _ = o.get_bounds(net.layers[lid - 1]["src"])
            assert np.all(src_lo > 0)       # the premise: every ReLU is stably active
        A = (pert[lid] - base[lid]).T     # [n_lid, n_in]
        c0 = base[lid][0] - A @ mid
        Ap, An = np.maximum(A, 0), np.minimum(A, 0)
        l_ref = Ap @ lo0 + An @ hi0 + c0
        u_ref = Ap @ hi0 + An @ lo0 + c0
        lo, hi = o.get_bounds(lid)
        scale = 1.0 + np.abs(u_ref)
        assert np.max(np.abs(lo - l_ref) / scale) < 1e-10, lid
        assert np.max(np.abs(hi - u_ref) / scale) < 1e-10, lid


def test_all_dead_network():
    net = tiny_fc(4)
    _shift_biases(net, -5.0)
    o = make_oracle(net)
    c = np.full(net.n_in, 0.5, np.float32)
    o.analyze(c, 0.1)
    lo, hi = o.get_bounds(net.out_layer)
    b = net.layers[-1]["b"].astype(np.float64)
    assert np.max(np.abs(lo - b)) < 1e-14 and np.max(np.abs(hi - b)) < 1e-14


def test_hand_computed_unstable_relu_example():
    g = json.load(open(os.path.join(GOLD, "hand_relu_example.json")))
    o = OracleNet(2, 1, 1)
    l1 = o.add_dense(0, np.array(g["W1"], np.float32), np.array(g["b1"], np.float32))
    r1 = o.add_relu(l1)
    l2 = o.add_dense(r1, np.array(g["W2"], np.float32), np.array(g["b2"], np.float32))
    o.analyze_box(g["box_lo"], g["box_hi"])
    lo, hi = o.get_bounds(l1)
    assert np.allclose(lo, g["hidden_lo"], atol=1e-14) and np.allclose(hi, g["hidden_hi"], atol=1e-14)
    gam, dlt, lam = o.get_relaxation(r1)
    assert np.allclose(gam, g["gamma"], atol=1e-15)
    assert np.allclose(dlt, g["delta"], atol=1e-15)
    assert list(lam) == g["lambda"]
    lo, hi = o.get_bounds(l2)
    assert np.allclose(lo, g["out_lo"], atol=1e-13), lo
    assert np.allclose(hi, g["out_hi"], atol=1e-13), hi
    assert np.all(lo <= np.array(g["out_lo"])) and np.all(hi >= np.array(g["out_hi"]))   # outward


def _toeplitz_equivalent(net):
    """Same network with every conv layer replaced by the dense layer of its Toeplitz matrix."""
    eq = wl.Net(net.name + "_dense", (net.n_in, 1, 1))
    for i, L in enumerate(net.layers, start=1):
        if L["type"] == "conv":
            A, b = affine_matrix(net, i)
            assert np.array_equal(A.astype(np.float32).astype(np.float64), A)
            eq.dense(L["src"], A.astype(np.float32), b.astype(np.float32))
        elif L["type"] == "dense":
            eq.dense(L["src"], L["W"], L["b"])
        elif L["type"] == "relu":
            eq.relu(L["src"])
        else:
            eq.add(L["a"], L["b"])
    return eq


@pytest.mark.parametrize("maker", [tiny_conv, tiny_resnet])
def test_conv_equals_its_toeplitz_dense_layer(maker):
    """A back-substitution step is a matrix product with the layer's matrix; for a convolution that
    matrix is its Toeplitz matrix (paper Section 2 'Backsubstitution as matrix multiplication')."""
    net = maker(7)
    eq = _toeplitz_equivalent(net)
    rng = np.random.default_rng(1)
    c = rng.random(net.n_in).astype(np.float32)
    o1, o2 = make_oracle(net), make_oracle(eq)
    o1.analyze(c, 0.03)
    o2.analyze(c, 0.03)
    for lid in analysed_layers(net):
        a, b = o1.get_bounds(lid), o2.get_bounds(lid)
        s = 1 + np.abs(a[1])
        assert np.max(np.abs(a[0] - b[0]) / s) < 1e-11 and np.max(np.abs(a[1] - b[1]) / s) < 1e-11, lid


def test_residual_block_equals_dense_net_carrying_the_skip():
    """x -> A1 x -> relu -> A2 (.) + x   equals the plain chain
       x -> [A1 x ; x] -> relu -> [A2 | I] (.)  when x >= 0 (the carried copy is a stably active ReLU,
       which DeepPoly treats exactly).  Candidates at the input only, because the chain has one more
       single-layer expression than the residual form."""
    rng = np.random.default_rng(3)
    n, m = 5, 5
    W0 = rng.standard_normal((n, 4)).astype(np.float32)
    b0 = rng.standard_normal(n).astype(np.float32)
    A1 = rng.standard_normal((m, n)).astype(np.float32)
    b1 = (rng.standard_normal(m) * 0.1).astype(np.float32)
    A2 = rng.standard_normal((n, m)).astype(np.float32)
    b2 = (rng.standard_normal(n) * 0.1).astype(np.float32)
    W3 = rng.standard_normal((3, n)).astype(np.float32)
    b3 = rng.standard_normal(3).astype(np.float32)

    res = wl.Net("res", (4, 1, 1))
    x = res.relu(res.dense(0, W0, b0))
    h = res.relu(res.dense(x, A1, b1))
    s = res.add(res.dense(h, A2, b2), x)
    res.dense(res.relu(s), W3, b3)

    ch = wl.Net("chain", (4, 1, 1))
    x = ch.relu(ch.dense(0, W0, b0))
    hx = ch.relu(ch.dense(x, np.vstack([A1, np.eye(n, dtype=np.float32)]), np.concatenate([b1, np.zeros(n, np.float32)])))
    s2 = ch.dense(hx, np.hstack([A2, np.eye(n, dtype=np.float32)]), b2)
    ch.dense(ch.relu(s2), W3, b3)

    c = rng.random(4).astype(np.float32)
    o1 = make_oracle(res, candidates=OracleNet.CAND_INPUT_ONLY)
    o2 = make_oracle(ch, candidates=OracleNet.CAND_INPUT_ONLY)
    o1.analyze(c, 0.2)
    # chain: layer by layer; the carried copies get the interval of x itself (with candidates at the
    # input only, back-substituting a copy of relu(a) through lam*a would give it a negative lower end)
    o2.set_ball(c, 0.2)
    xl, xu = o1.get_bounds(2)
    for lid in range(1, o2.num_layers):
        o2.analyze_layer(lid)
        if lid == 3:
            l3, u3 = o2.get_bounds(3)
            l3[m:], u3[m:] = xl, xu
            o2.set_bounds(3, l3, u3)
    lo1, hi1 = o1.get_bounds(s)
    lo2, hi2 = o2.get_bounds(s2)
    assert np.max(np.abs(lo1 - lo2)) < 1e-12 and np.max(np.abs(hi1 - hi2)) < 1e-12
    lo1, hi1 = o1.get_bounds(res.out_layer)
    lo2, hi2 = o2.get_bounds(ch.out_layer)
    assert np.max(np.abs(lo1 - lo2)) < 1e-11 and np.max(np.abs(hi1 - hi2)) < 1e-11
    sl, su = o1.get_bounds(s)
    al, au = o1.get_bounds(1)
    assert np.any((sl < 0) & (su > 0)) and np.any((al < 0) & (au > 0))   # the test is not vacuous


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.3), (tiny_conv, 0.1), (tiny_resnet, 0.05)])
def test_bounds_contain_sampled_and_corner_points(maker, eps):
    """Soundness by brute force: 1e5 random and vertex points of the box."""
    net = maker(21)
    o = make_oracle(net)
    rng = np.random.default_rng(8)
    c = rng.random(net.n_in).astype(np.float32)
    o.analyze(c, eps)
    lo0, hi0 = ball_box(c, eps)
    X = sample_box(lo0, hi0, 100_000, rng)
    vals = forward(net, X)
    n_unstable = 0
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        v = vals[lid]
        assert np.all(v.min(0) >= lo - 1e-12), lid
        assert np.all(v.max(0) <= hi + 1e-12), lid
        n_unstable += int(np.sum((lo < 0) & (hi > 0)))
    assert n_unstable > 0


def test_one_dimensional_input_exact_range_is_contained():
    """For a 1-D input the network is piecewise linear in x; its exact range over [lo,hi] is attained
    at an end point or at a kink.  Dense sampling plus all sign changes of hidden neurons gives it."""
    net = wl.fc_net("fc1d", [8, 8], n_in=1, n_out=2, seed=13)
    o = make_oracle(net)
    o.analyze_box([-1.0], [1.0])
    xs = np.linspace(-1, 1, 200_001)[:, None]
    vals = forward(net, xs)
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        assert np.all(vals[lid].min(0) >= lo - 1e-12) and np.all(vals[lid].max(0) <= hi + 1e-12)
    # the first layer is affine in x: its bounds are exact
    lo, hi = o.get_bounds(1)
    assert np.max(np.abs(vals[1].min(0) - lo)) < 1e-12 and np.max(np.abs(vals[1].max(0) - hi)) < 1e-12


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv, tiny_resnet])
def test_nested_boxes_give_nested_bounds(maker):
    """With the lower relaxation fixed (lam = 0 everywhere) every transformer is monotone in the box."""
    net = maker(17)
    rng = np.random.default_rng(4)
    c = rng.random(net.n_in).astype(np.float32)
    prev = None
    for eps in (0.01, 0.03, 0.1):
        o = make_oracle(net, lambda_policy=OracleNet.LAMBDA_ZERO)
        o.analyze(c, eps, clip_lo=-10.0, clip_hi=10.0)
        cur = {lid: o.get_bounds(lid) for lid in analysed_layers(net)}
        if prev is not None:
            for lid in cur:
                assert np.all(cur[lid][0] <= prev[lid][0] + 1e-12), lid
                assert np.all(cur[lid][1] >= prev[lid][1] - 1e-12), lid
        prev = cur


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv, tiny_resnet])
def test_all_candidates_never_looser_than_input_only(maker):
    net = maker(9)
    rng = np.random.default_rng(6)
    c = rng.random(net.n_in).astype(np.float32)
    oa = make_oracle(net, candidates=OracleNet.CAND_ALL)
    oi = make_oracle(net, candidates=OracleNet.CAND_INPUT_ONLY)
    # same relaxations in both runs: feed the first run's intervals into the second, layer by layer
    oa.analyze(c, 0.1)
    oi.set_ball(c, 0.1)
    for lid in range(1, oi.num_layers):
        if net.layers[lid - 1]["type"] == "relu":
            oi.analyze_layer(lid)
        elif lid in analysed_layers(net):
            rows = np.arange(net.n_neurons(lid), dtype=np.int32)
            lo_i, hi_i = oi.bound_rows(lid, rows)
            lo_a, hi_a = oa.get_bounds(lid)
            assert np.all(lo_a >= lo_i - 1e-12) and np.all(hi_a <= hi_i + 1e-12), lid
            oi.set_bounds(lid, lo_a, hi_a)


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.2), (tiny_conv, 0.05), (tiny_resnet, 0.02)])
@pytest.mark.parametrize("cand", [0, 1])
def test_second_implementation_agrees(maker, eps, cand):
    """An independent round-to-nearest NumPy DeepPoly (matrix form) lies inside the oracle's outward
    rounded intervals and within 1e-9 of them."""
    net = maker(31)
    rng = np.random.default_rng(12)
    c = rng.random(net.n_in).astype(np.float32)
    o = make_oracle(net, candidates=cand)
    o.analyze(c, eps)
    lo0, hi0 = o.get_bounds(0)
    ref = np_deeppoly(net, lo0, hi0, candidates=cand)
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        rl, ru = ref[lid]
        s = 1 + np.abs(ru) + np.abs(rl)
        assert np.max(np.abs(lo - rl) / s) < 1e-9 and np.max(np.abs(hi - ru) / s) < 1e-9, lid
        assert np.all(lo <= rl + 1e-9 * s) and np.all(hi >= ru - 1e-9 * s)


def test_certify_margins_against_second_implementation_and_samples():
    net = tiny_fc(41, widths=(8, 8), n_in=5, n_out=4)
    rng = np.random.default_rng(2)
    c = rng.random(net.n_in).astype(np.float32)
    o = make_oracle(net)
    o.analyze(c, 0.02)
    y = forward(net, c[None, :].astype(np.float64))[net.out_layer][0]
    label = int(np.argmax(y))
    ok, m = o.certify(label)
    others = [j for j in range(4) if j != label]
    R = np.zeros((3, 4))
    for r, j in enumerate(others):
        R[r, label], R[r, j] = 1.0, -1.0
    lo0, hi0 = o.get_bounds(0)
    ref = np_deeppoly(net, lo0, hi0, extra_rows=R)["extra"]
    assert np.max(np.abs(m - ref)) < 1e-10 and np.all(m <= ref + 1e-12)
    X = sample_box(lo0, hi0, 50_000, rng)
    out = forward(net, X)[net.out_layer]
    for r, j in enumerate(others):
        assert np.all(out[:, label] - out[:, j] >= m[r] - 1e-12)
    assert ok == bool(np.all(m > 0))
    # margins by back-substitution are at least as good as comparing the output intervals
    lo, hi = o.get_bounds(net.out_layer)
    for r, j in enumerate(others):
        assert m[r] >= lo[label] - hi[j] - 1e-12


def test_outward_rounding_is_really_outward():
    """Interval ends must bracket the exactly rounded value: with 1/3-like weights the lower and upper
    ends of the first layer differ although the box is a single point."""
    o = OracleNet(3, 1, 1)
    W = np.array([[1 / 3, 1 / 7, 1 / 11]], np.float32)
    o.add_dense(0, W, np.array([0.1], np.float32))
    x = np.array([1 / 3, 1 / 5, 1 / 7], np.float64)
    o.analyze_box(x, x)
    lo, hi = o.get_bounds(1)
    from fractions import Fraction
    exact = sum(Fraction(float(w)) * Fraction(float(v)) for w, v in zip(W[0], x)) + Fraction(float(np.float32(0.1)))
    assert Fraction(float(lo[0])) <= exact <= Fraction(float(hi[0]))
    assert lo[0] < hi[0] and hi[0] - lo[0] < 1e-15


def test_errors():
    o = OracleNet(4, 1, 1)
    o.add_dense(0, np.zeros((3, 4), np.float32), None)
    with pytest.raises(Exception):
        o.analyze_box([0, 0, 0, 1], [1, 1, 1, 0])       # lo > hi
    with pytest.raises(Exception):
        o.get_bounds(1)                                  # nothing analysed yet


def test_collapsed_and_literal_interval_coefficients():
    """The literal scheme (interval coefficients kept to the end) and the re-centred one are both sound;
    on a shallow net they agree to rounding noise, on a deep one the literal intervals blow up."""
    shallow = tiny_fc(5)
    rng = np.random.default_rng(3)
    c = rng.random(shallow.n_in).astype(np.float32)
    a, b = make_oracle(shallow), make_oracle(shallow)
    b.set_collapse(False)
    a.analyze(c, 0.1)
    b.analyze(c, 0.1)
    for lid in analysed_layers(shallow):
        (l1, u1), (l2, u2) = a.get_bounds(lid), b.get_bounds(lid)
        assert np.max(np.abs(l1 - l2)) < 1e-12 and np.max(np.abs(u1 - u2)) < 1e-12
    deep = wl.fc_net("deep_fc", [64] * 24, n_in=16, n_out=4, seed=2)
    c = rng.random(deep.n_in).astype(np.float32)
    a, b = make_oracle(deep), make_oracle(deep)
    b.set_collapse(False)
    a.analyze(c, 1e-4)
    # same relaxations for the literal run: layer by layer with the collapsed run's intervals
    b.set_ball(c, 1e-4)
    X = sample_box(*ball_box(c, 1e-4), 2000, rng)
    vals = forward(deep, X)
    widths = []
    for lid in range(1, b.num_layers):
        if deep.layers[lid - 1]["type"] == "relu":
            b.analyze_layer(lid)
            continue
        la, ua = a.get_bounds(lid)
        lb, ub = b.bound_rows(lid, np.arange(la.size, dtype=np.int32))
        v = vals[lid]
        assert np.all(v.min(0) >= la - 1e-12) and np.all(v.max(0) <= ua + 1e-12)
        assert np.all(v.min(0) >= lb - 1e-12) and np.all(v.max(0) <= ub + 1e-12)
        widths.append((np.mean(ua - la), np.mean(ub - lb)))
        b.set_bounds(lid, la, ua)
    # the literal intervals are never tighter (up to noise) and visibly wider at the deep end
    assert all(wb >= wa * (1 - 1e-9) for wa, wb in widths)
    assert widths[-1][1] > widths[-1][0] * (1 + 1e-6), widths[-1]


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (tiny_conv, 0.05), (tiny_resnet, 0.02)])
def test_linear_output_forms_against_second_implementation_and_samples(maker, eps):
    """Lower bounds of arbitrary linear forms of the outputs: equal to the NumPy DeepPoly's to 1e-9, below every
    sampled value of the form, and equal to the certification margins when the forms are y_label - y_j."""
    net = maker(17)
    rng = np.random.default_rng(23)
    c = rng.random(net.n_in).astype(np.float32)
    o = make_oracle(net)
    o.analyze(c, eps)
    n_out = net.n_neurons(net.out_layer)
    coef = rng.standard_normal((5, n_out))
    coef[1] = 0.0
    coef[2, 1:] = 0.0
    off = rng.standard_normal(5)
    lb = o.bound_outputs(coef, off)
    lo0, hi0 = o.get_bounds(0)
    ref = np_deeppoly(net, lo0, hi0, extra_rows=coef)["extra"] + off
    assert np.max(np.abs(lb - ref) / (1 + np.abs(ref))) < 1e-9
    assert abs(lb[1] - off[1]) < 1e-12                       # the zero form is its offset
    Y = forward(net, sample_box(lo0, hi0, 2000, rng))[net.out_layer]
    assert np.all(Y @ coef.T + off >= lb - 1e-12)
    label = 1
    rows = np.array([np.eye(n_out)[label] - np.eye(n_out)[j] for j in range(n_out) if j != label])
    _, margins = o.certify(label)
    assert np.array_equal(o.bound_outputs(rows), margins)
