"""Pins of the oracle's early-termination mode (paper Sections 3.2 and 4.2) against things that are not the
oracle: closed forms of the forward interval pass, the two extreme cases (nothing terminates / everything
does), a second implementation in matrix form, and sampled network outputs.  No GPU needed."""
import numpy as np
import pytest

import workloads as wl
from helpers import affine_matrix, ball_box, forward, np_deeppoly_early, sample_box
from oracle import OracleNet
from test_oracle_pins import _shift_biases, analysed_layers, make_oracle, tiny_conv, tiny_fc, tiny_resnet


def early_oracle(net):
    o = make_oracle(net)
    o.set_early_termination(True)
    return o


def affine_ids(net):
    return [i for i, L in enumerate(net.layers, start=1) if L["type"] != "relu"]


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.2), (tiny_conv, 0.05), (tiny_resnet, 0.02)])
def test_interval_image_is_the_closed_form(maker, eps):
    """Forward interval analysis of a layer: A+ l + A- u + b over the predecessor's intervals (sum layers: the sum
    of the two intervals), with A taken from forward passes of basis vectors."""
    net = maker(5)
    rng = np.random.default_rng(3)
    c = rng.random(net.n_in).astype(np.float32)
    o = early_oracle(net)
    o.analyze(c, eps)
    bounded = set(analysed_layers(net)) | {0}

    def known(q):
        return o.get_bounds(q) if q in bounded else o.get_interval_image(q)

    for lid in affine_ids(net):
        L = net.layers[lid - 1]
        ilo, ihi = o.get_interval_image(lid)
        if L["type"] == "add":
            (la, ua), (lb, ub) = known(L["a"]), known(L["b"])
            rl, ru = la + lb, ua + ub
        else:
            A, b = affine_matrix(net, lid)
            pl, pu = known(L["src"])
            rl = np.maximum(A, 0) @ pl + np.minimum(A, 0) @ pu + b
            ru = np.maximum(A, 0) @ pu + np.minimum(A, 0) @ pl + b
        s = 1 + np.abs(rl) + np.abs(ru)
        assert np.max(np.abs(ilo - rl) / s) < 1e-12 and np.max(np.abs(ihi - ru) / s) < 1e-12, lid
        if lid in bounded:      # back-substitution can only tighten the interval image
            lo, hi = o.get_bounds(lid)
            assert np.all(lo >= ilo) and np.all(hi <= ihi), lid


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv])
def test_nothing_terminates_gives_the_full_analysis(maker):
    """Zero biases and a box symmetric about 0: every hidden neuron's range contains 0 strictly, no neuron
    meets the criterion, and the procedure must return what the analysis without early termination returns."""
    net = maker(21)
    for L in net.layers:
        if "b" in L and L["type"] != "add":
            L["b"] = np.zeros_like(L["b"])
    lo0, hi0 = -np.ones(net.n_in), np.ones(net.n_in)
    full = make_oracle(net)
    full.analyze_box(lo0, hi0)
    early = early_oracle(net)
    early.analyze_box(lo0, hi0)
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    for lid in analysed_layers(net):
        if lid in feeds:
            assert np.all(early.get_term_layer(lid) == 0), lid      # the premise
        lf, uf = full.get_bounds(lid)
        le, ue = early.get_bounds(lid)
        s = 1 + np.abs(uf) + np.abs(lf)
        assert np.max(np.abs(lf - le) / s) < 1e-12 and np.max(np.abs(uf - ue) / s) < 1e-12, lid


@pytest.mark.parametrize("maker", [tiny_fc, tiny_conv, tiny_resnet])
def test_everything_terminates_at_once_when_all_relus_are_stable(maker):
    """All ReLUs stably active: no hidden neuron is back-substituted (its interval is the interval image), and
    the output layer, back-substituted through exact relaxations, is the interval image of the composed map."""
    net = maker(11)
    _shift_biases(net, 5.0)
    o = early_oracle(net)
    rng = np.random.default_rng(2)
    c = rng.random(net.n_in).astype(np.float32)
    eps = 0.05
    o.analyze(c, eps)
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    for lid in feeds:
        assert np.all(o.get_term_layer(lid) == lid)
        lo, hi = o.get_bounds(lid)
        ilo, ihi = o.get_interval_image(lid)
        assert np.array_equal(lo, ilo) and np.array_equal(hi, ihi) and np.all(lo > 0)
    lo0, hi0 = ball_box(c, eps)
    mid = 0.5 * (lo0 + hi0)
    last = len(net.layers)
    base = forward(net, mid[None, :])[last]
    A = (forward(net, mid[None, :] + np.eye(net.n_in))[last] - base).T
    c0 = base[0] - A @ mid
    l_ref = np.maximum(A, 0) @ lo0 + np.minimum(A, 0) @ hi0 + c0
    u_ref = np.maximum(A, 0) @ hi0 + np.minimum(A, 0) @ lo0 + c0
    lo, hi = o.get_bounds(last)
    assert np.all(o.get_term_layer(last) == 0)
    assert np.max(np.abs(lo - l_ref) / (1 + np.abs(l_ref))) < 1e-10
    assert np.max(np.abs(hi - u_ref) / (1 + np.abs(u_ref))) < 1e-10


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.05), (tiny_fc, 0.2), (tiny_conv, 0.03), (tiny_resnet, 0.01)])
def test_second_implementation_agrees(maker, eps):
    """The matrix-form NumPy version of the same procedure stops every neuron at the same layer and gives the same
    intervals to 1e-9; the oracle's outward-rounded ones contain it."""
    net = maker(33)
    rng = np.random.default_rng(14)
    c = rng.random(net.n_in).astype(np.float32)
    o = early_oracle(net)
    o.analyze(c, eps)
    lo0, hi0 = o.get_bounds(0)
    ref, term, _ = np_deeppoly_early(net, lo0, hi0)
    n_stopped = 0
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        rl, ru = ref[lid]
        s = 1 + np.abs(ru) + np.abs(rl)
        assert np.max(np.abs(lo - rl) / s) < 1e-9 and np.max(np.abs(hi - ru) / s) < 1e-9, lid
        assert np.all(lo <= rl + 1e-9 * s) and np.all(hi >= ru - 1e-9 * s)
        if lid in term:
            t = o.get_term_layer(lid)
            assert np.array_equal(t, term[lid]), lid
            n_stopped += int(np.sum(t != 0))
    assert n_stopped > 0      # the case exercises the criterion


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (tiny_conv, 0.05), (tiny_resnet, 0.02)])
def test_bounds_contain_sampled_outputs_and_stop_only_when_the_sign_is_proven(maker, eps):
    net = maker(8)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    o = early_oracle(net)
    o.analyze(c, eps)
    lo0, hi0 = o.get_bounds(0)
    vals = forward(net, sample_box(lo0, hi0, 400, rng))
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    for lid in analysed_layers(net):
        lo, hi = o.get_bounds(lid)
        assert np.all(vals[lid] >= lo - 1e-12) and np.all(vals[lid] <= hi + 1e-12), lid
        if lid in feeds:
            t = o.get_term_layer(lid)
            stopped = t != 0
            assert np.all((lo[stopped] >= 0) | (hi[stopped] <= 0)), lid


def test_forced_decisions_are_followed():
    """Replaying a run's own decisions reproduces it bit for bit; forcing every neuron down to the input gives the
    analysis without early termination (whose first candidate is the interval image)."""
    net = tiny_conv(4)
    rng = np.random.default_rng(9)
    c = rng.random(net.n_in).astype(np.float32)
    eps = 0.04
    a = early_oracle(net)
    a.analyze(c, eps)
    b = early_oracle(net)
    z = early_oracle(net)
    feeds = sorted({L["src"] for L in net.layers if L["type"] == "relu"})
    for lid in feeds:
        b.set_term_override(lid, a.get_term_layer(lid))
        z.set_term_override(lid, np.zeros(net.n_neurons(lid), np.int32))
    b.analyze(c, eps)
    z.analyze(c, eps)
    full = make_oracle(net)
    full.analyze(c, eps)
    for lid in analysed_layers(net):
        la, ua = a.get_bounds(lid)
        lb, ub = b.get_bounds(lid)
        assert np.array_equal(la, lb) and np.array_equal(ua, ub), lid
        lz, uz = z.get_bounds(lid)
        lf, uf = full.get_bounds(lid)
        s = 1 + np.abs(uf) + np.abs(lf)
        assert np.max(np.abs(lz - lf) / s) < 1e-12 and np.max(np.abs(uz - uf) / s) < 1e-12, lid
