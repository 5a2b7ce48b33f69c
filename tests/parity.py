"""Shared harness of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded arrays and compare every reported interval."""
from __future__ import annotations

import numpy as np

import workloads as wl
from oracle import OracleNet

REL_TOL = 1e-3          # a GPU bound may be looser than the oracle's by at most REL_TOL * (1 + |b|)
# ... and must contain it.  The oracle's relaxation slopes differ from the library's in the last float32 bits (the
# library's are float32 values computed from intervals that are wider by its rounding slack; every slope in [0,1] is
# sound, so neither analysis dominates the other in principle).  Measured on the five configurations, the ten small
# networks and the scaled 34-layer residual net: the library's interval contained the free-running oracle's in every
# one of the comparisons (worst violation <= 0); the bar leaves room for the slope effect only:
CONTAIN_TOL = 1e-6
# With early termination a stopped neuron keeps the intersection of its interval image and its candidates so far, and
# the two sides reach that intersection from slightly different slopes.  Measured over the GPU suite (2 877
# comparisons): worst violation 1.3e-6 in one build and 8.8e-6 in another that differs only in the order of some float64
# sums (scaled 34-layer residual net both times; 1.3e-7 on every other network): which neurons stop where moves with
# the last bits, and the figure with it.  Five times the worst seen:
EARLY_CONTAIN_TOL = 5e-5
# When the oracle is told to use the GPU's slopes and lower-line choices, every transformer is monotone
# in the intervals and the GPU intervals must contain the oracle's up to float64 rounding noise:
STRICT_CONTAIN_TOL = 1e-9


def analysed_layers(net: wl.Net):
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    return [i for i, L in enumerate(net.layers, start=1)
            if L["type"] == "relu" or i in feeds or i == len(net.layers)]


def affine_read_layers(net: wl.Net):
    """Layers that an affine layer reads directly (no ReLU in between): the library bounds them too (their intervals
    enter its rounding slack) and takes candidates there."""
    return sorted({L["src"] for L in net.layers if L["type"] in ("dense", "conv", "avgpool") and L["src"] > 0
                   and net.layers[L["src"] - 1]["type"] != "relu"})


def same_lower_lines(net: wl.Net, g1, g2, batch_index=0) -> bool:
    """Whether two GPU analyses chose the same lower relaxation line for every ReLU neuron.  The choice switches at
    u = -l, the only discontinuity of the analysis: two sound analyses whose intervals differ in the last digits can
    choose differently there, and their later bounds then differ by far more than rounding, in both directions."""
    for lid, L in enumerate(net.layers, start=1):
        if L["type"] == "relu" and not np.array_equal(g1.get_relu_lambda(lid, batch_index), g2.get_relu_lambda(lid, batch_index)):
            return False
    return True


def make_gpu(net: wl.Net):
    from paper_2007_10868_amd import Net
    g = Net(*net.input_shape)
    wl.build_into(net, g)
    return g


def make_oracle(net: wl.Net, **opts):
    """The oracle with the same set of bounded layers as the GPU library: the paper bounds the inputs of ReLU layers
    and the last layer; the library also bounds every layer that an affine layer reads (it needs their intervals for
    its rounding slack), which matters only where two affine layers follow each other without a ReLU.  Those layers
    are marked in the oracle as explicitly requested, so that both sides take the same candidates."""
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    for L in net.layers:
        if L["type"] in ("dense", "conv", "avgpool"):
            src = L["src"]
            if src > 0 and net.layers[src - 1]["type"] != "relu":
                o.request_bounds(src)
    if opts:
        o.set_options(**opts)
    return o


def oracle_with_gpu_ties(net: wl.Net, o: OracleNet, g, center, eps, batch_index=0, clip=(0.0, 1.0), tie=1e-4,
                         extra_layers=()):
    """Oracle analysis layer by layer.  The choice lam in {0,1} of the lower relaxation is the only
    discontinuity of the analysis: where the oracle's own interval is within `tie` of the switching
    point u = -l, it is told to take the GPU's choice.  Returns the number of such neurons.
    extra_layers: layers to bound besides the inputs of ReLU layers and the last layer."""
    o.set_ball(center, eps, clip[0], clip[1])
    forced = 0
    also = affine_read_layers(net)      # marked as requested by make_oracle: candidates are taken there on both sides
    for lid in range(1, o.num_layers):
        L = net.layers[lid - 1]
        if L["type"] == "relu":
            lo, hi = o.get_bounds(L["src"])
            near = (lo < 0) & (hi > 0) & (np.abs(hi + lo) <= tie * (hi - lo))
            if near.any():
                lam = g.get_relu_lambda(lid, batch_index)
                o.set_lambda_override(lid, np.where(near, lam, -1).astype(np.int8))
                forced += int(near.sum())
            else:
                o.set_lambda_override(lid, None)
            o.analyze_layer(lid)
        elif lid in analysed_layers(net) or lid in extra_layers or lid in also:
            o.analyze_layer(lid)
    return forced


def oracle_with_gpu_relaxation(net: wl.Net, o: OracleNet, g, center, eps, batch_index=0, clip=(0.0, 1.0)):
    """Oracle analysis layer by layer with the GPU's relaxation parameters (slope of the upper line, choice
    of the lower line) for every neuron that is unstable for the oracle; intercepts and everything else
    are the oracle's own, from its own (tighter) intervals."""
    o.set_ball(center, eps, clip[0], clip[1])
    for lid in range(1, o.num_layers):
        L = net.layers[lid - 1]
        if L["type"] == "relu":
            o.set_lambda_override(lid, g.get_relu_lambda(lid, batch_index))
            o.set_gamma_override(lid, g.get_relu_slopes(lid, batch_index).astype(np.float64))
            o.analyze_layer(lid)
        elif lid in analysed_layers(net) or lid in affine_read_layers(net):
            o.analyze_layer(lid)


def clear_overrides(net: wl.Net, o: OracleNet):
    for lid in range(1, o.num_layers):
        if net.layers[lid - 1]["type"] == "relu":
            o.set_lambda_override(lid, None)
            o.set_gamma_override(lid, None)


LOG = []       # (what, looseness / allowed, containment violation) of every comparison made, for reports


def compare_layer(glo, ghi, olo, ohi, what="", contain_tol=None):
    """Returns (max looseness / allowed, max containment violation / scale); asserts the bar."""
    glo, ghi = np.asarray(glo, np.float64), np.asarray(ghi, np.float64)
    assert np.all(np.isfinite(glo)) and np.all(np.isfinite(ghi)), what
    s_lo, s_hi = 1.0 + np.abs(olo), 1.0 + np.abs(ohi)
    loose = max(np.max((olo - glo) / s_lo), np.max((ghi - ohi) / s_hi))
    viol = max(np.max((glo - olo) / s_lo), np.max((ohi - ghi) / s_hi))
    LOG.append((what, float(loose / REL_TOL), float(viol)))
    assert loose <= REL_TOL, f"{what}: GPU bound looser than oracle by {loose:.3e} (relative), allowed {REL_TOL}"
    tol = CONTAIN_TOL if contain_tol is None else contain_tol
    assert viol <= tol, f"{what}: GPU bound inside the oracle bound by {viol:.3e} (relative), allowed {tol}"
    return loose / REL_TOL, viol


def compare_all(net, g, o, batch_index=0, what="", f64=True, contain_tol=None):
    worst = 0.0
    for lid in sorted(set(analysed_layers(net)) | set(affine_read_layers(net))):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = (g.get_bounds_f64 if f64 else g.get_bounds)(lid, batch_index)
        r, _ = compare_layer(glo, ghi, olo, ohi, f"{what} layer {lid}", contain_tol)
        worst = max(worst, r)
    return worst


def check_samples_inside(net, g, lo0, hi0, n, rng, batch_index=0, what=""):
    from helpers import forward, sample_box
    X = sample_box(lo0, hi0, n, rng)
    vals = forward(net, X)
    for lid in sorted(set(analysed_layers(net)) | set(affine_read_layers(net))):
        glo, ghi = g.get_bounds(lid, batch_index)
        v = vals[lid]
        assert np.all(v.min(0) >= glo.astype(np.float64)), f"{what} layer {lid}: sampled output below the lower bound"
        assert np.all(v.max(0) <= ghi.astype(np.float64)), f"{what} layer {lid}: sampled output above the upper bound"


def float_inference_layers(net: wl.Net):
    """Layers that carry bounds in float32-inference mode besides the usual ones: every layer an affine layer reads
    (its intervals enter the reader's error constant) and every sum layer (its rounding is relative to its interval)."""
    out = set()
    for i, L in enumerate(net.layers, start=1):
        if L["type"] in ("dense", "conv", "avgpool") and L["src"] > 0 and net.layers[L["src"] - 1]["type"] != "relu":
            out.add(L["src"])
        if L["type"] == "add":
            out.add(i)
    return sorted(out)


def bounded_affine_layers(net: wl.Net):
    """Layers that start back-substitutions (they have bounds and are no ReLU layers)."""
    return [i for i in analysed_layers(net) if net.layers[i - 1]["type"] != "relu"]


def oracle_early_with_gpu_decisions(net: wl.Net, o: OracleNet, g, center, eps, batch_index=0, clip=(0.0, 1.0),
                                    tie=1e-4):
    """Oracle in early-termination mode, layer by layer, stopping every neuron where the GPU stopped it (a
    neuron whose candidate is within rounding of 0 can be stopped by one side and not by the other, and what it
    keeps then differs by more than rounding), and taking the GPU's lower-line choice at near-ties as in
    oracle_with_gpu_ties.  Returns the number of forced lower-line choices."""
    o.set_early_termination(True)
    o.set_ball(center, eps, clip[0], clip[1])
    for lid in bounded_affine_layers(net):
        o.set_term_override(lid, g.get_term_layer(lid, batch_index))
    forced = 0
    for lid in range(1, o.num_layers):
        L = net.layers[lid - 1]
        if L["type"] == "relu":
            lo, hi = o.get_bounds(L["src"])
            near = (lo < 0) & (hi > 0) & (np.abs(hi + lo) <= tie * (hi - lo))
            if near.any():
                lam = g.get_relu_lambda(lid, batch_index)
                o.set_lambda_override(lid, np.where(near, lam, -1).astype(np.int8))
                forced += int(near.sum())
            else:
                o.set_lambda_override(lid, None)
        o.analyze_layer(lid)        # in this mode every layer is visited (interval image at least)
    return forced
