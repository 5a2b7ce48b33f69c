"""GPU parity of early termination (paper Sections 3.2 and 4.2): the HIP library against the oracle's
early-termination mode on the same seeded inputs.

What is compared: (1) with the oracle stopping every neuron where the GPU stopped it, all intervals agree to the
usual bar (GPU contains the oracle's, looser by at most 1e-3 * (1 + |b|)); (2) the oracle deciding for itself
stops (almost) every neuron at the same layer; (3) sampled network outputs lie inside; (4) a stopped neuron has
its sign proven."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box, forward
from parity import (EARLY_CONTAIN_TOL, analysed_layers, bounded_affine_layers, check_samples_inside, compare_all, make_gpu, make_oracle,
                    oracle_early_with_gpu_decisions)
from test_gpu_parity import mid_resnet, odd_fc, pad0_conv, rect_conv, tiny_conv, tiny_fc, tiny_resnet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def check_early(net, g, center, eps, batch_index=0, what="", samples=200, seed=0, max_mismatch=0.005):
    """g: analysed with early termination on.  Returns the number of neurons that stopped early."""
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    # (1) replayed decisions: full parity
    o = make_oracle(net)
    oracle_early_with_gpu_decisions(net, o, g, center, eps, batch_index)
    compare_all(net, g, o, batch_index, what, contain_tol=EARLY_CONTAIN_TOL)
    # (2) the oracle's own decisions
    of = make_oracle(net)
    of.set_early_termination(True)
    of.analyze(center, eps)
    total = differ = stopped = 0
    for lid in bounded_affine_layers(net):
        tg, to = g.get_term_layer(lid, batch_index), of.get_term_layer(lid)
        total += tg.size
        differ += int(np.sum(tg != to))
        if lid in feeds:
            stopped += int(np.sum(tg != 0))
            lo, hi = g.get_bounds_f64(lid, batch_index)
            s = tg != 0
            assert np.all((lo[s] >= 0) | (hi[s] <= 0)), f"{what} layer {lid}: stopped without a proven sign"
        else:
            assert np.all(tg == 0), f"{what} layer {lid}: rows of this layer must never stop"
    assert differ <= max(1, int(max_mismatch * total)), f"{what}: {differ} of {total} neurons stop at another layer"
    # (3) soundness
    lo0, hi0 = ball_box(center, eps)
    check_samples_inside(net, g, lo0, hi0, samples, np.random.default_rng(seed), batch_index, what)
    return stopped


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (odd_fc, 0.02), (tiny_conv, 0.05), (pad0_conv, 0.02),
                                       (rect_conv, 0.02), (tiny_resnet, 0.01), (mid_resnet, 0.004)])
def test_small_nets(maker, eps):
    net = maker(7)
    c = np.random.default_rng(21).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze(c, eps)
    stopped = check_early(net, g, c, eps, what=net.name)
    done, full = g.early_termination_stats()
    assert 0 <= done <= full
    print(f"{net.name}: {stopped} neurons stopped early, crossing work {done / max(full, 1):.3f} of full")


def test_switching_the_mode_off_restores_the_full_analysis():
    net = odd_fc(3)
    c = np.random.default_rng(4).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, 0.02)
    ref = {lid: g.get_bounds_f64(lid) for lid in analysed_layers(net)}
    g.set_early_termination(True)
    g.analyze(c, 0.02)
    g.set_early_termination(False)
    g.analyze(c, 0.02)
    for lid, (lo, hi) in ref.items():
        l2, h2 = g.get_bounds_f64(lid)
        assert np.array_equal(lo, l2) and np.array_equal(hi, h2)
    with pytest.raises(Exception):
        g.get_term_layer(bounded_affine_layers(net)[0])


def test_config0_batch_and_certify():
    net = wl.config(0)
    eps = net.eps
    X = np.stack([net.center(j) for j in range(4)])
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze_batch(X, eps)
    for b in range(X.shape[0]):
        check_early(net, g, X[b], eps, batch_index=b, what=f"config0[{b}]", samples=50)
    # certification rows are substituted down to the input: margins match the replayed oracle to the usual bar
    labels = [int(np.argmax(forward(net, X[b][None, :].astype(np.float64))[net.out_layer][0])) for b in range(4)]
    ver, mar = g.certify_batch(labels)
    o = make_oracle(net)
    oracle_early_with_gpu_decisions(net, o, g, X[1], eps, 1)
    _, om = o.certify(labels[1])
    m1 = np.asarray(mar[1], np.float64)
    assert np.all(m1 <= om + 2e-6 * (1 + np.abs(om))) and np.all(om - m1 <= 1e-3 * (1 + np.abs(om)))


def test_config1_rows_are_removed():
    net = wl.config(1)
    eps = net.eps
    X = np.stack([net.center(j) for j in range(3)])
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze_batch(X, eps)
    stopped = check_early(net, g, X[2], eps, batch_index=2, what="config1[2]", samples=50)
    done, full = g.early_termination_stats()
    print(f"config1: {stopped} neurons of input 2 stopped early; crossing work {done / full:.3f} of full")
    assert stopped > 0 and done <= full


def test_contracted_config1_most_work_is_removed():
    """The regime early termination is for (most ReLUs stable): the benchmark network with its weights scaled by 0.3,
    in the benchmark's launch configuration (all rows of a batch in the same launches, rows physically removed)."""
    net = wl.contracted(wl.config(1), 0.3)
    eps = net.eps
    X = np.stack([net.center(j) for j in range(8)])
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze_batch(X, eps)
    done, full = g.early_termination_stats()
    print(f"contracted config1: crossing work {done / full:.3f} of full")
    assert done < 0.6 * full
    for b in (0, 7):
        stopped = check_early(net, g, X[b], eps, batch_index=b, what=f"contracted config1[{b}]", samples=50)
        assert stopped > 1000
    # batched == one by one, bit for bit, also when rows are removed
    g1 = make_gpu(net)
    g1.set_early_termination(True)
    g1.analyze(X[7], eps)
    for lid in bounded_affine_layers(net):
        a, b = g.get_bounds_f64(lid, 7)
        c, d = g1.get_bounds_f64(lid)
        assert np.array_equal(a, c) and np.array_equal(b, d)
        assert np.array_equal(g.get_term_layer(lid, 7), g1.get_term_layer(lid))


def test_chunked_batched_conv():
    """Small workspace: many chunks, each with its own task list."""
    net = wl.config(2)
    eps = net.eps
    X = np.stack([net.center(j) for j in range(2)])
    g = make_gpu(net)
    g.set_early_termination(True)
    mn, full = g.workspace_size(2)
    ws = torch.empty(max(mn * 300, full // 7), dtype=torch.uint8, device="cuda")
    g.set_workspace(ws)
    g.analyze_batch(X, eps)
    ref = make_gpu(net)
    ref.set_early_termination(True)
    ref.analyze_batch(X, eps)
    for lid in analysed_layers(net):
        for b in range(2):
            a, c = g.get_bounds_f64(lid, b), ref.get_bounds_f64(lid, b)
            assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1]), (lid, b)   # chunking changes nothing
    check_early(net, g, X[1], eps, batch_index=1, what="config2[1]", samples=50)


def test_scaled_resnet():
    net = wl.scaled_resnet(8, 16)
    eps = net.eps
    c = net.center(0)
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze(c, eps)
    stopped = check_early(net, g, c, eps, what=net.name, samples=20)
    done, full = g.early_termination_stats()
    print(f"{net.name}: {stopped} neurons stopped early; crossing work {done / full:.3f} of full")


def test_contracted_resnet34_every_neuron_with_replayed_decisions():
    """The 1M-neuron residual configuration in the regime early termination is for: every weight times 0.05, so that
    99.9 % of the ReLU inputs have a decided sign and almost every row stops at once (50 ms per input on the GPU).  The
    oracle in its early-termination mode then finishes a whole pass in well under a minute, so EVERY interval of EVERY
    layer is compared (966 666 back-substituted neurons, decisions replayed), the oracle's own decisions are compared
    with the library's, and sampled outputs are checked."""
    net = wl.contracted(wl.config(4), 0.05)
    c = net.center(0)
    g = make_gpu(net)
    g.set_early_termination(True)
    g.analyze(c, net.eps)
    stopped = check_early(net, g, c, net.eps, what="resnet34 x0.05", samples=32)
    done, full = g.early_termination_stats()
    n_relu_in = sum(net.n_neurons(L["src"]) for L in net.layers if L["type"] == "relu")
    print(f"contracted resnet34: {stopped} of {n_relu_in} ReLU inputs stopped early; crossing work {done / full:.5f} of full")
    assert stopped > 0.99 * n_relu_in and done < 0.01 * full
