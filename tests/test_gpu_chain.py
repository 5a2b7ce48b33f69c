"""The fused chain kernel (one launch per start layer for chains of narrow dense layers, coefficient blocks in LDS)
against the oracle, against the general kernels, and its own invariants (batched == single bit for bit, which layers
take it)."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box
from parity import (analysed_layers, check_samples_inside, compare_all, make_gpu, make_oracle, oracle_with_gpu_relaxation,
                    oracle_with_gpu_ties, same_lower_lines, STRICT_CONTAIN_TOL)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def launches(g, X, eps):
    g.profile_enable(True)
    g.analyze_batch(X, eps)
    prof = g.profile_read()
    g.profile_enable(False)
    return prof["cross"]["launches"], prof["scan"]["launches"]


NETS = [
    ("fc_6x100", lambda: wl.config(0), None),
    ("tiny", lambda: wl.fc_net("tiny_fc", [6, 6], n_in=4, n_out=3, seed=1), 0.1),
    ("odd", lambda: wl.fc_net("odd_fc", [37, 101, 19], n_in=23, n_out=7, seed=1), 0.05),          # odd K: 8-byte weight loads
    ("quad", lambda: wl.fc_net("quad_fc", [24, 28, 40, 20, 52], n_in=36, n_out=8, seed=1), 0.03),
    ("wide_in", lambda: wl.fc_net("wide_in", [256, 17, 256], n_in=1024, n_out=10, seed=2), 0.002),   # the size limits themselves
    ("deep", lambda: wl.fc_net("deep16", [48] * 15, n_in=30, n_out=5, seed=3), 0.002),               # 16 steps: the longest chain
]


@pytest.mark.parametrize("name,maker,eps", NETS, ids=[n[0] for n in NETS])
def test_fused_chain_matches_oracle_and_general_kernels(name, maker, eps):
    net = maker()
    eps = net.eps if eps is None else eps
    rng = np.random.default_rng(12)
    X = rng.random((5, net.n_in)).astype(np.float32)
    g = make_gpu(net)
    n_dense = sum(1 for L in net.layers if L["type"] == "dense")
    cross, scan = launches(g, X, eps)
    assert (cross, scan) == (n_dense - 1, 0), (cross, scan)    # every start layer went through the fused kernel, once (the first
                                                                # one has no product in it and is not counted as a crossing launch)
    fused = {l: [g.get_bounds_f64(l, b) for b in range(5)] for l in analysed_layers(net)}
    for b in (0, 4):
        o = make_oracle(net)
        oracle_with_gpu_ties(net, o, g, X[b], eps, batch_index=b)
        worst = compare_all(net, g, o, batch_index=b, what=f"{name} fused, box {b}")
        oracle_with_gpu_relaxation(net, o, g, X[b], eps, batch_index=b)
        compare_all(net, g, o, batch_index=b, what=f"{name} fused, box {b} (GPU slopes)", contain_tol=STRICT_CONTAIN_TOL)
        lo0, hi0 = ball_box(X[b], eps)
        check_samples_inside(net, g, lo0, hi0, 2000, rng, batch_index=b, what=name)
    print(name, "fused chain: worst looseness / allowed =", worst)
    # one box alone: the same bits (a row's arithmetic does not depend on what else is in the launch)
    g.analyze(X[3], eps)
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l)
        assert np.array_equal(lo, fused[l][3][0]) and np.array_equal(hi, fused[l][3][1]), l
    # the general kernels on the same boxes: same analysis up to the order of the float64 sums
    h = make_gpu(net)
    h.set_chain_fusion(False)
    cross, scan = launches(h, X, eps)
    assert scan > 0
    g.analyze_batch(X, eps)
    for b in range(5):
        if not same_lower_lines(net, g, h, b):
            continue                # a lower-line choice at u = -l fell differently: the later bounds may differ by more
        for l in analysed_layers(net):
            (lo, hi), (lo2, hi2) = g.get_bounds_f64(l, b), h.get_bounds_f64(l, b)
            assert np.max(np.abs(lo - lo2) / (1 + np.abs(lo2))) < 2e-5 and np.max(np.abs(hi - hi2) / (1 + np.abs(hi2))) < 2e-5, (l, b)


def test_which_layers_take_the_fused_path():
    """Decided by the network alone: more than 256 neurons in the start layer itself or in a hidden layer below it, or a
    non-dense layer below, send a start layer to the general kernels; modes the fused kernel does not implement switch
    it off altogether."""
    rng = np.random.default_rng(0)
    net = wl.fc_net("mixed", [64, 300, 64], n_in=50, n_out=6, seed=4)     # start layer 1 is a chain, 3 is 300 wide, 5 and 7 cross 300
    X = rng.random((2, net.n_in)).astype(np.float32)
    g = make_gpu(net)
    cross, scan = launches(g, X, 0.01)
    assert cross == 1 + (2 + 3) and scan == 2 + (3 + 4)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, X[1], 0.01, batch_index=1)
    compare_all(net, g, o, batch_index=1, what="mixed")
    for mode in ("early", "float", "f64"):
        h = make_gpu(wl.config(0))
        {"early": lambda: h.set_early_termination(True), "float": lambda: h.set_float_inference(True),
         "f64": lambda: h.set_coefficient_storage(64)}[mode]()
        Xc = rng.random((2, 784)).astype(np.float32)
        cross, scan = launches(h, Xc, 0.02)
        assert scan > 0, mode


def test_config0_certify_after_fused_analysis_and_graph_replay():
    net = wl.config(0)
    X = np.stack([net.center(j) for j in range(net.n_inputs)])
    g = make_gpu(net)
    g.analyze_batch(X, net.eps)
    ref = {l: [g.get_bounds_f64(l, b) for b in range(len(X))] for l in analysed_layers(net)}
    labels = [int(np.argmax(sum(ref[net.out_layer][b]))) for b in range(len(X))]
    ok, margins = g.certify_batch(labels)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, X[6], net.eps, batch_index=6)
    _, m_o = o.certify(labels[6])
    assert np.all(margins[6] <= m_o + 2e-6 * (1 + np.abs(m_o))) and np.all(m_o - margins[6] <= 1e-3 * (1 + np.abs(m_o)))
    g.set_graph_replay(True)
    for _ in range(3):
        g.analyze_batch(X, net.eps)
        torch.cuda.synchronize()
        for l in analysed_layers(net):
            for b in (0, 9):
                lo, hi = g.get_bounds_f64(l, b)
                assert np.array_equal(lo, ref[l][b][0]) and np.array_equal(hi, ref[l][b][1])
