"""Graph replay (gp_set_graph_replay): the captured pass must give the eager pass's bits on every replay, with eager work
and synchronisations of the same process in between, and must be rebuilt when anything it depends on changes."""
import numpy as np
import pytest
import torch

import workloads as wl
from parity import analysed_layers, make_gpu
from test_gpu_parity import tiny_conv, tiny_resnet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def all_bounds(g, net, batch):
    return [[g.get_bounds_f64(l, b) for b in range(batch)] for l in analysed_layers(net)]


def same(a, b):
    return all(np.array_equal(x[0], y[0]) and np.array_equal(x[1], y[1]) for la, lb in zip(a, b) for x, y in zip(la, lb))


@pytest.mark.parametrize("maker", [lambda: wl.config(0), tiny_conv, tiny_resnet, lambda: wl.config(2)])
def test_replays_equal_eager(maker):
    net = maker()
    rng = np.random.default_rng(1)
    eps = net.eps if net.eps > 0 else 0.02
    sets = [rng.random((3, net.n_in)).astype(np.float32) for _ in range(3)]
    eager = make_gpu(net)
    want = []
    for X in sets:
        eager.analyze_batch(X, eps)
        want.append(all_bounds(eager, net, 3))
    g = make_gpu(net)
    g.set_graph_replay(True)
    for rep in range(3):                       # the first pass of rep 0 captures, everything after replays
        for X, w in zip(sets, want):
            g.analyze_batch(X, eps)
            assert same(all_bounds(g, net, 3), w), (net.name, rep)
            # eager work of the same process between the replays
            eager.analyze_batch(X[:1], eps)
            torch.cuda.synchronize()
        label = np.array([0, 1, 2], np.int32) % net.n_neurons(net.out_layer)
        ok_g, m_g = g.certify_batch(label)     # certification rows run eagerly on the replayed bounds
        eager.analyze_batch(sets[-1], eps)
        ok_e, m_e = eager.certify_batch(label)
        assert np.array_equal(m_g, m_e)


def test_graph_is_rebuilt_when_its_inputs_change():
    net = wl.config(0)
    rng = np.random.default_rng(2)
    X = rng.random((4, net.n_in)).astype(np.float32)
    eager = make_gpu(net)
    g = make_gpu(net)
    g.set_graph_replay(True)

    def check(batch, eps, what):
        g.analyze_batch(X[:batch], eps)
        eager.analyze_batch(X[:batch], eps)
        assert same(all_bounds(g, net, batch), all_bounds(eager, net, batch)), what

    check(4, 0.02, "first capture")
    check(4, 0.02, "replay")
    check(4, 0.01, "other eps")
    check(2, 0.01, "other batch")
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    g.set_workspace(ws)
    check(2, 0.01, "caller workspace")
    check(2, 0.01, "replay with caller workspace")
    s = torch.cuda.Stream()
    g.set_stream(s)
    check(2, 0.01, "other stream")
    g.set_stream(torch.cuda.current_stream())
    g.set_float_inference(True)
    eager.set_float_inference(True)
    check(2, 0.01, "float32-inference mode")
    check(2, 0.01, "replay in float32-inference mode")
    g.set_early_termination(True)
    eager.set_early_termination(True)
    check(2, 0.01, "early termination runs eagerly")
    g.set_early_termination(False)
    eager.set_early_termination(False)
    check(2, 0.01, "back to replay")
    g.set_graph_replay(False)
    check(2, 0.01, "switched off")
