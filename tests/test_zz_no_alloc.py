"""The allocation-free entry point gp_analyze_batch_dev_static against gp_analyze_batch_dev: same bits, on two calls
in a row, the second on fewer boxes; its refusals.  Collected last on purpose (a failure here hides no other test)."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as wl
from parity import analysed_layers, make_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def _reference(net, centers, eps):
    g = make_gpu(net)
    g.analyze_batch_dev(torch.tensor(centers, device="cuda"), eps)
    return {l: [g.get_bounds_f64(l, b) for b in range(centers.shape[0])] for l in analysed_layers(net)}


@pytest.mark.parametrize("cfg,first,second", [(1, 16, 5), (2, 12, 3), (0, 10, 3)])
def test_static_workspace_call_gives_the_same_bits_twice_in_a_row(cfg, first, second):
    """FC 9x500 with 16 boxes needs 101 MB of workspace, so the 32 MiB static array forces row chunks; small conv takes
    the narrow-layer kernels; FC 6x100 goes through the fused chain kernel, which needs no workspace at all.  Reference: gp_analyze_batch_dev on a net of its own."""
    net = wl.config(cfg)
    centers = np.stack([net.center(j) for j in range(first)])
    ref_first = _reference(net, centers, net.eps)
    ref_second = _reference(net, centers[7:7 + second], net.eps)
    n_out = net.n_neurons(net.out_layer)
    g = make_gpu(net)
    g.set_stream(torch.cuda.current_stream())
    g.analyze_batch_dev(torch.tensor(centers, device="cuda"), net.eps)          # sizes the per-layer arrays
    for cs, ref in ((centers, ref_first), (centers[7:7 + second], ref_second)):
        t = torch.tensor(cs, device="cuda")
        lo = torch.full((cs.shape[0], n_out), float("nan"), dtype=torch.float64, device="cuda")
        hi = torch.full_like(lo, float("nan"))
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()          # the driver's count: sees the library's own hipMalloc too
        g.analyze_batch_dev_static(t, net.eps, lo, hi)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] >= free_before
        lo, hi = lo.cpu().numpy(), hi.cpu().numpy()
        for b in range(cs.shape[0]):
            assert np.array_equal(lo[b], ref[net.out_layer][b][0]) and np.array_equal(hi[b], ref[net.out_layer][b][1]), b
            for l in analysed_layers(net):
                glo, ghi = g.get_bounds_f64(l, b)
                assert np.array_equal(glo, ref[l][b][0]) and np.array_equal(ghi, ref[l][b][1]), (l, b)


def test_static_workspace_call_with_channels_and_positions_in_the_output():
    """A last layer with several positions: the caller's arrays are numbered C,H,W like every array of the boundary."""
    rng = np.random.default_rng(3)
    net = wl.Net("conv_out", (2, 6, 6))
    W1 = (rng.standard_normal((4, 2, 3, 3)) * 0.3).astype(np.float32)
    W2 = (rng.standard_normal((3, 4, 3, 3)) * 0.3).astype(np.float32)
    net.conv(net.relu(net.conv(0, W1, np.zeros(4, np.float32), 1, 1)), W2, (rng.standard_normal(3) * 0.1).astype(np.float32), 2, 0)
    centers = rng.random((3, net.n_in)).astype(np.float32)
    ref = _reference(net, centers, 0.03)
    g = make_gpu(net)
    t = torch.tensor(centers, device="cuda")
    g.analyze_batch_dev(t, 0.03)
    n_out = net.n_neurons(net.out_layer)
    lo = torch.empty((3, n_out), dtype=torch.float64, device="cuda")
    hi = torch.empty_like(lo)
    g.analyze_batch_dev_static(t, 0.03, lo, hi)
    for b in range(3):
        assert np.array_equal(lo[b].cpu().numpy(), ref[net.out_layer][b][0])
        assert np.array_equal(hi[b].cpu().numpy(), ref[net.out_layer][b][1])


def test_static_workspace_call_refuses_instead_of_allocating():
    from paper_2007_10868_amd import GpuPolyError
    net = wl.config(0)
    g = make_gpu(net)
    n_out = net.n_neurons(net.out_layer)
    t = torch.tensor(np.stack([net.center(j) for j in range(4)]), device="cuda")
    lo = torch.empty((4, n_out), dtype=torch.float64, device="cuda")
    hi = torch.empty_like(lo)
    with pytest.raises(GpuPolyError) as e:          # no analysis yet: no per-layer arrays
        g.analyze_batch_dev_static(t, net.eps, lo, hi)
    assert e.value.status == 3
    g.analyze_batch_dev(t[:2].contiguous(), net.eps)
    with pytest.raises(GpuPolyError) as e:          # more boxes than the arrays were sized for
        g.analyze_batch_dev_static(t, net.eps, lo, hi)
    assert e.value.status == 3
    g.analyze_batch_dev_static(t[:2].contiguous(), net.eps, lo[:2], hi[:2])
    g.analyze_batch_dev(t, net.eps)
    g.profile_enable(True)
    with pytest.raises(GpuPolyError) as e:
        g.analyze_batch_dev_static(t, net.eps, lo, hi)
    assert e.value.status == 3
    g.profile_enable(False)
    g.analyze_batch_dev_static(t, net.eps, lo, hi)
    # a row that cannot fit the static array: 2 x 1200 x 1200 neurons in front of a dense head (46 MB per row pair)
    big = wl.Net("big_rows", (1, 1200, 1200))
    c1 = big.conv(0, np.ones((2, 1, 1, 1), np.float32), np.zeros(2, np.float32), 1, 0)
    r1 = big.relu(c1)
    rng = np.random.default_rng(0)
    big.dense(r1, (rng.standard_normal((2, 2 * 1200 * 1200)) * 1e-3).astype(np.float32), np.zeros(2, np.float32))
    gb = make_gpu(big)
    tb = torch.zeros((1, big.n_in), dtype=torch.float32, device="cuda")
    lob = torch.empty((1, 2), dtype=torch.float64, device="cuda")
    with pytest.raises(GpuPolyError) as e:          # refused from the topology alone, before any device state exists
        gb.analyze_batch_dev_static(tb, 0.01, lob, lob.clone())
    assert e.value.status == 7 and "static workspace" in str(e.value)
