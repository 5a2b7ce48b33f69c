"""GPU parity of the step onto layers with at most 4 channels behind a strided layer (Algorithm 1, short K per output
pixel: one lane per output pixel, the rows' blocks staged in LDS): every number of image channels, channel counts of
the crossed layer with and without whole 4-channel groups, filters that leave some parity classes without taps, windows
large enough for several groups of items per work-group, one box and a batch."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box
from parity import analysed_layers, check_samples_inside, compare_all, make_gpu, make_oracle, oracle_with_gpu_ties

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


# (image channels, image size, convolutions (c_out, k, stride, pad), hidden dense widths)
CASES = [
    (1, 12, [(8, 4, 2, 1), (8, 3, 1, 1)], [16]),            # grayscale, K per pixel 2*2*8
    (2, 11, [(6, 3, 2, 0), (4, 3, 1, 0)], [12]),            # 6 channels: no 4-channel groups; odd image size
    (3, 16, [(16, 4, 2, 1), (8, 4, 2, 1)], [20]),           # the small conv net's shape, reduced
    (4, 10, [(12, 5, 3, 2), (8, 3, 1, 1)], []),             # stride 3, 5x5: classes with one and with two taps per axis
    (3, 9, [(8, 2, 2, 0), (8, 2, 1, 0)], [10]),             # 2x2 stride 2: one tap per class
    (3, 40, [(4, 4, 2, 1), (4, 3, 2, 1)], [8]),             # 20x20 windows: more than 256 items per class and row
    (1, 14, [(4, 3, 1, 1), (4, 3, 1, 1)], [10]),            # stride 1, K = 36: one class
    (1, 100, [(2, 2, 2, 0)], []),                           # a 50x50 window does not fit the work-group's LDS: another form runs
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_image_step_matches_oracle(case):
    ci, hw, convs, denses = CASES[case]
    net = wl.conv_net(f"img{case}", (ci, hw, hw), convs, denses, n_out=4, seed=400 + case)
    rng = np.random.default_rng(900 + case)
    c = rng.random(net.n_in).astype(np.float32)
    eps = 0.02
    g = make_gpu(net)
    g.analyze(c, eps)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, c, eps)
    compare_all(net, g, o, what=net.name)
    lo0, hi0 = ball_box(c, eps)
    check_samples_inside(net, g, lo0, hi0, 2_000, rng, what=net.name)


@pytest.mark.parametrize("case", [0, 2, 5])
def test_image_step_batched_equals_single(case):
    ci, hw, convs, denses = CASES[case]
    net = wl.conv_net(f"img{case}", (ci, hw, hw), convs, denses, n_out=4, seed=400 + case)
    rng = np.random.default_rng(950 + case)
    cs = rng.random((5, net.n_in)).astype(np.float32)
    gb = make_gpu(net)
    gb.analyze_batch(cs, 0.02)
    gs = make_gpu(net)
    for j in range(5):
        gs.analyze(cs[j], 0.02)
        for lid in analysed_layers(net):
            lo1, hi1 = gs.get_bounds_f64(lid)
            lo2, hi2 = gb.get_bounds_f64(lid, j)
            assert np.array_equal(lo1, lo2) and np.array_equal(hi1, hi2), (net.name, j, lid)


LARGE = [
    # conv 6 channels (no 4-channel groups): rows of 150 and of 18 coefficients made by the scans of large launches
    ("conv6", lambda: wl.conv_net("gen_conv6", (2, 13, 13), [(6, 3, 1, 0), (4, 5, 1, 0)], [12], n_out=4, seed=431), 50, False),
    # conv 8 channels: 16-byte groups; the dense start layer's rows range over a 12x12x8 block (chunks of 512 coefficients)
    ("conv8", lambda: wl.conv_net("gen_conv8", (3, 13, 13), [(8, 2, 1, 0)], [170], n_out=4, seed=432), 50, False),
    # dense rows with the fused chain kernel switched off
    ("dense", lambda: wl.fc_net("gen_fc", [120, 96], n_in=40, n_out=5, seed=433), 90, True),
]


@pytest.mark.parametrize("name,maker,batch,chain_off", LARGE, ids=[c[0] for c in LARGE])
def test_rows_made_by_the_scan_equal_the_stored_ones(name, maker, batch, chain_off):
    """Launches of more than 16 384 rows let the scan compute a start layer's own matrix rows instead of reading them back
    (and never store the rows over the input): the bounds must be the bits of the two-kernel form, which the same
    boxes take when they are analysed one at a time; one box is also compared with the oracle."""
    net = maker()
    rng = np.random.default_rng(77)
    cs = rng.random((batch, net.n_in)).astype(np.float32)
    eps = 0.02
    gb = make_gpu(net)
    gs = make_gpu(net)
    if chain_off:
        gb.set_chain_fusion(False)
        gs.set_chain_fusion(False)
    gb.analyze_batch(cs, eps)
    for j in (0, batch // 2, batch - 1):
        gs.analyze(cs[j], eps)
        for lid in analysed_layers(net):
            lo1, hi1 = gs.get_bounds_f64(lid)
            lo2, hi2 = gb.get_bounds_f64(lid, j)
            assert np.array_equal(lo1, lo2) and np.array_equal(hi1, hi2), (net.name, j, lid)
    j = batch - 1
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, gb, cs[j], eps, batch_index=j)
    compare_all(net, gb, o, batch_index=j, what=net.name)
