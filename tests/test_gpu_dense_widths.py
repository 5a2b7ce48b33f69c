"""GPU parity on chains of dense layers of randomly drawn widths (3 to 400 inputs, 5 to 330 neurons per layer) with 1 to
130 boxes per pass.  The width of a layer is the length of the contraction of the crossing below it, so the draws vary
the number of 16-channel steps (1 to 25: the branch-free steady part of the loop runs for none, some or most of
them), the ragged last step (widths that are no multiple of 16, and of 4: scalar loads) and, through the number of rows
of a launch, the tile shape (32x32, 64x32, 64x64).  Both coefficient storages are compared with the oracle given the
same relaxation slopes: float32 storage to 1e-3 (the bar of Section 4's soundness discussion as the test suite reads
it: looser by at most 1e-3 * (1 + |bound|)), float64 storage to 1e-8; neither may lie inside the oracle's interval by
more than 1e-12."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box
from parity import (affine_read_layers, analysed_layers, check_samples_inside, make_gpu, make_oracle,
                    oracle_with_gpu_relaxation)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def dense_chain(seed):
    rng = np.random.default_rng(seed)
    net = wl.Net(f"dense_chain_{seed}", (1, 1, int(rng.integers(3, 400))))

    def dense(src, n_out):
        n = net.n_neurons(src)
        Wt = (rng.standard_normal((n_out, n)) * np.sqrt(2.0 / n)).astype(np.float32)
        return net.dense(src, Wt, (rng.standard_normal(n_out) * 0.1).astype(np.float32))

    cur = 0
    for _ in range(int(rng.integers(2, 5))):
        cur = net.relu(dense(cur, int(rng.integers(5, 330))))
    dense(cur, int(rng.integers(2, 40)))
    net.eps = float(rng.choice([0.001, 0.004, 0.01]))
    return net


@pytest.mark.parametrize("seed", range(32))
def test_dense_chain(seed):
    net = dense_chain(seed)
    rng = np.random.default_rng(50_000 + seed)
    nb = int([1, 2, 7, 40, 130][seed % 5])
    X = rng.random((nb, net.n_in)).astype(np.float32)
    layers = sorted(set(analysed_layers(net)) | set(affine_read_layers(net)))
    # float32 storage twice: start layers whose chain is narrow enough take the fused chain kernel by default; with it
    # switched off every layer takes the general crossing and scan kernels
    for bits, bar, fused in ((32, 1e-3, True), (32, 1e-3, False), (64, 1e-8, False)):
        g = make_gpu(net)
        g.set_coefficient_storage(bits)
        g.set_chain_fusion(fused)
        g.analyze_batch(X, net.eps)
        for b in sorted({0, nb - 1, int(rng.integers(0, nb))}):
            o = make_oracle(net)
            oracle_with_gpu_relaxation(net, o, g, X[b], net.eps, batch_index=b)
            for lid in layers:
                olo, ohi = o.get_bounds(lid)
                glo, ghi = g.get_bounds_f64(lid, b)
                loose = max(np.max((olo - glo) / (1 + np.abs(olo))), np.max((ghi - ohi) / (1 + np.abs(ohi))))
                inside = max(np.max((glo - olo) / (1 + np.abs(olo))), np.max((ohi - ghi) / (1 + np.abs(ohi))))
                assert loose <= bar and inside <= 1e-12, (bits, fused, seed, nb, b, lid, loose, inside)


def test_accumulation_roundoff_hook_only_widens_and_stays_sound():
    """The study hook that prices the accumulation-error term at another unit roundoff (Section 4.1, explicit error
    term): the default is 2^-50 (setting it changes nothing), a larger unit gives bounds that contain the default ones
    and are looser by no more than the ratio of the units allows, out-of-range units are refused."""
    from paper_2007_10868_amd import GpuPolyError
    net = wl.fc_net("roundoff_fc", [96, 80, 64], n_in=50, n_out=6, seed=21)
    rng = np.random.default_rng(3)
    c = rng.random(net.n_in).astype(np.float32)
    eps = 0.01
    g = make_gpu(net)
    g.set_chain_fusion(False)
    g.analyze(c, eps)
    base = {l: g.get_bounds_f64(l) for l in analysed_layers(net)}
    g.debug_set_accumulation_roundoff(2.0 ** -50)
    g.analyze(c, eps)
    for l in base:
        lo, hi = g.get_bounds_f64(l)
        assert np.array_equal(lo, base[l][0]) and np.array_equal(hi, base[l][1]), l
    g.debug_set_accumulation_roundoff(2.0 ** -24)
    g.analyze(c, eps)
    grew = False
    for l in base:
        lo, hi = g.get_bounds_f64(l)
        assert (lo <= base[l][0]).all() and (hi >= base[l][1]).all(), l
        grew = grew or (hi > base[l][1]).any()
        # float32-unit slack: still small against the bounds themselves on a net of this size
        assert np.max(hi - base[l][1]) <= 1e-2 * (1.0 + np.max(np.abs(base[l][1]))), l
    assert grew
    lo0, hi0 = ball_box(c, eps)
    check_samples_inside(net, g, lo0, hi0, 2000, rng, what="roundoff 2^-24")
    for bad in (2.0 ** -60, 2.0 ** -4, float("nan")):
        with pytest.raises(GpuPolyError):
            g.debug_set_accumulation_roundoff(bad)
