"""Float64 coefficient storage (the paper evaluates a single and a double precision build, Section 5): the same
analysis with the blocks held in float64.  What the float32 storage loses is then gone, so the GPU intervals agree
with the oracle's to 1e-9 when both use the same relaxation slopes: a bar a million times tighter than the one the
float32 mode is held to, which pins the GPU arithmetic itself rather than its rounding slack."""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box, forward
from parity import (analysed_layers, affine_read_layers, check_samples_inside, compare_all, make_gpu, make_oracle,
                    oracle_with_gpu_relaxation, oracle_with_gpu_ties, same_lower_lines)
from test_gpu_avgpool import lenet_like, pooled_shortcut
from test_gpu_early_term import check_early
from test_gpu_parity import mid_resnet, odd_fc, pad0_conv, quad_fc, rect_conv, strip_conv, tiny_conv, tiny_fc, tiny_resnet

pytestmark = pytest.mark.gpu

F64_TOL = 1e-9          # |GPU bound - oracle bound| <= F64_TOL * (1 + |bound|), same relaxation on both sides


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def layers_of(net):
    return sorted(set(analysed_layers(net)) | set(affine_read_layers(net)))


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (odd_fc, 0.05), (quad_fc, 0.03), (tiny_conv, 0.05), (pad0_conv, 0.03),
                                       (tiny_resnet, 0.02), (mid_resnet, 0.01), (rect_conv, 0.04), (strip_conv, 0.004),
                                       (lenet_like, 0.03), (pooled_shortcut, 0.01)])
def test_float64_storage_agrees_with_the_oracle_to_1e9(maker, eps):
    net = maker(1)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_coefficient_storage(64)
    g.analyze(c, eps)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, c, eps)
    compare_all(net, g, o, what=net.name)                          # the usual bar first (oracle's own slopes)
    lo0, hi0 = ball_box(c, eps)
    check_samples_inside(net, g, lo0, hi0, 5_000, rng, what=net.name)
    oracle_with_gpu_relaxation(net, o, g, c, eps)                  # same slopes on both sides
    worst = 0.0
    for lid in layers_of(net):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = g.get_bounds_f64(lid)
        assert np.all(glo <= olo + 1e-12 * (1 + np.abs(olo))) and np.all(ghi >= ohi - 1e-12 * (1 + np.abs(ohi))), (net.name, lid)
        d = max(np.max((olo - glo) / (1 + np.abs(olo))), np.max((ghi - ohi) / (1 + np.abs(ohi))))
        worst = max(worst, d)
        assert d <= F64_TOL, f"{net.name} layer {lid}: float64-storage bound looser than the oracle's by {d:.3e}"
    print(net.name, "float64 storage: worst looseness", worst)
    # and it is never looser than the float32 storage by more than rounding noise
    g32 = make_gpu(net)
    g32.analyze(c, eps)
    y = forward(net, c[None].astype(np.float64))[net.out_layer][0]
    label = int(np.argmax(y))
    m64, m32 = g.certify(label)[1], g32.certify(label)[1]
    m_o = o.certify(label)[1]
    assert np.all(m64 <= m_o + 1e-6 * (1 + np.abs(m_o)))            # margins are reported in float32, rounded down
    assert np.all(m_o - m64 <= 1e-6 * (1 + np.abs(m_o)))
    assert np.all(m32 <= m_o + 1e-4 * (1 + np.abs(m_o)))


def test_switching_storage_back_and_forth_and_batches():
    net = mid_resnet(2)
    g = make_gpu(net)
    centers = np.stack([np.random.default_rng(40 + j).random(net.n_in).astype(np.float32) for j in range(3)])
    g.analyze_batch(centers, 0.01)
    ref32 = [g.get_bounds_f64(net.out_layer, b) for b in range(3)]
    g.set_coefficient_storage(64)
    g.analyze_batch(centers, 0.01)
    b64 = {l: [g.get_bounds_f64(l, b) for b in range(3)] for l in analysed_layers(net)}
    for b in range(3):
        lo, hi = b64[net.out_layer][b]
        assert np.all(lo >= ref32[b][0] - 1e-9) and np.all(hi <= ref32[b][1] + 1e-9)      # tighter than float32 storage
        assert np.max(ref32[b][1] - hi) < 1e-3 and np.max(ref32[b][1] - hi) > 0
        g.analyze(centers[b], 0.01)                                                       # batched == single, bit for bit
        for l in analysed_layers(net):
            lo1, hi1 = g.get_bounds_f64(l)
            assert np.array_equal(lo1, b64[l][b][0]) and np.array_equal(hi1, b64[l][b][1])
    mn, full = g.workspace_size(1)
    mn32, full32 = make_gpu(net).workspace_size(1)
    assert full > 1.9 * full32 - (1 << 20)
    small = torch.empty(mn * 41 + 4096, dtype=torch.uint8, device="cuda")                # chunked == unchunked
    g.set_workspace(small)
    g.analyze(centers[2], 0.01)
    for l in analysed_layers(net):
        lo1, hi1 = g.get_bounds_f64(l)
        assert np.array_equal(lo1, b64[l][2][0]) and np.array_equal(hi1, b64[l][2][1])
    g.set_workspace(None)
    g.set_coefficient_storage(32)
    g.analyze_batch(centers, 0.01)
    for b in range(3):
        lo, hi = g.get_bounds_f64(net.out_layer, b)
        assert np.array_equal(lo, ref32[b][0]) and np.array_equal(hi, ref32[b][1])
    from paper_2007_10868_amd import GpuPolyError
    with pytest.raises(GpuPolyError) as e:
        g.set_coefficient_storage(16)
    assert e.value.status == 1


@pytest.mark.parametrize("maker,eps", [(odd_fc, 0.02), (tiny_conv, 0.05), (mid_resnet, 0.005), (lenet_like, 0.03)])
def test_float64_storage_with_early_termination_and_float_inference(maker, eps):
    net = maker(2)
    c = np.random.default_rng(6).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.set_coefficient_storage(64)
    g.set_early_termination(True)
    g.analyze(c, eps)
    check_early(net, g, c, eps, what=net.name + " early, float64 storage", samples=300, seed=1)
    g.set_early_termination(False)
    g.set_float_inference(True)
    g.analyze(c, eps)
    from parity import compare_layer, float_inference_layers
    o = make_oracle(net)
    o.set_float_inference(True)
    oracle_with_gpu_ties(net, o, g, c, eps, extra_layers=float_inference_layers(net))
    for lid in sorted(set(analysed_layers(net)) | set(float_inference_layers(net))):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = g.get_bounds_f64(lid)
        compare_layer(glo, ghi, olo, ohi, f"{net.name} layer {lid}")


def test_config1_sampled_neurons_in_float64_storage():
    """FC 9x500, 4 inputs batched: every layer's bounds against the oracle with the GPU's relaxation.  The slack of a
    crossing is (K + 8) * 2^-50 per unit of |coefficient| * |neuron|, and the interval widths of this random network
    grow about 25-fold per layer, so the bar here is 1e-7 (measured: 1.4e-9 at worst)."""
    net = wl.config(1)
    g = make_gpu(net)
    g.set_coefficient_storage(64)
    centers = np.stack([net.center(j) for j in range(4)])
    g.analyze_batch(centers, net.eps)
    o = make_oracle(net)
    oracle_with_gpu_relaxation(net, o, g, centers[3], net.eps, batch_index=3)
    for lid in layers_of(net):
        olo, ohi = o.get_bounds(lid)
        glo, ghi = g.get_bounds_f64(lid, 3)
        d = max(np.max((olo - glo) / (1 + np.abs(olo))), np.max((ghi - ohi) / (1 + np.abs(ohi))))
        v = max(np.max((glo - olo) / (1 + np.abs(olo))), np.max((ohi - ghi) / (1 + np.abs(ohi))))
        assert d <= 1e-7 and v <= 1e-12, (lid, d, v)


def _strip5_conv(seed=0):
    from test_gpu_parity import strip5_conv
    return strip5_conv(seed)


@pytest.mark.parametrize("maker,eps,batch", [(strip_conv, 0.004, 2), (_strip5_conv, 0.002, 2), (lambda s: wl.config(2), 2.0 / 255.0, 3),
                                             (lambda s: wl.config(3), 1.0 / 255.0, 1), (lambda s: wl.scaled_resnet(8, 16), 0.002, 2),
                                             (lambda s: wl.lenet_pool(), 1.0 / 255.0, 1)])
def test_float32_storage_tracks_float64_storage(maker, eps, batch):
    """The narrow-layer kernels (direct MFMA, one lane per pixel, strips of pixels) exist for float32 storage only; the
    float64 storage runs every layer through the general kernel and is within 1e-9 of the oracle.  So the float32
    results must contain the float64 results (up to what slightly different slopes do: the float32 intervals are wider
    by their slack, the slopes follow) and exceed them by no more than the float32 slack, which grows with depth (measured:
    3e-6 on three-layer networks, 3e-5 on the deep ones; bar 2e-4): a check of those kernels at full size, several times
    tighter than the 1e-3 bar and without the oracle's run time."""
    net = maker(1)
    centers = np.stack([np.random.default_rng(50 + j).random(net.n_in).astype(np.float32) for j in range(batch)])
    g64 = make_gpu(net)
    g64.set_coefficient_storage(64)
    g64.analyze_batch(centers, eps)
    g32 = make_gpu(net)
    g32.analyze_batch(centers, eps)
    worst = 0.0
    for b in range(batch):
        assert same_lower_lines(net, g32, g64, b), "a tie of the lower-line choice fell differently: pick another seed"
        for lid in layers_of(net):
            lo64, hi64 = g64.get_bounds_f64(lid, b)
            lo32, hi32 = g32.get_bounds_f64(lid, b)
            s_lo, s_hi = 1 + np.abs(lo64), 1 + np.abs(hi64)
            loose = max(np.max((lo64 - lo32) / s_lo), np.max((hi32 - hi64) / s_hi))
            inside = max(np.max((lo32 - lo64) / s_lo), np.max((hi64 - hi32) / s_hi))
            worst = max(worst, loose)
            assert loose <= 2e-4, f"{net.name} box {b} layer {lid}: float32 storage looser than float64 storage by {loose:.3e}"
            assert inside <= 1e-5, f"{net.name} box {b} layer {lid}: float32 storage inside float64 storage by {inside:.3e}"
    print(net.name, "float32 vs float64 storage: worst", worst)
