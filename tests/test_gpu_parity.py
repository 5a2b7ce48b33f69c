"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on
the same seeded inputs; plus soundness by sampling and the library's own edge cases.

Bar (stated by the benchmark spec): every GPU interval contains every sampled concrete output and the
oracle's interval, and is looser than the oracle's by at most 1e-3 * (1 + |b|)."""
import ctypes as C
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import ball_box, forward
from parity import (REL_TOL, STRICT_CONTAIN_TOL, analysed_layers, check_samples_inside, clear_overrides, compare_all,
                    compare_layer, make_gpu, make_oracle, oracle_with_gpu_relaxation, oracle_with_gpu_ties)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    torch.cuda.init()


def tiny_fc(seed=0):
    return wl.fc_net("tiny_fc", [6, 6], n_in=4, n_out=3, seed=seed)


def odd_fc(seed=0):          # widths that are no multiple of 4: scalar load paths, ragged tiles
    return wl.fc_net("odd_fc", [37, 101, 19], n_in=23, n_out=7, seed=seed)


def quad_fc(seed=0):         # widths = 4, 8, 12 (mod 16): every length of the transposed last K tile of dense layers
    return wl.fc_net("quad_fc", [24, 28, 40, 20, 52], n_in=36, n_out=8, seed=seed)


def tiny_conv(seed=0):       # channel counts 2,3,4: unaligned paths; stride 2 with an even kernel
    return wl.conv_net("tiny_conv", (2, 6, 6), [(3, 3, 1, 1), (4, 4, 2, 1)], [8], n_out=3, seed=seed)


def pad0_conv(seed=0):       # no padding, window never clipped before it covers the layer
    return wl.conv_net("pad0_conv", (1, 12, 12), [(4, 3, 1, 0), (8, 3, 2, 0), (8, 2, 1, 0)], [16], n_out=5, seed=seed)


def tiny_resnet(seed=0):
    return wl.resnet("tiny_res", (2, 8, 8), channels=(3, 4), blocks=(2, 1), n_out=3, seed=seed)


def mid_resnet(seed=0):      # 16x16, two stages, identity and 1x1-stride-2 shortcuts, several M tiles
    return wl.resnet("mid_res", (3, 16, 16), channels=(8, 16), blocks=(2, 2), n_out=10, seed=seed)


def strip_conv(seed=0):
    """Wide layers (32 and 16 channels) behind a 3-channel image, 3x3 stride-1 filters, a rectangular image whose width
    is no multiple of 8: the narrow-layer kernels (direct MFMA, strip of output pixels) with ragged strips and borders."""
    return wl.conv_net("strip_conv", (3, 7, 11), [(32, 3, 1, 1), (16, 3, 1, 1), (32, 3, 1, 0)], [12], n_out=4, seed=seed)


def strip5_conv(seed=0):
    """The same with 5x5 filters (the other filter width the strip kernel is built for)."""
    return wl.conv_net("strip5_conv", (3, 9, 13), [(32, 5, 1, 2), (16, 5, 1, 2), (32, 5, 1, 0)], [12], n_out=4, seed=seed)


def rect_conv(seed=0):
    """Rectangular image, kh != kw, stride_h != stride_w, pad_h != pad_w."""
    rng = np.random.default_rng(seed)
    net = wl.Net("rect", (3, 9, 14))

    def cv(src, co, kh, kw):
        ci = net.shape_of(src)[0]
        W = (rng.standard_normal((co, ci, kh, kw)) * np.sqrt(2.0 / (ci * kh * kw))).astype(np.float32)
        b = (rng.standard_normal(co) * 0.1).astype(np.float32)
        return W, b
    # Net.conv only knows square strides/pads: describe the layers by hand
    W, b = cv(0, 5, 3, 2)
    net.layers.append(dict(type="conv", src=0, W=W, b=b, stride=(1, 2), pad=(1, 0), shape=(5, 9, 7)))
    net.layers.append(dict(type="relu", src=1, shape=(5, 9, 7)))
    W, b = cv(2, 6, 2, 3)
    net.layers.append(dict(type="conv", src=2, W=W, b=b, stride=(2, 1), pad=(0, 1), shape=(6, 4, 7)))
    net.layers.append(dict(type="relu", src=3, shape=(6, 4, 7)))
    W = (rng.standard_normal((4, 6 * 4 * 7)) * 0.1).astype(np.float32)
    net.layers.append(dict(type="dense", src=4, W=W, b=np.zeros(4, np.float32), shape=(4, 1, 1)))
    return net


def run_pair(net, center, eps, clip=(0.0, 1.0)):
    g = make_gpu(net)
    g.analyze(center, eps, clip[0], clip[1])
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, center, eps, clip=clip)
    return g, o


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cols", [16, 4])
def test_mfma_f64_error_model(cols):
    """The crossing kernel's slack assumes |MFMA sum - exact sum| <= (K+8) * 2^-50 * sum|terms|, for the 16-column
    instruction and for the 4-column one.  Checked against exact rational arithmetic on float32-valued operands with
    heavy cancellation."""
    from paper_2007_10868_amd import load_library
    lib = load_library()
    rng = np.random.default_rng(0)
    K = 512
    A = (rng.standard_normal((16, K)) * np.exp2(rng.integers(-20, 20, (16, K)))).astype(np.float32).astype(np.float64)
    B = rng.standard_normal((K, cols)).astype(np.float32).astype(np.float64)
    A[:, 1::2] = -A[:, 0::2]           # cancellation
    B[1::2, :] = B[0::2, :] * (1 + 2.0 ** -20)
    B = B.astype(np.float32).astype(np.float64)
    tA, tB = torch.tensor(A, device="cuda"), torch.tensor(B, device="cuda")
    tD = torch.zeros(16, cols, dtype=torch.float64, device="cuda")
    fn = lib.gp_debug_mfma_f64 if cols == 16 else lib.gp_debug_mfma_f64_4col
    st = fn(C.c_void_p(tA.data_ptr()), C.c_void_p(tB.data_ptr()), C.c_void_p(tD.data_ptr()), K,
                               C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    torch.cuda.synchronize()
    D = tD.cpu().numpy()
    worst = 0.0
    for i in range(16):
        for j in range(0, cols, 5 if cols == 16 else 1):
            terms = [Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(K)]
            exact = sum(terms)
            mag = sum(abs(t) for t in terms)
            err = abs(Fraction(float(D[i, j])) - exact)
            assert err <= Fraction((K + 8) * 2.0 ** -50) * mag, (i, j, float(err), float(mag))
            worst = max(worst, float(err / mag))
    # plain layout check against NumPy as well
    assert np.allclose(D, A @ B, rtol=0, atol=1e-9 * np.abs(A).max())
    print("worst |err|/sum|terms| =", worst)


@pytest.mark.parametrize("maker,eps", [(tiny_fc, 0.1), (odd_fc, 0.05), (quad_fc, 0.03), (tiny_conv, 0.05), (pad0_conv, 0.03),
                                       (tiny_resnet, 0.02), (mid_resnet, 0.01), (rect_conv, 0.04), (strip_conv, 0.004), (strip5_conv, 0.002)])
def test_small_networks_match_oracle_and_contain_samples(maker, eps):
    net = maker(1)
    rng = np.random.default_rng(5)
    c = rng.random(net.n_in).astype(np.float32)
    g, o = run_pair(net, c, eps)
    worst = compare_all(net, g, o, what=net.name)
    compare_all(net, g, o, what=net.name + " (float32 output)", f64=False)
    lo0, hi0 = ball_box(c, eps)
    check_samples_inside(net, g, lo0, hi0, 20_000, rng, what=net.name)
    n_uns = sum(int(np.sum((o.get_bounds(l)[0] < 0) & (o.get_bounds(l)[1] > 0))) for l in analysed_layers(net))
    assert n_uns > 0
    print(net.name, "worst looseness / allowed =", worst)
    # same relaxation parameters on both sides: the GPU intervals must contain the oracle's, strictly
    oracle_with_gpu_relaxation(net, o, g, c, eps)
    compare_all(net, g, o, what=net.name + " (GPU slopes)", contain_tol=STRICT_CONTAIN_TOL)


SMALL_NETS = [(tiny_fc, 0.1), (odd_fc, 0.05), (quad_fc, 0.03), (tiny_conv, 0.05), (pad0_conv, 0.03), (tiny_resnet, 0.02),
              (mid_resnet, 0.01), (rect_conv, 0.04), (strip_conv, 0.004), (strip5_conv, 0.002)]


@pytest.mark.parametrize("maker,eps", SMALL_NETS)
def test_small_networks_match_the_literal_interval_coefficient_oracle(maker, eps):
    """The same comparison against the oracle in the paper's literal scheme (Section 4.1: every coefficient stays an
    interval until the end of the back-substitution, nothing is re-centred on the way).  On networks of this depth the
    two oracle modes agree to rounding noise, so the library must meet the same bar against either."""
    net = maker(1)
    c = np.random.default_rng(5).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, eps)
    o = make_oracle(net)
    o.set_collapse(False)
    oracle_with_gpu_ties(net, o, g, c, eps)
    worst = compare_all(net, g, o, what=net.name + " (literal oracle)")
    print(net.name, "against the literal oracle: worst looseness / allowed =", worst)


@pytest.mark.parametrize("cfg,inputs", [(0, (0, 9)), (1, (0,)), (2, (0,))])
def test_configs_match_the_literal_interval_coefficient_oracle(cfg, inputs):
    """Configurations FC 6x100, FC 9x500 and small conv against the literal scheme of Section 4.1."""
    net = wl.config(cfg)
    g = make_gpu(net)
    o = make_oracle(net)
    o.set_collapse(False)
    for j in inputs:
        c = net.center(j)
        g.analyze(c, net.eps)
        oracle_with_gpu_ties(net, o, g, c, net.eps)
        worst = compare_all(net, g, o, what=f"{net.name} input {j} (literal oracle)")
        print(net.name, "input", j, "against the literal oracle: worst looseness / allowed =", worst)


def test_failed_allocation_at_a_larger_batch_leaves_the_net_usable():
    """A batch whose per-layer arrays do not fit the device fails with GP_ERR_NOMEM; the next analysis at the earlier
    batch size must allocate afresh and give the same bits as before (no kernel ever runs on freed or missing arrays)."""
    from paper_2007_10868_amd import GpuPolyError, load_library
    net = odd_fc(2)
    c = np.random.default_rng(9).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, 0.02)
    ref = {l: g.get_bounds_f64(l) for l in analysed_layers(net)}
    lib = load_library()
    huge = 1 << 28                      # 101 neurons x 2^28 boxes x 8 bytes = 217 GB per array: the second one cannot fit
    one_center = torch.zeros(net.n_in, dtype=torch.float32, device="cuda")
    # (the library fails while sizing its arrays, before it reads a single centre)
    st = lib.gp_analyze_batch_dev(g._h, huge, C.c_void_p(one_center.data_ptr()), 0.02, 0.0, 1.0)
    assert st == 4, st
    with pytest.raises(GpuPolyError) as e:
        g.get_bounds_f64(net.out_layer)
    assert e.value.status == 3          # no successful analysis any more
    g.analyze(c, 0.02)
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l)
        assert np.array_equal(lo, ref[l][0]) and np.array_equal(hi, ref[l][1]), l


def test_config0_fc6x100_all_inputs_and_certify():
    net = wl.config(0)
    g = make_gpu(net)
    o = make_oracle(net)
    rng = np.random.default_rng(0)
    for j in range(net.n_inputs):
        c = net.center(j)
        g.analyze(c, net.eps)
        oracle_with_gpu_ties(net, o, g, c, net.eps)
        compare_all(net, g, o, what=f"fc6x100 input {j}")
        y = forward(net, c[None, :].astype(np.float64))[net.out_layer][0]
        label = int(np.argmax(y))
        ok_g, m_g = g.certify(label)
        ok_o, m_o = o.certify(label)
        compare_layer(m_g, m_g, m_o, m_g, f"fc6x100 input {j} margins")      # lower ends only
        assert np.all(m_g.astype(np.float64) <= m_o + 2e-6 * (1 + np.abs(m_o)))
        assert ok_g == bool(np.all(m_g > 0))
        if ok_g:
            assert ok_o
        if j == 0:
            lo0, hi0 = ball_box(c, net.eps)
            check_samples_inside(net, g, lo0, hi0, 5_000, rng, what="fc6x100")


def test_config1_fc9x500_single_and_batched():
    net = wl.config(1)
    g = make_gpu(net)
    o = make_oracle(net)
    centers = np.stack([net.center(j) for j in range(4)])
    g.analyze(centers[0], net.eps)
    single = {l: g.get_bounds_f64(l) for l in analysed_layers(net)}
    oracle_with_gpu_ties(net, o, g, centers[0], net.eps)
    worst = compare_all(net, g, o, what="fc9x500 input 0")
    print("fc9x500 worst looseness / allowed =", worst)
    # the batched pass must give, for every box, what the single pass gives (same kernels, same order)
    g.analyze_batch(centers, net.eps)
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l, 0)
        assert np.array_equal(lo, single[l][0]) and np.array_equal(hi, single[l][1]), l
    oracle_with_gpu_ties(net, o, g, centers[3], net.eps, batch_index=3)
    compare_all(net, g, o, batch_index=3, what="fc9x500 input 3 (batched)")
    # device-resident centres
    t = torch.tensor(centers, device="cuda")
    g.analyze_batch_dev(t, net.eps)
    lo, hi = g.get_bounds_f64(net.out_layer, 3)
    olo, ohi = o.get_bounds(net.out_layer)
    compare_layer(lo, hi, olo, ohi, "fc9x500 device centres")


def test_config1_in_the_benchmark_launch_configuration():
    """The workload exactly as bench.py times it: all 100 inputs of FC 9x500 in one batched pass, centres resident on
    the device, workspace from a torch tensor sized the way bench.py sizes it.  Full oracle parity on three of the
    inputs, bit-equality with a single-input pass, sampled outputs for every tenth input."""
    net = wl.config(1)
    batch = net.n_inputs
    g = make_gpu(net)
    centers = np.stack([net.center(j) for j in range(batch)])
    t = torch.tensor(centers, device="cuda")
    g.set_stream(torch.cuda.current_stream())
    _, full = g.workspace_size(batch)
    free, _ = torch.cuda.mem_get_info()
    ws = torch.empty(int(min(full, free * 0.6)), dtype=torch.uint8, device="cuda")
    g.set_workspace(ws)
    g.analyze_batch_dev(t, net.eps)
    o = make_oracle(net)
    for b in (0, 57, 99):
        oracle_with_gpu_ties(net, o, g, centers[b], net.eps, batch_index=b)
        compare_all(net, g, o, batch_index=b, what=f"fc9x500 x100, input {b}")
    rng = np.random.default_rng(3)
    for b in range(0, batch, 10):
        lo0, hi0 = ball_box(centers[b], net.eps)
        check_samples_inside(net, g, lo0, hi0, 200, rng, batch_index=b, what=f"fc9x500 x100, input {b}")
    batched = {l: g.get_bounds_f64(l, 57) for l in analysed_layers(net)}
    g1 = make_gpu(net)
    g1.analyze(centers[57], net.eps)
    for l in analysed_layers(net):
        lo, hi = g1.get_bounds_f64(l)
        assert np.array_equal(lo, batched[l][0]) and np.array_equal(hi, batched[l][1]), l


def test_config2_small_conv():
    net = wl.config(2)
    g = make_gpu(net)
    o = make_oracle(net)
    rng = np.random.default_rng(1)
    for j in (0, 7):
        c = net.center(j)
        g.analyze(c, net.eps)
        oracle_with_gpu_ties(net, o, g, c, net.eps)
        worst = compare_all(net, g, o, what=f"conv_small input {j}")
    lo0, hi0 = ball_box(c, net.eps)
    check_samples_inside(net, g, lo0, hi0, 2_000, rng, what="conv_small")
    print("conv_small worst looseness / allowed =", worst)


@pytest.mark.parametrize("make, rows", [(mid_resnet, 37), (strip_conv, 37), (strip_conv, 200), (strip5_conv, 37), (strip5_conv, 200)])
def test_row_chunking_gives_identical_bounds(make, rows):
    """A workspace that holds only a few rows forces the chunked path (Section 4.2, memory management).  Which
    crossing kernel a chunk gets may depend on how its rows are aligned; the bounds may not."""
    net = make(3)
    c = np.random.default_rng(2).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, 0.01)
    ref = {l: g.get_bounds_f64(l) for l in analysed_layers(net)}
    mn, full = g.workspace_size(1)
    small = torch.empty(mn * rows + 4096, dtype=torch.uint8, device="cuda")   # a few rows at a time: ragged chunks
    assert small.numel() < full
    g.set_workspace(small)
    g.analyze(c, 0.01)
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l)
        assert np.array_equal(lo, ref[l][0]) and np.array_equal(hi, ref[l][1]), l
    g.set_workspace(torch.empty(1024, dtype=torch.uint8, device="cuda"))
    from paper_2007_10868_amd import GpuPolyError
    with pytest.raises(GpuPolyError) as e:
        g.analyze(c, 0.01)
    assert e.value.status == 7
    g.set_workspace(None)
    g.analyze(c, 0.01)                     # still usable after the failure
    assert np.array_equal(g.get_bounds_f64(net.out_layer)[0], ref[net.out_layer][0])


def test_batched_conv_matches_single_and_certify_batch():
    net = wl.config(2)
    g = make_gpu(net)
    centers = np.stack([net.center(j) for j in range(3)])
    g.analyze_batch(centers, net.eps)
    batched = [g.get_bounds_f64(net.out_layer, b) for b in range(3)]
    labels = [int(np.argmax((lo + hi) / 2)) for lo, hi in batched]
    ok_b, m_b = g.certify_batch(labels)
    for b in range(3):
        g.analyze(centers[b], net.eps)
        lo, hi = g.get_bounds_f64(net.out_layer)
        assert np.array_equal(lo, batched[b][0]) and np.array_equal(hi, batched[b][1])
        ok, m = g.certify(labels[b])
        assert np.array_equal(m, m_b[b]) and ok == ok_b[b]
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, centers[2], net.eps)
    _, m_o = o.certify(labels[2])
    assert np.all(m_b[2] <= m_o + 2e-6 * (1 + np.abs(m_o)))
    assert np.all(m_o - m_b[2] <= REL_TOL * (1 + np.abs(m_o)))


def test_stream_and_workspace_from_torch():
    net = tiny_conv(2)
    c = np.random.default_rng(3).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, 0.05)
    ref = g.get_bounds_f64(net.out_layer)
    s = torch.cuda.Stream()
    g.set_stream(s)
    _, full = g.workspace_size(1)
    g.set_workspace(torch.empty(full, dtype=torch.uint8, device="cuda"))
    g.analyze(c, 0.05)
    got = g.get_bounds_f64(net.out_layer)
    assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])


def test_degenerate_cases():
    # eps = 0: every interval collapses onto the concrete forward pass
    net = tiny_resnet(4)
    c = np.random.default_rng(4).random(net.n_in).astype(np.float32)
    g = make_gpu(net)
    g.analyze(c, 0.0)
    vals = forward(net, c[None, :].astype(np.float64))
    for l in analysed_layers(net):
        lo, hi = g.get_bounds_f64(l)
        v = vals[l][0]
        assert np.all(lo <= v) and np.all(v <= hi)
        assert np.max(hi - lo) < 1e-5 * (1 + np.max(np.abs(v)))
    # a single affine layer: closed form of the first layer
    one = wl.fc_net("one", [], n_in=9, n_out=4, seed=3)
    g1 = make_gpu(one)
    x = np.random.default_rng(1).random(9).astype(np.float32)
    g1.analyze(x, 0.25, -5.0, 5.0)
    W, b = one.layers[0]["W"].astype(np.float64), one.layers[0]["b"].astype(np.float64)
    lo0, hi0 = ball_box(x, 0.25, -5.0, 5.0)
    l_ref = np.maximum(W, 0) @ lo0 + np.minimum(W, 0) @ hi0 + b
    u_ref = np.maximum(W, 0) @ hi0 + np.minimum(W, 0) @ lo0 + b
    lo, hi = g1.get_bounds_f64(1)
    assert np.all(lo <= l_ref) and np.all(hi >= u_ref)
    assert np.max(l_ref - lo) < 1e-6 and np.max(hi - u_ref) < 1e-6
    # the box is clipped: centre at the clip end, huge eps
    g1.analyze(np.ones(9, np.float32), 100.0, 0.0, 1.0)
    lo, hi = g1.get_bounds_f64(0)
    assert np.all(lo == 0.0) and np.all(hi == 1.0)
    # explicit box
    g1.analyze_box(lo0.astype(np.float32) - 1e-3, hi0.astype(np.float32) + 1e-3)
    lo, hi = g1.get_bounds_f64(1)
    assert np.all(lo <= l_ref) and np.all(hi >= u_ref)


def test_overflow_is_reported():
    """Bounds beyond the float64 range are an error, never a number.  (A float32 overflow of single
    coefficients only loses the later candidates: the earlier ones stay valid and finite.)"""
    from paper_2007_10868_amd import GpuPolyError
    net = wl.fc_net("big", [8] * 10, n_in=4, n_out=2, seed=0)
    for L in net.layers:
        if L["type"] == "dense":
            L["W"] = (L["W"] * np.float32(1e36)).astype(np.float32)
    g = make_gpu(net)
    with pytest.raises(GpuPolyError) as e:
        g.analyze(np.full(4, 0.5, np.float32), 0.1)
    assert e.value.status == 6
    mild = wl.fc_net("mild", [8, 8, 8], n_in=4, n_out=2, seed=0)
    for L in mild.layers:
        if L["type"] == "dense":
            L["W"] = (L["W"] * np.float32(1e30)).astype(np.float32)
    g = make_gpu(mild)
    c = np.full(4, 0.5, np.float32)
    g.analyze(c, 0.1)                       # coefficients overflow float32 on the way down
    lo0, hi0 = ball_box(c, 0.1)
    check_samples_inside(mild, g, lo0, hi0, 2_000, np.random.default_rng(0), what="mild overflow")


def test_config3_deep_conv_one_input():
    """~150k neurons, windows that grow until they cover the image, stride-2 layers, 4096->512 dense head."""
    net = wl.config(3)
    g = make_gpu(net)
    o = make_oracle(net)
    c = net.center(0)
    g.analyze(c, net.eps)
    forced = oracle_with_gpu_ties(net, o, g, c, net.eps)
    worst = compare_all(net, g, o, what="conv_deep input 0")
    lo0, hi0 = ball_box(c, net.eps)
    check_samples_inside(net, g, lo0, hi0, 200, np.random.default_rng(3), what="conv_deep")
    print("conv_deep worst looseness / allowed =", worst, "lambda ties forced:", forced)


def stratified_rows(shape, count, rng):
    """Rows (C,H,W-flattened neuron indices) of a layer of the given shape that cover the cases its kernels treat
    differently: the four corners and the edge midpoints (dependence windows clipped and shifted at the borders), the
    positions one step inside a corner, positions of either parity (a stride-2 shortcut reads every other position),
    the centre and random interior positions; at each position the first, the last and a random channel (first and
    last row of a tile, ragged channel tiles).  `count` rows at most, taken round-robin over the positions so that
    a small count still holds every kind."""
    C, H, W = shape
    if C * H * W <= count:
        return np.arange(C * H * W, dtype=np.int32)
    pos = [(0, 0), (0, W - 1), (H - 1, 0), (H - 1, W - 1),                       # corners
           (0, W // 2), (H - 1, W // 2), (H // 2, 0), (H // 2, W - 1),           # edge midpoints
           (min(1, H - 1), min(1, W - 1)), (max(H - 2, 0), max(W - 2, 0)),       # one step inside
           (min(1, H - 1), min(2, W - 1)), (min(2, H - 1), min(1, W - 1)),       # odd/even and even/odd
           (H // 2, W // 2)]
    pos += [(int(rng.integers(0, H)), int(rng.integers(0, W))) for _ in range(3)]
    pos = list(dict.fromkeys(pos))
    rows = []
    for p in range(4):
        for i, (y, x) in enumerate(pos):
            kind = (p + i) % 4          # first channel, last channel, two random ones: every pass mixes the kinds
            c = 0 if kind == 0 else C - 1 if kind == 1 else int(rng.integers(0, C))
            rows.append((c * H + y) * W + x)
    rows = list(dict.fromkeys(rows))[:count]
    return np.sort(np.array(rows, dtype=np.int32))


def _sampled_rows_against_teacher_forced_oracle(net, g, o, c, eps, rows_per_layer, rng, what, batch_index=0):
    """The oracle gets the GPU's intervals of all earlier layers as data (teacher forcing) and bounds a
    stratified sample of rows of each analysed layer on its own; the two must agree to the usual bar."""
    o.set_ball(c, eps)
    worst, n_rows = 0.0, 0
    for lid in range(1, o.num_layers):
        L = net.layers[lid - 1]
        if L["type"] == "relu":
            o.analyze_layer(lid)            # relaxation from the forced intervals of its input
            continue
        if lid not in analysed_layers(net):
            continue
        glo, ghi = g.get_bounds_f64(lid, batch_index)
        rows = stratified_rows(net.shape_of(lid), rows_per_layer, rng)
        olo, ohi = o.bound_rows(lid, rows)
        r, _ = compare_layer(glo[rows], ghi[rows], olo, ohi, f"{what} layer {lid}")
        worst = max(worst, r)
        n_rows += rows.size
        o.set_bounds(lid, glo, ghi)
    return worst, n_rows


def test_scaled_resnet34_full_parity():
    """Same depth and topology as the 34-layer residual configuration, channels / 8, 16x16 input:
    every interval of every analysed layer against the full oracle."""
    net = wl.scaled_resnet(8, 16)
    g = make_gpu(net)
    o = make_oracle(net)
    c = net.center(0)
    g.analyze(c, net.eps)
    forced = oracle_with_gpu_ties(net, o, g, c, net.eps)
    worst = compare_all(net, g, o, what=net.name)
    lo0, hi0 = ball_box(c, net.eps)
    check_samples_inside(net, g, lo0, hi0, 500, np.random.default_rng(4), what=net.name)
    print(net.name, "worst looseness / allowed =", worst, "ties forced:", forced)
    oracle_with_gpu_relaxation(net, o, g, c, net.eps)
    compare_all(net, g, o, what=net.name + " (GPU slopes)", contain_tol=STRICT_CONTAIN_TOL)


@pytest.mark.parametrize("j,rows_per_layer", [(0, 64), (1, 32)])
def test_config4_resnet34_sampled_rows(j, rows_per_layer):
    """The full 1M-neuron configuration: the whole oracle pass would take hours, so a stratified sample of rows
    (corners, edges, interior, first and last channels) of every analysed layer is bounded by the oracle with teacher
    forcing, and every neuron is checked against sampled concrete outputs."""
    net = wl.config(4)
    g = make_gpu(net)
    o = make_oracle(net)
    c = net.center(j)
    g.analyze(c, net.eps)
    rng = np.random.default_rng(5 + j)
    worst, n_rows = _sampled_rows_against_teacher_forced_oracle(net, g, o, c, net.eps, rows_per_layer, rng, f"resnet34 input {j}")
    lo0, hi0 = ball_box(c, net.eps)
    check_samples_inside(net, g, lo0, hi0, 64, rng, what="resnet34")
    print(f"resnet34 input {j}: {n_rows} sampled rows, worst looseness / allowed = {worst}")


def _workspace_like_bench(g, batch):
    g.set_stream(torch.cuda.current_stream())
    _, full = g.workspace_size(batch)
    free, _ = torch.cuda.mem_get_info()
    ws = torch.empty(int(min(full, free * 0.6)), dtype=torch.uint8, device="cuda")
    g.set_workspace(ws)
    return ws


def test_config2_in_the_benchmark_launch_configuration():
    """Small conv exactly as bench.py times it: all 100 inputs in one batched pass, centres resident on the device,
    workspace from a torch tensor.  Full oracle parity on two of the inputs, sampled outputs on every tenth, and
    bit-equality of a batched result with a single-input pass."""
    net = wl.config(2)
    batch = net.n_inputs
    g = make_gpu(net)
    centers = np.stack([net.center(j) for j in range(batch)])
    ws = _workspace_like_bench(g, batch)
    g.analyze_batch_dev(torch.tensor(centers, device="cuda"), net.eps)
    o = make_oracle(net)
    for b in (3, 99):
        oracle_with_gpu_ties(net, o, g, centers[b], net.eps, batch_index=b)
        compare_all(net, g, o, batch_index=b, what=f"conv_small x100, input {b}")
    rng = np.random.default_rng(8)
    for b in range(0, batch, 10):
        lo0, hi0 = ball_box(centers[b], net.eps)
        check_samples_inside(net, g, lo0, hi0, 200, rng, batch_index=b, what=f"conv_small x100, input {b}")
    batched = {l: g.get_bounds_f64(l, 99) for l in analysed_layers(net)}
    g1 = make_gpu(net)
    g1.analyze(centers[99], net.eps)
    for l in analysed_layers(net):
        lo, hi = g1.get_bounds_f64(l)
        assert np.array_equal(lo, batched[l][0]) and np.array_equal(hi, batched[l][1]), l
    del ws


def test_config3_in_the_benchmark_launch_configuration():
    """Deep conv exactly as bench.py times it: all 20 inputs in one batched pass.  Full oracle parity on one input of
    the batch, a stratified sample of rows per layer (teacher forcing) on another, sampled outputs on four, and
    bit-equality of a batched result with a single-input pass."""
    net = wl.config(3)
    batch = net.n_inputs
    g = make_gpu(net)
    centers = np.stack([net.center(j) for j in range(batch)])
    ws = _workspace_like_bench(g, batch)
    g.analyze_batch_dev(torch.tensor(centers, device="cuda"), net.eps)
    o = make_oracle(net)
    oracle_with_gpu_ties(net, o, g, centers[19], net.eps, batch_index=19)
    worst = compare_all(net, g, o, batch_index=19, what="conv_deep x20, input 19")
    rng = np.random.default_rng(9)
    o2 = make_oracle(net)
    w2, n_rows = _sampled_rows_against_teacher_forced_oracle(net, g, o2, centers[7], net.eps, 64, rng,
                                                             "conv_deep x20, input 7", batch_index=7)
    for b in (0, 7, 13, 19):
        lo0, hi0 = ball_box(centers[b], net.eps)
        check_samples_inside(net, g, lo0, hi0, 100, rng, batch_index=b, what=f"conv_deep x20, input {b}")
    batched = {l: g.get_bounds_f64(l, 7) for l in analysed_layers(net)}
    g1 = make_gpu(net)
    g1.analyze(centers[7], net.eps)
    for l in analysed_layers(net):
        lo, hi = g1.get_bounds_f64(l)
        assert np.array_equal(lo, batched[l][0]) and np.array_equal(hi, batched[l][1]), l
    print("conv_deep x20: worst looseness / allowed =", worst, "; sampled rows:", n_rows, "worst", w2)
    del ws


@pytest.mark.parametrize("maker,eps", [(odd_fc, 0.02), (tiny_conv, 0.05), (mid_resnet, 0.005)])
def test_linear_output_forms(maker, eps):
    """gp_bound_outputs: lower bounds of arbitrary linear forms of the outputs against the oracle's (never above it
    beyond rounding, looser by at most the usual bar), below sampled values, and equal to gp_certify on its rows."""
    net = maker(5)
    rng = np.random.default_rng(31)
    X = rng.random((2, net.n_in)).astype(np.float32)
    g = make_gpu(net)
    g.analyze_batch(X, eps)
    n_out = net.n_neurons(net.out_layer)
    coef = rng.standard_normal((6, n_out)).astype(np.float32)
    coef[1] = 0.0
    off = rng.standard_normal(6).astype(np.float32)
    lb = g.bound_outputs(coef, off, batch=2).astype(np.float64)
    for b in range(2):
        o = make_oracle(net)
        oracle_with_gpu_ties(net, o, g, X[b], eps, batch_index=b)
        ref = o.bound_outputs(coef.astype(np.float64), off.astype(np.float64))
        assert np.all(lb[b] <= ref + 2e-6 * (1 + np.abs(ref))), (b, lb[b], ref)
        assert np.all(ref - lb[b] <= REL_TOL * (1 + np.abs(ref))), (b, lb[b], ref)
        lo0, hi0 = ball_box(X[b], eps)
        from helpers import sample_box
        Y = forward(net, sample_box(lo0, hi0, 500, rng))[net.out_layer]
        assert np.all(Y @ coef.T.astype(np.float64) + off >= lb[b])
    label = 2
    rows = np.array([np.eye(n_out)[label] - np.eye(n_out)[j] for j in range(n_out) if j != label], np.float32)
    _, margins = g.certify_batch([label, label])
    assert np.array_equal(g.bound_outputs(rows, batch=2), margins)
