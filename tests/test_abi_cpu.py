"""Host-side checks of the HIP library that need no GPU: it loads, exports every declared symbol,
validates arguments, and plans dependence windows as the paper's formulas say."""
import ctypes as C
import json
import os
import re

import numpy as np
import pytest
import torch

import workloads as wl
from paper_2007_10868_amd import GpuPolyError, Net, lib_path, load_library
from paper_2007_10868_amd.gpupoly import EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "gpupoly.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(gp_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(EXPORTS), declared ^ set(EXPORTS)
    lib = C.CDLL(lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert b"gfx950" in load_library().gp_version()


def test_dependence_window_example_of_the_paper():
    """Section 4.3: W^1 = 3, W^2 = 4 for the 3x3 then 2x2 filters of the figure of Section 3.1."""
    g = json.load(open(os.path.join(GOLD, "dependence_window_example.json")))
    (h0, w0, c0) = g["layer_shapes_hwc"][0]
    n = Net(c0, h0, w0)
    cur = 0
    cin = c0
    for f, s, shp in zip(g["filters"], g["strides"], g["layer_shapes_hwc"][1:]):
        cur = n.add_conv2d(cur, np.ones((shp[2], cin, f, f), np.float32), None, s, 0)
        cin = shp[2]
        assert n.layer_size(cur) == shp[0] * shp[1] * shp[2]
    plan = n.debug_plan(cur)
    wins = [(p["window_h"], p["window_w"], p["channels"]) for p in plan if p["kind"] in (0, 1)]
    assert wins[0] == (g["W0"], g["W0"], 2)
    assert wins[1] == (g["W1"], g["W1"], 2) and wins[1][0] * wins[1][1] * wins[1][2] == g["size1"]
    assert wins[2] == (g["W2"], g["W2"], 2) and wins[2][0] * wins[2][1] * wins[2][2] == g["size2"]
    assert all(p["acc_stride_h"] == 1 for p in plan)


def test_window_recurrence_with_stride_and_padding():
    """W' = (W-1)*s + f (eq. 4) and accumulated stride S' = s*S (eq. 9), clipped to the layer."""
    net = wl.config(3)
    g = Net(*net.input_shape)
    wl.build_into(net, g)
    # start at the last conv (layer 11: 64x8x8 after two stride-2 convs)
    plan = [p for p in g.debug_plan(11) if p["kind"] in (0, 1)]
    W, S = 1, 1
    convs = [L for L in net.layers[:11] if L["type"] == "conv"][::-1]
    assert plan[0]["window_h"] == 1
    for p, L in zip(plan[1:], convs):
        W = (W - 1) * L["stride"] + L["W"].shape[2]
        S *= L["stride"]
        H = net.shape_of(L["src"])[1]
        assert p["window_h"] == min(W, H), (p, W, H)
        if W < H:
            assert p["acc_stride_h"] == S
    assert plan[-1]["channels"] == 3


def test_average_pooling_plans_like_a_convolution_with_the_same_window():
    """The dependence window of a row grows through a pooling layer as through a convolution (eq. 4: W' = (W-1)*s + f;
    eq. 9: S' = s*S), channels pass through, and rows of a pooling layer itself start from a one-hot block."""
    net = wl.pool_net("p", (3, 32, 32), [("conv", 8, 3, 1, 1), ("pool", 2, 2, 0), ("conv", 16, 3, 1, 0), ("pool", 3, 2, 1)],
                      [20], n_out=5, seed=0)
    g = Net(*net.input_shape)
    wl.build_into(net, g)
    assert [g.layer_size(i) for i in (3, 6)] == [8 * 16 * 16, 16 * 7 * 7]
    plan = [p for p in g.debug_plan(6) if p["kind"] in (0, 1)]           # rows of the second pooling layer
    assert (plan[0]["layer"], plan[0]["window_h"], plan[0]["channels"]) == (6, 1, 16)
    W, S = 1, 1
    expect = []
    for lid in (6, 4, 3, 1):
        L = net.layers[lid - 1]
        k = L["kernel"] if L["type"] == "avgpool" else L["W"].shape[2]
        W, S = (W - 1) * L["stride"] + k, S * L["stride"]
        expect.append((lid, W, S, net.shape_of(L["src"])[0]))
    got = [(p["layer"], p["window_h"], p["acc_stride_h"], p["channels"]) for p in plan[1:]]
    assert got == expect == [(6, 3, 2, 16), (4, 5, 2, 8), (3, 10, 4, 8), (1, 12, 4, 3)]
    with pytest.raises(GpuPolyError) as e:
        g.add_avgpool2d(7, 2)                               # layer 7 is 20x1x1: window larger than the input
    assert e.value.status == 2
    with pytest.raises(GpuPolyError) as e:
        g.add_avgpool2d(2, 2, 1, 2)                         # padding as large as the window
    assert e.value.status == 2
    with pytest.raises(GpuPolyError) as e:
        g.add_avgpool2d(2, 0)
    assert e.value.status == 1


def test_residual_plan_merges_branches():
    net = wl.scaled_resnet(8, 16)
    g = Net(*net.input_shape)
    wl.build_into(net, g)
    adds = [i for i, L in enumerate(net.layers, start=1) if L["type"] == "add"]
    plan = g.debug_plan(adds[1])
    kinds = [p["kind"] for p in plan]
    assert kinds.count(3) == 2                      # forks at both sum layers on the way down
    assert sum(p["merged"] for p in plan) == 2      # ... and both are joined again at the block heads
    assert plan[-1]["layer"] == 1 and plan[-1]["channels"] == 3
    mn, full = g.workspace_size(1)
    assert 0 < mn <= full


def test_argument_errors():
    n = Net(4, 1, 1)
    with pytest.raises(GpuPolyError) as e:
        n.add_dense(3, np.zeros((2, 4), np.float32))
    assert e.value.status == 1
    with pytest.raises(GpuPolyError) as e:
        n.add_dense(0, np.full((2, 4), np.nan, np.float32))
    assert e.value.status == 6
    a = n.add_dense(0, np.zeros((3, 4), np.float32))
    b = n.add_dense(0, np.zeros((2, 4), np.float32))
    with pytest.raises(GpuPolyError) as e:
        n.add_residual(a, b)
    assert e.value.status == 2
    with pytest.raises(GpuPolyError) as e:
        n.get_bounds(a)                                   # nothing analysed yet
    assert e.value.status == 3
    with pytest.raises(GpuPolyError) as e:
        n.analyze(np.zeros(4, np.float32), -1.0)
    assert e.value.status == 1
    with pytest.raises(GpuPolyError) as e:
        n.analyze_box(np.ones(4, np.float32), np.zeros(4, np.float32))
    assert e.value.status == 1
    with pytest.raises(GpuPolyError) as e:
        n.analyze(np.array([0, np.inf, 0, 0], np.float32), 0.1)
    assert e.value.status == 6
    m = Net(2, 4, 4)
    with pytest.raises(GpuPolyError) as e:
        m.add_conv2d(0, np.zeros((2, 2, 7, 7), np.float32), None, 1, 0)   # kernel larger than the input
    assert e.value.status == 2
    lib = load_library()
    assert lib.gp_net_create(0, 1, 1, C.byref(C.c_void_p())) == 1
    assert lib.gp_num_layers(None) == -1


def test_layers_beyond_the_32_bit_offsets_of_the_kernels_are_refused():
    """The crossing kernels address a layer's weights (also their float64 copy) through 32-bit byte offsets: a layer of
    2^28 weights or more is an error at construction, before a single weight is read."""
    lib = load_library()
    h = C.c_void_p()
    assert lib.gp_net_create(1 << 14, 1, 1, C.byref(h)) == 0
    dummy = (C.c_float * 4)()
    lid = C.c_int32(-1)
    assert lib.gp_add_dense(h, 0, 1 << 14, dummy, None, C.byref(lid)) == 2
    assert b"2^28" in lib.gp_last_error(h)
    lib.gp_net_destroy(h)
    assert lib.gp_net_create(1 << 13, 4, 4, C.byref(h)) == 0
    assert lib.gp_add_conv2d(h, 0, 1 << 12, 3, 3, 1, 1, 1, 1, dummy, None, C.byref(lid)) == 2     # 2^13 * 2^12 * 9 weights
    lib.gp_net_destroy(h)


def test_allocation_free_call_refuses_rows_beyond_its_static_workspace_from_the_topology_alone():
    big = wl.Net("big_rows", (1, 1200, 1200))
    r1 = big.relu(big.conv(0, np.ones((2, 1, 1, 1), np.float32), np.zeros(2, np.float32), 1, 0))
    big.dense(r1, np.zeros((2, 2 * 1200 * 1200), np.float32), np.zeros(2, np.float32))
    g = Net(*big.input_shape)
    wl.build_into(big, g)
    lib = load_library()
    fake = C.c_void_p(256)          # never dereferenced: the call fails while it sizes the plans
    assert lib.gp_analyze_batch_dev_static(g._h, 1, fake, 0.01, 0.0, 1.0, fake, fake) == 7
    assert b"static workspace" in lib.gp_last_error(g._h)
    assert lib.gp_analyze_batch_dev_static(g._h, 0, fake, 0.01, 0.0, 1.0, fake, fake) == 1
    assert lib.gp_analyze_batch_dev_static(g._h, 1, fake, 0.01, 0.0, 1.0, None, fake) == 1


def test_unsupported_topology_is_reported_not_guessed():
    n = Net(4, 1, 1)
    a = n.add_dense(0, np.eye(4, dtype=np.float32))
    r = n.add_relu(a)
    s = n.add_residual(r, r)                # x + x
    n.add_dense(s, np.eye(4, dtype=np.float32))
    with pytest.raises(GpuPolyError) as e:
        n.debug_plan(4)
    assert e.value.status == 8


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful without a GPU")
def test_no_gpu_is_an_error_not_a_fallback():
    n = Net(4, 1, 1)
    n.add_dense(0, np.eye(4, dtype=np.float32))
    with pytest.raises(GpuPolyError) as e:
        n.analyze(np.zeros(4, np.float32), 0.1)
    assert e.value.status == 5


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: asking the benchmark for more must end with a message, not with a number."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_early_termination_calls_without_analysis():
    g = Net(4)
    g.add_dense(0, np.ones((3, 4), np.float32))
    g.set_early_termination(True)
    with pytest.raises(GpuPolyError) as e:
        g.get_term_layer(1)
    assert e.value.status == 3          # GP_ERR_STATE: nothing analysed yet
    with pytest.raises(GpuPolyError):
        g.early_termination_stats()
    g.set_early_termination(False)
