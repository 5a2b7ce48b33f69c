"""Seeded synthetic networks and input boxes for the DeepPoly back-substitution tests and benchmark.

This module only draws random weights / inputs and lists topologies.  It holds none of the
verifier's arithmetic; both the CPU oracle and the HIP path are fed from it so that they see the
very same arrays.  The five numbered configurations stand in for the paper's MNIST / CIFAR10
workloads (Section 5, Table 1): same input shapes (28x28x1, 32x32x3 images in [0,1]) and the same
families of topology (fully connected, convolutional, residual; 3 K - 1 M neurons), but with
random He-normal weights and uniform random images, because neither the datasets nor the trained
weights are available.

Conventions
  * layer id 0 is the input; every add_* call creates the next id.
  * dense weight: float32 [out, in], `in` is the CHW-flattened predecessor.
  * conv weight : float32 [c_out, c_in, kh, kw]; bias float32 [c_out].
  * "N(0, v)" in the configuration list is read as a variance, so biases have std 0.1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Any, Dict, List, Tuple

import numpy as np


@dataclass
class Net:
    name: str
    input_shape: Tuple[int, int, int]            # (C, H, W); flat inputs are (n, 1, 1)
    layers: List[Dict[str, Any]] = field(default_factory=list)   # layers[i] creates id i+1
    eps: float = 0.0
    n_inputs: int = 1
    input_seed_base: int = 0

    # ---- topology helpers -------------------------------------------------------------
    def shape_of(self, lid: int) -> Tuple[int, int, int]:
        if lid == 0:
            return self.input_shape
        return self.layers[lid - 1]["shape"]

    def _push(self, d: Dict[str, Any]) -> int:
        self.layers.append(d)
        return len(self.layers)

    def dense(self, src: int, W: np.ndarray, b: np.ndarray) -> int:
        return self._push(dict(type="dense", src=src, W=W, b=b, shape=(W.shape[0], 1, 1)))

    def conv(self, src: int, W: np.ndarray, b: np.ndarray, stride: int, pad: int) -> int:
        c, h, w = self.shape_of(src)
        co, ci, kh, kw = W.shape
        assert ci == c
        ho = (h + 2 * pad - kh) // stride + 1
        wo = (w + 2 * pad - kw) // stride + 1
        return self._push(dict(type="conv", src=src, W=W, b=b, stride=stride, pad=pad,
                               shape=(co, ho, wo)))

    def avgpool(self, src: int, kernel: int, stride: int = 0, pad: int = 0) -> int:
        c, h, w = self.shape_of(src)
        stride = stride or kernel
        ho = (h + 2 * pad - kernel) // stride + 1
        wo = (w + 2 * pad - kernel) // stride + 1
        return self._push(dict(type="avgpool", src=src, kernel=kernel, stride=stride, pad=pad, shape=(c, ho, wo)))

    def relu(self, src: int) -> int:
        return self._push(dict(type="relu", src=src, shape=self.shape_of(src)))

    def add(self, a: int, b: int) -> int:
        assert self.shape_of(a) == self.shape_of(b)
        return self._push(dict(type="add", a=a, b=b, shape=self.shape_of(a)))

    @property
    def n_in(self) -> int:
        c, h, w = self.input_shape
        return c * h * w

    @property
    def out_layer(self) -> int:
        return len(self.layers)

    def n_neurons(self, lid: int) -> int:
        c, h, w = self.shape_of(lid)
        return c * h * w

    # ---- inputs -------------------------------------------------------------------------
    def center(self, j: int) -> np.ndarray:
        """Image j of this configuration: uniform[0,1], float32, CHW-flattened."""
        rng = np.random.default_rng(self.input_seed_base + j)
        return rng.random(self.n_in).astype(np.float32)


def build_into(net: Net, target) -> List[int]:
    """Replays the topology on any object with add_dense/add_conv2d/add_avgpool2d/add_relu/add_residual.

    Returns the ids the target handed back (they must equal 1..len(layers))."""
    ids = []
    for L in net.layers:
        t = L["type"]
        if t == "dense":
            ids.append(target.add_dense(L["src"], L["W"], L["b"]))
        elif t == "conv":
            ids.append(target.add_conv2d(L["src"], L["W"], L["b"], L["stride"], L["pad"]))
        elif t == "avgpool":
            ids.append(target.add_avgpool2d(L["src"], L["kernel"], L["stride"], L["pad"]))
        elif t == "relu":
            ids.append(target.add_relu(L["src"]))
        elif t == "add":
            ids.append(target.add_residual(L["a"], L["b"]))
        else:
            raise ValueError(t)
    assert ids == list(range(1, len(net.layers) + 1)), ids
    return ids


# ---- random draws ---------------------------------------------------------------------------
BIAS_STD = 0.1     # "N(0, 0.01)" read as a variance


def _dense_params(rng, n_out, n_in, scale=1.0):
    W = (rng.standard_normal((n_out, n_in)) * np.sqrt(2.0 / n_in) * scale).astype(np.float32)
    b = (rng.standard_normal(n_out) * BIAS_STD).astype(np.float32)
    return W, b


def _conv_params(rng, c_out, c_in, k, scale=1.0):
    fan_in = c_in * k * k
    W = (rng.standard_normal((c_out, c_in, k, k)) * np.sqrt(2.0 / fan_in) * scale).astype(np.float32)
    b = (rng.standard_normal(c_out) * BIAS_STD).astype(np.float32)
    return W, b


def fc_net(name, widths, n_in=784, n_out=10, seed=0, eps=0.0, n_inputs=1, input_seed_base=0) -> Net:
    rng = np.random.default_rng(seed)
    net = Net(name, (n_in, 1, 1), eps=eps, n_inputs=n_inputs, input_seed_base=input_seed_base)
    cur, fan = 0, n_in
    for wd in widths:
        W, b = _dense_params(rng, wd, fan)
        cur = net.relu(net.dense(cur, W, b))
        fan = wd
    W, b = _dense_params(rng, n_out, fan)
    net.dense(cur, W, b)
    return net


def conv_net(name, input_shape, convs, denses, n_out=10, seed=0, eps=0.0, n_inputs=1,
             input_seed_base=0) -> Net:
    """convs: list of (c_out, k, stride, pad), each followed by ReLU; denses: hidden widths (+ReLU)."""
    rng = np.random.default_rng(seed)
    net = Net(name, input_shape, eps=eps, n_inputs=n_inputs, input_seed_base=input_seed_base)
    cur = 0
    for (co, k, s, p) in convs:
        ci = net.shape_of(cur)[0]
        W, b = _conv_params(rng, co, ci, k)
        cur = net.relu(net.conv(cur, W, b, s, p))
    fan = net.n_neurons(cur)
    for wd in denses:
        W, b = _dense_params(rng, wd, fan)
        cur = net.relu(net.dense(cur, W, b))
        fan = wd
    W, b = _dense_params(rng, n_out, fan)
    net.dense(cur, W, b)
    return net


def pool_net(name, input_shape, stages, denses, n_out=10, seed=0, eps=0.0, n_inputs=1, input_seed_base=0) -> Net:
    """stages: ("conv", c_out, k, stride, pad) (followed by ReLU) or ("pool", k, stride, pad) (average pooling);
    denses: hidden widths (+ReLU).  The LeNet family: convolutions with sub-sampling by averages in between."""
    rng = np.random.default_rng(seed)
    net = Net(name, input_shape, eps=eps, n_inputs=n_inputs, input_seed_base=input_seed_base)
    cur = 0
    for st in stages:
        if st[0] == "conv":
            _, co, k, s, p = st
            W, b = _conv_params(rng, co, net.shape_of(cur)[0], k)
            cur = net.relu(net.conv(cur, W, b, s, p))
        else:
            _, k, s, p = st
            cur = net.avgpool(cur, k, s, p)
    fan = net.n_neurons(cur)
    for wd in denses:
        W, b = _dense_params(rng, wd, fan)
        cur = net.relu(net.dense(cur, W, b))
        fan = wd
    W, b = _dense_params(rng, n_out, fan)
    net.dense(cur, W, b)
    return net


def resnet(name, input_shape=(3, 32, 32), channels=(64, 128, 256, 512), blocks=(3, 4, 6, 3),
           n_out=10, seed=0, eps=0.0, n_inputs=1, input_seed_base=0, second_conv_scale=0.2, pool_head=False) -> Net:
    """Basic-block residual net: stem conv3x3+ReLU; per block conv3x3-ReLU-conv3x3, sum with the
    shortcut (identity, or a 1x1 stride-2 conv when the stage halves the resolution), ReLU.
    Batch-norm is taken as folded into the conv weights.  The head is global average pooling
    followed by a dense layer; average pooling is linear, so the two are handed over as ONE dense
    layer whose weight is W[o][c] / (H*W) replicated over the H*W positions of channel c
    (exact when H*W is a power of two).  pool_head: the same network with the pooling as a layer of its own."""
    rng = np.random.default_rng(seed)
    net = Net(name, input_shape, eps=eps, n_inputs=n_inputs, input_seed_base=input_seed_base)
    W, b = _conv_params(rng, channels[0], input_shape[0], 3)
    cur = net.relu(net.conv(0, W, b, 1, 1))
    c_prev = channels[0]
    for si, (ch, nb) in enumerate(zip(channels, blocks)):
        for bi in range(nb):
            down = (si > 0 and bi == 0)
            stride = 2 if down else 1
            W1, b1 = _conv_params(rng, ch, c_prev, 3)
            W2, b2 = _conv_params(rng, ch, ch, 3, scale=second_conv_scale)
            if down or c_prev != ch:
                Ws, bs = _conv_params(rng, ch, c_prev, 1)
            block_in = cur
            h = net.relu(net.conv(block_in, W1, b1, stride, 1))
            h = net.conv(h, W2, b2, 1, 1)
            if down or c_prev != ch:
                sc = net.conv(block_in, Ws, bs, stride, 0)
            else:
                sc = block_in
            cur = net.relu(net.add(h, sc))
            c_prev = ch
    c, hh, ww = net.shape_of(cur)
    Wh, bh = _dense_params(rng, n_out, c)
    if pool_head:
        assert hh == ww
        net.dense(net.avgpool(cur, hh), Wh, bh)
        return net
    Wfold = np.repeat(Wh / np.float32(hh * ww), hh * ww, axis=1).astype(np.float32)  # CHW order
    net.dense(cur, Wfold, bh)
    return net


# ---- the five benchmark configurations --------------------------------------------------------
def config(i: int) -> Net:
    """i in 0..4 = the five configurations of the benchmark description, in its order."""
    wseed = 1000 + i
    ibase = 2000 + 100 * i
    if i == 0:
        return fc_net("fc_6x100", [100] * 6, seed=wseed, eps=0.02, n_inputs=10, input_seed_base=ibase)
    if i == 1:
        return fc_net("fc_9x500", [500] * 9, seed=wseed, eps=0.01, n_inputs=100, input_seed_base=ibase)
    if i == 2:
        return conv_net("conv_small", (3, 32, 32), [(16, 4, 2, 1), (32, 4, 2, 1)], [100],
                        seed=wseed, eps=2.0 / 255.0, n_inputs=100, input_seed_base=ibase)
    if i == 3:
        return conv_net("conv_deep", (3, 32, 32),
                        [(32, 3, 1, 1), (32, 3, 1, 1), (64, 3, 2, 1), (64, 3, 1, 1), (64, 3, 1, 1),
                         (64, 3, 2, 1)], [512], seed=wseed, eps=1.0 / 255.0, n_inputs=20,
                        input_seed_base=ibase)
    if i == 4:
        return resnet("resnet34", seed=wseed, eps=0.5 / 255.0, n_inputs=10, input_seed_base=ibase)
    raise ValueError(i)


def lenet_pool() -> Net:
    """Not one of the five configurations: a CIFAR-sized LeNet-family network with average pooling as sub-sampling
    (conv5x5-32, ReLU, 2x2 average, conv5x5-64, ReLU, 2x2 average, dense 512, ReLU, dense 10), the workload the
    pooling step of the library is measured on."""
    return pool_net("lenet_pool", (3, 32, 32), [("conv", 32, 5, 1, 2), ("pool", 2, 2, 0), ("conv", 64, 5, 1, 2), ("pool", 2, 2, 0)],
                    [512], n_out=10, seed=1100, eps=1.0 / 255.0, n_inputs=20, input_seed_base=2900)


def contracted(net: Net, weight_scale: float) -> Net:
    """The same network with every weight matrix / filter multiplied by `weight_scale` (biases kept).  With random
    He-normal weights the interval widths grow from layer to layer and every ReLU is unstable after the first few;
    a factor well below 1 stops that growth and leaves most ReLUs stable, which is the regime of the paper's robustly
    trained networks (Section 5), where early termination removes most of the work."""
    out = Net(f"{net.name}_w{weight_scale:g}", net.input_shape, eps=net.eps, n_inputs=net.n_inputs,
              input_seed_base=net.input_seed_base)
    for L in net.layers:
        d = dict(L)
        if d["type"] in ("dense", "conv"):
            d["W"] = (d["W"] * np.float32(weight_scale)).astype(np.float32)
        out.layers.append(d)
    return out


def scaled_resnet(div: int, spatial: int = 32, blocks=(3, 4, 6, 3), seed: int = 1004, eps=0.5 / 255.0) -> Net:
    """Same depth and topology as configuration 4 with channels divided by `div`."""
    ch = tuple(max(1, c // div) for c in (64, 128, 256, 512))
    return resnet(f"resnet34_div{div}_s{spatial}", (3, spatial, spatial), ch, blocks, seed=seed, eps=eps,
                  n_inputs=2, input_seed_base=2400)
