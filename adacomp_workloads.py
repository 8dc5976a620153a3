"""Seeded synthetic gradient workloads: layer tables and dW generators.

This module serves both the CPU oracle's tests and the GPU path's tests / bench.  It holds no
part of the compression method: only tensor shapes, bin lengths and random number recipes.

The five workloads stand in for the gradients the AdaComp paper trains on (section "Methodology":
MNIST / CIFAR10 CNNs, ResNet-50, a char-LSTM, a speech DNN); real gradients need those datasets,
so the values here are random draws with the stated per-layer distributions.  Bin lengths follow
the paper's Table 2: 50 for convolutional layers, 500 for fully connected and recurrent ones.

Every draw comes from numpy's counter-based Philox generator keyed by
(seed, workload, learner, step, layer, block), so a value depends only on its coordinates and
never on how many threads produced it or in which order.
"""
from __future__ import annotations

import functools
import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

L_T_CONV = 50
L_T_FC = 500
_BLOCK = 1 << 22  # elements per independently keyed block


@dataclass(frozen=True)
class Layer:
    name: str
    n_elems: int
    L_T: int
    elem_offset: int = 0


@dataclass(frozen=True)
class Workload:
    index: int          # 1..5, position in the list of benchmark configurations
    name: str
    layers: tuple       # of Layer, elem_offset filled in
    n_learners: int
    n_steps: int
    dist: str           # "normal" | "laplace" | "normal_outliers" | "normal_spikes"

    @property
    def n_total(self) -> int:
        """Length of the flat buffer (end of the layer that lies last; layer starts are multiples of 4)."""
        return max(l.elem_offset + l.n_elems for l in self.layers)

    @property
    def n_params(self) -> int:
        return sum(l.n_elems for l in self.layers)

    def table(self):
        """[(elem_offset, n_elems, L_T)] as the C interfaces take it."""
        return [(l.elem_offset, l.n_elems, l.L_T) for l in self.layers]


def _place(layers):
    out, off = [], 0
    for name, n, lt in layers:
        out.append(Layer(name, int(n), int(lt), off))
        off += (int(n) + 3) // 4 * 4
    return tuple(out)


def _resnet50_layers():
    """Weight tensors of ResNet-50 by rule: 7x7 stem, four stages of bottleneck blocks
    (1x1, 3x3, 1x1 x4) with a 1x1 projection in each stage's first block, then the FC layer."""
    layers = [("conv1", 7 * 7 * 3 * 64, L_T_CONV)]
    c_in = 64
    for stage, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), start=2):
        for b in range(blocks):
            p = f"layer{stage}.{b}"
            layers.append((p + ".conv1", c_in * width, L_T_CONV))
            layers.append((p + ".conv2", 3 * 3 * width * width, L_T_CONV))
            layers.append((p + ".conv3", width * 4 * width, L_T_CONV))
            if b == 0:
                layers.append((p + ".downsample", c_in * 4 * width, L_T_CONV))
            c_in = 4 * width
    layers.append(("fc", 2048 * 1000, L_T_FC))
    return layers


@functools.lru_cache(maxsize=None)
def workload(index: int) -> Workload:
    if index == 1:
        return Workload(1, "fc_mnist", _place([("fc1", 784 * 500, L_T_FC), ("fc2", 500 * 10, L_T_FC)]),
                        1, 5, "normal")
    if index == 2:
        return Workload(2, "cifar_cnn", _place([
            ("conv1", 5 * 5 * 3 * 64, L_T_CONV), ("conv2", 5 * 5 * 64 * 64, L_T_CONV),
            ("conv3", 5 * 5 * 64 * 128, L_T_CONV), ("fc1", 2048 * 384, L_T_FC),
            ("fc2", 384 * 192, L_T_FC), ("fc3", 192 * 10, L_T_FC)]), 4, 20, "normal")
    if index == 3:
        return Workload(3, "resnet50", _place(_resnet50_layers()), 8, 10, "laplace")
    if index == 4:
        return Workload(4, "char_lstm", _place([
            ("lstm1", 4 * 512 * (65 + 512), L_T_FC), ("lstm2", 4 * 512 * (512 + 512), L_T_FC),
            ("softmax", 512 * 65, L_T_FC)]), 8, 50, "normal_outliers")
    if index == 5:
        return Workload(5, "speech_dnn", _place(
            [(f"fc{i}", 4096 * 4096, L_T_FC) for i in range(1, 7)] + [("out", 4096 * 5999, L_T_FC)]),
            16, 10, "normal_spikes")
    raise ValueError("workload index must be 1..5")


def with_bin_lengths(wl: Workload, conv_L_T: int, fc_L_T: int, n_learners=None, n_steps=None) -> Workload:
    """The same layer shapes, distributions and random draws as ``wl`` with other bin lengths: the
    paper's stress tests keep the network and change only L_T (Fig. 2(a): 800 for convolutional
    and 8000 for fully connected layers on the CIFAR10 CNN; section "Robustness of the AdaComp
    Technique": 5000, and 200 / 300 for local selection).  Layers whose name starts with "conv" or
    contains ".conv" / ".downsample" take conv_L_T, the others fc_L_T."""
    def is_conv(name):
        return name.startswith("conv") or ".conv" in name or ".downsample" in name
    layers = tuple(Layer(l.name, l.n_elems, int(conv_L_T if is_conv(l.name) else fc_L_T), l.elem_offset)
                   for l in wl.layers)
    return Workload(wl.index, f"{wl.name}_LT{conv_L_T}_{fc_L_T}", layers,
                    wl.n_learners if n_learners is None else n_learners,
                    wl.n_steps if n_steps is None else n_steps, wl.dist)


def custom(name, layers, n_learners=1, n_steps=1, dist="normal") -> Workload:
    """A workload over an arbitrary [(name, n_elems, L_T)] list (edge-case tests)."""
    return Workload(0, name, _place(layers), n_learners, n_steps, dist)


def custom_placed(name, layers, n_learners=1, n_steps=1, dist="normal") -> Workload:
    """Like custom, with the element offset of every layer given: [(name, n_elems, L_T, elem_offset)],
    in any order, with any gaps (offsets must be multiples of 4 and the layers must not overlap)."""
    placed = tuple(Layer(nm, int(n), int(lt), int(off)) for nm, n, lt, off in layers)
    assert all(l.elem_offset % 4 == 0 for l in placed)
    return Workload(0, name, placed, n_learners, n_steps, dist)


def _rng(seed, wl_index, learner, step, layer, block, salt=0):
    key1 = ((wl_index & 0xF) << 60) | ((salt & 0xF) << 56) | ((learner & 0xFFF) << 44) | \
           ((step & 0xFFFF) << 28) | ((layer & 0xFFF) << 16) | (block & 0xFFFF)
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), key1]))


def layer_params(wl: Workload, seed: int = 0):
    """Per-layer distribution parameter, drawn once per layer from the seed and shared by every
    learner and step: sigma (normal kinds) or b (laplace)."""
    out = []
    for li, _ in enumerate(wl.layers):
        u = _rng(seed, wl.index, 0, 0, li, 0, salt=1).random()
        if wl.dist == "normal" and wl.index == 2:
            out.append(10.0 ** (-4.0 + 2.0 * u))          # log-uniform in [1e-4, 1e-2]
        elif wl.dist == "laplace":
            out.append(10.0 ** (-5.0 + 3.0 * u))          # log-uniform in [1e-5, 1e-2]
        else:
            out.append(1e-3)
    return out


SPIKE_FRACTION = 0.005
SPIKE_SIGMA = 0.1
OUTLIER_PROB = 0.01
OUTLIER_FACTOR = 100.0


@functools.lru_cache(maxsize=64)
def _spike_positions(wl_index: int, seed: int, layer: int, n: int):
    """Fixed positions of the sparse-spike pattern of one layer (same for all learners, steps)."""
    k = int(round(SPIKE_FRACTION * n))
    rng = _rng(seed, wl_index, 0, 0, layer, 0, salt=2)
    pos = np.unique(rng.integers(0, n, size=k, dtype=np.int64))
    return pos


def _fill_block(view, wl, seed, learner, step, li, blk, param):
    rng = _rng(seed, wl.index, learner, step, li, blk)
    n = view.size
    if wl.dist == "laplace":
        u = rng.random(n, dtype=np.float32)
        u -= np.float32(0.5)                               # (-0.5, 0.5)
        mag = np.abs(u)
        np.minimum(mag, np.float32(0.49999997), out=mag)   # keep log(1 - 2|u|) finite at u = -0.5
        mag *= np.float32(-2.0)
        np.log1p(mag, out=mag)                             # log(1 - 2|u|) <= 0
        mag *= np.float32(-param)
        np.copysign(mag, u, out=view)
        return
    rng.standard_normal(n, dtype=np.float32, out=view)
    view *= np.float32(param)
    if wl.dist == "normal_outliers":
        mask = rng.random(n, dtype=np.float32) < np.float32(OUTLIER_PROB)
        view[mask] *= np.float32(OUTLIER_FACTOR)


def gradient(wl: Workload, learner: int, step: int, seed: int = 0, out=None, threads: int = 1):
    """dW of one learner at one step as a flat float32 array of wl.n_total elements
    (elements between layers, if any, are zero)."""
    if out is None:
        out = np.zeros(wl.n_total, np.float32)
    else:
        assert out.dtype == np.float32 and out.size == wl.n_total
    params = layer_params(wl, seed)
    jobs = []
    for li, layer in enumerate(wl.layers):
        for blk in range(math.ceil(layer.n_elems / _BLOCK)):
            lo = layer.elem_offset + blk * _BLOCK
            hi = min(layer.elem_offset + layer.n_elems, lo + _BLOCK)
            jobs.append((out[lo:hi], wl, seed, learner, step, li, blk, params[li]))
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(lambda a: _fill_block(*a), jobs))
    else:
        for a in jobs:
            _fill_block(*a)
    if wl.dist == "normal_spikes":
        for li, layer in enumerate(wl.layers):
            pos = _spike_positions(wl.index, seed, li, layer.n_elems)
            v = _rng(seed, wl.index, learner, step, li, 0, salt=3).standard_normal(pos.size, dtype=np.float32)
            v *= np.float32(SPIKE_SIGMA)
            out[layer.elem_offset + pos] += v
    return out
