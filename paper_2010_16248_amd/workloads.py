"""Synthetic workloads: tensor-shape sets and seeded gradient generators.

This module serves the tests, the benchmark and the CPU oracle's callers alike.
It holds NONE of the method's arithmetic (no error feedback, no compression, no
norms, no regime test): only the shapes of the gradient sets and the random
numbers that stand in for real gradients.

The shape sets follow the models the paper trains (Section 5.1 "Dataset and
Models"; parameter totals in the appendix tables "Total parameters when training
Cifar-10" and "... WikiText-2").  Only tensor shapes are used: the paper's
datasets are not needed, and all values are seeded and synthetic.

Layer convention: a convolution weight of shape out x in x kh x kw is the matrix
out x (in*kh*kw), row-major; a 1-D tensor (bias, batch-norm weight/bias) has
rows = 1, is_matrix = 0.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

SEED_BASE = 20101624

METHOD_POWERSGD = 0
METHOD_TOPK = 1
METHOD_BATCH = 2


@dataclass(frozen=True)
class Layer:
    offset: int
    rows: int
    cols: int
    is_matrix: int

    @property
    def numel(self) -> int:
        return self.rows * self.cols


def make_layers(shapes: Sequence[Tuple[int, int, int]]) -> List[Layer]:
    """Concatenate (rows, cols, is_matrix) shapes into a flat layout."""
    out, off = [], 0
    for r, c, m in shapes:
        out.append(Layer(off, int(r), int(c), int(m)))
        off += int(r) * int(c)
    return out


def total_params(layers: Sequence[Layer]) -> int:
    return sum(l.numel for l in layers)


# --------------------------------------------------------------------------
# shape sets
# --------------------------------------------------------------------------

def tiny4_shapes():
    """Four small matrices of the smallest configuration (all compressed)."""
    return [(64, 576, 1), (128, 1152, 1), (256, 2304, 1), (10, 512, 1)]


def resnet18_shapes(n_classes: int = 10):
    """ResNet-18 for 32x32 inputs: 21 matrices + 41 vectors, 11 173 962 parameters
    at 10 classes (appendix table of parameter totals)."""
    s = []

    def conv(o, i, k):
        s.append((o, i * k * k, 1))

    def bn(c):
        s.append((1, c, 0))
        s.append((1, c, 0))

    conv(64, 3, 3)
    bn(64)
    inp = 64
    for width in (64, 128, 256, 512):
        for block in range(2):
            conv(width, inp, 3)
            bn(width)
            conv(width, width, 3)
            bn(width)
            if block == 0 and inp != width:
                conv(width, inp, 1)  # projection shortcut
                bn(width)
            inp = width
    s.append((n_classes, 512, 1))
    s.append((1, n_classes, 0))
    return s


def vgg19bn_shapes(n_classes: int = 10):
    """VGG-19 with batch norm for 32x32 inputs and a 512-512-classes head:
    19 matrices + 51 vectors, 20 565 834 parameters at 10 classes."""
    s = []
    inp = 3
    for width, reps in ((64, 2), (128, 2), (256, 4), (512, 4), (512, 4)):
        for _ in range(reps):
            s.append((width, inp * 9, 1))
            s.extend([(1, width, 0)] * 3)  # conv bias, bn weight, bn bias
            inp = width
    for o, i in ((512, 512), (512, 512), (n_classes, 512)):
        s.append((o, i, 1))
        s.append((1, o, 0))
    return s


def lstm_shapes():
    """Two-layer LSTM language-model set as six dense tensors: embedding, four
    recurrent weight matrices, decoder (51 265 536 parameters)."""
    return [(32768, 672, 1)] + [(2688, 672, 1)] * 4 + [(32768, 672, 1)]


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    method: int
    shapes: list
    n_workers: int
    # PowerSGD: ranks; TopK: numerators over k_den.  "crit" = level used inside
    # critical regimes (less compression), "noncrit" = outside.
    level_crit: int
    level_noncrit: int
    k_den: int = 100
    eta: float = 0.5
    window_steps: int = 10
    n_windows: int = 2
    dist: str = "normal"          # "normal" | "laplace" | "lstm"
    scale_lo: float = 1e-4
    scale_hi: float = 1e-2
    fixed_scale: float = 0.0      # > 0: one scale for every layer
    seed: int = SEED_BASE
    window_scale_even: Sequence[float] = field(default_factory=list)
    window_scale_odd: Sequence[float] = field(default_factory=list)
    batch_multiplier: int = 1     # batch-size mode: floor(B_high / B_low)

    @property
    def layers(self) -> List[Layer]:
        return make_layers(self.shapes)

    @property
    def n_params(self) -> int:
        return total_params(self.layers)


def workload(name: str) -> Workload:
    if name == "tiny_powersgd":
        return Workload(name, METHOD_POWERSGD, tiny4_shapes(), 2, 2, 1,
                        window_steps=10, n_windows=2, fixed_scale=0.01, seed=SEED_BASE + 1)
    if name == "resnet18_topk":
        return Workload(name, METHOD_TOPK, resnet18_shapes(), 4, 10, 1,
                        dist="laplace", window_steps=20, n_windows=3, seed=SEED_BASE + 2)
    if name == "resnet18_powersgd":
        return Workload(name, METHOD_POWERSGD, resnet18_shapes(), 4, 4, 1,
                        window_steps=20, n_windows=3, seed=SEED_BASE + 3)
    if name == "vgg19_powersgd":
        return Workload(name, METHOD_POWERSGD, vgg19bn_shapes(), 1, 4, 2,
                        window_steps=50, n_windows=6, seed=SEED_BASE + 4,
                        window_scale_even=[1.00, 0.30, 0.28, 0.84, 0.28, 0.27],
                        window_scale_odd=[1.00, 0.30, 0.28, 0.28, 0.84, 0.28])
    if name == "lstm_topk":
        return Workload(name, METHOD_TOPK, lstm_shapes(), 16, 10, 1,
                        dist="lstm", window_steps=100, n_windows=3, seed=SEED_BASE + 5,
                        window_scale_even=[1.00, 0.40, 0.38],
                        window_scale_odd=[1.00, 0.40, 0.38])
    if name == "resnet18_topk_k99":
        # the levels the paper itself trains with (Section 5.4, TopK tables): K 99 % inside
        # critical regimes, K 25 % outside; ResNet-18 with 100 classes
        return Workload(name, METHOD_TOPK, resnet18_shapes(100), 4, 99, 25,
                        dist="laplace", window_steps=20, n_windows=3, seed=SEED_BASE + 7)
    if name == "lstm_topk_k99":
        # K 99 % / 2 % on the LSTM set (appendix figure of the language model)
        return Workload(name, METHOD_TOPK, lstm_shapes(), 4, 99, 2,
                        dist="lstm", window_steps=100, n_windows=3, seed=SEED_BASE + 8,
                        window_scale_even=[1.00, 0.40, 0.38],
                        window_scale_odd=[1.00, 0.40, 0.38])
    if name == "resnet18_batch":
        # batch-size mode: B_low = 512, B_high = 4096 (Section 5); a "step" is one micro-batch
        return Workload(name, METHOD_BATCH, resnet18_shapes(), 4, 1, 1,
                        window_steps=20, n_windows=3, seed=SEED_BASE + 6, batch_multiplier=8)
    raise KeyError(name)


WORKLOAD_NAMES = ["tiny_powersgd", "resnet18_topk", "resnet18_powersgd",
                  "vgg19_powersgd", "lstm_topk", "resnet18_batch", "resnet18_topk_k99",
                  "lstm_topk_k99"]


# --------------------------------------------------------------------------
# seeded generators (inputs only)
# --------------------------------------------------------------------------

def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed)] + [int(k) for k in key])))


def layer_scales(wl: Workload) -> np.ndarray:
    """Per-layer value scale: log-uniform in [scale_lo, scale_hi], or fixed."""
    n = len(wl.shapes)
    if wl.fixed_scale > 0:
        return np.full(n, wl.fixed_scale, dtype=np.float64)
    u = _rng(wl.seed, 7001).random(n)
    return np.exp(np.log(wl.scale_lo) + u * (np.log(wl.scale_hi) - np.log(wl.scale_lo)))


def window_scale(wl: Workload, layer_index: int, window: int) -> float:
    seq = wl.window_scale_even if layer_index % 2 == 0 else wl.window_scale_odd
    if not seq:
        return 1.0
    return float(seq[min(window, len(seq) - 1)])


def gradient(wl: Workload, worker: int, step: int, window: int = 0) -> np.ndarray:
    """One worker's flat fp32 gradient for one step (all layers concatenated)."""
    layers = wl.layers
    n = total_params(layers)
    rng = _rng(wl.seed + 1000 * worker, 1, step)
    sc = layer_scales(wl)
    if wl.dist == "laplace":
        g = rng.laplace(0.0, 1.0, n)
    else:
        g = rng.standard_normal(n)
    out = np.empty(n, dtype=np.float32)
    for li, l in enumerate(layers):
        s = sc[li] * window_scale(wl, li, window)
        seg = g[l.offset:l.offset + l.numel]
        if wl.dist == "lstm" and li == 0:
            # embedding: 5 % of rows non-zero, entries N(0, 1e-3^2)
            rows = _rng(wl.seed + 1000 * worker, 2, step).random(l.rows) < 0.05
            m = (seg.reshape(l.rows, l.cols) * (1e-3 * window_scale(wl, li, window)))
            m[~rows, :] = 0.0
            out[l.offset:l.offset + l.numel] = m.reshape(-1).astype(np.float32)
        else:
            out[l.offset:l.offset + l.numel] = (seg * s).astype(np.float32)
    return out


def q_init(wl_or_layers, r_max: int, seed: int = SEED_BASE) -> np.ndarray:
    """Initial right factors: for every matrix layer an (cols x r_max) block of
    N(0,1) entries, row-major, blocks concatenated in layer order."""
    layers = wl_or_layers.layers if isinstance(wl_or_layers, Workload) else wl_or_layers
    total = sum(l.cols * r_max for l in layers if l.is_matrix)
    return _rng(seed, 9001).standard_normal(total).astype(np.float32)


def random_layers(seed: int, n_layers: int, max_rows: int = 40, max_cols: int = 300,
                  p_vector: float = 0.3) -> List[Layer]:
    """Ragged, mostly 16-byte-misaligned layer sets for edge-case tests."""
    rng = _rng(seed, 4242)
    shapes = []
    for _ in range(n_layers):
        if rng.random() < p_vector:
            shapes.append((1, int(rng.integers(1, max_cols)), 0))
        else:
            shapes.append((int(rng.integers(1, max_rows)), int(rng.integers(1, max_cols)), 1))
    return make_layers(shapes)
