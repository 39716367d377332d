"""Seeded synthetic inputs shaped like the paper's workloads, and their work counts.

This module holds NO arithmetic of the method: only shapes, random tensors and MAC
counting.  It imports neither the GPU binding nor the CPU oracle, so both can be fed
the same bytes.  The tensors stand in for MNIST (1x28x28, Section IV), CIFAR-10
(3x32x32, Section V) and ImageNet resized to 256x256 (Section VI): only the shapes
and rough value ranges of those data sets are used.

Every tensor comes from numpy's PCG64 seeded with [18040451, config, tensor_id].
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED = 18040451


def rng(cfg: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng([SEED, cfg, tensor_id])


@dataclass(frozen=True)
class ConvSpec:
    """One stride-1 convolution layer on an NCHW minibatch (Section II-A: N images, K kernels)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    pad: int = 0
    act: str = "identity"  # identity | sigmoid | relu
    pool: int = 1          # 1 = none, 2 = 2x2 stride-2 max pool

    @property
    def Ho(self) -> int:
        return self.H + 2 * self.pad - self.R + 1

    @property
    def Wo(self) -> int:
        return self.W + 2 * self.pad - self.S + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C, self.R, self.S)

    @property
    def y_shape(self):
        return (self.N, self.K, self.Ho // self.pool, self.Wo // self.pool)

    def macs_nominal(self) -> int:
        return self.N * self.K * self.C * self.R * self.S * self.Ho * self.Wo

    def macs_exact(self) -> int:
        """Multiply-adds of one pass, not counting products with padding zeros."""
        def taps(L, Lo, F):
            # sum over output positions and filter taps of [input index in range]
            return sum(1 for i in range(Lo) for r in range(F) if 0 <= i + r - self.pad < L)
        return self.N * self.K * self.C * taps(self.H, self.Ho, self.R) * taps(self.W, self.Wo, self.S)


@dataclass(frozen=True)
class DenseSpec:
    in_: int
    out: int
    act: str = "identity"


@dataclass
class ConvWorkload:
    cfg: int
    name: str
    conv: ConvSpec
    x: np.ndarray
    w: np.ndarray
    bias: np.ndarray
    dy: np.ndarray

    def flop(self) -> int:
        return 2 * 3 * self.conv.macs_exact()


@dataclass
class CrbmWorkload:
    cfg: int
    name: str
    conv: ConvSpec
    v0: np.ndarray
    W: np.ndarray
    b: np.ndarray
    c: np.ndarray
    u: np.ndarray
    lr: float

    def flop(self) -> int:
        return 2 * 5 * self.conv.macs_exact()


@dataclass
class CnnWorkload:
    cfg: int
    name: str
    conv: List[ConvSpec]
    dense: List[DenseSpec]
    classes: int
    lr: float
    x: np.ndarray
    labels: np.ndarray
    params: List[np.ndarray] = field(default_factory=list)  # conv w0,b0,...; dense W0,b0,...

    @property
    def batch(self) -> int:
        return self.conv[0].N if self.conv else int(self.x.shape[0])

    def conv_flop(self) -> int:
        """fwd + wgrad for every conv layer, + full bwd for all but the first (no consumer)."""
        return 2 * sum(c.macs_exact() * (2 if i == 0 else 3) for i, c in enumerate(self.conv))

    def dense_flop(self) -> int:
        return 2 * 3 * sum(self.batch * d.in_ * d.out for d in self.dense)

    def flop(self) -> int:
        return self.conv_flop() + self.dense_flop()

    def clone_params(self) -> List[np.ndarray]:
        return [p.copy() for p in self.params]


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def config1(batch: int = 8) -> ConvWorkload:
    """Single conv layer fwd+bwd: 1x28x28 U[0,1), 8 filters 5x5 N(0, 0.01), sigmoid, no pool."""
    cs = ConvSpec(batch, 1, 28, 28, 8, 5, 5, 0, "sigmoid", 1)
    return ConvWorkload(
        1, "c1_single_conv", cs,
        x=_f32(rng(1, 0).random(cs.x_shape)),
        w=_f32(rng(1, 1).normal(0.0, 0.01, cs.w_shape)),
        bias=_f32(rng(1, 2).normal(0.0, 0.01, (cs.K,))),
        dy=_f32(rng(1, 3).normal(0.0, 1.0, cs.y_shape)))


def config3(batch: int = 64) -> CrbmWorkload:
    """Conv RBM CD-1 step: binary visibles Bernoulli(0.2), 40 filters 9x9 N(0, 0.01)."""
    cs = ConvSpec(batch, 1, 28, 28, 40, 9, 9, 0, "sigmoid", 1)
    return CrbmWorkload(
        3, "c3_crbm_cd1", cs,
        v0=_f32(rng(3, 0).random(cs.x_shape) < 0.2),
        W=_f32(rng(3, 1).normal(0.0, 0.01, cs.w_shape)),
        b=np.zeros((cs.K,), np.float32),
        c=np.zeros((cs.C,), np.float32),
        u=_f32(rng(3, 2).random(cs.y_shape, dtype=np.float32)),
        lr=0.01)


def _cnn(cfg: int, name: str, conv: List[ConvSpec], dense: List[DenseSpec], classes: int, lr: float,
         x_kind: str, conv_sigma: Optional[float]) -> CnnWorkload:
    """Weights: conv filters N(0, conv_sigma) when given, else N(0, sqrt(2/fan_in)); dense
    weights N(0, sqrt(2/fan_in)); biases N(0, 0.01) so that the bias path carries signal."""
    c0 = conv[0]
    g = rng(cfg, 0)
    x = g.random(c0.x_shape, dtype=np.float32) if x_kind == "uniform" else g.standard_normal(c0.x_shape, dtype=np.float32)
    labels = rng(cfg, 1).integers(0, classes, size=(c0.N,)).astype(np.int32)
    params: List[np.ndarray] = []
    tid = 2
    for c in conv:
        sigma = conv_sigma if conv_sigma is not None else float(np.sqrt(2.0 / (c.C * c.R * c.S)))
        params.append(_f32(rng(cfg, tid).normal(0.0, sigma, c.w_shape)))
        params.append(_f32(rng(cfg, tid + 1).normal(0.0, 0.01, (c.K,))))
        tid += 2
    for d in dense:
        sigma = float(np.sqrt(2.0 / d.in_))
        params.append(_f32(rng(cfg, tid).standard_normal((d.out, d.in_), dtype=np.float32) * np.float32(sigma)))
        params.append(_f32(rng(cfg, tid + 1).normal(0.0, 0.01, (d.out,))))
        tid += 2
    return CnnWorkload(cfg, name, conv, dense, classes, lr, _f32(x), labels, params)


def config2(batch: int = 100) -> CnnWorkload:
    """Small CNN on 1x28x28: conv 8@5x5 ReLU, pool 2, conv 8@5x5 ReLU, pool 2, dense 150, dense 10."""
    conv = [ConvSpec(batch, 1, 28, 28, 8, 5, 5, 0, "relu", 2), ConvSpec(batch, 8, 12, 12, 8, 5, 5, 0, "relu", 2)]
    dense = [DenseSpec(128, 150, "relu"), DenseSpec(150, 10, "identity")]
    return _cnn(2, "c2_small_cnn", conv, dense, 10, 0.1, "uniform", 0.01)


def config4(batch: int = 100) -> CnnWorkload:
    """Color CNN on 3x32x32: conv 12@5x5 pad 2, pool 2, conv 24@3x3 pad 1, pool 2, dense 64, dense 10."""
    conv = [ConvSpec(batch, 3, 32, 32, 12, 5, 5, 2, "relu", 2), ConvSpec(batch, 12, 16, 16, 24, 3, 3, 1, "relu", 2)]
    dense = [DenseSpec(1536, 64, "relu"), DenseSpec(64, 10, "identity")]
    return _cnn(4, "c4_color_cnn", conv, dense, 10, 0.001, "normal", None)


def config5(batch: int = 128, image: int = 256, hidden: int = 2048, classes: int = 1000) -> CnnWorkload:
    """Large-image CNN on 3x256x256: 4 x [conv 3x3 pad 1 (16,16,32,32) ReLU + pool 2], dense 2048, dense 1000.

    `image`, `hidden`, `classes` shrink the same architecture for oracle-sized parity cases."""
    assert image % 16 == 0
    chans = [3, 16, 16, 32, 32]
    conv, side = [], image
    for i in range(4):
        conv.append(ConvSpec(batch, chans[i], side, side, chans[i + 1], 3, 3, 1, "relu", 2))
        side //= 2
    dense = [DenseSpec(32 * side * side, hidden, "relu"), DenseSpec(hidden, classes, "identity")]
    return _cnn(5, "c5_large_image_cnn", conv, dense, classes, 0.001, "normal", None)


# ---- the networks as the paper describes them (inference workloads; seeds 11..13)

def paper_mnist_cnn(batch: int = 100) -> CnnWorkload:
    """Section IV-B: 1x28x28, conv 8@5x5 + pool 2, conv 8@5x5 + pool 2, dense 150, dense 10; sigmoid
    everywhere but the softmax output."""
    conv = [ConvSpec(batch, 1, 28, 28, 8, 5, 5, 0, "sigmoid", 2), ConvSpec(batch, 8, 12, 12, 8, 5, 5, 0, "sigmoid", 2)]
    dense = [DenseSpec(128, 150, "sigmoid"), DenseSpec(150, 10, "identity")]
    return _cnn(11, "paper_mnist_cnn", conv, dense, 10, 0.1, "uniform", None)


def paper_cifar_cnn(batch: int = 100) -> CnnWorkload:
    """Section V: 3x32x32, conv 12@5x5 + pool 2, conv 24@3x3 + pool 2 (no padding), dense 64, dense 10; ReLU."""
    conv = [ConvSpec(batch, 3, 32, 32, 12, 5, 5, 0, "relu", 2), ConvSpec(batch, 12, 14, 14, 24, 3, 3, 0, "relu", 2)]
    dense = [DenseSpec(24 * 6 * 6, 64, "relu"), DenseSpec(64, 10, "identity")]
    return _cnn(12, "paper_cifar_cnn", conv, dense, 10, 0.001, "normal", None)


def paper_imagenet_cnn(batch: int = 128, image: int = 256, hidden: int = 2048, classes: int = 1000) -> CnnWorkload:
    """Section VI: 3 x image x image, five blocks of conv 3x3 (16, 16, 32, 32, 32 kernels, zero-padded to
    keep the size) + ReLU + pool 2, dense `hidden` ReLU, dense `classes`.  `image`, `hidden`, `classes`
    shrink the same architecture for oracle-sized parity cases."""
    assert image % 32 == 0
    chans = [3, 16, 16, 32, 32, 32]
    conv, side = [], image
    for i in range(5):
        conv.append(ConvSpec(batch, chans[i], side, side, chans[i + 1], 3, 3, 1, "relu", 2))
        side //= 2
    dense = [DenseSpec(32 * side * side, hidden, "relu"), DenseSpec(hidden, classes, "identity")]
    return _cnn(13, "paper_imagenet_cnn", conv, dense, classes, 0.001, "normal", None)


def paper_mnist_dense(batch: int = 100, sizes=(784, 500, 250, 10)) -> CnnWorkload:
    """Section IV-A: fully-connected 784-500-250-10, sigmoid hidden layers, softmax output,
    mini-batches of 100, learning rate 0.1 (momentum 0.9 is an argument of the step).
    Inputs uniform in [0, 1) like grey-scale pixels; weights N(0, sqrt(2/fan_in)), biases N(0, 0.01)."""
    dense = [DenseSpec(sizes[i], sizes[i + 1], "sigmoid" if i + 2 < len(sizes) else "identity") for i in range(len(sizes) - 1)]
    x = rng(14, 0).random((batch, sizes[0]), dtype=np.float32)
    labels = rng(14, 1).integers(0, sizes[-1], size=(batch,)).astype(np.int32)
    params: List[np.ndarray] = []
    tid = 2
    for d in dense:
        params.append(_f32(rng(14, tid).standard_normal((d.out, d.in_), dtype=np.float32) * np.float32(np.sqrt(2.0 / d.in_))))
        params.append(_f32(rng(14, tid + 1).normal(0.0, 0.01, (d.out,))))
        tid += 2
    return CnnWorkload(14, "paper_mnist_dense", [], dense, sizes[-1], 0.1, _f32(x), labels, params)


@dataclass
class RbmWorkload:
    """Fully-connected RBM step: v0 [batch, n_vis], W [n_hid, n_vis], u [batch, n_hid]."""
    name: str
    batch: int
    n_vis: int
    n_hid: int
    visible: str
    v0: np.ndarray
    W: np.ndarray
    b: np.ndarray
    c: np.ndarray
    u: np.ndarray
    lr: float

    def flop(self) -> int:
        return 2 * 5 * self.batch * self.n_vis * self.n_hid


def dense_rbm(batch: int = 100, n_vis: int = 784, n_hid: int = 500, visible: str = "binary", seed: int = 15) -> RbmWorkload:
    """The first layer of Section IV-A's network as an RBM (Section II): binary inputs with about a
    fifth of the pixels on (or standard-normal inputs for Gaussian visible units), W ~ N(0, 0.05),
    small random biases."""
    g = rng(seed, 0)
    v0 = (g.random((batch, n_vis)) < 0.2).astype(np.float32) if visible == "binary" else \
        g.standard_normal((batch, n_vis), dtype=np.float32)
    return RbmWorkload(f"dense_rbm_{visible}", batch, n_vis, n_hid, visible, _f32(v0),
                       _f32(rng(seed, 1).normal(0.0, 0.05, (n_hid, n_vis))), _f32(rng(seed, 2).normal(0.0, 0.1, (n_hid,))),
                       _f32(rng(seed, 3).normal(0.0, 0.1, (n_vis,))), _f32(rng(seed, 4).random((batch, n_hid), dtype=np.float32)), 0.05)


def crbm_units(cs: ConvSpec, visible: str, hidden_pool: int, seed: int = 16) -> CrbmWorkload:
    """A CRBM step on any shape: binary (30 % on) or standard-normal visibles, filters N(0, 0.05),
    small random biases, one uniform number per hidden unit (hidden_pool 1) or per 2x2 block (2)."""
    g = rng(seed, 0)
    v0 = (g.random(cs.x_shape) < 0.3).astype(np.float32) if visible == "binary" else g.standard_normal(cs.x_shape, dtype=np.float32)
    ushape = (cs.N, cs.K, cs.Ho // hidden_pool, cs.Wo // hidden_pool)
    return CrbmWorkload(0, f"crbm_{visible}_pool{hidden_pool}", cs, _f32(v0), _f32(rng(seed, 1).normal(0.0, 0.05, cs.w_shape)),
                        _f32(rng(seed, 2).normal(0.0, 0.1, (cs.K,))), _f32(rng(seed, 3).normal(0.0, 0.1, (cs.C,))),
                        _f32(rng(seed, 4).random(ushape, dtype=np.float32)), 0.01)


def large_filter_layer(batch: int = 64) -> ConvWorkload:
    """A layer with large filters (32 -> 32 channels, 12x12 filters, 32x32 output maps from 43x43
    inputs): the case Section II-A sends through the Fourier transform.  Gradients N(0, 1), filters
    N(0, sqrt(2/fan_in)); x and bias are not used by the backward-data pass and stay empty."""
    cs = ConvSpec(batch, 32, 43, 43, 32, 12, 12, 0, "identity", 1)
    return ConvWorkload(17, "large_filter_full_convolution", cs, x=np.zeros((0,), np.float32),
                        w=_f32(rng(17, 1).normal(0.0, np.sqrt(2.0 / (cs.C * cs.R * cs.S)), cs.w_shape)),
                        bias=np.zeros((0,), np.float32), dy=_f32(rng(17, 3).normal(0.0, 1.0, cs.y_shape)))


def forward_flop(w: CnnWorkload) -> int:
    """Exact multiply-adds x 2 of one inference pass."""
    return 2 * sum(c.macs_exact() for c in w.conv) + 2 * sum(w.batch * d.in_ * d.out for d in w.dense)


def with_batch(cs: ConvSpec, n: int) -> ConvSpec:
    return replace(cs, N=n)


ALL = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
