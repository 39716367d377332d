"""A bounded, seeded sweep of random layer shapes and small random networks through the same
GPU-vs-oracle checks as the hand-picked parity cases.

The shapes come from a fixed pseudo-random sequence, so every run tests the same cases; each is a
test of its own, named by its shape.  The generator leans towards the shapes the library's
dispatch rules distinguish: padded 3x3 layers with 4-, 8- and 16-channel chunks (and channel counts
whose filter slices no longer fit the LDS, which must fall through to the generic kernel), whole and
ragged 8 x 32 / 16 x 32 tiles, one to three output channels (the banded-filter kernel), filter sizes
with one to nine tap tiles in the filter-gradient kernel, pooled and unpooled layers of every
activation.  The networks mix pooled and unpooled ReLU layers, so the decisions "unit on/off"
that the GPU takes from its own fp32 values are checked against the oracle's and handed to it.
A third family are stacks of padded 3x3 ReLU + pooling layers with 16 or 32 channels behind a first
layer of one, three or sixteen channels (the shape of Section VI's network, on maps from 16 to 256
columns wide, whole and ragged against the kernels' 32- and 64-column segments): these reach the
streaming forms, the first-layer kernels and the launches that a layer's filter gradient and
backward-data pass share inside the training step.
"""
import random

import numpy as np
import pytest

pytest.importorskip("torch")

from paper_1804_04512_amd import workloads as wl
from paper_1804_04512_amd.workloads import ConvSpec, DenseSpec

import test_gpu_parity as T

pytestmark = pytest.mark.gpu

N_LAYERS, N_NETS, N_STACKS = 40, 10, 8


def layer_cases(count=N_LAYERS, seed=20241):
    rnd = random.Random(seed)
    cases = []
    while len(cases) < count:
        kind = len(cases) % 4
        if kind == 0:
            # padded 3x3 layers on tile-friendly maps: the specialised engines and their limits
            R = S = 3
            pad = 1
            C = rnd.choice([3, 4, 8, 12, 16, 16, 24, 32, 32, 48, 64, 128])
            K = rnd.choice([8, 16, 16, 24, 32, 32, 40])
            H = rnd.choice([8, 12, 16, 24, 32, 40])
            W = rnd.choice([16, 32, 32, 64, 68, 96])
        elif kind == 1:
            # few channels in: the backward-data pass has one to three output channels
            R = rnd.choice([3, 5, 7, 9])
            S = rnd.choice([R, R, rnd.choice([3, 5, 7])])
            pad = rnd.randint(0, min(R, S) - 1)
            C = rnd.choice([1, 1, 2, 3])
            K = rnd.choice([1, 2, 5, 8, 12, 16, 24, 40])
            H = rnd.randint(max(R - 2 * pad, 1) + 1, 48)
            W = rnd.randint(max(S - 2 * pad, 1) + 1, 70)
        else:
            R = rnd.choice([1, 2, 3, 3, 4, 5, 5, 7, 9, 12])
            S = rnd.choice([R, R, R, rnd.choice([1, 2, 3, 5, 7])])
            pad = rnd.randint(0, min(R, S) - 1)
            C = rnd.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 24, 32, 33, 40])
            K = rnd.choice([1, 2, 3, 5, 8, 12, 16, 17, 24, 32, 33, 40, 50])
            H = rnd.randint(max(R - 2 * pad, 1), 70)
            W = rnd.choice([rnd.randint(max(S - 2 * pad, 1), 75), rnd.choice([8, 16, 24, 32, 36, 40, 64, 68])])
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        Ho, Wo = H + 2 * pad - R + 1, W + 2 * pad - S + 1
        pool = 2 if (Ho % 2 == 0 and Wo % 2 == 0 and rnd.random() < 0.6) else 1
        act = rnd.choice(["identity", "sigmoid", "relu", "relu"])
        N = rnd.randint(1, 4)
        if N * C * H * W * K * R * S > 3e8:   # keeps one oracle pass under about a second
            continue
        cases.append(ConvSpec(N, C, H, W, K, R, S, pad, act, pool))
    return cases


def net_cases(count=N_NETS, seed=20242):
    rnd = random.Random(seed)
    cases = []
    while len(cases) < count:
        B = rnd.choice([1, 2, 3, 5, 8, 16, 33])
        C = rnd.choice([1, 3, 4, 8])
        H = rnd.choice([16, 20, 24, 28, 32, 36, 40, 48])
        W = rnd.choice([H, H, rnd.choice([16, 24, 32, 40, 44])])
        conv, ok = [], True
        for _ in range(rnd.randint(1, 3)):
            R = rnd.choice([3, 3, 3, 5, 1, 2])
            pad = rnd.randint(0, R - 1)
            K = rnd.choice([3, 5, 8, 12, 16, 24, 32, 40])
            Ho, Wo = H + 2 * pad - R + 1, W + 2 * pad - R + 1
            if Ho < 1 or Wo < 1:
                ok = False
                break
            pool = 2 if (Ho % 2 == 0 and Wo % 2 == 0 and rnd.random() < 0.6) else 1
            act = rnd.choice(["relu", "relu", "relu", "sigmoid", "identity"])
            conv.append(ConvSpec(B, C, H, W, K, R, R, pad, act, pool))
            C, H, W = K, Ho // pool, Wo // pool
        feat = C * H * W
        if not ok or feat > 20000:
            continue
        dense, classes = [], rnd.choice([2, 5, 10, 37, 100])
        nd = rnd.randint(1, 3)
        for q in range(nd):
            out = classes if q == nd - 1 else rnd.choice([7, 32, 64, 100, 150, 257])
            dense.append(DenseSpec(feat, out, "identity" if q == nd - 1 else rnd.choice(["relu", "sigmoid"])))
            feat = out
        cases.append((conv, dense, classes, rnd.choice(["uniform", "normal"])))
    return cases


def stack_cases(count=N_STACKS, seed=20243):
    rnd = random.Random(seed)
    cases = []
    while len(cases) < count:
        B = rnd.choice([1, 2, 3, 4, 6, 8, 12, 16, 24])
        C = rnd.choice([1, 3, 3, 16])
        H = rnd.choice([16, 32, 48, 64, 96, 128])
        W = rnd.choice([16, 32, 40, 64, 72, 96, 128, 136, 192, 256])
        if B * H * W > 1600000:   # keeps the oracle's step within a few seconds
            continue
        conv = []
        for _ in range(rnd.randint(2, 4)):
            if H % 2 or W % 2:
                break
            K = rnd.choice([16, 16, 32])
            conv.append(ConvSpec(B, C, H, W, K, 3, 3, 1, "relu", 2))
            C, H, W = K, H // 2, W // 2
        if len(conv) < 2 or C * H * W > 40000:
            continue
        classes = rnd.choice([10, 37, 100])
        cases.append((conv, [DenseSpec(C * H * W, 64, "relu"), DenseSpec(64, classes, "identity")], classes, "normal"))
    return cases


LAYERS = layer_cases()
NETS = net_cases()
STACKS = stack_cases()


def layer_id(c):
    return f"N{c.N}C{c.C}_{c.H}x{c.W}_K{c.K}_{c.R}x{c.S}p{c.pad}_{c.act}_pool{c.pool}"


def net_id(case):
    conv, dense, classes, kind = case
    return "B%d_" % conv[0].N + "_".join(f"c{c.C}-{c.K}k{c.R}p{c.pad}{c.act[0]}{c.pool}" for c in conv) + \
        "_" + "-".join(str(d.out) for d in dense) + "_" + kind[0]


@pytest.mark.parametrize("i", range(N_LAYERS), ids=[layer_id(c) for c in LAYERS])
def test_sweep_layer_trio(i):
    cs = LAYERS[i]
    print(f"sweep layer {i}: {cs}", flush=True)
    x, w, b, dy = T.rand_layer(cs, 5000 + i)
    T.check_trio(cs, x, w, b, dy)


@pytest.mark.parametrize("i", range(N_NETS), ids=[net_id(c) for c in NETS])
def test_sweep_network_step(i):
    conv, dense, classes, kind = NETS[i]
    print(f"sweep network {i}: {net_id(NETS[i])}", flush=True)
    w = wl._cnn(100 + i, "sweep", conv, dense, classes, 0.05, kind, None)
    T.check_cnn(w)
    T.check_forward(w)


def stack_id(case):
    conv = case[0]
    return f"B{conv[0].N}_{conv[0].H}x{conv[0].W}_" + "-".join([str(conv[0].C)] + [str(c.K) for c in conv])


@pytest.mark.parametrize("i", range(N_STACKS), ids=[stack_id(c) for c in STACKS])
def test_sweep_pooled_3x3_stack_step(i):
    conv, dense, classes, kind = STACKS[i]
    print(f"sweep stack {i}: {stack_id(STACKS[i])}", flush=True)
    T.check_cnn(wl._cnn(300 + i, "sweep", conv, dense, classes, 0.02, kind, None))
