"""Seeded synthetic inputs and the workload (layer) lists, shared by tests and bench.py.

This module holds none of the method's arithmetic: it only draws random tensors, rounds them
once to bfloat16 bit patterns (the same bits are then handed to the device path and, widened
exactly, to the CPU oracle) and lists the layer shapes of the two networks the paper evaluates
(AlexNet and VGG-16, Section 4.1).  The tensors stand in for the ImageNet-style images, trained
weights and labels those networks imply; none of that data is needed for throughput or parity.

Recipe: tensor `t` of workload `c` comes from numpy.random.default_rng([181101532, c, t]);
images and upstream gradients ~ N(0,1); weights ~ N(0, 2/fan_in) (variance; fan_in = C*R*S or
in_features); labels uniform over the classes.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 181101532


def rng(config: int, tensor: int):
    return np.random.default_rng([SEED_BASE, int(config), int(tensor)])


def f32_to_bf16_bits(a):
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def normal_bf16(g, shape, std=1.0):
    """N(0, std^2) samples as bfloat16 bit patterns (uint16)."""
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return f32_to_bf16_bits(a)


def he_weight_bf16(g, shape):
    """Weights ~ N(0, 2/fan_in); shape is KRSC (conv) or [out][in] (FC)."""
    fan_in = int(np.prod(shape[1:]))
    return normal_bf16(g, shape, std=float(np.sqrt(2.0 / fan_in)))


def labels(g, batch, classes=1000):
    return g.integers(0, classes, size=batch, dtype=np.int32)


def out_dim(n_in, pad, win, stride):
    return (n_in + 2 * pad - win) // stride + 1


# ---- workloads ---------------------------------------------------------------------------------
# conv layer: (name, C, K, R, stride, pad, pool_after) with pool = (window, stride) or None;
# every conv is followed by ReLU.  Input images are 224x224x3.

ALEXNET_CONVS = [
    ("conv1", 3, 64, 11, 4, 2, (3, 2)),
    ("conv2", 64, 192, 5, 1, 2, (3, 2)),
    ("conv3", 192, 384, 3, 1, 1, None),
    ("conv4", 384, 256, 3, 1, 1, None),
    ("conv5", 256, 256, 3, 1, 1, (3, 2)),
]

_VGG_BLOCKS = [(64, 2), (128, 2), (256, 3), (512, 3), (512, 3)]


def _vgg_convs():
    out, c = [], 3
    for bi, (k, reps) in enumerate(_VGG_BLOCKS, start=1):
        for j in range(1, reps + 1):
            out.append((f"conv{bi}_{j}", c, k, 3, 1, 1, (2, 2) if j == reps else None))
            c = k
    return out


VGG16_CONVS = _vgg_convs()

# FC head: (name, in, out, relu)
ALEXNET_FCS = [("fc6", 9216, 4096, True), ("fc7", 4096, 4096, True), ("fc8", 4096, 1000, False)]
VGG16_FCS = [("fc6", 25088, 4096, True), ("fc7", 4096, 4096, True), ("fc8", 4096, 1000, False)]

NETS = {"alexnet": (ALEXNET_CONVS, ALEXNET_FCS), "vgg16": (VGG16_CONVS, VGG16_FCS)}


def conv_shapes(convs, image=224):
    """Walk a conv list; yields dicts with the geometry of every layer (per image)."""
    h = image
    out = []
    for (name, c, k, r, st, pad, pool) in convs:
        p = out_dim(h, pad, r, st)
        d = dict(name=name, H=h, W=h, C=c, K=k, R=r, S=r, stride=st, pad=pad, P=p, Q=p, pool=pool)
        h = p
        if pool is not None:
            h = out_dim(h, 0, pool[0], pool[1])
        d["out_hw"] = h
        out.append(d)
    return out


def step_flops_per_image(net):
    """Direct-convolution FLOP count of one training step per image: every pass counts
    2*P*Q*K*C*R*S (taps in the padding included); fwd + dgrad + wgrad, with the first
    layer's dgrad left out; FC layers count 2*in*out per pass, three passes."""
    convs, fcs = NETS[net]
    total = 0
    for i, d in enumerate(conv_shapes(convs)):
        f = 2 * d["P"] * d["Q"] * d["K"] * d["C"] * d["R"] * d["S"]
        total += 3 * f if i > 0 else 2 * f
    for (_, n_in, n_out, _) in fcs:
        total += 3 * 2 * n_in * n_out
    return total
