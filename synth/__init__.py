"""Seeded synthetic inputs for the SqueezeNet forward path.

This module only draws numbers and names shapes; it holds none of the method's
arithmetic.  Both the CPU oracle's tests and the GPU tests take their tensors
from here so that the two sides see the same values.

The paper runs one 224x224 RGB photograph through trained SqueezeNet
(section "Convolutional Neural Networks").  Neither the photographs nor the
trained weights are available, and the arithmetic does not depend on them, so
seeded tensors of the same shapes stand in: pixel-like uniform[0,1) inputs (or
normal(0,1) for the reduced-precision sweep), He-normal kernels with standard
deviation sqrt(2 / (Cin*K*K)), which keeps activations O(1) through all 26
convolutions, and biases uniform[-0.1, 0.1].

Draw order for a seed is fixed: the input first, then for each convolution in
network order its kernel and then its bias.
"""
from __future__ import annotations

import numpy as np

# (name, Cin, Cout, K, stride, pad, input height) of the 26 convolutions, network order.
_FIRES = (("fire2", 96, 16, 64, 55), ("fire3", 128, 16, 64, 55), ("fire4", 128, 32, 128, 55),
          ("fire5", 256, 32, 128, 27), ("fire6", 256, 48, 192, 27), ("fire7", 384, 48, 192, 27),
          ("fire8", 384, 64, 256, 27), ("fire9", 512, 64, 256, 13))


def conv_layers():
    layers = [("conv1", 3, 96, 7, 2, 2, 224)]
    for name, cin, sq, e, h in _FIRES:
        layers.append((name + "/sq", cin, sq, 1, 1, 0, h))
        layers.append((name + "/e1", sq, e, 1, 1, 0, h))
        layers.append((name + "/e3", sq, e, 3, 1, 1, h))
    layers.append(("conv10", 512, 1000, 1, 1, 0, 13))
    return layers


def second_network_layers():
    """Convolution shapes of a second, different CNN (the paper's scheme is meant for any CNN,
    section "Introduction"): the five convolutions of the classic 2012 ImageNet network in its
    ungrouped single-tower form -- 11x11 stride 4, 5x5 pad 2 and three 3x3 pad 1 layers on
    227 -> 55 -> 27 -> 13 feature maps.  Same tuple layout as conv_layers()."""
    return [("c1_11x11s4", 3, 96, 11, 4, 0, 227), ("c2_5x5p2", 96, 256, 5, 1, 2, 27),
            ("c3_3x3p1", 256, 384, 3, 1, 1, 13), ("c4_3x3p1", 384, 384, 3, 1, 1, 13),
            ("c5_3x3p1", 384, 256, 3, 1, 1, 13)]


def fire_layers():
    return list(_FIRES)


def uniform01(rng, shape):
    return rng.random(shape, dtype=np.float32)


def normal01(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def he_normal(rng, cout, cin, k):
    std = np.float32(np.sqrt(2.0 / (cin * k * k)))
    return rng.standard_normal((cout, cin, k, k), dtype=np.float32) * std


def bias(rng, cout):
    return (rng.random(cout, dtype=np.float32) * np.float32(0.2) - np.float32(0.1)).astype(np.float32)


def conv_params(rng, cout, cin, k):
    w = he_normal(rng, cout, cin, k)
    b = bias(rng, cout)
    return w, b


def squeezenet_params(rng):
    """52 arrays: kernel, bias for each convolution in network order."""
    out = []
    for _, cin, cout, k, _, _, _ in conv_layers():
        w, b = conv_params(rng, cout, cin, k)
        out += [w, b]
    return out


def config_fire2(seed: int = 0, n: int = 1):
    """Workload 1: one fire2 module, input n x 96 x 55 x 55 uniform[0,1)."""
    rng = np.random.default_rng(seed)
    x = uniform01(rng, (n, 96, 55, 55))
    w_sq, b_sq = conv_params(rng, 16, 96, 1)
    w_e1, b_e1 = conv_params(rng, 64, 16, 1)
    w_e3, b_e3 = conv_params(rng, 64, 16, 3)
    return dict(x=x, w_sq=w_sq, b_sq=b_sq, w_e1=w_e1, b_e1=b_e1, w_e3=w_e3, b_e3=b_e3)


def config_conv1(seed: int = 1, n: int = 1, size: int = 224):
    """Workload 2: conv1 (96 kernels 7x7, stride 2) then max pooling 3x3 stride 2.
    size=224 goes with pad 2, size=227 with pad 0; both give 111 x 111."""
    rng = np.random.default_rng(seed)
    x = uniform01(rng, (n, 3, size, size))
    w, b = conv_params(rng, 96, 3, 7)
    return dict(x=x, w=w, b=b, pad=2 if size == 224 else 0)


def config_squeezenet(seed: int = 2, n: int = 1):
    """Workloads 3 (n=1, seed 2) and 4 (n=64, seed 3): the whole network."""
    rng = np.random.default_rng(seed)
    x = uniform01(rng, (n, 3, 224, 224))
    return dict(x=x, params=squeezenet_params(rng))


def config_layer_sweep(seed: int = 4, n: int = 256, only=None, layers=None):
    """Workload 5: every convolution shape on its own, normal(0,1) inputs.
    Yields (name, x, w, b, stride, pad) one layer at a time (the tensors are large).
    Each layer has its own stream, keyed by (seed, layer name), so a selection of
    layers sees the same numbers as the full sweep.  `layers` replaces the SqueezeNet
    list (second_network_layers() for the second workload)."""
    for name, cin, cout, k, s, p, h in (conv_layers() if layers is None else layers):
        if only is not None and name not in only:
            continue
        lrng = np.random.default_rng([seed, hash_name(name)])
        x = normal01(lrng, (n, cin, h, h))
        w, b = conv_params(lrng, cout, cin, k)
        yield name, x, w, b, s, p


def hash_name(name: str) -> int:
    """Stable small integer for a layer name (Python's hash() is salted)."""
    v = 0
    for ch in name.encode():
        v = (v * 131 + ch) % 1000003
    return v
