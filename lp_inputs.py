"""Seeded synthetic inputs with the shapes and value distributions of the VGG16
workloads (the paper evaluates on ImageNet images and trained VGG16 weights,
Sec. 2.2-2.5; neither is available, so these stand in for them).

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark.  It holds no arithmetic of the method: only shapes and random draws.
All tensors are float32, activations NCHW, weights [Cout][Cin][R][S], FC
weights [Nout][K]; generator = numpy PCG64 seeded per tensor.
"""
import math

import numpy as np

# (name, Cin, Cout, input H=W, 2x2 max-pool after this layer)
VGG16_CONV = [
    ("conv1_1", 3, 64, 224, False),
    ("conv1_2", 64, 64, 224, True),
    ("conv2_1", 64, 128, 112, False),
    ("conv2_2", 128, 128, 112, True),
    ("conv3_1", 128, 256, 56, False),
    ("conv3_2", 256, 256, 56, False),
    ("conv3_3", 256, 256, 56, True),
    ("conv4_1", 256, 512, 28, False),
    ("conv4_2", 512, 512, 28, False),
    ("conv4_3", 512, 512, 28, True),
    ("conv5_1", 512, 512, 14, False),
    ("conv5_2", 512, 512, 14, False),
    ("conv5_3", 512, 512, 14, True),
]

# Giga1Net convolution layers (Table 1 of the paper): (name, Cin, Cout, kernel size, input
# width = height, zero padding, 2x2 max-pool after).  The table gives kernel sizes, channel counts,
# input sizes and where the pools are, not the paddings; the paddings here are the ones that make
# each layer's input size equal the previous layer's (pooled) output size at stride 1.
GIGA1NET_CONV = [
    ("conv1", 3, 16, 1, 224, 0, True),
    ("conv2", 16, 16, 7, 112, 1, True),
    ("conv3", 16, 32, 7, 54, 0, True),
    ("conv4", 32, 64, 5, 24, 1, False),
    ("conv5", 64, 64, 5, 22, 1, False),
    ("conv6", 64, 64, 5, 20, 1, False),
    ("conv7", 64, 128, 3, 18, 1, False),
    ("conv8", 128, 128, 3, 18, 1, False),
    ("conv9", 128, 128, 3, 18, 1, False),
    ("conv10", 128, 128, 3, 18, 1, False),
    ("conv11", 128, 128, 3, 18, 1, True),
]

# (name, K, Nout, ReLU after)
VGG16_FC = [
    ("fc6", 25088, 4096, True),
    ("fc7", 4096, 4096, True),
    ("fc8", 4096, 1000, False),
]


def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def normal(shape, std, seed, stream=0):
    return (_rng(seed, stream).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def relu_normal(shape, seed, stream=0):
    """ReLU(N(0,1)): about half the entries are exactly zero."""
    return np.maximum(_rng(seed, stream).standard_normal(shape, dtype=np.float32), np.float32(0))


def uniform01(shape, seed, stream=0):
    return _rng(seed, stream).random(shape, dtype=np.float32)


def he_normal_conv(cout, cin, r, s, seed, stream=0):
    return normal((cout, cin, r, s), math.sqrt(2.0 / (cin * r * s)), seed, stream)


def config1(seed=0):
    """Single conv layer: batch 1, 16->16 channels, 16x16, 3x3; x ReLU(N(0,1)), w N(0, std 0.1)."""
    x = relu_normal((1, 16, 16, 16), seed, 0)
    w = normal((16, 16, 3, 3), 0.1, seed, 1)
    return x, w


def config2(seed=1, batch=8, hw=224):
    """conv1_2-shaped layer: 64->64 channels, 3x3, He-normal weights, ReLU(N(0,1)) activations."""
    x = relu_normal((batch, 64, hw, hw), seed, 0)
    w = he_normal_conv(64, 64, 3, 3, seed, 1)
    return x, w


def vgg16_conv_weights(seed=2, layers=None):
    """He-normal weights for the 13 conv layers (or the named subset), in order."""
    out = []
    for i, (name, cin, cout, _, _) in enumerate(VGG16_CONV):
        if layers is None or name in layers:
            out.append(he_normal_conv(cout, cin, 3, 3, seed, 100 + i))
    return out


def giga1net_conv_weights(seed=5):
    """He-normal weights [Cout,Cin,k,k] for the eleven Giga1Net conv layers."""
    return [he_normal_conv(cout, cin, k, k, seed, 100 + i) for i, (_, cin, cout, k, *_rest) in enumerate(GIGA1NET_CONV)]


def config3_input(seed=2, batch=32, hw=224):
    """Image batch ~U(0,1), [batch,3,hw,hw]."""
    return uniform01((batch, 3, hw, hw), seed, 0)


CONFIG4_LAYERS = [n for (n, *_rest) in VGG16_CONV[4:]]  # conv3_1 .. conv5_3


def config4_layer(index, seed=3, batch=64):
    """index into VGG16_CONV[4:]; returns (name, x, w) with x ReLU(N(0,1)) at the layer's true shape."""
    name, cin, cout, hw, _ = VGG16_CONV[4 + index]
    x = relu_normal((batch, cin, hw, hw), seed, 10 + index)
    w = he_normal_conv(cout, cin, 3, 3, seed, 100 + index)
    return name, x, w


def config5_input(seed=4, batch=256, k=25088):
    return relu_normal((batch, k), seed, 0)


def config5_weights(seed=4, dims=None):
    """N(0, std 0.01) weights for fc6/fc7/fc8 (or a list of (K, Nout) overrides)."""
    dims = dims or [(k, n) for (_, k, n, _) in VGG16_FC]
    return [normal((n, k), 0.01, seed, 100 + i) for i, (k, n) in enumerate(dims)]
