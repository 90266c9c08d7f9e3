"""Synthetic convolution workloads and their seeded input generators.

This module holds none of the convolution's arithmetic: it names layer shapes
and draws seeded random tensors.  It is the only module that both the GPU
tests and the CPU-oracle tests share, so that both sides see the same inputs.

The layer shapes stand in for the workloads the paper measures (Figures 1-3:
the convolution layers of ResNet-50 at batch 1/4/32; section 3 also names
VGG): VGG-16-style 3x3 stacks and ResNet-50-style 7x7/1x1/3x3 layers.  Values
are i.i.d. synthetic (no dataset, no trained weights).
"""
from collections import namedtuple

import numpy as np

PAD_VALID = 0
PAD_SAME = 1

BASE_SEED = 190404174

Layer = namedtuple(
    "Layer",
    "name batch in_rows in_cols channels features window_rows window_cols "
    "stride_rows stride_cols padding dist group")


def _layer(name, n, hw, c, k, win, stride, padding, dist, group):
    return Layer(name, n, hw, hw, c, k, win, win, stride, stride, padding, dist, group)


_VGG = [(224, 64, 64), (112, 128, 128), (56, 256, 256), (28, 512, 512), (14, 512, 512)]

LAYERS = {}


def _add(layer):
    LAYERS[layer.name] = layer


# Group 0: the tiny case.
_add(_layer("T1", 1, 8, 4, 4, 3, 1, PAD_SAME, "uniform", 0))
# Group 1: VGG-16-style 3x3 sweep, stride 1, SAME, batch 1 and 16.
for _n in (1, 16):
    for _hw, _c, _k in _VGG:
        _add(_layer("V%d-N%d" % (_hw, _n), _n, _hw, _c, _k, 3, 1, PAD_SAME, "uniform", 1))
# Group 2: ResNet-50-style layers, batch 32, normal(0,1) values.
_add(_layer("R7x7", 32, 224, 3, 64, 7, 2, PAD_SAME, "normal", 2))
_add(_layer("R1x1a", 32, 56, 64, 256, 1, 1, PAD_SAME, "normal", 2))
_add(_layer("R1x1b", 32, 56, 256, 64, 1, 1, PAD_SAME, "normal", 2))
_add(_layer("R3x3", 32, 56, 64, 64, 3, 1, PAD_SAME, "normal", 2))
_add(_layer("R1x1s2", 32, 28, 512, 1024, 1, 2, PAD_SAME, "normal", 2))
# Group 3: large-batch 3x3 throughput layer and its VALID / stride-2 variants.
_add(_layer("L-same", 64, 56, 256, 256, 3, 1, PAD_SAME, "uniform", 3))
_add(_layer("L-valid", 64, 56, 256, 256, 3, 1, PAD_VALID, "uniform", 3))
_add(_layer("L-s2", 64, 56, 256, 256, 3, 2, PAD_SAME, "uniform", 3))
_add(_layer("L-s2valid", 64, 56, 256, 256, 3, 2, PAD_VALID, "uniform", 3))

# Group 4 (bf16 inputs, fp32 accumulate) reuses these shapes with uniform values.
BF16_LAYERS = ["V224-N16", "V112-N16", "V56-N16", "V28-N16", "V14-N16",
               "R3x3", "R1x1a", "R1x1b", "R1x1s2"]

VGG_N16 = ["V224-N16", "V112-N16", "V56-N16", "V28-N16", "V14-N16"]

# Group 5: the distinct convolution shapes of ResNet-50 at batch 32 (the workload of the paper's
# Figure 1; batch 1 and 4 below), derived from the architecture's published definition: a 7x7 stride-2 stem and four
# stages of bottleneck blocks (1x1 reduce, 3x3, 1x1 expand, 1x1 projection shortcuts) at 56, 28,
# 14 and 7 pixels with 64/128/256/512 bottleneck channels.  Both common placements of the
# stage's stride 2 are listed (on the first 1x1, or on the 3x3): 20 + 6 = 26 shapes.
# (image size, C, K, window, stride)
_RN50 = [
    (224, 3, 64, 7, 2),
    (56, 64, 64, 1, 1), (56, 64, 64, 3, 1), (56, 64, 256, 1, 1), (56, 256, 64, 1, 1),
    (56, 256, 128, 1, 2), (28, 128, 128, 3, 1), (28, 128, 512, 1, 1), (56, 256, 512, 1, 2),
    (28, 512, 128, 1, 1),
    (28, 512, 256, 1, 2), (14, 256, 256, 3, 1), (14, 256, 1024, 1, 1), (28, 512, 1024, 1, 2),
    (14, 1024, 256, 1, 1),
    (14, 1024, 512, 1, 2), (7, 512, 512, 3, 1), (7, 512, 2048, 1, 1), (14, 1024, 2048, 1, 2),
    (7, 2048, 512, 1, 1),
    # stride on the 3x3 instead of the first 1x1
    (56, 256, 128, 1, 1), (56, 128, 128, 3, 2), (28, 512, 256, 1, 1), (28, 256, 256, 3, 2),
    (14, 1024, 512, 1, 1), (14, 512, 512, 3, 2),
]
RESNET50 = {}
for _i, (_hw, _c, _k, _win, _st) in enumerate(_RN50):
    _name = "RN50-%02d-%dx%d-%dto%d-%dx%ds%d" % (_i + 1, _hw, _hw, _c, _k, _win, _win, _st)
    RESNET50[_name] = _layer(_name, 32, _hw, _c, _k, _win, _st, PAD_SAME, "normal", 5)
# The same 26 shapes at the two other batch sizes of the paper's Figures 2 and 3.
RESNET50_BATCHES = (1, 4, 32)
RESNET50_BY_BATCH = {32: RESNET50}
for _n in (1, 4):
    RESNET50_BY_BATCH[_n] = {}
    for _name, _l in RESNET50.items():
        _nm = "%s-N%d" % (_name, _n)
        RESNET50_BY_BATCH[_n][_nm] = _l._replace(name=_nm, batch=_n)
ALL_LAYERS = dict(LAYERS)
for _n in RESNET50_BATCHES:
    ALL_LAYERS.update(RESNET50_BY_BATCH[_n])
VGG_N1 = ["V224-N1", "V112-N1", "V56-N1", "V28-N1", "V14-N1"]


def layer_seed(layer):
    """Seed of a layer's generator: base seed + group, then a per-name offset."""
    if layer.name in LAYERS:
        return BASE_SEED + layer.group * 1000 + sorted(LAYERS).index(layer.name)
    base = layer.name.rsplit("-N", 1)[0] if layer.batch != 32 else layer.name
    offset = 0 if layer.batch == 32 else 100 * layer.batch
    return BASE_SEED + layer.group * 1000 + offset + sorted(RESNET50).index(base)


def round_to_bf16(x):
    """Round float32 values to the nearest bf16 (ties to even).

    Returns (float32 array holding the rounded values, uint16 array of bf16 bits).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    bits = u.astype(np.uint16)
    widened = (bits.astype(np.uint32) << 16).view(np.float32)
    return widened.reshape(x.shape), bits.reshape(x.shape)


def draw(shape, dist, rng):
    """One float32 tensor: 'uniform' = U[-1,1), 'normal' = N(0,1),
    'ints' = integers in [-4,4] (exact in fp32 and bf16), 'ones' = all 1."""
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "ints":
        return rng.integers(-4, 5, size=shape).astype(np.float32)
    if dist == "ones":
        return np.ones(shape, dtype=np.float32)
    raise ValueError("unknown distribution %r" % (dist,))


def make_inputs(layer, dist=None, seed=None, batch=None):
    """(input NHWC float32, filter HWCF float32) for a layer, from its seed.

    Input and filter are consecutive draws of one generator.  `dist` overrides
    the layer's value distribution, `batch` its batch size.
    """
    dist = dist or layer.dist
    rng = np.random.default_rng(layer_seed(layer) if seed is None else seed)
    n = layer.batch if batch is None else batch
    x = draw((n, layer.in_rows, layer.in_cols, layer.channels), dist, rng)
    f = draw((layer.window_rows, layer.window_cols, layer.channels, layer.features), dist, rng)
    return x, f


def make_case(shape_in, shape_f, dist, seed):
    """Inputs for an ad-hoc shape: NHWC input shape, HWCF filter shape."""
    rng = np.random.default_rng(seed)
    return draw(shape_in, dist, rng), draw(shape_f, dist, rng)
