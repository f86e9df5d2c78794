"""Seeded synthetic inputs and workload descriptions shared by the tests, the
benchmark and the smoke check.

Holds no arithmetic of the method: only plain hyper-parameter tables and
numpy.random.default_rng draws.  The oracle and the HIP binding each turn the
tables into their own configuration objects.

The paper trains on ImageNet ILSVRC-2012 (Section 1, Section 3), which is not
available here; the synthetic tensors below take its shapes (stored 3x256x256
uint8 pictures, 227x227 crops, 1000 classes) and stand in for it.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 14122302

# (cout, k, stride, pad, groups, lrn, pool)
ALEXNET = {
    "name": "alexnet",
    "in_c": 3, "crop": 227, "raw": 256,
    "conv": [
        (96, 11, 4, 0, 1, 1, 1),
        (256, 5, 1, 2, 2, 1, 1),
        (384, 3, 1, 1, 1, 0, 0),
        (384, 3, 1, 1, 2, 0, 0),
        (256, 3, 1, 1, 2, 0, 1),
    ],
    "fc": [4096, 4096, 1000],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

# Small net with the same layer census: 63 -> conv1(7,s2) 29 -> pool 14 -> conv2 14
# -> pool 6 -> conv3/4/5 6 -> pool 2; flatten 32*2*2 = 128 -> 256 -> 256 -> 10.
MINI = {
    "name": "mini",
    "in_c": 3, "crop": 63, "raw": 63,
    "conv": [
        (16, 7, 2, 0, 1, 1, 1),
        (32, 5, 1, 2, 2, 1, 1),
        (48, 3, 1, 1, 1, 0, 0),
        (48, 3, 1, 1, 2, 0, 0),
        (32, 3, 1, 1, 2, 0, 1),
    ],
    "fc": [256, 256, 10],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

# A mid-sized net whose tensors span several GEMM tiles with ragged tails and
# which needs a real crop window (raw > crop).  Used by parity tests only.
MIDI = {
    "name": "midi",
    "in_c": 3, "crop": 67, "raw": 80,
    "conv": [
        (24, 11, 4, 0, 1, 1, 1),
        (40, 5, 1, 2, 2, 1, 1),
        (72, 3, 1, 1, 1, 0, 0),
        (72, 3, 1, 1, 2, 0, 0),
        (40, 3, 1, 1, 2, 0, 1),
    ],
    "fc": [200, 136, 37],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

# 3x3 unit-stride layers with every padding (0, 1, 2) over map sizes that are not multiples of the 4x4 tiles
# of the transformed path: 31 -> 29 -> 31 -> 31 (pool 15) -> 13 -> 15 (pool 7); flatten 8*7*7 = 392.
PADS = {
    "name": "pads",
    "in_c": 3, "crop": 31, "raw": 31,
    "conv": [
        (8, 3, 1, 0, 1, 0, 0),
        (16, 3, 1, 2, 1, 0, 0),
        (16, 3, 1, 1, 2, 0, 1),
        (24, 3, 1, 0, 1, 0, 0),
        (8, 3, 1, 2, 2, 0, 1),
    ],
    "fc": [32, 16, 5],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

# Degenerate sizes: 15 -> conv1(3,s2) 7 -> pool 3 -> conv2 3 -> pool 1 -> conv3/4/5 on 1x1 maps; flatten 8.
TINY = {
    "name": "tiny",
    "in_c": 3, "crop": 15, "raw": 15,
    "conv": [
        (8, 3, 2, 0, 1, 1, 1),
        (8, 3, 1, 1, 2, 1, 1),
        (8, 3, 1, 1, 1, 0, 0),
        (8, 3, 1, 1, 2, 0, 0),
        (8, 3, 1, 1, 2, 0, 0),
    ],
    "fc": [12, 8, 3],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

# Channel counts, group sizes and layer widths that are no multiples of four, a 1x1 kernel and three groups:
# every kernel that has a 16-byte form falls back to its 4-byte form.
# 33 -> conv1(5,s2,p1) 16 -> pool 7 -> conv2 7 -> pool 3 -> conv3/4 3 -> conv5(1x1) 3 -> pool 1; flatten 7.
ODD = {
    "name": "odd",
    "in_c": 3, "crop": 33, "raw": 35,
    "conv": [
        (6, 5, 2, 1, 1, 1, 1),
        (10, 3, 1, 1, 2, 1, 1),
        (9, 3, 1, 1, 1, 0, 0),
        (15, 3, 1, 1, 3, 0, 0),
        (7, 1, 1, 0, 1, 0, 1),
    ],
    "fc": [13, 11, 3],
    "lrn": (5, 2.0, 1e-4, 0.75),
    "dropout_p": 0.5, "lr": 0.01, "momentum": 0.9, "weight_decay": 5e-4,
}

WORKLOADS = {"alexnet": ALEXNET, "mini": MINI, "midi": MIDI, "pads": PADS, "tiny": TINY, "odd": ODD}


def make_params(shapes, seed: int, bias_value: float = 0.0, std: float = 0.01):
    """Weights N(0, std^2), biases constant; returned as float32 arrays keyed
    like `shapes` (name -> shape, names ending in .w or .b)."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shp in shapes.items():
        if name.endswith(".w"):
            out[name] = (rng.standard_normal(shp) * std).astype(np.float32)
        else:
            out[name] = np.full(shp, bias_value, np.float32)
    return out


def make_random_like(shapes, seed: int, std: float = 1.0):
    """N(0, std^2) float32 tensor for every entry of `shapes` (momentum, biases ...)."""
    rng = np.random.default_rng(seed)
    return {k: (rng.standard_normal(s) * std).astype(np.float32) for k, s in shapes.items()}


def make_float_batch(batch: int, c: int, h: int, w: int, classes: int, seed: int):
    """Already-preprocessed input uniform[-1,1] and uniform labels."""
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1.0, 1.0, size=(batch, c, h, w)).astype(np.float32)
    labels = rng.integers(0, classes, size=batch).astype(np.int32)
    return x, labels


def make_raw_batch(batch: int, c: int, raw_h: int, raw_w: int, classes: int, seed: int):
    """Stored pictures uint8 uniform[0,255] and uniform labels."""
    rng = np.random.default_rng(seed)
    raw = rng.integers(0, 256, size=(batch, c, raw_h, raw_w), dtype=np.uint8)
    labels = rng.integers(0, classes, size=batch).astype(np.int32)
    return raw, labels


def make_mean_image(c: int, raw_h: int, raw_w: int, seed: int):
    """Non-constant mean image uniform[100,140) so indexing mistakes show."""
    rng = np.random.default_rng(seed)
    return rng.uniform(100.0, 140.0, size=(c, raw_h, raw_w)).astype(np.float32)


def make_normal(shape, seed: int, std: float = 1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(np.float32)
