"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module holds no arithmetic of the convolution method itself: it only
draws the int8 tensors that both the GPU library and the CPU oracle are fed
with, so the two sides see bit-identical inputs without sharing any code of
the method.

Generator: the splitmix64 stream (Steele, Lea, Flood, "Fast splittable
pseudorandom number generators", OOPSLA 2014).  Element k of a tensor filled
in memory order is the top byte of the k-th 64-bit output, reinterpreted as a
signed byte, i.e. i.i.d. uniform on [-128, 127] -- the value range the paper
states for quantised weights and activations (section 6: signed 8-bit integers).
"""
from __future__ import annotations

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, count: int) -> np.ndarray:
    """First `count` outputs of splitmix64 started from `seed` (uint64 array)."""
    with np.errstate(over="ignore"):
        k = np.arange(1, count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + k * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def int8_tensor(seed: int, shape) -> np.ndarray:
    """int8 tensor of `shape`, uniform on [-128,127], filled in C order."""
    count = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(count, dtype=np.int8)
    chunk = 1 << 22
    for lo in range(0, count, chunk):
        hi = min(count, lo + chunk)
        with np.errstate(over="ignore"):
            k = np.arange(lo + 1, hi + 1, dtype=np.uint64)
            z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + k * _GAMMA
            z = (z ^ (z >> np.uint64(30))) * _M1
            z = (z ^ (z >> np.uint64(27))) * _M2
            z = z ^ (z >> np.uint64(31))
        out[lo:hi] = (z >> np.uint64(56)).astype(np.uint8).view(np.int8)
    return out.reshape(shape)


# ---------------------------------------------------------------------------
# Workload descriptions.  Layer shapes follow the paper's experiment section
# (VGG16 3x3 layers of Table 4 at the standard VGG16 widths, a 5x5 layer like
# the Inception-v3 ones named there) with synthetic values; nothing here comes
# from the datasets or trained weights the paper measured on.
# ---------------------------------------------------------------------------

def layer_config(idx: int) -> dict:
    """Single-layer workloads 1..4 (dict of N,C,K,H,W,r,m,pad,moduli,seed_x,seed_w)."""
    table = {
        1: dict(N=1, C=16, K=16, H=16, W=16, r=3, m=8, pad=1, moduli=(251, 241, 239)),
        2: dict(N=1, C=256, K=256, H=56, W=56, r=3, m=8, pad=1, moduli=(251, 241, 239, 233)),
        3: dict(N=1, C=128, K=128, H=28, W=28, r=5, m=12, pad=2, moduli=(251, 241, 239, 233)),
        4: dict(N=1, C=512, K=512, H=28, W=28, r=3, m=14, pad=1, moduli=(65521, 65519)),
    }
    cfg = dict(table[idx])
    cfg["name"] = f"config{idx}"
    cfg["seed_x"] = 1000 * idx + 1
    cfg["seed_w"] = 1000 * idx + 2
    return cfg


def layer_tensors(cfg: dict):
    """(x, w) int8 arrays of a single-layer workload: x [N,C,H,W], w [K,C,r,r]."""
    x = int8_tensor(cfg["seed_x"], (cfg["N"], cfg["C"], cfg["H"], cfg["W"]))
    w = int8_tensor(cfg["seed_w"], (cfg["K"], cfg["C"], cfg["r"], cfg["r"]))
    return x, w


# VGG16 convolution stack: (name, C, K, H=W of the layer's input, pool after?)
VGG16_LAYERS = (
    ("conv1_1", 3, 64, 224, False), ("conv1_2", 64, 64, 224, True),
    ("conv2_1", 64, 128, 112, False), ("conv2_2", 128, 128, 112, True),
    ("conv3_1", 128, 256, 56, False), ("conv3_2", 256, 256, 56, False), ("conv3_3", 256, 256, 56, True),
    ("conv4_1", 256, 512, 28, False), ("conv4_2", 512, 512, 28, False), ("conv4_3", 512, 512, 28, True),
    ("conv5_1", 512, 512, 14, False), ("conv5_2", 512, 512, 14, False), ("conv5_3", 512, 512, 14, False),
)


def vgg16_stack(batch: int = 8, hw: int = 224):
    """Workload 5: list of per-layer dicts for the 13-layer 3x3 stack.

    `hw` scales the input plane (224 for the full workload; a smaller multiple
    of 16 gives the same stack on a reduced plane for quick parity runs).
    The requantisation shift of each layer is fixed here so that every user of
    the workload applies the same one: s = round(log2(74*sqrt(9*C))), which
    keeps the int8 activations of uniform random layers spread over the int8
    range without collapsing to zero.
    """
    import math
    layers = []
    scale = hw / 224.0
    for li, (name, C, K, H, pool) in enumerate(VGG16_LAYERS):
        h = int(round(H * scale))
        shift = int(round(math.log2(74.0 * math.sqrt(9.0 * C))))
        moduli = (251, 241, 239) if C == 3 else (251, 241, 239, 233)
        layers.append(dict(name=name, N=batch, C=C, K=K, H=h, W=h, r=3, m=8, pad=1,
                           moduli=moduli, shift=shift, pool=pool,
                           seed_w=5000 + 10 * li + 2))
    return layers


VGG16_SEED_X = 5001
