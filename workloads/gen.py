"""Seeded synthetic tensors for a workload.

Draw order (fixed, so both consumers read the same bytes): image, then for
every conv layer its weight then its bias, then labels, then the mask
permutation.  Everything comes from numpy.random.default_rng(seed).

The paper times its networks on random images and random kernels (Sec. 5.1:
run time depends only on image size and network structure), so synthetic
tensors of the right shapes are the paper's own workload.
"""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from .nets import Net, Config, CONFIGS


@dataclass
class Workload:
    net: Net
    image: np.ndarray            # float32 [N, C0, H, W], unpadded, U[-1, 1]
    weights: List[np.ndarray]    # float32 [K, C, k, k] per conv layer
    biases: List[np.ndarray]     # float32 [K] per conv layer
    labels: np.ndarray           # int32 [N, H, W]
    mask: np.ndarray             # uint8 [N, H, W], exactly round(frac*N*H*W) ones
    dtype: str = "f32"


def make_params(net: Net, rng: np.random.Generator, bias_std: float = 0.0):
    """Weights (He-normal or N(0, 0.05)) and biases for every conv layer."""
    ws, bs = [], []
    for (K, C, kh, kw) in net.conv_shapes():
        if net.init == "he":
            std = np.sqrt(2.0 / (C * kh * kw))
        elif net.init == "n0.05":
            std = 0.05
        else:
            raise ValueError(net.init)
        ws.append((rng.standard_normal((K, C, kh, kw)) * std).astype(np.float32))
        if bias_std > 0.0:
            bs.append((rng.standard_normal(K) * bias_std).astype(np.float32))
        else:
            rng.standard_normal(K)      # keep the stream position independent of bias_std
            bs.append(np.zeros(K, np.float32))
    return ws, bs


def pick_mask(rng: np.random.Generator, shape, frac: float) -> np.ndarray:
    """Exactly round(frac * size) distinct pixels from a seeded permutation."""
    total = int(np.prod(shape))
    count = int(round(frac * total))
    mask = np.zeros(total, np.uint8)
    if count > 0:
        mask[rng.permutation(total)[:count]] = 1
    return mask.reshape(shape)


def make_workload(net: Net, N: int, H: int, W: int, mask_frac: float, seed: int = 0,
                  bias_std: float = 0.0, positive_frac: float = -1.0,
                  dtype: str = "f32") -> Workload:
    rng = np.random.default_rng(seed)
    image = rng.uniform(-1.0, 1.0, size=(N, net.C0, H, W)).astype(np.float32)
    ws, bs = make_params(net, rng, bias_std)
    if positive_frac >= 0.0:
        labels = (rng.random((N, H, W)) < positive_frac).astype(np.int32)
    else:
        labels = rng.integers(0, net.classes, size=(N, H, W)).astype(np.int32)
    mask = pick_mask(rng, (N, H, W), mask_frac)
    return Workload(net, image, ws, bs, labels, mask, dtype)


def config_workload(i: int, bias_std: float = 0.0) -> Workload:
    c: Config = CONFIGS[i]
    return make_workload(c.net, c.N, c.H, c.W, c.mask_frac, c.seed, bias_std,
                         c.positive_frac, c.dtype)


def sample_pixels(N: int, H: int, W: int, count: int, seed: int = 1) -> np.ndarray:
    """int32 [P, 3] (n, i, j): the four corners and edge midpoints of image 0, then
    seeded uniform pixels over the batch, without duplicates."""
    fixed = [(0, 0, 0), (0, 0, W - 1), (0, H - 1, 0), (0, H - 1, W - 1),
             (0, 0, W // 2), (0, H - 1, W // 2), (0, H // 2, 0), (0, H // 2, W - 1)]
    seen, out = set(), []
    for p in fixed:
        if p not in seen:
            seen.add(p)
            out.append(p)
    rng = np.random.default_rng(seed)
    total = N * H * W
    count = min(count, total)
    while len(out) < count:
        f = int(rng.integers(0, total))
        p = (f // (H * W), (f // W) % H, f % W)
        if p not in seen:
            seen.add(p)
            out.append(p)
    return np.asarray(out[:max(count, 0)], np.int32).reshape(-1, 3)
