"""Cube classifiers for video and seeded synthetic clips (the paper's closing
section: the method carried over to video with 3-D convolution and pooling).

A network is the list of layers of the ORIGINAL cube classifier: it looks at
patch_t frames of patch x patch pixels and must end in a 1 x 1 x 1 map with
`classes` channels.  Pure data and seeded random tensors: no arithmetic of the
method lives here.

Draw order: video, then for every conv layer its weight then its bias, then
labels, then the mask permutation (numpy.random.default_rng(seed)).
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

from .nets import CONV, MAXPOOL, AVGPOOL, ACT_NONE, ACT_RELU, ACT_TANH  # noqa: F401
from .gen import pick_mask


@dataclass(frozen=True)
class Layer3:
    kind: int          # CONV / MAXPOOL / AVGPOOL
    K: int             # output channels (conv)
    k: int             # square spatial kernel size
    s: int             # spatial stride
    kt: int            # temporal kernel size
    st: int            # temporal stride
    act: int = ACT_NONE


def conv3(K, k, kt, s=1, st=1, act=ACT_NONE):
    return Layer3(CONV, K, k, s, kt, st, act)


def maxpool3(k, kt, s=None, st=None):
    return Layer3(MAXPOOL, 0, k, k if s is None else s, kt, kt if st is None else st)


def avgpool3(k, kt, s=None, st=None):
    return Layer3(AVGPOOL, 0, k, k if s is None else s, kt, kt if st is None else st)


@dataclass(frozen=True)
class VideoNet:
    name: str
    C0: int
    patch_t: int                 # nt: frames of a cube
    patch: int                   # n: the cube is nt x n x n
    layers: Tuple[Layer3, ...]
    init: str = "he"

    def conv_shapes(self) -> List[Tuple[int, int, int, int, int]]:
        """(K, C, kt, k, k) for every conv layer, in order."""
        out, c = [], self.C0
        for L in self.layers:
            if L.kind == CONV:
                out.append((L.K, c, L.kt, L.k, L.k))
                c = L.K
        return out

    @property
    def classes(self) -> int:
        return self.conv_shapes()[-1][0]


@dataclass
class VideoWorkload:
    net: VideoNet
    video: np.ndarray            # float32 [N, C0, T, H, W], unpadded, U[-1, 1]
    weights: List[np.ndarray]    # float32 [K, C, kt, k, k] per conv layer
    biases: List[np.ndarray]     # float32 [K]
    labels: np.ndarray           # int32 [N, T, H, W]
    mask: np.ndarray             # uint8 [N, T, H, W]
    dtype: str = "f32"


def make_video_params(net: VideoNet, rng: np.random.Generator, bias_std: float = 0.0):
    ws, bs = [], []
    for (K, C, kt, kh, kw) in net.conv_shapes():
        std = np.sqrt(2.0 / (C * kt * kh * kw)) if net.init == "he" else 0.05
        ws.append((rng.standard_normal((K, C, kt, kh, kw)) * std).astype(np.float32))
        if bias_std > 0.0:
            bs.append((rng.standard_normal(K) * bias_std).astype(np.float32))
        else:
            rng.standard_normal(K)
            bs.append(np.zeros(K, np.float32))
    return ws, bs


def make_video_workload(net: VideoNet, N: int, T: int, H: int, W: int, mask_frac: float, seed: int = 0,
                        bias_std: float = 0.0, dtype: str = "f32") -> VideoWorkload:
    rng = np.random.default_rng(seed)
    video = rng.uniform(-1.0, 1.0, size=(N, net.C0, T, H, W)).astype(np.float32)
    ws, bs = make_video_params(net, rng, bias_std)
    labels = rng.integers(0, net.classes, size=(N, T, H, W)).astype(np.int32)
    mask = pick_mask(rng, (N, T, H, W), mask_frac)
    return VideoWorkload(net, video, ws, bs, labels, mask, dtype)


_R = ACT_RELU

# a small cube classifier for tests that check every voxel: 6 frames of 10 x 10 pixels
TINY_VIDEO = VideoNet("tinycube", 2, 6, 10, (
    conv3(6, 3, 2, act=_R),                 # -> 5 x 8 x 8
    maxpool3(2, 2, s=2, st=1),              # -> 4 x 4 x 4
    conv3(8, 3, 2, act=_R),                 # -> 3 x 2 x 2
    conv3(5, 2, 3)), init="n0.05")          # -> 1 x 1 x 1

# temporal and spatial strides that differ, an average pool, tanh: 9 frames of 11 x 11 pixels
STRIDED_VIDEO = VideoNet("stridedcube", 3, 9, 11, (
    conv3(5, 3, 3, s=2, st=2, act=ACT_TANH),    # -> 4 x 5 x 5
    avgpool3(2, 2, s=1, st=1),                  # -> 3 x 4 x 4
    conv3(7, 2, 1, act=_R),                     # -> 3 x 3 x 3
    maxpool3(3, 3, s=3, st=3),                  # -> 1 x 1 x 1
    conv3(4, 1, 1)), init="n0.05")

# The measured video workload: a clip classifier in the style of the scene-labelling network, 14 frames of
# 22 x 22 pixels per labelled voxel (temporal and spatial strides 2 in both pools).
CLIP_NET = VideoNet("clip14x22", 3, 14, 22, (
    conv3(32, 3, 3, act=_R), maxpool3(2, 2),
    conv3(64, 3, 3, act=_R), maxpool3(2, 2),
    conv3(128, 3, 2, act=_R),
    conv3(256, 2, 1, act=_R),       # fc 128*2*2 -> 256
    conv3(10, 1, 1)))               # fc 256 -> 10


@dataclass(frozen=True)
class VideoConfig:
    net: VideoNet
    N: int
    T: int
    H: int
    W: int
    mask_frac: float
    dtype: str = "f32"
    seed: int = 0


VIDEO_CONFIGS = (
    VideoConfig(TINY_VIDEO, 1, 5, 12, 14, 0.10),
    VideoConfig(CLIP_NET, 1, 16, 256, 256, 0.01),
)


def video_workload(i: int, bias_std: float = 0.0) -> VideoWorkload:
    c = VIDEO_CONFIGS[i]
    return make_video_workload(c.net, c.N, c.T, c.H, c.W, c.mask_frac, c.seed, bias_std, c.dtype)
