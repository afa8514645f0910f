"""Descriptions of the original (strided, patch-input) CNNs used as workloads.

A network is the list of layers of the ORIGINAL patch classifier (the one the
paper's Fig. 1(a) scans patch by patch): stride-s convolutions, stride-s
pools, and fully connected layers written as convolutions whose kernel covers
the whole remaining map (Sec. 3.4, last paragraph).  Fed an n x n patch it
must end in a 1 x 1 map with `classes` channels.

Pure data: nothing here knows about dilation, padding or any arithmetic.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

CONV, MAXPOOL, AVGPOOL = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_TANH = 0, 1, 2


@dataclass(frozen=True)
class Layer:
    kind: int          # CONV / MAXPOOL / AVGPOOL
    K: int             # output channels (conv); ignored for pools
    k: int             # square kernel size
    s: int             # stride in the original CNN
    act: int = ACT_NONE  # pointwise non-linearity applied after a conv


def conv(K, k, s=1, act=ACT_NONE):
    return Layer(CONV, K, k, s, act)


def maxpool(k, s=None):
    return Layer(MAXPOOL, 0, k, k if s is None else s)


def avgpool(k, s=None):
    return Layer(AVGPOOL, 0, k, k if s is None else s)


@dataclass(frozen=True)
class Net:
    name: str
    C0: int                      # input channels
    patch: int                   # n: the original CNN takes n x n patches
    layers: Tuple[Layer, ...]
    init: str = "he"             # "he" or "n0.05"

    def channels(self) -> List[int]:
        """Channel count after each layer."""
        out, c = [], self.C0
        for L in self.layers:
            if L.kind == CONV:
                c = L.K
            out.append(c)
        return out

    def patch_sizes(self) -> List[int]:
        """Spatial size of the patch CNN's map after each layer (valid, floor)."""
        out, m = [], self.patch
        for L in self.layers:
            m = (m - L.k) // L.s + 1
            out.append(m)
        return out

    @property
    def classes(self) -> int:
        return self.channels()[-1]

    def conv_shapes(self) -> List[Tuple[int, int, int, int]]:
        """(K, C, k, k) for every conv layer, in order."""
        out, c = [], self.C0
        for L in self.layers:
            if L.kind == CONV:
                out.append((L.K, c, L.k, L.k))
                c = L.K
        return out


# ---------------------------------------------------------------------------
# The five benchmark networks, and the paper's own Plain CNN_1 (Table 1).  ReLU follows every conv / fc except the last;
# pools whose type a configuration leaves open are max pools.
# ---------------------------------------------------------------------------
_R = ACT_RELU

_TINY = Net("tiny16", 3, 16, (
    conv(8, 5, 1, _R), maxpool(2, 2),
    conv(16, 3, 1, _R), maxpool(2, 2),
    conv(10, 2, 1)), init="n0.05")

_SCENE = Net("scene60", 3, 60, (
    conv(32, 5, 1, _R), maxpool(2, 2),
    conv(64, 5, 1, _R), maxpool(2, 2),
    conv(128, 5, 1, _R), maxpool(2, 2),
    conv(256, 4, 1, _R),        # fc 2048 -> 256
    conv(33, 1, 1)))            # fc 256 -> 33

_WIDE = Net("wide92", 3, 92, (
    conv(64, 5, 1, _R), maxpool(2, 2),
    conv(128, 5, 1, _R), maxpool(2, 2),
    conv(256, 5, 1, _R), maxpool(2, 2),
    conv(256, 3, 1, _R), maxpool(2, 2),
    conv(512, 3, 1, _R),        # fc 2304 -> 512
    conv(2, 1, 1)))             # fc 512 -> 2

_STRIDED = Net("strided67", 3, 67, (
    conv(48, 7, 2, _R), maxpool(3, 2),
    conv(96, 5, 1, _R), avgpool(3, 2),
    conv(192, 3, 1, _R),
    conv(21, 3, 1)))            # fc 192*3*3 -> 21


# Plain CNN_1 of the paper's experiments (Table 1; Sec. 5.1): 133 x 133 patches, 32 outputs.  The table lists
# tanh after each pool; it is applied before the pool here, in the convolution's epilogue: tanh is monotonic,
# so the pooled values are the same, and in whole-image form both maps have the same size.
_T = ACT_TANH
def _plain(pool1):
    n = 6 + pool1 * (3 + 2 * 7 - 1) - 1       # 133, 69, 37 for pool1 = 8, 4, 2
    return Net("plain%d" % n, 3, n, (
        conv(50, 6, 1, _T), maxpool(pool1, pool1),
        conv(50, 3, 1, _T), maxpool(2, 2),
        conv(32, 7, 1)))


_PLAIN = _plain(8)
# Table 4's variants: pool1 4x4 / 4 and 2x2 / 2 make the network take 69 x 69 and 37 x 37 patches
_PLAIN69, _PLAIN37 = _plain(4), _plain(2)


@dataclass(frozen=True)
class Config:
    net: Net
    N: int
    H: int
    W: int
    mask_frac: float
    dtype: str = "f32"           # "f32" or "bf16" (bf16 inputs, fp32 accumulate)
    positive_frac: float = -1.0  # >=0: Bernoulli labels (2 classes)
    seed: int = 0


CONFIGS = (
    Config(_TINY, 1, 40, 40, 0.10),
    Config(_SCENE, 1, 512, 512, 0.05),
    Config(_SCENE, 4, 1024, 1024, 0.01),
    Config(_WIDE, 1, 1024, 1024, 0.02, dtype="bf16", positive_frac=0.3),
    Config(_STRIDED, 1, 2048, 2048, 0.01),
    # the paper's own workload: 256 x 256 labelled pixels (3 x 388 x 388 padded), errors of 1024 chosen pixels
    Config(_PLAIN, 1, 256, 256, 1024.0 / 65536.0),
    Config(_PLAIN69, 1, 256, 256, 1024.0 / 65536.0),
    Config(_PLAIN37, 1, 256, 256, 1024.0 / 65536.0),
)


def config_net(i: int) -> Net:
    return CONFIGS[i].net
