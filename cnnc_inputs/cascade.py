"""Shapes of the three cascade networks and seeded weight blobs for them.

The three-stage cascade follows Section 3 of the paper (three CNNs of growing
size, convolution stride 1, pooling stride 2, the activation of eq. (1) after
every hidden layer).  The paper's own layer shapes were printed only in its
Figure 1; the shapes used here are the benchmark's default cascade:

  stage 1: 12x12 -> conv3x3 1->4 -> pool2 -> conv3x3 4->8 -> fc 72->1
  stage 2: 24x24 -> conv5x5 1->8 -> pool2 -> conv3x3 8->16 -> pool2
           -> fc 256->32 -> fc 32->1
  stage 3: 48x48 -> conv5x5 1->16 -> pool2 -> conv5x5 16->32 -> pool2
           -> conv3x3 32->32 -> fc 1568->64 -> fc 64->1

A fully connected layer is described like a convolution whose kernel covers
its whole input map (feature order [channel][row][col]), so one record type
serves all layers.

Weight blob layout (float32, one blob per stage): for every conv / fc layer in
order, weights [cout][cin][k][k] in C order followed by bias[cout].
"""
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

CONV, POOL, FC = 0, 1, 2
ACT_NONE, ACT_RATIONAL, ACT_SCALED_TANH, ACT_TANH = 0, 1, 2, 3


@dataclass(frozen=True)
class Layer:
    kind: int   # CONV, POOL or FC
    cin: int    # input channels
    cout: int   # output channels (POOL: == cin)
    k: int      # kernel side (POOL: 2; FC: side of the input map)
    act: int    # ACT_* applied to the layer output

    @property
    def n_weights(self) -> int:
        return 0 if self.kind == POOL else self.cout * self.cin * self.k * self.k

    @property
    def n_params(self) -> int:
        return 0 if self.kind == POOL else self.n_weights + self.cout

    @property
    def fan_in(self) -> int:
        return self.cin * self.k * self.k


@dataclass(frozen=True)
class Stage:
    in_size: int
    layers: Sequence[Layer]

    @property
    def n_params(self) -> int:
        return sum(l.n_params for l in self.layers)

    def shapes(self):
        """(channels, side) of the map after every layer, starting with the input."""
        c, s = 1, self.in_size
        out = [(c, s)]
        for l in self.layers:
            if l.kind == CONV:
                c, s = l.cout, s - l.k + 1
            elif l.kind == POOL:
                assert s % 2 == 0
                s //= 2
            else:
                assert s == l.k and c == l.cin
                c, s = l.cout, 1
            out.append((c, s))
        return out


def default_cascade(act: int = ACT_RATIONAL) -> List[Stage]:
    """The benchmark's default three-stage cascade; `act` is the hidden activation."""
    s1 = Stage(12, (
        Layer(CONV, 1, 4, 3, act), Layer(POOL, 4, 4, 2, ACT_NONE),
        Layer(CONV, 4, 8, 3, act), Layer(FC, 8, 1, 3, ACT_NONE)))
    s2 = Stage(24, (
        Layer(CONV, 1, 8, 5, act), Layer(POOL, 8, 8, 2, ACT_NONE),
        Layer(CONV, 8, 16, 3, act), Layer(POOL, 16, 16, 2, ACT_NONE),
        Layer(FC, 16, 32, 4, act), Layer(FC, 32, 1, 1, ACT_NONE)))
    s3 = Stage(48, (
        Layer(CONV, 1, 16, 5, act), Layer(POOL, 16, 16, 2, ACT_NONE),
        Layer(CONV, 16, 32, 5, act), Layer(POOL, 32, 32, 2, ACT_NONE),
        Layer(CONV, 32, 32, 3, act), Layer(FC, 32, 64, 7, act),
        Layer(FC, 64, 1, 1, ACT_NONE)))
    return [s1, s2, s3]


def draw_weights(cascade: Sequence[Stage], seed: int, bias_sd: float = 0.0) -> List[np.ndarray]:
    """One float32 blob per stage, weights ~ N(0, 1/fan_in).

    Draw order: stage 1 to 3, layer by layer, each weight array in C order as
    float64 standard normals scaled by fan_in**-0.5 and rounded to float32.
    Biases are zero (the benchmark's rule) unless `bias_sd` > 0, which tests use
    to make the bias terms observable; those are drawn from a second generator
    so the weights do not depend on `bias_sd`.
    """
    rng = np.random.default_rng(seed)
    brng = np.random.default_rng([seed, 0xB1A5])
    blobs = []
    for st in cascade:
        parts = []
        for l in st.layers:
            if l.kind == POOL:
                continue
            w = rng.standard_normal(l.n_weights) * (l.fan_in ** -0.5)
            b = brng.standard_normal(l.cout) * bias_sd if bias_sd > 0 else np.zeros(l.cout)
            parts += [w.astype(np.float32), b.astype(np.float32)]
        blobs.append(np.concatenate(parts))
    return blobs


def uniform_weights(cascade: Sequence[Stage], values: Sequence[Sequence[float]]) -> List[np.ndarray]:
    """Blobs in which every weight of a layer has one value and biases are 0.

    `values[s][j]` is the value for the j-th weighted layer of stage s.
    """
    blobs = []
    for st, vals in zip(cascade, values):
        parts, j = [], 0
        for l in st.layers:
            if l.kind == POOL:
                continue
            parts += [np.full(l.n_weights, vals[j], np.float32), np.zeros(l.cout, np.float32)]
            j += 1
        blobs.append(np.concatenate(parts))
    return blobs


# --------------------------------------------------------------------------
# First stage in the paper's own geometry (Section 3.1: no fully connected layer, convolution stride 1,
# pooling stride 2; Section 3.3: 27 x 31 window, 4 pixel step).  The shapes were printed only in the
# paper's Figure 1.  Chosen here: square kernels that take a 27 x 31 window to one response,
#   conv 4x4 1->4, pool 2, conv 3x3 4->11, pool 2, conv 5x6 (w x h) 11->1,
# which has 806 parameters (the paper states 797; no list of square kernels with full connections
# between maps gives exactly that).
@dataclass(frozen=True)
class RLayer:
    kind: int   # CONV or POOL
    cin: int
    cout: int
    kw: int     # kernel width (POOL: 2)
    kh: int     # kernel height (POOL: 2)
    act: int

    @property
    def n_weights(self) -> int:
        return 0 if self.kind == POOL else self.cout * self.cin * self.kw * self.kh

    @property
    def n_params(self) -> int:
        return 0 if self.kind == POOL else self.n_weights + self.cout

    @property
    def fan_in(self) -> int:
        return self.cin * self.kw * self.kh


@dataclass(frozen=True)
class ScanNet:
    win_w: int
    win_h: int
    step: int
    layers: Sequence[RLayer]

    @property
    def n_params(self) -> int:
        return sum(l.n_params for l in self.layers)


SCAN_C2 = 11


def paper_stage1(act: int = ACT_RATIONAL) -> ScanNet:
    return ScanNet(27, 31, 4, (
        RLayer(CONV, 1, 4, 4, 4, act), RLayer(POOL, 4, 4, 2, 2, ACT_NONE),
        RLayer(CONV, 4, SCAN_C2, 3, 3, act), RLayer(POOL, SCAN_C2, SCAN_C2, 2, 2, ACT_NONE),
        RLayer(CONV, SCAN_C2, 1, 5, 6, ACT_NONE)))


def draw_scan_weights(net: ScanNet, seed: int, bias_sd: float = 0.0) -> np.ndarray:
    """float32 blob: per conv layer weights [cout][cin][kh][kw] ~ N(0, 1/fan_in), then bias[cout]."""
    rng = np.random.default_rng([seed, 0x5CA4])
    brng = np.random.default_rng([seed, 0x5CA4, 0xB1A5])
    parts = []
    for l in net.layers:
        if l.kind == POOL:
            continue
        w = rng.standard_normal(l.n_weights) * (l.fan_in ** -0.5)
        b = brng.standard_normal(l.cout) * bias_sd if bias_sd > 0 else np.zeros(l.cout)
        parts += [w.astype(np.float32), b.astype(np.float32)]
    return np.concatenate(parts)


# The selective unit's networks in the paper's geometry (Section 3.3: the analysed region is scaled to 51 x 55
# and each of CNN_2, CNN_3 gives a 5 x 5 response map).  Chosen: a 35 x 39 window scanned with the 4 pixel step
# of two pools, (51 - 35) / 4 + 1 = 5, with the same layer pattern as the first network:
#   conv 4x4 1->c1, pool 2, conv 3x3 c1->c2, pool 2, conv 7x8 (w x h) c2->1
# CNN_2: c1, c2 = 4, 19 (1,836 parameters; the paper: 1,819).  CNN_3: 5, 28 (2,942; the paper: 2,923).
REGION_W, REGION_H, REGION_MARGIN = 51, 55, 12


def _region_net(c1: int, c2: int, act: int) -> ScanNet:
    return ScanNet(35, 39, 4, (
        RLayer(CONV, 1, c1, 4, 4, act), RLayer(POOL, c1, c1, 2, 2, ACT_NONE),
        RLayer(CONV, c1, c2, 3, 3, act), RLayer(POOL, c2, c2, 2, 2, ACT_NONE),
        RLayer(CONV, c2, 1, 7, 8, ACT_NONE)))


def paper_stage2(act: int = ACT_RATIONAL) -> ScanNet:
    return _region_net(4, 19, act)


def paper_stage3(act: int = ACT_RATIONAL) -> ScanNet:
    return _region_net(5, 28, act)
