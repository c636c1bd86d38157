"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds *no arithmetic of the method*: it only names the benchmark
layers and draws x / w / dy from fixed distributions.  It is the one module
that both the CPU oracle's tests and the GPU path's tests / benchmark use, so
that both sides see identical arrays.

Shapes follow the networks the paper trains (ResNet-18/50, MobileNetV2,
InceptionV3; Tables 6-7).  The paper's datasets are not available, so the
value distributions are stand-ins: activations are (clipped) normal, weights
Kaiming-normal, output gradients heavy-tailed Student-t with a few large
outliers -- the "sharp and wide" shape of Sec.3.2, characteristic C1.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)
    groups: int = 1
    x_dist: str = "normal"        # normal | relu | relu6
    dy_df: float = 3.0            # Student-t degrees of freedom
    dy_scale: float = 1e-3
    dy_outliers: bool = True      # 0.01 % of entries multiplied by 100

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad[0] - self.R) // self.stride[0] + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad[1] - self.S) // self.stride[1] + 1

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C // self.groups, self.R, self.S)

    @property
    def y_shape(self):
        return (self.N, self.K, self.P, self.Q)

    @property
    def macs(self) -> int:
        """Multiply-accumulates of one of the three convolution passes."""
        return self.N * self.K * self.P * self.Q * (self.C // self.groups) * self.R * self.S


# Index = position in the benchmark's config list.
CONFIGS: Dict[int, List[Layer]] = {
    0: [Layer("tiny3x3", 2, 16, 16, 16, 32, 3, 3, pad=(1, 1), x_dist="normal", dy_scale=1e-3)],
    1: [Layer("resnet18_3x3", 64, 64, 56, 56, 64, 3, 3, pad=(1, 1), x_dist="relu", dy_scale=1e-4)],
    2: [Layer("r50_1x1_reduce", 128, 1024, 14, 14, 256, 1, 1),
        Layer("r50_3x3", 128, 256, 14, 14, 256, 3, 3, pad=(1, 1)),
        Layer("r50_1x1_expand", 128, 256, 14, 14, 1024, 1, 1)],
    3: [Layer("mbv2_expand", 64, 24, 56, 56, 144, 1, 1, x_dist="relu6", dy_df=2.0, dy_scale=1e-4,
              dy_outliers=False),
        Layer("mbv2_depthwise", 64, 144, 56, 56, 144, 3, 3, pad=(1, 1), groups=144, x_dist="relu6",
              dy_df=2.0, dy_scale=1e-4, dy_outliers=False),
        Layer("mbv2_project", 64, 144, 56, 56, 24, 1, 1, x_dist="relu6", dy_df=2.0, dy_scale=1e-4,
              dy_outliers=False)],
    4: [Layer("inc_1x7", 64, 768, 17, 17, 768, 1, 7, pad=(0, 3)),
        Layer("inc_7x1", 64, 768, 17, 17, 768, 7, 1, pad=(3, 0)),
        Layer("inc_3x3_s2", 64, 768, 17, 17, 192, 3, 3, stride=(2, 2), pad=(0, 0))],
    # beyond the benchmark's list: a fully connected layer (the paper replaces conv AND fc layers,
    # Sec.4 setup) is the 1x1 convolution of a 1x1 image; ResNet-50's classifier at batch 256
    5: [Layer("r50_fc", 256, 2048, 1, 1, 1000, 1, 1)],
    # ... and ResNet-50's strided layers (Fig.10 times every convolution of that network): the 7x7
    # stem on 3 channels, the 3x3 and the 1x1 shortcut that halve the image
    6: [Layer("r50_stem", 16, 3, 224, 224, 64, 7, 7, stride=(2, 2), pad=(3, 3), x_dist="normal", dy_scale=1e-4),
        Layer("r50_3x3_s2", 64, 128, 56, 56, 128, 3, 3, stride=(2, 2), pad=(1, 1), x_dist="relu", dy_scale=1e-4),
        Layer("r50_shortcut_s2", 32, 256, 56, 56, 512, 1, 1, stride=(2, 2), x_dist="relu", dy_scale=1e-4)],
}


def resnet50_layers(N: int = 64):
    """[(how often the shape occurs, Layer)] for every convolution of ResNet-50 on 224 x 224 images
    (stride on the 3x3 of a bottleneck) and its classifier: the per-layer workload of Fig.10."""
    def L(name, C, H, K, R, s=1):
        return Layer(name, N, C, H, H, K, R, R, stride=(s, s), pad=(R // 2, R // 2), x_dist="relu", dy_scale=1e-4)
    out = [(1, L("stem_7x7_s2", 3, 224, 64, 7, 2))]
    H, Cin = 56, 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        s = 1 if stage == 0 else 2
        tag = f"s{stage + 1}"
        # first block: reduces from the previous stage's width, strided 3x3, projection shortcut
        out += [(1, L(f"{tag}_1x1_in", Cin, H, width, 1)), (1, L(f"{tag}_3x3_first", width, H, width, 3, s)),
                (1, L(f"{tag}_shortcut", Cin, H, 4 * width, 1, s))]
        H //= s
        out += [(blocks, L(f"{tag}_1x1_expand", width, H, 4 * width, 1)),
                (blocks - 1, L(f"{tag}_1x1_reduce", 4 * width, H, width, 1)),
                (blocks - 1, L(f"{tag}_3x3", width, H, width, 3))]
        Cin = 4 * width
    out.append((1, Layer("fc", N, 2048, 1, 1, 1000, 1, 1, x_dist="relu", dy_scale=1e-4)))
    return out

# Default clip candidates of the search: ratio_j = 2^(-j/4), j = 0..31 (j = 0 is "no clipping").
def default_ratios(n_cand: int = 32) -> np.ndarray:
    return np.exp2(-np.arange(n_cand, dtype=np.float64) / 4.0).astype(np.float32)


def _rng(seed: int, cfg: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg, layer, tensor])))


def make_x(L: Layer, cfg: int, li: int, seed: int = 0) -> np.ndarray:
    r = _rng(seed, cfg, li, 0)
    x = r.standard_normal(L.x_shape, dtype=np.float32)
    if L.x_dist == "relu":
        np.maximum(x, 0.0, out=x)
    elif L.x_dist == "relu6":
        np.clip(x, 0.0, 6.0, out=x)
    return x


def make_w(L: Layer, cfg: int, li: int, seed: int = 0) -> np.ndarray:
    r = _rng(seed, cfg, li, 1)
    fan_in = (L.C // L.groups) * L.R * L.S
    w = r.standard_normal(L.w_shape, dtype=np.float32)
    w *= np.float32(np.sqrt(2.0 / fan_in))
    return w


def make_dy(L: Layer, cfg: int, li: int, seed: int = 0) -> np.ndarray:
    r = _rng(seed, cfg, li, 2)
    n = int(np.prod(L.y_shape))
    dy = r.standard_t(L.dy_df, size=n).astype(np.float32)
    dy *= np.float32(L.dy_scale)
    if L.dy_outliers:
        k = int(round(1e-4 * n))
        if k > 0:
            pos = r.choice(n, size=k, replace=False)
            dy[pos] *= np.float32(100.0)
    return dy.reshape(L.y_shape)


def make_layer_inputs(cfg: int, li: int, seed: int = 0):
    L = CONFIGS[cfg][li]
    return L, make_x(L, cfg, li, seed), make_w(L, cfg, li, seed), make_dy(L, cfg, li, seed)


def mobilenetv2_layers(N: int = 32):
    """[(how often, Layer)] for every convolution of MobileNetV2 (width 1.0, 224 x 224 images): the
    3x3 stride-2 stem, per inverted-residual block the 1x1 expansion, the 3x3 depthwise layer
    (stride 2 in the first block of four stages) and the 1x1 projection, and the last 1x1 layer."""
    out = []

    def add(name, C, H, K, R, s, g=1):
        L = Layer(name, N, C, H, H, K, R, R, stride=(s, s), pad=(R // 2, R // 2), groups=g, x_dist="relu6",
                  dy_df=2.0, dy_scale=1e-4, dy_outliers=False)
        for i, (cnt, Lo) in enumerate(out):
            if Lo == L:
                out[i] = (cnt + 1, Lo)
                return
        out.append((1, L))

    add("stem_3x3_s2", 3, 224, 32, 3, 2)
    H, Cin = 112, 32
    for t, c, n, s in ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)):
        for i in range(n):
            st = s if i == 0 else 1
            hid = Cin * t
            if t != 1:
                add(f"expand_{Cin}_{hid}_at{H}", Cin, H, hid, 1, 1)
            add(f"depthwise_{hid}_at{H}_s{st}", hid, H, hid, 3, st, hid)
            H //= st
            add(f"project_{hid}_{c}_at{H}", hid, H, c, 1, 1)
            Cin = c
    add("last_1x1", 320, 7, 1280, 1, 1)
    return out


def inceptionv3_layers(N: int = 32):
    """[(1, Layer)] for the distinct kinds of convolution in InceptionV3 (299 x 299 images): the
    unpadded 3x3 stem layers, 1x1 / 5x5 / 3x3 branches at 35 x 35, the unpadded stride-2 reductions,
    the 1x7 / 7x1 pairs at 17 x 17, the 1x3 / 3x1 pairs at 8 x 8 and the classifier."""
    sh = [("stem_3x3_s2", 3, 299, 32, 3, 3, 2, 0, 0), ("stem_3x3", 32, 149, 32, 3, 3, 1, 0, 0),
          ("stem_3x3_pad", 32, 147, 64, 3, 3, 1, 1, 1), ("stem_1x1", 64, 73, 80, 1, 1, 1, 0, 0),
          ("stem_3x3_192", 80, 73, 192, 3, 3, 1, 0, 0),
          ("a_1x1_64", 192, 35, 64, 1, 1, 1, 0, 0), ("a_1x1_48", 192, 35, 48, 1, 1, 1, 0, 0),
          ("a_5x5", 48, 35, 64, 5, 5, 1, 2, 2), ("a_3x3_64_96", 64, 35, 96, 3, 3, 1, 1, 1),
          ("a_3x3_96_96", 96, 35, 96, 3, 3, 1, 1, 1), ("a_1x1_288", 288, 35, 64, 1, 1, 1, 0, 0),
          ("reduce_a_3x3_s2", 288, 35, 384, 3, 3, 2, 0, 0), ("reduce_a_3x3_s2_96", 96, 35, 96, 3, 3, 2, 0, 0),
          ("b_1x1_128", 768, 17, 128, 1, 1, 1, 0, 0), ("b_1x7_128", 128, 17, 128, 1, 7, 1, 0, 3),
          ("b_7x1_192", 128, 17, 192, 7, 1, 1, 3, 0), ("b_1x7_160", 160, 17, 160, 1, 7, 1, 0, 3),
          ("b_1x1_192", 768, 17, 192, 1, 1, 1, 0, 0),
          ("reduce_b_3x3_s2_320", 192, 17, 320, 3, 3, 2, 0, 0), ("reduce_b_3x3_s2_192", 192, 17, 192, 3, 3, 2, 0, 0),
          ("c_1x1_320", 1280, 8, 320, 1, 1, 1, 0, 0), ("c_1x3", 384, 8, 384, 1, 3, 1, 0, 1),
          ("c_3x1", 384, 8, 384, 3, 1, 1, 1, 0), ("c_3x3_448", 448, 8, 384, 3, 3, 1, 1, 1),
          ("c_1x1_2048", 2048, 8, 448, 1, 1, 1, 0, 0), ("fc", 2048, 1, 1000, 1, 1, 1, 0, 0)]
    return [(1, Layer(name, N, C, H, H, K, R, S, stride=(s, s), pad=(ph, pw), x_dist="relu", dy_scale=1e-4))
            for name, C, H, K, R, S, s, ph, pw in sh]
