"""Layer shapes and seeded synthetic inputs for the lowered Conv / FC hot path.

This module holds no arithmetic of the method: it only names layer shapes and draws random tensors.
Both the GPU tests/benchmark and the CPU oracle are fed from here, so both see identical bytes.

The shapes are those of ResNet-50 and VGG-19 layers (the two networks of the paper's evaluation,
Section 7).  The trained models and images are not used: values are seeded synthetic draws with
the stated distributions.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Tuple

import numpy as np

SEED_BASE = 180500907

ACT_NONE = 0
ACT_RELU = 1


@dataclasses.dataclass(frozen=True)
class ConvLayer:
    """NHWC input [n,h,w,c], filter [k,r,s,c/groups] (Section 3.5 listing, Section 5.2 filter layout)."""
    name: str
    n: int
    h: int
    w: int
    c: int
    k: int
    r: int
    s: int
    stride: int = 1
    pad: int = 0
    groups: int = 1
    act: int = ACT_RELU
    add: bool = False      # the element-wise chain has a tensor-add link (residual add) before the activation

    @property
    def oh(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def ow(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def gemm(self) -> Tuple[int, int, int]:
        """(M, N, K) of the contraction the layer lowers to."""
        return self.n * self.oh * self.ow, self.k, self.r * self.s * (self.c // self.groups)

    @property
    def ops(self) -> int:
        m, n, k = self.gemm
        return 2 * m * n * k

    def alg_bytes(self, elem: int, bias_elem: int = 4) -> int:
        """Each tensor once: input + filter + bias + output (+ the addend of the chain)."""
        x = self.n * self.h * self.w * self.c
        wt = self.k * self.r * self.s * (self.c // self.groups)
        y = self.n * self.oh * self.ow * self.k
        return (x + wt + y * (2 if self.add else 1)) * elem + self.k * bias_elem

    def with_batch(self, n: int) -> "ConvLayer":
        return dataclasses.replace(self, n=n, name=f"{self.name.split('@b')[0]}@b{n}")


@dataclasses.dataclass(frozen=True)
class FcLayer:
    """a [M,K] times w [K,N] plus bias [N] (Section 3.4: MatMul followed by a broadcasted add)."""
    name: str
    M: int
    K: int
    N: int
    act: int = ACT_RELU

    @property
    def gemm(self) -> Tuple[int, int, int]:
        return self.M, self.N, self.K

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K

    def alg_bytes(self, elem: int, bias_elem: int = 4) -> int:
        return (self.M * self.K + self.K * self.N + self.M * self.N) * elem + self.N * bias_elem


def config1_layer() -> ConvLayer:
    return ConvLayer("cfg1_3x3_c16_k16_32", 1, 32, 32, 16, 16, 3, 3, 1, 1)


def resnet50_layers(batch: int) -> List[ConvLayer]:
    """The five ResNet-50-shaped layers: stem 7x7/2, the 56x56 bottleneck trio, the 7x7-map 3x3."""
    b = batch
    return [
        ConvLayer(f"rn_7x7s2_c3_k64_224@b{b}", b, 224, 224, 3, 64, 7, 7, 2, 3),
        ConvLayer(f"rn_1x1_c256_k64_56@b{b}", b, 56, 56, 256, 64, 1, 1, 1, 0),
        ConvLayer(f"rn_3x3_c64_k64_56@b{b}", b, 56, 56, 64, 64, 3, 3, 1, 1),
        ConvLayer(f"rn_1x1_c64_k256_56@b{b}", b, 56, 56, 64, 256, 1, 1, 1, 0),
        ConvLayer(f"rn_3x3_c512_k512_7@b{b}", b, 7, 7, 512, 512, 3, 3, 1, 1),
    ]


def resnet50_block_tails(batch: int) -> List[ConvLayer]:
    """The last convolution of a bottleneck block in each of the four stages, with the block's
    residual add and Relu stacked on it (Section 5.2): 1x1 expand, + shortcut, max."""
    b = batch
    return [
        ConvLayer(f"rn_tail_1x1_c64_k256_56@b{b}", b, 56, 56, 64, 256, 1, 1, 1, 0, add=True),
        ConvLayer(f"rn_tail_1x1_c128_k512_28@b{b}", b, 28, 28, 128, 512, 1, 1, 1, 0, add=True),
        ConvLayer(f"rn_tail_1x1_c256_k1024_14@b{b}", b, 14, 14, 256, 1024, 1, 1, 1, 0, add=True),
        ConvLayer(f"rn_tail_1x1_c512_k2048_7@b{b}", b, 7, 7, 512, 2048, 1, 1, 1, 0, add=True),
    ]


def resnet50_bottleneck(batch: int) -> List[ConvLayer]:
    """One identity-shortcut bottleneck block of the 56x56 stage as a chain: 1x1 reduce, 3x3, 1x1
    expand whose chain adds the block input and applies Relu.  Each layer reads its predecessor."""
    b = batch
    return [
        ConvLayer(f"rn_block_1x1_c256_k64_56@b{b}", b, 56, 56, 256, 64, 1, 1, 1, 0),
        ConvLayer(f"rn_block_3x3_c64_k64_56@b{b}", b, 56, 56, 64, 64, 3, 3, 1, 1),
        ConvLayer(f"rn_block_1x1_c64_k256_56@b{b}", b, 56, 56, 64, 256, 1, 1, 1, 0, add=True),
    ]


def depthwise_layers(batch: int) -> List[ConvLayer]:
    """Depthwise 3x3 layers (groups == channels: every channel has its own 3x3 filter) on the feature-map sizes
    of a 224 x 224 classification network that halves the map and doubles the channels stage by stage."""
    b = batch
    shapes = [(112, 32, 1), (112, 64, 2), (56, 128, 1), (56, 128, 2), (28, 256, 1), (28, 256, 2), (14, 512, 1),
              (14, 512, 2), (7, 1024, 1)]
    return [ConvLayer(f"dw_3x3s{st}_c{c}_{hw}@b{b}", b, hw, hw, c, c, 3, 3, st, 1, groups=c) for hw, c, st in shapes]


def addend_f32(layer: ConvLayer, seed: int) -> np.ndarray:
    """Shortcut tensor of a block tail: unit-variance activations of the output's shape."""
    rng = np.random.default_rng(seed + 500)
    return rng.standard_normal(size=(layer.n, layer.oh, layer.ow, layer.k), dtype=np.float32)


def addend_q(layer: ConvLayer, seed: int, y_scale: float):
    """-> int8 shortcut codes, scale, offset: a post-Relu tensor on roughly the output's scale."""
    rng = np.random.default_rng(seed + 500)
    r_scale = float(np.float32(y_scale * rng.uniform(0.5, 1.5)))
    r_off = -128
    codes = np.clip(np.rint(np.abs(rng.standard_normal(size=(layer.n, layer.oh, layer.ow, layer.k))) / r_scale)
                    + r_off, -128, 127).astype(np.int8)
    return codes, r_scale, r_off


def vgg19_conv_layers(batch: int = 16) -> List[ConvLayer]:
    b = batch
    return [
        ConvLayer(f"vgg_3x3_c64_224@b{b}", b, 224, 224, 64, 64, 3, 3, 1, 1),
        ConvLayer(f"vgg_3x3_c128_112@b{b}", b, 112, 112, 128, 128, 3, 3, 1, 1),
        ConvLayer(f"vgg_3x3_c256_56@b{b}", b, 56, 56, 256, 256, 3, 3, 1, 1),
        ConvLayer(f"vgg_3x3_c512_28@b{b}", b, 28, 28, 512, 512, 3, 3, 1, 1),
        ConvLayer(f"vgg_3x3_c512_14@b{b}", b, 14, 14, 512, 512, 3, 3, 1, 1),
    ]


def vgg19_fc_layers(batch: int = 16) -> List[FcLayer]:
    return [
        FcLayer(f"vgg_fc_25088_4096@m{batch}", batch, 25088, 4096, ACT_RELU),
        FcLayer(f"vgg_fc_4096_4096@m{batch}", batch, 4096, 4096, ACT_RELU),
        FcLayer(f"vgg_fc_4096_1000@m{batch}", batch, 4096, 1000, ACT_NONE),
    ]


def fc_sweep_layers() -> List[FcLayer]:
    return [FcLayer(f"fc_{m}x{k}x{n}", m, k, n, ACT_RELU)
            for (m, k, n) in [(1, 2048, 1000), (64, 2048, 1000), (256, 4096, 4096), (1024, 9216, 4096)]]


def layer_seed(config_index: int, layer_index: int) -> int:
    return SEED_BASE + 1000 * config_index + layer_index


# ---------------------------------------------------------------------------------------------------
# Random tensors.  dist "uniform"       : x, w ~ U(-1,1), bias ~ U(-0.1,0.1).
#                  dist "uniform_fan_in": x ~ U(-1,1), w ~ U(-1,1)/sqrt(fan_in), bias ~ U(-0.1,0.1)
#                                         (outputs stay O(1) however deep the reduction is, as
#                                         in a trained network).
#                  dist "fan_in"        : x ~ N(0,1), w and bias ~ N(0,1)/sqrt(fan_in).
# ---------------------------------------------------------------------------------------------------

def _draw(rng: np.random.Generator, shape, dist: str, fan_in: int, is_bias=False, is_input=False):
    if dist in ("uniform", "uniform_fan_in"):
        lim = 0.1 if is_bias else 1.0
        t = rng.uniform(-lim, lim, size=shape).astype(np.float32)
        if dist == "uniform_fan_in" and not is_bias and not is_input:
            t *= np.float32(1.0 / math.sqrt(fan_in))
        return t
    if dist == "fan_in":
        t = rng.standard_normal(size=shape, dtype=np.float32)
        if not is_input:
            t *= np.float32(1.0 / math.sqrt(fan_in))
        return t
    raise ValueError(dist)


def conv_inputs_f32(layer: ConvLayer, seed: int, dist: str = "fan_in"):
    """-> x [n,h,w,c], w [k,r,s,c/groups], bias [k], all float32, C-contiguous."""
    rng = np.random.default_rng(seed)
    cg = layer.c // layer.groups
    fan_in = layer.r * layer.s * cg
    x = _draw(rng, (layer.n, layer.h, layer.w, layer.c), dist, fan_in, is_input=True)
    w = _draw(rng, (layer.k, layer.r, layer.s, cg), dist, fan_in)
    b = _draw(rng, (layer.k,), dist, fan_in, is_bias=True)
    return x, w, b


def fc_inputs_f32(layer: FcLayer, seed: int, dist: str = "fan_in"):
    """-> a [M,K], w [K,N], bias [N]."""
    rng = np.random.default_rng(seed)
    a = _draw(rng, (layer.M, layer.K), dist, layer.K, is_input=True)
    w = _draw(rng, (layer.K, layer.N), dist, layer.K)
    b = _draw(rng, (layer.N,), dist, layer.K, is_bias=True)
    return a, w, b


@dataclasses.dataclass(frozen=True)
class QParams:
    """Scale/offset of the three quantized tensors of one operator (Section 4.1 tensor type)."""
    x_scale: float
    x_off: int
    w_scale: float
    w_off: int
    y_scale: float
    y_off: int


def _draw_qparams(rng: np.random.Generator, fan_in: int, w_off: int) -> QParams:
    f32 = lambda v: float(np.float32(v))
    x_scale = f32(rng.uniform(0.01, 0.1))
    x_off = int(rng.integers(-20, 21))
    # filter codes below have a standard deviation of 30 codes; real filters one of 1/sqrt(fan_in)
    w_scale = f32(1.0 / (30.0 * math.sqrt(fan_in)))
    y_scale = f32(rng.uniform(0.01, 0.1))
    y_off = int(rng.integers(-20, 21))
    return QParams(x_scale, x_off, w_scale, w_off, y_scale, y_off)


def _draw_codes(rng, shape, mean: float, std: float, lo: int, hi: int) -> np.ndarray:
    """int8 codes with a discretised, saturated normal distribution."""
    t = rng.standard_normal(size=shape, dtype=np.float32)
    t *= np.float32(std)
    t += np.float32(mean)
    np.rint(t, out=t)
    np.clip(t, lo, hi, out=t)
    return t.astype(np.int8)


def conv_inputs_q(layer: ConvLayer, seed: int, dist: str = "normal", w_off: int = 0):
    """-> xq int8 [n,h,w,c], wq int8 [k,r,s,c/groups], bias_q int32 [k], QParams.

    dist "normal": activations are codes spread around x_off with a standard deviation of
    1/x_scale codes (a unit-variance real tensor), filters around w_off with 30 codes, bias codes
    with the spread of a real bias of 1/sqrt(fan_in).  dist "uniform": every int8 code equally
    likely (activations and filters), which drives many outputs into saturation.
    """
    rng = np.random.default_rng(seed)
    cg = layer.c // layer.groups
    fan_in = layer.r * layer.s * cg
    qp = _draw_qparams(rng, fan_in, w_off)
    xs, ws = (layer.n, layer.h, layer.w, layer.c), (layer.k, layer.r, layer.s, cg)
    if dist == "normal":
        xq = _draw_codes(rng, xs, qp.x_off, 1.0 / qp.x_scale, -128, 127)
        wq = _draw_codes(rng, ws, w_off, 30.0, -127, 127)
    elif dist == "uniform":
        xq = rng.integers(-128, 128, size=xs, dtype=np.int8)
        wq = rng.integers(-127, 128, size=ws, dtype=np.int8)
    else:
        raise ValueError(dist)
    bias_std = (1.0 / math.sqrt(fan_in)) / (qp.x_scale * qp.w_scale)
    bias_q = np.rint(rng.standard_normal(size=(layer.k,)) * bias_std).astype(np.int32)
    return xq, wq, bias_q, qp


def fc_inputs_q(layer: FcLayer, seed: int, dist: str = "normal", w_off: int = 0):
    """-> aq int8 [M,K], wq int8 [K,N], bias_q int32 [N], QParams."""
    rng = np.random.default_rng(seed)
    qp = _draw_qparams(rng, layer.K, w_off)
    if dist == "normal":
        aq = _draw_codes(rng, (layer.M, layer.K), qp.x_off, 1.0 / qp.x_scale, -128, 127)
        wq = _draw_codes(rng, (layer.K, layer.N), w_off, 30.0, -127, 127)
    elif dist == "uniform":
        aq = rng.integers(-128, 128, size=(layer.M, layer.K), dtype=np.int8)
        wq = rng.integers(-127, 128, size=(layer.K, layer.N), dtype=np.int8)
    else:
        raise ValueError(dist)
    bias_std = (1.0 / math.sqrt(layer.K)) / (qp.x_scale * qp.w_scale)
    bias_q = np.rint(rng.standard_normal(size=(layer.N,)) * bias_std).astype(np.int32)
    return aq, wq, bias_q, qp


def sample_output_indices(layer: ConvLayer, seed: int, n_random: int = 20000) -> np.ndarray:
    """Flat indices into y [n,oh,ow,k] for sampled checks at full size: every output of the four
    border rows/columns of the first and last image plus n_random uniformly drawn ones."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    oh, ow, k = layer.oh, layer.ow, layer.k
    total = layer.n * oh * ow * k
    picks = [rng.integers(0, total, size=n_random, dtype=np.int64)]
    for n in sorted({0, layer.n - 1}):
        ys, xs = np.meshgrid(np.arange(oh), np.arange(ow), indexing="ij")
        border = (ys == 0) | (ys == oh - 1) | (xs == 0) | (xs == ow - 1)
        pix = (n * oh + ys[border]) * ow + xs[border]
        picks.append((pix[:, None] * k + np.arange(k)[None, :]).reshape(-1).astype(np.int64))
    return np.unique(np.concatenate(picks))
