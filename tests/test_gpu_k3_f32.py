"""The fp32 3x3 stride-1 kernel for many channels (16 x 16 pixel tiles x 128 output channels, the input walked
in 32-channel chunks whose patch is scaled and cut into two fp16 planes in LDS, three fp16 MFMAs per product) through the
C ABI against the CPU oracle, element by element, at |gpu - oracle| <= 1e-5 + 1e-4 |oracle|: one, two (even)
and three (odd) channel chunks, both tile shapes (16 x 16 pixels x 128 channels, 16 x 32 x 64), ragged pixel and channel tiles, every kind of padding, more tiles than CUs
(persistent workgroups, patch prefetch across tiles), the tensor-add link, no bias; for more than 64 output
channels both the kernel whose pixel tile is shaped per layer (every count of pixel blocks, forced tile shapes) and
the fixed 16 x 16 one.  The planner's shape
conditions are lifted through a tuning knob so that small shapes reach the kernel.
"""
import re

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  c  k  pads (top, left, bottom, right)
SHAPES = [
    (1, 16, 16, 64, 128, (1, 1, 1, 1)),     # one tile, two chunks
    (2, 20, 37, 96, 128, (1, 1, 1, 1)),     # three chunks (odd: the slab ring ends on the other buffer), ragged tiles
    (1, 18, 18, 128, 200, (0, 0, 0, 0)),    # no padding, ragged second channel tile
    (3, 13, 14, 64, 72, (1, 0, 0, 1)),      # asymmetric padding, one ragged channel tile
    (1, 3, 40, 256, 136, (0, 1, 0, 1)),     # one output row, eight chunks
    (1, 33, 3, 64, 130, (1, 0, 1, 0)),      # one output column
    (1, 12, 12, 64, 128, (2, 3, 2, 1)),     # padding wider than the filter needs
    (9, 56, 56, 64, 128, (1, 1, 1, 1)),     # 144 tiles
    (5, 112, 112, 64, 96, (1, 1, 1, 1)),    # 245 tiles
    (3, 112, 112, 128, 256, (1, 1, 1, 1)),  # 294 tiles: some workgroups take two (prefetch across tiles)
    # 64 output channels or fewer: the 16 x 32 pixel tile with 64 channels
    (1, 16, 32, 64, 64, (1, 1, 1, 1)),      # exactly one tile
    (2, 21, 45, 96, 64, (1, 1, 1, 1)),      # ragged tiles, three chunks
    (1, 18, 70, 64, 40, (0, 0, 0, 0)),      # no padding, ragged channel tile
    (3, 9, 33, 128, 64, (1, 0, 0, 1)),      # asymmetric padding
    (1, 40, 3, 64, 16, (1, 0, 1, 0)),       # one output column
    (6, 112, 112, 64, 64, (1, 1, 1, 1)),    # 168 tiles
    (5, 224, 224, 64, 64, (1, 1, 1, 1)),    # 490 tiles: workgroups take two (prefetch across tiles)
]


def _case(i):
    n, h, w, c, k, pd = SHAPES[i]
    rng = np.random.default_rng(34000 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(k, 3, 3, c)) / np.sqrt(9 * c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b, pd


def _expected_variant(k, form, variant):
    if k <= 64:
        return variant == "conv_k3_f32_f16x3_16x32x64"
    if form == "fixed":
        return variant == "conv_k3_f32_f16x3"
    # the tile shape picked for the layer; a pick of 16 x 16 goes to the fixed-tile kernel
    return re.fullmatch(r"conv_k3_f32_f16x3(_\d+x\d+)?", variant) is not None


@pytest.mark.parametrize("i", range(len(SHAPES)))
@pytest.mark.parametrize("form", ["shaped", "fixed"])
def test_conv_k3_f32(i, form, knobs):
    G = _gpu()
    knobs.set("F32_K3_ANY", 1)
    knobs.set("F32_K3C64", 0)               # the 64-input-channel kernel would take the largest C = 64 case
    knobs.set("F32_K3V", 1 if form == "shaped" else 0)
    x, wt, b, pd = _case(i)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.conv2d_f32(x, wt, bias, (1, 1), pd, 1, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, bias, desc, act)
        assert _expected_variant(wt.shape[0], form, variant), variant
        G.assert_close_f32(got, ref, f"case {i} act {act} [{variant}]")


# th, tw: every count of pixel blocks (5 to 8), tiles that fill their last block and tiles that do not, the widest
# and the narrowest, rows that wrap inside a 32-pixel block at every phase, a tile larger than the whole map
TILE_SHAPES = [(16, 16), (7, 28), (8, 28), (14, 16), (4, 56), (9, 28), (5, 27), (6, 30), (3, 64), (13, 13), (2, 3),
               (28, 8), (40, 40)]


@pytest.mark.parametrize("shape", TILE_SHAPES, ids=lambda s: f"{s[0]}x{s[1]}")
@pytest.mark.parametrize("i", [1, 3, 6, 7])
def test_conv_k3_f32_every_tile_shape(i, shape, knobs):
    G = _gpu()
    knobs.set("F32_K3_ANY", 1)
    knobs.set("F32_K3C64", 0)
    th, tw = shape
    knobs.set("F32_K3_TH", th)
    knobs.set("F32_K3_TW", tw)
    x, wt, b, pd = _case(i)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
    if (th, tw) == (40, 40):                # not a shape the kernel has (more than 256 pixels): the planner's own pick
        assert re.fullmatch(r"conv_k3_f32_f16x3(_\d+x\d+)?", variant), variant
    else:
        assert variant == f"conv_k3_f32_f16x3_{th}x{tw}", variant
    G.assert_close_f32(got, ref, f"case {i} tile {th}x{tw}")


@pytest.mark.parametrize("i", [1, 2, 3, 11, 12])
@pytest.mark.parametrize("in_place", [False, True])
def test_conv_k3_f32_tensor_add_link(i, in_place, knobs):
    G = _gpu()
    knobs.set("F32_K3_ANY", 1)
    x, wt, b, pd = _case(i)
    n, h, w, _ = x.shape
    oh, ow = h + pd[0] + pd[2] - 2, w + pd[1] + pd[3] - 2
    add = np.random.default_rng(34100 + i).uniform(-1, 1, size=(n, oh, ow, wt.shape[0])).astype(np.float32)
    ref = oracle.conv2d_f32_add(x, wt, b, add, (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, G.make_desc(x.shape, wt.shape, (1, 1), pd, 1), wl.ACT_RELU,
                                          in_place=in_place)
    assert variant.startswith("conv_k3_f32_f16x3") and variant.endswith("_add"), variant
    G.assert_close_f32(got, ref, f"case {i} add link in_place {in_place}")


def test_conv_k3_f32_is_the_planners_choice_only_where_the_map_tiles_well(knobs):
    G = _gpu()
    x, wt, b, pd = _case(1)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)            # 12 tiles, 20 x 37 map: not taken
    assert not variant.startswith("conv_k3_f32"), variant
    G.assert_close_f32(got, ref, f"[{variant}]")
    knobs.set("F32_K3_ANY", 1)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU, use_workspace=False)
    assert not variant.startswith("conv_k3_f32"), variant
    G.assert_close_f32(got, ref, f"no workspace [{variant}]")
    knobs.set("F32_K3", 0)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
    assert not variant.startswith("conv_k3_f32"), variant
    G.assert_close_f32(got, ref, f"switched off [{variant}]")
