"""The fp32 3x3 / 64-input-channel kernel (16 x 16 pixel tiles, the input patch scaled and cut into two fp16 planes
in LDS, three fp16 MFMAs per product) through the C ABI against the CPU oracle, element by element, at
|gpu - oracle| <= 1e-5 + 1e-4 |oracle|: maps that are and are not multiples of the tile, one pixel wide or
high, padding 0 / 1 / asymmetric / wider than the filter needs, ragged and several channel tiles, more
tiles than CUs (persistent workgroups walk several, the next patch prefetched), the tensor-add link in and
out of place, no bias.  The planner's tile threshold is lowered through a tuning knob so that small
shapes reach the kernel; results never depend on it.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  k  pads (top, left, bottom, right)
SHAPES = [
    (1, 16, 16, 64, (1, 1, 1, 1)),      # exactly one tile
    (2, 20, 37, 64, (1, 1, 1, 1)),      # ragged tiles in both directions
    (1, 18, 18, 64, (0, 0, 0, 0)),      # no padding: 16 x 16 outputs
    (1, 9, 50, 72, (1, 1, 1, 1)),       # ragged channel tile (64 + 8)
    (3, 13, 14, 128, (1, 0, 0, 1)),     # asymmetric padding, two channel tiles
    (1, 3, 40, 64, (0, 1, 0, 1)),       # one output row
    (1, 33, 3, 200, (1, 0, 1, 0)),      # one output column, four channel tiles with a ragged last
    (1, 12, 12, 64, (2, 3, 2, 1)),      # padding wider than the filter needs
    (5, 56, 56, 64, (1, 1, 1, 1)),      # 80 tiles
    (2, 224, 100, 64, (1, 1, 1, 1)),    # 196 tiles: more than... fewer than CUs; see below for the persistent walk
    (6, 112, 112, 64, (1, 1, 1, 1)),    # 294 tiles: some workgroups take two
    (4, 80, 80, 160, (1, 1, 1, 1)),     # 300 tiles in three channel tiles: a workgroup's second tile is another channel
                                        # tile (its first slabs are issued ahead of the first tile's stores)
    (3, 150, 150, 64, (1, 1, 1, 1)),    # 300 tiles, ragged: lanes outside the output in every tile of the last row/column
]


def _case(i):
    n, h, w, k, pd = SHAPES[i]
    rng = np.random.default_rng(33000 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, 64)).astype(np.float32)
    wt = (rng.standard_normal(size=(k, 3, 3, 64)) / np.sqrt(576)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b, pd


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_conv_k3c64_f32(i, knobs):
    G = _gpu()
    knobs.set("F32_K3C64_MIN_TILES", 1)
    x, wt, b, pd = _case(i)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.conv2d_f32(x, wt, bias, (1, 1), pd, 1, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, bias, desc, act)
        assert variant == "conv_k3c64_f32_f16x3", variant
        G.assert_close_f32(got, ref, f"case {i} act {act} [{variant}]")


@pytest.mark.parametrize("i", [1, 3, 4])
@pytest.mark.parametrize("in_place", [False, True])
def test_conv_k3c64_f32_tensor_add_link(i, in_place, knobs):
    G = _gpu()
    knobs.set("F32_K3C64_MIN_TILES", 1)
    x, wt, b, pd = _case(i)
    n, h, w, _ = x.shape
    oh, ow = h + pd[0] + pd[2] - 2, w + pd[1] + pd[3] - 2
    add = np.random.default_rng(33100 + i).uniform(-1, 1, size=(n, oh, ow, wt.shape[0])).astype(np.float32)
    ref = oracle.conv2d_f32_add(x, wt, b, add, (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, G.make_desc(x.shape, wt.shape, (1, 1), pd, 1), wl.ACT_RELU,
                                          in_place=in_place)
    assert variant == "conv_k3c64_f32_f16x3_add", variant
    G.assert_close_f32(got, ref, f"case {i} add link in_place {in_place}")


def test_conv_k3c64_f32_is_taken_only_with_a_workspace_and_enough_tiles(knobs):
    G = _gpu()
    x, wt, b, pd = _case(1)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)            # 12 tiles: below the planner's threshold
    assert not variant.startswith("conv_k3c64_f32"), variant
    G.assert_close_f32(got, ref, f"[{variant}]")
    knobs.set("F32_K3C64_MIN_TILES", 1)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU, use_workspace=False)
    assert not variant.startswith("conv_k3c64_f32"), variant
    G.assert_close_f32(got, ref, f"no workspace [{variant}]")
    knobs.set("F32_K3C64", 0)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
    assert not variant.startswith("conv_k3c64_f32"), variant
    G.assert_close_f32(got, ref, f"switched off [{variant}]")
