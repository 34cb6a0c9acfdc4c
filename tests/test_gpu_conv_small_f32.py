"""The single-launch fp32 kernel for convolutions on few pixels with a short reduction (wavefronts
split the reduction, operands straight from global memory in MFMA layout, partial sums reduced in LDS)
through the C ABI against the CPU oracle: 1x1 and 3x3 filters, strides, every kind of padding, ragged
pixel and channel counts, the shortest and the longest reduction it takes, with and without bias;
and shapes just outside its range take the other kernels.  |gpu - oracle| <= 1e-5 + 1e-4 |oracle|.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  c  k  r  s  stride  pads(t,l,b,r)
SMALL_CONV = [
    (1, 56, 56, 256, 64, 1, 1, (1, 1), (0, 0, 0, 0)),      # batch-1 1x1 reduce of a residual block
    (1, 56, 56, 64, 64, 3, 3, (1, 1), (1, 1, 1, 1)),       # batch-1 3x3: nine groups per wavefront
    (2, 9, 11, 16, 20, 3, 3, (1, 1), (1, 1, 1, 1)),        # reduction 144: 18 groups on 8 wavefronts (3 each, two idle), ragged channels
    (1, 13, 7, 128, 36, 1, 1, (1, 1), (0, 0, 0, 0)),       # the shortest reduction it takes (128), ragged pixels
    (3, 10, 10, 8, 8, 5, 3, (2, 1), (2, 0, 1, 2)),         # reduction 120 is below the minimum: generic kernel
    (1, 12, 12, 64, 40, 3, 3, (2, 2), (0, 1, 1, 0)),       # stride 2, one-sided padding
    (2, 6, 6, 80, 12, 2, 4, (1, 1), (1, 3, 0, 0)),         # reduction 640, the longest it takes; padding wider than the filter allows
    (1, 5, 5, 32, 4, 5, 5, (1, 1), (2, 2, 2, 2)),          # reduction 800: above the maximum, generic kernel
    (1, 1, 1, 128, 4, 1, 1, (1, 1), (0, 0, 0, 0)),         # one pixel, one channel group
    (4, 7, 7, 24, 68, 3, 3, (1, 1), (1, 1, 1, 1)),         # three channel blocks, the last with 4 channels
]
TAKEN = [True, True, True, True, False, True, True, False, True, True]


@pytest.mark.parametrize("i", range(len(SMALL_CONV)))
def test_conv2d_small_f32(i):
    G = _gpu()
    n, h, w, c, k, r, s, st, pd = SMALL_CONV[i]
    rng = np.random.default_rng(9700 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, r, s, c)) / np.sqrt(r * s * c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, st, pd, 1)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.conv2d_f32(x, wt, b, st, pd, 1, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act, use_workspace=use_ws)
            assert (variant == "conv_small_f32") == TAKEN[i], variant
            G.assert_close_f32(got, ref, f"small conv {SMALL_CONV[i]} act {act} ws {use_ws} [{variant}]")
    got, _ = G.gpu_conv2d_f32(x, wt, None, desc, wl.ACT_NONE)
    G.assert_close_f32(got, oracle.conv2d_f32(x, wt, None, st, pd, 1, act=wl.ACT_NONE), f"small conv {i} without bias")


def test_conv2d_small_f32_not_taken_with_many_tiles_or_odd_channels():
    G = _gpu()
    rng = np.random.default_rng(9790)
    for shape in [(8, 56, 56, 64, 64, 1, 1), (1, 20, 20, 20, 16, 3, 3), (1, 20, 20, 16, 18, 3, 3)]:
        n, h, w, c, k, r, s = shape
        x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
        wt = (rng.uniform(-1, 1, size=(k, r, s, c)) / np.sqrt(r * s * c)).astype(np.float32)
        b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
        pd = (r // 2,) * 4
        desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
        ref = oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_RELU)
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
        assert variant != "conv_small_f32", (shape, variant)
        G.assert_close_f32(got, ref, f"conv {shape} [{variant}]")


# The same kernel with the reduction also sliced over the grid (partial sums to the workspace, the
# finishing kernel sums them in split order): deep reductions on very few pixels.
# n  h  w  c  k  r  s  stride  pads
SPLIT_CONV = [
    (1, 7, 7, 512, 512, 3, 3, (1, 1), (1, 1, 1, 1)),       # the batch-1 3x3 of the last stage: 8 slices x 32 tiles
    (1, 14, 14, 256, 256, 3, 3, (1, 1), (1, 1, 1, 1)),     # 4 slices x 56 tiles
    (2, 5, 6, 96, 36, 3, 3, (1, 1), (1, 1, 1, 1)),         # 864 indices: a full slice and a half one; ragged pixels and channels
    (1, 4, 9, 648, 8, 1, 1, (1, 1), (0, 0, 0, 0)),         # 648 indices, 8 more than one workgroup takes: second slice of one group
    (3, 3, 3, 40, 20, 5, 5, (2, 2), (2, 2, 2, 2)),         # 5x5 stride 2 on a 3x3 map: most taps are padding
]


@pytest.mark.parametrize("i", range(len(SPLIT_CONV)))
def test_conv2d_small_f32_split(i, knobs):
    G = _gpu()
    knobs.set("F32_SMALL_MIN_WGS", "1")     # take the sliced form at any size
    n, h, w, c, k, r, s, st, pd = SPLIT_CONV[i]
    rng = np.random.default_rng(9750 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, r, s, c)) / np.sqrt(r * s * c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, st, pd, 1)
    oh, ow = oracle.out_dim(h, r, st[0], pd[0], pd[2]), oracle.out_dim(w, s, st[1], pd[1], pd[3])
    add = rng.uniform(-1, 1, size=(n, oh, ow, k)).astype(np.float32)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.conv2d_f32(x, wt, b, st, pd, 1, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act)
        assert variant == "conv_small_f32_splitk", variant
        G.assert_close_f32(got, ref, f"sliced small conv {SPLIT_CONV[i]} act {act} [{variant}]")
        # without a workspace the reduction cannot be sliced over the grid: another kernel, same result
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act, use_workspace=False)
        assert variant != "conv_small_f32_splitk", variant
        G.assert_close_f32(got, ref, f"sliced small conv {SPLIT_CONV[i]} act {act} no workspace [{variant}]")
        # the add link is applied by the finishing kernel
        ref = oracle.conv2d_f32_add(x, wt, b, add, st, pd, 1, act=act)
        got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, desc, act)
        assert variant == "conv_small_f32_splitk", variant
        G.assert_close_f32(got, ref, f"sliced small conv + add {SPLIT_CONV[i]} act {act} [{variant}]")


def test_conv2d_small_f32_split_is_the_planner_choice():
    """Without any override the batch-1 3x3 512->512 on a 7x7 map takes the sliced form."""
    G = _gpu()
    n, h, w, c, k, r, s, st, pd = SPLIT_CONV[0]
    rng = np.random.default_rng(9760)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, r, s, c)) / np.sqrt(r * s * c)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, st, pd, 1)
    got, variant = G.gpu_conv2d_f32(x, wt, None, desc, wl.ACT_RELU)
    assert variant == "conv_small_f32_splitk", variant
    G.assert_close_f32(got, oracle.conv2d_f32(x, wt, None, st, pd, 1, act=wl.ACT_RELU), "planner-chosen sliced small conv")
