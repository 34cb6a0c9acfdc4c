"""The fp32 contraction over planes (operands scaled by a power of two and cut into two fp16 planes by a packing
pass, three fp16 MFMAs per product, fp32 accumulation) through the C ABI against the CPU oracle, element by element, at
|gpu - oracle| <= 1e-5 + 1e-4 |oracle|: both tile widths, ragged pixel and channel tiles, channel counts
that are not a multiple of the 32-index slab, groups, strides, padding on every side, FullyConnected
with ragged K and N ([K][N] weights transposed by the packing pass), the tensor-add link, a split
reduction with its finishing kernel, reductions long enough for the second accumulator set, wide value
ranges, and the fall-back when the workspace is missing or too small.  The planner's size thresholds are
lowered through the tuning knobs so that small shapes reach the kernel; results never depend on them.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


def _take_p3(knobs, bn=None, split=None):
    knobs.set("F32_P3_MIN_M", 1)
    knobs.set("F32_P3_RATIO", 0)
    if bn:
        knobs.set("F32_P3_BN", bn)
    if split:
        knobs.set("F32_SPLIT", split)


# n  h  w  c  k  r  s  stride  pad  groups
CONV_SHAPES = [
    (2, 14, 14, 64, 128, 3, 3, 1, 1, 1),     # M = 392: ragged last pixel tile; one channel tile
    (1, 19, 17, 32, 200, 3, 3, 1, 1, 1),     # ragged channel tile (200 = 128 + 72), one slab per tap
    (1, 12, 13, 40, 96, 3, 3, 1, 1, 1),      # 40 channels: slab tail of 8 inside every tap
    (2, 15, 15, 72, 136, 5, 5, 2, 2, 1),     # 5x5 stride 2, three slabs per tap with a tail, padding 2
    (1, 20, 20, 64, 64, 3, 3, 1, 0, 1),      # no padding; 64 channels out
    (3, 9, 11, 128, 72, 1, 1, 1, 0, 1),      # pointwise, ragged channel tile of the 128-wide form
    (1, 16, 16, 64, 192, 3, 3, 1, 1, 2),     # two groups: 32 channels in, 96 out per group
    (1, 10, 30, 48, 160, 3, 1, 1, 1, 1),     # 3x1 filter, padding wider than the filter needs on the width
    (1, 28, 28, 256, 128, 3, 3, 1, 1, 1),    # 72 slabs: second accumulator set (long reduction)
    (1, 7, 7, 512, 256, 3, 3, 1, 1, 1),      # M = 49: one partial pixel tile
]


def _conv_case(i):
    n, h, w, c, k, r, s, st, pd, g = CONV_SHAPES[i]
    rng = np.random.default_rng(31000 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(k, r, s, c // g)) / np.sqrt(r * s * c // g)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b, (st, st), (pd, pd, pd, pd), g


@pytest.mark.parametrize("i", range(len(CONV_SHAPES)))
@pytest.mark.parametrize("bn", [128, 64])
def test_conv_p3(i, bn, knobs):
    G = _gpu()
    _take_p3(knobs, bn=bn)
    x, wt, b, st, pd, g = _conv_case(i)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.conv2d_f32(x, wt, bias, st, pd, g, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, bias, desc, act)
        assert variant.startswith(f"igemm_f32_p3_128x{bn}"), variant
        G.assert_close_f32(got, ref, f"conv case {i} bn {bn} act {act} [{variant}]")


@pytest.mark.parametrize("i", [0, 3, 8, 9])
@pytest.mark.parametrize("split", [2, 5])
def test_conv_p3_split_reduction(i, split, knobs):
    G = _gpu()
    _take_p3(knobs, split=split)
    x, wt, b, st, pd, g = _conv_case(i)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
    assert variant.startswith("igemm_f32_p3"), variant
    G.assert_close_f32(got, ref, f"conv case {i} split {split} [{variant}]")


def test_conv_p3_asymmetric_padding_and_strides(knobs):
    G = _gpu()
    _take_p3(knobs)
    rng = np.random.default_rng(31100)
    x = rng.uniform(-1, 1, size=(2, 13, 18, 64)).astype(np.float32)
    wt = (rng.standard_normal(size=(130, 3, 4, 64)) / np.sqrt(3 * 4 * 64)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(130,)).astype(np.float32)
    st, pd = (2, 1), (0, 2, 1, 3)                       # top, left, bottom, right
    ref = oracle.conv2d_f32(x, wt, b, st, pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, G.make_desc(x.shape, wt.shape, st, pd, 1), wl.ACT_RELU)
    assert variant.startswith("igemm_f32_p3"), variant
    G.assert_close_f32(got, ref, f"asymmetric padding [{variant}]")


@pytest.mark.parametrize("in_place", [False, True])
def test_conv_p3_tensor_add_link(in_place, knobs):
    G = _gpu()
    _take_p3(knobs)
    x, wt, b, st, pd, g = _conv_case(1)
    rng = np.random.default_rng(31200)
    n, h, w, _ = x.shape
    add = rng.uniform(-1, 1, size=(n, h, w, wt.shape[0])).astype(np.float32)
    ref = oracle.conv2d_f32_add(x, wt, b, add, st, pd, g, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, G.make_desc(x.shape, wt.shape, st, pd, g), wl.ACT_RELU,
                                          in_place=in_place)
    assert variant.startswith("igemm_f32_p3"), variant
    G.assert_close_f32(got, ref, f"add link in_place {in_place} [{variant}]")


FC_SHAPES = [(300, 512, 256), (129, 72, 200), (257, 1032, 65), (1024, 2048, 384), (64, 40, 1000), (130, 4104, 130)]


@pytest.mark.parametrize("shape", FC_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("split", [0, 3])
def test_fc_p3(shape, split, knobs):
    G = _gpu()
    _take_p3(knobs, split=split or None)
    M, K, N = shape
    layer = wl.FcLayer("p3", M, K, N)
    a, w, b = wl.fc_inputs_f32(layer, 31300 + M + K + N, dist="uniform_fan_in")
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.fc_f32(a, w, bias, act=act)
        got, variant = G.gpu_fc_f32(a, w, bias, act)
        assert variant.startswith("igemm_f32_p3"), variant
        G.assert_close_f32(got, ref, f"fc {shape} split {split} act {act} [{variant}]")


def test_p3_wide_value_range_is_held_to_fp32_accuracy(knobs):
    """Magnitudes over 24 binades in one tensor, exact powers of two and values whose low pieces are zero:
    the pieces are exact whatever the exponent, so the error stays at the size of fp32 rounding
    (componentwise: |gpu - exact| <= 4 * 2^-22 * (|A||W| + |b|))."""
    G = _gpu()
    _take_p3(knobs)
    M, K, N = 260, 264, 136
    rng = np.random.default_rng(31400)
    a = (rng.uniform(-1, 1, size=(M, K)) * np.exp2(rng.integers(-12, 12, size=(M, K)))).astype(np.float32)
    w = (rng.uniform(-1, 1, size=(K, N)) * np.exp2(rng.integers(-12, 12, size=(K, N)))).astype(np.float32)
    a[::7, ::5] = np.exp2(rng.integers(-10, 10, size=a[::7, ::5].shape)).astype(np.float32)   # single-piece values
    w[::3, ::11] = 0.0
    b = rng.uniform(-1, 1, size=(N,)).astype(np.float32)
    got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_NONE)
    assert variant.startswith("igemm_f32_p3"), variant
    exact = a.astype(np.float64) @ w.astype(np.float64) + b.astype(np.float64)
    scale = np.abs(a).astype(np.float64) @ np.abs(w).astype(np.float64) + np.abs(b).astype(np.float64)
    err = np.abs(got.astype(np.float64) - exact)
    assert np.all(np.isfinite(got))
    worst = float((err / scale).max())
    assert worst <= 4 * 2.0 ** -22, worst


def test_p3_error_is_no_larger_than_the_fp32_matrix_core_path(knobs):
    """Same layer through both kernels: the piece-product form's error against the fp64 oracle stays within
    twice that of v_mfma_f32_32x32x2_f32 accumulation (both are fp32-level; neither is reduced precision)."""
    G = _gpu()
    x, wt, b, st, pd, g = _conv_case(8)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=wl.ACT_NONE).astype(np.float64)
    _take_p3(knobs)
    got_p3, v_p3 = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_NONE)
    knobs.set("F32_P3", 0)
    got_f32, v_f32 = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_NONE)
    assert v_p3.startswith("igemm_f32_p3") and not v_f32.startswith("igemm_f32_p3"), (v_p3, v_f32)
    e_p3 = np.abs(got_p3 - ref)
    e_f32 = np.abs(got_f32 - ref)
    assert e_p3.max() <= 2 * e_f32.max() + 1e-7, (e_p3.max(), e_f32.max())
    assert np.sqrt((e_p3 ** 2).mean()) <= 2 * np.sqrt((e_f32 ** 2).mean()) + 1e-8


def test_p3_needs_the_workspace_and_falls_back_without_it(knobs):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    _take_p3(knobs)
    x, wt, b, st, pd, g = _conv_case(0)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=wl.ACT_RELU)
    need = glowmi.conv2d_workspace_bytes(desc)
    planes = 6 * (x.size + wt.size)
    assert need >= planes, (need, planes)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU, use_workspace=False)
    assert not variant.startswith("igemm_f32_p3"), variant
    G.assert_close_f32(got, ref, f"no workspace [{variant}]")
    # one byte short: the call must not touch the workspace at all
    xd, wd, bd = G.dev(x), G.dev(wt), G.dev(b)
    ws = torch.full((need - 1,), 0x5a, dtype=torch.uint8, device="cuda:0")
    y = G.poison(ref.shape, torch.float32)
    glowmi.conv2d(xd, wd, bd, y, desc, wl.ACT_RELU, ws)
    torch.cuda.synchronize()
    assert not glowmi.last_variant().startswith("igemm_f32_p3")
    assert bool((ws == 0x5a).all()), "a workspace that is too small was written to"
    G.assert_close_f32(y.cpu().numpy(), ref, "short workspace")
