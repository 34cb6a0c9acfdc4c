"""Every tile form of the two generic implicit-GEMM kernels through the C ABI against the CPU oracle.
The planner takes only some of the forms by itself (the others are kept for measurements and are
selected with an environment variable), so each one is forced here on shapes with ragged tails in every
dimension, with and without a workspace for a split reduction.  fp32 within 1e-5 + 1e-4|oracle|, int8
bit-exact.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  c  k  r  s  stride  pads(t,l,b,r)  groups
CONV = [
    (2, 12, 12, 3, 5, 7, 7, (2, 2), (3, 3, 3, 3), 1),          # 3 channels: element-wise gather
    (3, 19, 17, 24, 40, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # ragged M, N and K tails (Kgemm = 216)
    (2, 7, 7, 128, 136, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # deep reduction, ragged N, split reduction
    (5, 16, 16, 32, 160, 3, 3, (2, 2), (0, 1, 1, 0), 1),       # stride 2, mixed pads, two 128-wide N tiles
    (1, 10, 10, 32, 48, 1, 1, (1, 1), (0, 0, 0, 0), 2),        # two groups
]
FC = [(130, 272, 144), (5, 64, 16), (33, 4096, 64), (70, 100, 36)]


@pytest.mark.parametrize("i", range(len(CONV)))
@pytest.mark.parametrize("tile", ["0", "1", "2", "3", "4", "5"])
def test_conv2d_f32_forced_tile(i, tile, knobs):
    G = _gpu()
    knobs.set("F32_TILE", tile)
    n, h, w, c, k, r, s, st, pd, g = CONV[i]
    layer = wl.ConvLayer(f"forced{i}", n, h, w, c, k, r, s, 1, 0, g)
    x, wt, b = wl.conv_inputs_f32(layer, 9100 + i, dist="uniform")
    ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=wl.ACT_RELU)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    for use_ws in (True, False):
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU, use_workspace=use_ws)
        assert variant.startswith("igemm_f32_"), variant
        G.assert_close_f32(got, ref, f"conv {i} tile {tile} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("shape", FC, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("tile", ["0", "1", "2", "3", "4", "5"])
def test_fc_f32_forced_tile(shape, tile, knobs):
    G = _gpu()
    knobs.set("F32_TILE", tile)
    M, K, N = shape
    a, w, b = wl.fc_inputs_f32(wl.FcLayer("forced", M, K, N), 9200 + M + K + N, dist="uniform_fan_in")
    ref = oracle.fc_f32(a, w, b, act=wl.ACT_NONE)
    for use_ws in (True, False):
        got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_NONE, use_workspace=use_ws)
        assert variant.startswith("igemm_f32_"), variant
        G.assert_close_f32(got, ref, f"fc {shape} tile {tile} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("i", range(len(CONV)))
@pytest.mark.parametrize("tile", ["0", "1", "2", "3"])
@pytest.mark.parametrize("w_off", [0, -7])
def test_qconv2d_forced_tile(i, tile, w_off, knobs):
    G = _gpu()
    knobs.set("I8_TILE", tile)
    n, h, w, c, k, r, s, st, pd, g = CONV[i]
    layer = wl.ConvLayer(f"forced{i}", n, h, w, c, k, r, s, 1, 0, g)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9300 + i, dist="uniform", w_off=w_off)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         st, pd, g, act=wl.ACT_RELU)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, g)
    for use_ws in (True, False):
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, wl.ACT_RELU, use_workspace=use_ws)
        assert variant.startswith("igemm_i8_") and "wide" not in variant, variant
        G.assert_equal_i8(got, ref, f"qconv {i} tile {tile} w_off {w_off} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("shape", FC, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("tile", ["0", "1", "2", "3"])
def test_qfc_forced_tile(shape, tile, knobs):
    G = _gpu()
    knobs.set("I8_TILE", tile)
    M, K, N = shape
    aq, wq, bq, qp = wl.fc_inputs_q(wl.FcLayer("forced", M, K, N), 9400 + M + K + N, dist="normal", w_off=2)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=wl.ACT_NONE)
    for use_ws in (True, False):
        got, variant = G.gpu_qfc(aq, wq, bq, qp, wl.ACT_NONE, use_workspace=use_ws)
        assert variant.startswith("igemm_i8_") and "wide" not in variant, variant
        G.assert_equal_i8(got, ref, f"qfc {shape} tile {tile} ws {use_ws} [{variant}]")
