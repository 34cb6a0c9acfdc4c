"""The first-layer kernels (7x7 stride 2 on 3 input channels, fp32 and int8) through the C ABI against
the CPU oracle on more shapes than the generic shape list holds: ragged tiles in both directions,
one-sided and no padding, output-channel counts that are not multiples of 16 or 64, several channel
slices, a map smaller than one tile, more tiles than persistent workgroups, and the layer's real size
(224 x 224).  fp32: |gpu - oracle| <= 1e-5 + 1e-4 |oracle|; int8: bit-exact.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  k  pads(t,l,b,r)
FIRST_LAYER = [
    (1, 224, 224, 64, (3, 3, 3, 3)),      # the layer itself
    (3, 37, 53, 64, (3, 3, 3, 3)),        # ragged tiles in both directions
    (2, 40, 40, 80, (3, 3, 3, 3)),        # two channel slices, the second with one run of 16
    (1, 33, 47, 70, (2, 3, 3, 2)),        # channel count that is no multiple of 16: byte stores
    (2, 21, 64, 16, (0, 0, 0, 0)),        # unpadded
    (1, 7, 7, 64, (3, 3, 3, 3)),          # map smaller than one tile
    (1, 9, 200, 32, (3, 0, 0, 3)),        # one tile row, many tile columns, one-sided padding
    (40, 50, 50, 64, (3, 3, 3, 3)),       # more tiles than persistent workgroups
    (1, 16, 16, 200, (3, 3, 3, 3)),       # four channel slices, the last of 8 channels
]


# both forms: products on the fp32 matrix cores, and three exact bf16 pieces per operand with six piece products
@pytest.mark.parametrize("i", range(len(FIRST_LAYER)))
@pytest.mark.parametrize("form", [("fp32", 0), ("bf16x6", 1)], ids=lambda f: f[0])
def test_first_layer_f32(i, form, knobs):
    G = _gpu()
    knobs.set("F32_SMALLC_BF16", form[1])
    n, h, w, k, pd = FIRST_LAYER[i]
    rng = np.random.default_rng(9900 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, 3)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, 7, 7, 3)) / 12).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, (2, 2), pd, 1)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.conv2d_f32(x, wt, b, (2, 2), pd, 1, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act)
        assert variant.startswith("conv_smallc_f32") and variant.endswith("bf16x6") == bool(form[1]), variant
        G.assert_close_f32(got, ref, f"first layer fp32 {FIRST_LAYER[i]} act {act} [{variant}]")


@pytest.mark.parametrize("i", range(len(FIRST_LAYER)))
@pytest.mark.parametrize("dist,x_off", [("normal", None), ("uniform", -11)])
def test_first_layer_int8(i, dist, x_off):
    G = _gpu()
    n, h, w, k, pd = FIRST_LAYER[i]
    layer = wl.ConvLayer(f"first{i}", n, h, w, 3, k, 7, 7, 2, 3, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9950 + i, dist=dist, w_off=0)
    if x_off is not None:
        qp = wl.QParams(qp.x_scale, x_off, qp.w_scale, qp.w_off, qp.y_scale, qp.y_off)
    desc = G.make_desc(xq.shape, wq.shape, (2, 2), pd, 1)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                             (2, 2), pd, 1, act=act)
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, act)
        assert variant.startswith("conv_smallc_i8"), variant
        G.assert_equal_i8(got, ref, f"first layer int8 {FIRST_LAYER[i]} {dist} act {act} [{variant}]")
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, None, qp.y_scale, qp.y_off,
                         (2, 2), pd, 1, act=wl.ACT_NONE)
    got, _ = G.gpu_qconv2d(xq, wq, None, qp, desc, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"first layer int8 {FIRST_LAYER[i]} without bias")


@pytest.mark.parametrize("mr_exp", [-1, -3])
def test_first_layer_int8_multipliers(mr_exp):
    """Both requantize forms (64-bit for multipliers from 1/4 up, multiply-high below)."""
    G = _gpu()
    rng = np.random.default_rng(9980 + mr_exp)
    xq = rng.integers(-20, 21, size=(2, 30, 30, 3), dtype=np.int8)
    wq = rng.integers(-9, 10, size=(64, 7, 7, 3), dtype=np.int8)
    bq = rng.integers(-50, 50, size=(64,), dtype=np.int32)
    qp = wl.QParams(0.8, 2, float(2.0 ** mr_exp), 0, 8.0, -3)
    pd = (3, 3, 3, 3)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (2, 2), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (2, 2), pd, 1), wl.ACT_RELU)
    assert variant.startswith("conv_smallc_i8"), variant
    assert len(np.unique(ref)) > 8
    G.assert_equal_i8(got, ref, f"first layer int8 multiplier {0.8 * 2.0 ** mr_exp / 8}")
