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


# both forms: products on the fp32 matrix cores, and two scaled fp16 pieces per operand with three piece products
@pytest.mark.parametrize("i", range(len(FIRST_LAYER)))
@pytest.mark.parametrize("form", [("fp32", 0), ("f16x3", 1)], ids=lambda f: f[0])
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
        assert variant.startswith("conv_smallc_f32") and variant.endswith("f16x3") == bool(form[1]), variant
        G.assert_close_f32(got, ref, f"first layer fp32 {FIRST_LAYER[i]} act {act} [{variant}]")


def _first_layer_f16(knobs, seed, n=2, h=37, w=53, k=80):
    knobs.set("F32_SMALLC_BF16", 1)
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, size=(n, h, w, 3)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, 7, 7, 3)) / 12).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b


def _run_first_layer(x, wt, b):
    G = _gpu()
    desc = G.make_desc(x.shape, wt.shape, (2, 2), (3, 3, 3, 3), 1)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_NONE)
    assert variant == "conv_smallc_f32_7x7s2c3_f16x3", variant
    return got


@pytest.mark.parametrize("ex,ew", [(80, -90), (-100, 40), (100, -90), (-50, -50)])
def test_first_layer_f16_power_of_two_scaling_changes_only_the_scale(ex, ew, knobs):
    """The fp16-piece form scales every patch and every workgroup's filters by a power of two of their own: scaling an
    operand by a power of two scales the result by it and changes nothing else, bit for bit."""
    x, wt, b = _first_layer_f16(knobs, 9990)
    base = _run_first_layer(x, wt, b)
    got = _run_first_layer(np.ldexp(x, ex).astype(np.float32), np.ldexp(wt, ew).astype(np.float32),
                           np.ldexp(b, ex + ew).astype(np.float32))
    assert np.all(np.isfinite(got))
    assert np.array_equal(np.ldexp(got.astype(np.float64), -(ex + ew)), base.astype(np.float64))


def test_first_layer_f16_wide_value_range_and_special_operands(knobs):
    """Magnitudes over 24 binades inside each tensor to the componentwise fp32-level bound; all-zero operands give the
    bias; an infinity makes the outputs it reaches non-finite and leaves no wrong finite value anywhere."""
    x, wt, b = _first_layer_f16(knobs, 9991)
    rng = np.random.default_rng(9992)
    xs = (x * np.exp2(rng.integers(-12, 12, size=x.shape))).astype(np.float32)
    ws = (wt * np.exp2(rng.integers(-12, 12, size=wt.shape))).astype(np.float32)
    ws[::3, :, :, 1] = 0.0
    pd = (3, 3, 3, 3)
    got = _run_first_layer(xs, ws, b)
    exact = oracle.conv2d_f32(xs, ws, b, (2, 2), pd, 1, act=wl.ACT_NONE).astype(np.float64)
    scale = oracle.conv2d_f32(np.abs(xs), np.abs(ws), np.abs(b), (2, 2), pd, 1, act=wl.ACT_NONE).astype(np.float64)
    assert np.all(np.isfinite(got))
    assert float((np.abs(got - exact) / scale).max()) <= 4 * 2.0 ** -22 + 2.0 ** -24
    got = _run_first_layer(np.zeros_like(x), wt, b)
    assert np.array_equal(got, np.broadcast_to(b, got.shape))
    got = _run_first_layer(x, np.zeros_like(wt), b)
    assert np.array_equal(got, np.broadcast_to(b, got.shape))
    xi = x.copy()
    xi[1, 20, 30, 1] = np.inf
    got = _run_first_layer(xi, wt, b)
    ref = oracle.conv2d_f32(xi, wt, b, (2, 2), pd, 1, act=wl.ACT_NONE)
    reached = ~np.isfinite(ref)
    assert reached.any() and not np.isfinite(got[reached]).any()
    rest = ~reached & ~np.isnan(got)
    assert np.all(np.abs(got[rest] - ref[rest]) <= 1e-5 + 1e-4 * np.abs(ref[rest]))


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
