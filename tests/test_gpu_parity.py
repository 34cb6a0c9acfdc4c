"""Element-by-element parity of the HIP path (through the C ABI) against the CPU oracle on seeded
inputs, at sizes the oracle finishes in seconds and that still span several tiles and ragged tails.

fp32: |gpu - oracle| <= 1e-5 + 1e-4 |oracle|.  int8: bit-exact.
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
CONV_SHAPES = [
    (1, 32, 32, 16, 16, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # config 1
    (2, 9, 8, 4, 6, 3, 3, (2, 2), (1, 1, 1, 1), 1),            # tiny, vector path with c = 4
    (1, 8, 11, 2, 3, 5, 3, (2, 1), (2, 0, 1, 2), 1),           # scalar path, asymmetric pads
    (3, 6, 6, 4, 6, 3, 3, (1, 2), (1, 2, 0, 1), 2),            # groups 2, scalar (cg = 2)
    (2, 12, 12, 3, 5, 7, 7, (2, 2), (3, 3, 3, 3), 1),          # stem-like 7x7/2 with c = 3
    (1, 10, 10, 32, 48, 1, 1, (1, 1), (0, 0, 0, 0), 2),        # 1x1 grouped, vector
    (2, 30, 30, 3, 64, 7, 7, (2, 2), (3, 3, 3, 3), 1),         # stem shape, small map
    (3, 19, 17, 24, 40, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # ragged M and K tails (Kgemm = 216)
    (2, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # several M tiles
    (1, 28, 28, 64, 256, 1, 1, (1, 1), (0, 0, 0, 0), 1),       # 128-wide N tiles
    (2, 7, 7, 128, 136, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # deep K, ragged N (136), split-K
    (5, 16, 16, 32, 160, 3, 3, (2, 2), (0, 1, 1, 0), 1),       # stride 2, mixed pads
    (1, 40, 36, 16, 8, 3, 3, (1, 1), (2, 2, 2, 2), 1),         # pad larger than needed
    (4, 5, 5, 16, 32, 5, 5, (1, 1), (0, 0, 0, 0), 1),          # filter covers the whole map
    (2, 6, 6, 64, 64, 3, 3, (1, 1), (1, 1, 1, 1), 16),         # 16 groups of 4 channels
]


def _conv_case(i, dist="uniform"):
    n, h, w, c, k, r, s, st, pd, g = CONV_SHAPES[i]
    rng = np.random.default_rng(1000 + i)
    lim = 1.0 if dist == "uniform" else None
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, r, s, c // g)) / np.sqrt(r * s * c // g)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b, st, pd, g


@pytest.mark.parametrize("i", range(len(CONV_SHAPES)))
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_NONE])
def test_conv2d_f32(i, act):
    G = _gpu()
    x, wt, b, st, pd, g = _conv_case(i)
    ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=act)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    for use_ws in (True, False):
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act, use_workspace=use_ws)
        G.assert_close_f32(got, ref, f"conv case {i} act {act} ws {use_ws} [{variant}]")


def test_conv2d_f32_no_bias():
    G = _gpu()
    x, wt, b, st, pd, g = _conv_case(7)
    ref = oracle.conv2d_f32(x, wt, None, st, pd, g, act=wl.ACT_RELU)
    got, _ = G.gpu_conv2d_f32(x, wt, None, G.make_desc(x.shape, wt.shape, st, pd, g), wl.ACT_RELU)
    G.assert_close_f32(got, ref, "conv without bias")


def test_conv2d_f32_config1():
    G = _gpu()
    layer = wl.config1_layer()
    x, wt, b = wl.conv_inputs_f32(layer, wl.layer_seed(0, 0), dist="uniform")
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_RELU)
    got, _ = G.gpu_conv2d_f32(x, wt, b, G.desc_of(layer), wl.ACT_RELU)
    G.assert_close_f32(got, ref, "config 1")


@pytest.mark.parametrize("li", range(5))
def test_conv2d_f32_resnet_batch1(li):
    G = _gpu()
    layer = wl.resnet50_layers(1)[li]
    x, wt, b = wl.conv_inputs_f32(layer, wl.layer_seed(1, li))
    pd = (layer.pad,) * 4
    ref = oracle.conv2d_f32(x, wt, b, (layer.stride,) * 2, pd, 1, act=layer.act)
    for use_ws in (True, False):
        got, variant = G.gpu_conv2d_f32(x, wt, b, G.desc_of(layer), layer.act, use_workspace=use_ws)
        G.assert_close_f32(got, ref, f"{layer.name} ws {use_ws} [{variant}]")


# Pointwise-convolution kernel (LDS-resident filter slice, A fragments straight from global memory).
# n  h  w  c  k  stride
PW_SHAPES = [
    (2, 20, 21, 64, 256, 1),      # M = 840: ragged last pixel block, all four channel groups
    (1, 33, 31, 64, 72, 1),       # ragged N: one full 64-channel group + 8 channels
    (3, 17, 19, 128, 200, 2),     # stride 2, C = 128, two filter slices, ragged N
    (2, 15, 15, 128, 64, 1),      # C = 128, one channel group
    (1, 13, 29, 128, 330, 2),     # C = 128, three slices, ragged N, stride 2
    (1, 9, 9, 64, 520, 1),        # three slices, the last with a single channel group of 8
    (2, 12, 12, 64, 64, 1),       # one channel group out of the slice's four
    (1, 1, 5, 64, 64, 1),         # fewer pixels than one block
    (2, 15, 17, 256, 64, 1),      # C = 256: four chunks per reduction, one channel group per slice
    (1, 11, 13, 256, 136, 2),     # C = 256, three slices, ragged N, stride 2
]


# Both forms of the pointwise kernel: products on the fp32 matrix cores, and every operand cut into three
# bf16 pieces with six piece products on the bf16 matrix cores (same tolerance: both are fp32-level).
PW_FORMS = [("fp32", 0), ("bf16x6", 1)]


@pytest.mark.parametrize("shape", PW_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_NONE])
@pytest.mark.parametrize("form", PW_FORMS, ids=lambda f: f[0])
def test_conv2d_f32_pointwise(shape, act, form, knobs):
    G = _gpu()
    knobs.set("F32_PW_MIN_ITEMS", "1")     # take the pointwise kernel at any size
    knobs.set("F32_PW_BF16", form[1])
    n, h, w, c, k, st = shape
    rng = np.random.default_rng(4000 + 7 * c + k)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, 1, 1, c)) / np.sqrt(c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    ref = oracle.conv2d_f32(x, wt, b, (st, st), (0, 0, 0, 0), 1, act=act)
    desc = G.make_desc(x.shape, wt.shape, (st, st), (0, 0, 0, 0), 1)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act)
    assert variant.startswith("conv_pw_f32") and ("bf16x6" in variant) == bool(form[1]), variant
    G.assert_close_f32(got, ref, f"pointwise {shape} act {act} [{variant}]")
    got, variant = G.gpu_conv2d_f32(x, wt, None, desc, act)
    G.assert_close_f32(got, oracle.conv2d_f32(x, wt, None, (st, st), (0, 0, 0, 0), 1, act=act),
                       f"pointwise {shape} without bias")


def test_conv2d_f32_pointwise_not_taken_with_bottom_padding(knobs):
    """A 1x1 convolution padded at the bottom/right reads outside the image: generic kernel."""
    G = _gpu()
    knobs.set("F32_PW_MIN_ITEMS", "1")
    rng = np.random.default_rng(4100)
    x = rng.uniform(-1, 1, size=(1, 9, 9, 64)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(64, 1, 1, 64)) / 8).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(64,)).astype(np.float32)
    pads = (0, 0, 1, 2)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), pads, 1, act=wl.ACT_NONE)
    got, variant = G.gpu_conv2d_f32(x, wt, b, G.make_desc(x.shape, wt.shape, (1, 1), pads, 1), wl.ACT_NONE)
    assert not variant.startswith("conv_pw_f32"), variant
    G.assert_close_f32(got, ref, "1x1 with bottom/right padding")


FC_SHAPES = [(1, 64, 8), (5, 37, 11), (16, 512, 1000), (3, 1000, 257), (64, 2048, 1000), (1, 2048, 1000),
             (130, 260, 132), (33, 4096, 64), (256, 300, 520)]


@pytest.mark.parametrize("shape", FC_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_NONE])
def test_fc_f32(shape, act):
    G = _gpu()
    M, K, N = shape
    rng = np.random.default_rng(2000 + M + K + N)
    a = rng.uniform(-1, 1, size=(M, K)).astype(np.float32)
    w = (rng.uniform(-1, 1, size=(K, N)) / np.sqrt(K)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(N,)).astype(np.float32)
    ref = oracle.fc_f32(a, w, b, act=act)
    for use_ws in (True, False):
        got, variant = G.gpu_fc_f32(a, w, b, act, use_workspace=use_ws)
        G.assert_close_f32(got, ref, f"fc {shape} act {act} ws {use_ws} [{variant}]")


def _qconv_case(i, dist, w_off):
    n, h, w, c, k, r, s, st, pd, g = CONV_SHAPES[i]
    layer = wl.ConvLayer(f"case{i}", n, h, w, c, k, r, s, 1, 0, g)
    return wl.conv_inputs_q(layer, 3000 + i, dist=dist, w_off=w_off), st, pd, g


@pytest.mark.parametrize("i", range(len(CONV_SHAPES)))
@pytest.mark.parametrize("dist,w_off", [("normal", 0), ("uniform", 0), ("normal", -7)])
def test_qconv2d(i, dist, w_off):
    G = _gpu()
    (xq, wq, bq, qp), st, pd, g = _qconv_case(i, dist, w_off)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, g)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                             st, pd, g, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, act, use_workspace=use_ws)
            G.assert_equal_i8(got, ref, f"qconv case {i} {dist} w_off {w_off} act {act} ws {use_ws} [{variant}]")


# int8 pointwise kernel: output channels in multiples of 16, filter offset 0.
# n  h  w  c  k  stride
PWQ_SHAPES = [
    (2, 20, 21, 64, 256, 1),      # ragged last pixel block, four channel groups
    (1, 33, 31, 64, 80, 1),       # ragged N: one full group + 16 channels
    (3, 17, 19, 128, 208, 2),     # stride 2, C = 128
    (2, 15, 15, 256, 64, 1),      # C = 256, one channel group
    (1, 13, 29, 256, 336, 2),     # C = 256, three slices of 128, ragged, stride 2
    (1, 9, 9, 64, 528, 1),        # three slices, the last with a single run of 16 channels
    (1, 1, 5, 128, 48, 1),        # fewer pixels than one block
]


@pytest.mark.parametrize("shape", PWQ_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dist", ["normal", "uniform"])
def test_qconv2d_pointwise(shape, dist, knobs):
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", "1")      # take the pointwise kernel at any size
    n, h, w, c, k, st = shape
    layer = wl.ConvLayer("pw", n, h, w, c, k, 1, 1, st, 0, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 5000 + 3 * c + k, dist=dist, w_off=0)
    desc = G.make_desc(xq.shape, wq.shape, (st, st), (0, 0, 0, 0), 1)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                             (st, st), (0, 0, 0, 0), 1, act=act)
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, act)
        assert variant.startswith("conv_pw_i8"), variant
        G.assert_equal_i8(got, ref, f"pointwise int8 {shape} {dist} act {act} [{variant}]")
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, None, qp.y_scale, qp.y_off,
                         (st, st), (0, 0, 0, 0), 1, act=wl.ACT_NONE)
    got, _ = G.gpu_qconv2d(xq, wq, None, qp, desc, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"pointwise int8 {shape} without bias")


@pytest.mark.parametrize("mr_exp", [-1, 1, -3, -8])
def test_qconv2d_pointwise_multipliers(mr_exp, knobs):
    """Both requantize forms of the pointwise kernel (64-bit for multipliers from 1/4 up)."""
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", "1")
    rng = np.random.default_rng(170 + mr_exp)
    xq = rng.integers(-6, 7, size=(2, 9, 9, 64), dtype=np.int8)
    wq = rng.integers(-5, 6, size=(48, 1, 1, 64), dtype=np.int8)
    bq = rng.integers(-50, 50, size=(48,), dtype=np.int32)
    qp = wl.QParams(0.8, 1, float(2.0 ** mr_exp), 0, 1.0, -3)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), (0, 0, 0, 0), 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (1, 1), (0, 0, 0, 0), 1),
                                 wl.ACT_RELU)
    assert variant.startswith("conv_pw_i8"), variant
    G.assert_equal_i8(got, ref, f"pointwise int8 multiplier 0.8*2^{mr_exp}")


def test_qconv2d_pointwise_not_taken_with_filter_offset(knobs):
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", "1")
    layer = wl.ConvLayer("pw", 1, 9, 9, 64, 64, 1, 1, 1, 0, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 5999, dist="normal", w_off=5)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), (0, 0, 0, 0), 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (1, 1), (0, 0, 0, 0), 1),
                                 wl.ACT_RELU)
    assert not variant.startswith("conv_pw_i8"), variant
    G.assert_equal_i8(got, ref, "1x1 int8 with a filter offset")


def test_qconv2d_zero_point_padding():
    """Input constantly at its offset: every output, borders included, is requantize(bias)."""
    G = _gpu()
    rng = np.random.default_rng(5)
    xq = np.full((2, 9, 9, 16), 11, np.int8)
    wq = rng.integers(-127, 128, size=(24, 3, 3, 16), dtype=np.int8)
    bq = rng.integers(-4000, 4000, size=(24,), dtype=np.int32)
    qp = wl.QParams(0.05, 11, 0.01, 0, 0.02, -5)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), (1, 1, 1, 1), 1)
    assert np.all(ref == ref[0, 0, 0, :])
    got, _ = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (1, 1), (1, 1, 1, 1), 1), wl.ACT_NONE)
    G.assert_equal_i8(got, ref, "zero-point padding")


@pytest.mark.parametrize("li", range(5))
def test_qconv2d_resnet_batch1(li):
    G = _gpu()
    layer = wl.resnet50_layers(1)[li]
    xq, wq, bq, qp = wl.conv_inputs_q(layer, wl.layer_seed(3, li))
    pd = (layer.pad,) * 4
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (layer.stride,) * 2, pd, 1, act=layer.act)
    for use_ws in (True, False):
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.desc_of(layer), layer.act, use_workspace=use_ws)
        G.assert_equal_i8(got, ref, f"{layer.name} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("shape", FC_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dist,w_off", [("normal", 0), ("uniform", 3)])
def test_qfc(shape, dist, w_off):
    G = _gpu()
    M, K, N = shape
    layer = wl.FcLayer("case", M, K, N)
    aq, wq, bq, qp = wl.fc_inputs_q(layer, 4000 + M + K + N, dist=dist, w_off=w_off)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_qfc(aq, wq, bq, qp, act, use_workspace=use_ws)
            G.assert_equal_i8(got, ref, f"qfc {shape} {dist} act {act} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("mr_exp", [-1, 0, 1, 2, -2, -3, -8])
def test_quantized_large_and_small_multipliers(mr_exp):
    """Combined multipliers around and above 1/4 take the kernel's 64-bit requantize form, smaller
    ones its multiply-high form; both must agree with the oracle bit for bit."""
    G = _gpu()
    rng = np.random.default_rng(70 + mr_exp)
    xq = rng.integers(-6, 7, size=(2, 9, 9, 16), dtype=np.int8)
    wq = rng.integers(-5, 6, size=(40, 3, 3, 16), dtype=np.int8)
    bq = rng.integers(-50, 50, size=(40,), dtype=np.int32)
    # sx*sw/sy = 0.8 * 2^mr_exp (not a power of two, so the mantissa is a full 31-bit number)
    qp = wl.QParams(0.8, 1, float(2.0 ** mr_exp), 0, 1.0, -3)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_RELU)
    assert (ref > -3).any()
    got, _ = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (1, 1), (1, 1, 1, 1), 1), wl.ACT_RELU)
    G.assert_equal_i8(got, ref, f"qconv multiplier 0.8*2^{mr_exp}")
    aq = rng.integers(-4, 5, size=(5, 64), dtype=np.int8)
    wf = rng.integers(-4, 5, size=(64, 48), dtype=np.int8)
    bf = rng.integers(-20, 20, size=(48,), dtype=np.int32)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wf, qp.w_scale, qp.w_off, bf, qp.y_scale, qp.y_off, act=wl.ACT_NONE)
    got, _ = G.gpu_qfc(aq, wf, bf, qp, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"qfc multiplier 0.8*2^{mr_exp}")


# ---------------------------------------------------------------------------------------------------
# element-wise chain with a tensor add (residual add + Relu in the producing kernel)
# ---------------------------------------------------------------------------------------------------
CHAIN_CASES = [0, 3, 4, 7, 8, 9, 10, 11]     # generic tiles, groups, stem shape, split-K, ragged tails


@pytest.mark.parametrize("i", CHAIN_CASES)
@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_NONE])
def test_conv2d_chain_f32(i, act):
    G = _gpu()
    x, wt, b, st, pd, g = _conv_case(i)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    oh, ow = oracle.out_dim(x.shape[1], wt.shape[1], st[0], pd[0], pd[2]), oracle.out_dim(x.shape[2], wt.shape[2], st[1], pd[1], pd[3])
    add = np.random.default_rng(6000 + i).uniform(-1, 1, size=(x.shape[0], oh, ow, wt.shape[0])).astype(np.float32)
    ref = oracle.conv2d_f32_add(x, wt, b, add, st, pd, g, act=act)
    for use_ws in (True, False):
        for in_place in (False, True):
            got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, desc, act, use_workspace=use_ws, in_place=in_place)
            G.assert_close_f32(got, ref, f"chain case {i} act {act} ws {use_ws} in-place {in_place} [{variant}]")
    # a chain without the add link is the plain operator
    got, _ = G.gpu_conv2d_f32_chain(x, wt, b, None, desc, act)
    G.assert_close_f32(got, oracle.conv2d_f32(x, wt, b, st, pd, g, act=act), f"chain case {i} without addend")


@pytest.mark.parametrize("shape", PW_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("form", PW_FORMS, ids=lambda f: f[0])
def test_conv2d_chain_f32_pointwise(shape, form, knobs):
    G = _gpu()
    knobs.set("F32_PW_MIN_ITEMS", "1")
    knobs.set("F32_PW_BF16", form[1])
    n, h, w, c, k, st = shape
    rng = np.random.default_rng(6100 + 7 * c + k)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, 1, 1, c)) / np.sqrt(c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, (st, st), (0, 0, 0, 0), 1)
    oh, ow = (h - 1) // st + 1, (w - 1) // st + 1
    add = rng.uniform(-1, 1, size=(n, oh, ow, k)).astype(np.float32)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.conv2d_f32_add(x, wt, b, add, (st, st), (0, 0, 0, 0), 1, act=act)
        for in_place in (False, True):
            got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, desc, act, in_place=in_place)
            assert variant.startswith("conv_pw_f32") and variant.endswith("_add"), variant
            assert ("bf16x6" in variant) == bool(form[1]), variant
            G.assert_close_f32(got, ref, f"pointwise chain {shape} act {act} in-place {in_place} [{variant}]")


@pytest.mark.parametrize("i", CHAIN_CASES)
@pytest.mark.parametrize("dist,w_off", [("normal", 0), ("uniform", 0), ("normal", -7)])
def test_qconv2d_chain(i, dist, w_off):
    G = _gpu()
    (xq, wq, bq, qp), st, pd, g = _qconv_case(i, dist, w_off)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, g)
    oh, ow = oracle.out_dim(xq.shape[1], wq.shape[1], st[0], pd[0], pd[2]), oracle.out_dim(xq.shape[2], wq.shape[2], st[1], pd[1], pd[3])
    rng = np.random.default_rng(6200 + i)
    rq = rng.integers(-128, 128, size=(xq.shape[0], oh, ow, wq.shape[0]), dtype=np.int8)
    # addend scales on both sides of the accumulator's: multipliers well above and below one
    for r_scale, r_off in ((float(np.float32(qp.y_scale * 0.7)), 9), (float(np.float32(qp.x_scale * qp.w_scale * 0.3)), -4)):
        for act in (wl.ACT_RELU, wl.ACT_NONE):
            ref = oracle.qconv2d_add(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, rq, r_scale, r_off,
                                     qp.y_scale, qp.y_off, st, pd, g, act=act)
            for use_ws, in_place in ((True, False), (False, True)):
                got, variant = G.gpu_qconv2d_chain(xq, wq, bq, qp, rq, r_scale, r_off, desc, act,
                                                   use_workspace=use_ws, in_place=in_place)
                G.assert_equal_i8(got, ref, f"qchain case {i} {dist} w_off {w_off} r_scale {r_scale} act {act} "
                                            f"ws {use_ws} in-place {in_place} [{variant}]")


@pytest.mark.parametrize("shape", PWQ_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_chain_pointwise(shape, knobs):
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", "1")
    n, h, w, c, k, st = shape
    layer = wl.ConvLayer("pw", n, h, w, c, k, 1, 1, st, 0, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 6300 + 3 * c + k, dist="normal", w_off=0)
    desc = G.make_desc(xq.shape, wq.shape, (st, st), (0, 0, 0, 0), 1)
    oh, ow = (h - 1) // st + 1, (w - 1) // st + 1
    rq = np.random.default_rng(6300 + k).integers(-128, 128, size=(n, oh, ow, k), dtype=np.int8)
    r_scale, r_off = float(np.float32(qp.y_scale * 0.6)), -11
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d_add(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, rq, r_scale, r_off,
                                 qp.y_scale, qp.y_off, (st, st), (0, 0, 0, 0), 1, act=act)
        for in_place in (False, True):
            got, variant = G.gpu_qconv2d_chain(xq, wq, bq, qp, rq, r_scale, r_off, desc, act, in_place=in_place)
            assert variant.startswith("conv_pw_i8") and variant.endswith("_add"), variant
            G.assert_equal_i8(got, ref, f"pointwise qchain {shape} act {act} in-place {in_place} [{variant}]")


# ---------------------------------------------------------------------------------------------------
# conversions at the borders of the integer islands: quantize / dequantize / rescale on the device
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("count", [1, 15, 16, 17, 4096, 100003, 1 << 21])
def test_quantize_dequantize_rescale(count):
    import torch
    import paper_1805_00907_amd as glowmi
    rng = np.random.default_rng(7000 + count % 97)
    scale, off = float(np.float32(rng.uniform(0.01, 0.1))), int(rng.integers(-30, 31))
    x = (rng.standard_normal(size=count) * 3.0).astype(np.float32)
    # exact ties and values far outside the range exercise rounding to even and saturation
    x[: min(count, 8)] = (np.array([0.5, 1.5, 2.5, -0.5, -1.5, 1e6, -1e6, 0.0], np.float32) * np.float32(scale))[: min(count, 8)]
    xd = torch.from_numpy(x).to("cuda:0")
    qd = torch.full((count + 64,), 77, dtype=torch.int8, device="cuda:0")
    glowmi.quantize(xd, qd, glowmi.QParam(scale, off), count=count)
    torch.cuda.synchronize()
    q = qd.cpu().numpy()
    np.testing.assert_array_equal(q[:count], oracle.quantize_f32(x, scale, off))
    assert np.all(q[count:] == 77), "write past the end"

    vd = torch.full((count + 64,), float("nan"), dtype=torch.float32, device="cuda:0")
    glowmi.dequantize(qd, vd, glowmi.QParam(scale, off), count=count)
    torch.cuda.synchronize()
    v = vd.cpu().numpy()
    np.testing.assert_array_equal(v[:count], oracle.dequantize_f32(q[:count], scale, off))
    assert np.all(np.isnan(v[count:])), "write past the end"

    for s_out, o_out in ((float(np.float32(scale * 2.3)), -7), (float(np.float32(scale * 0.11)), 12), (scale, off)):
        rd = torch.full((count + 64,), 55, dtype=torch.int8, device="cuda:0")
        glowmi.rescale(qd, glowmi.QParam(scale, off), rd, glowmi.QParam(s_out, o_out), count=count)
        torch.cuda.synchronize()
        r = rd.cpu().numpy()
        np.testing.assert_array_equal(r[:count], oracle.rescale(q[:count], scale, off, s_out, o_out))
        assert np.all(r[count:] == 55), "write past the end"
    # in place
    rd = qd.clone()
    glowmi.rescale(rd, glowmi.QParam(scale, off), rd, glowmi.QParam(0.05, 3), count=count)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(rd.cpu().numpy()[:count], oracle.rescale(q[:count], scale, off, 0.05, 3))


# ---------------------------------------------------------------------------------------------------
# a bottleneck block as one sequence out of one arena (1x1 reduce -> 3x3 -> 1x1 expand + shortcut + Relu)
# ---------------------------------------------------------------------------------------------------
def _block_layers(n, hw, c, mid):
    return [wl.ConvLayer("b1", n, hw, hw, c, mid, 1, 1, 1, 0), wl.ConvLayer("b2", n, hw, hw, mid, mid, 3, 3, 1, 1),
            wl.ConvLayer("b3", n, hw, hw, mid, c, 1, 1, 1, 0, add=True)]


@pytest.mark.parametrize("n,hw,c,mid", [(2, 9, 32, 8), (3, 14, 256, 64), (1, 28, 128, 64)])
def test_sequence_f32_bottleneck(n, hw, c, mid, knobs):
    """Every layer of the sequence against the oracle fed with the GPU's own previous activation
    (prefix sequences are deterministic), to the single-operator tolerance; plus replays of the
    captured graph against the eager result."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    knobs.set("F32_PW_MIN_ITEMS", "1")
    specs = _block_layers(n, hw, c, mid)
    data = [wl.conv_inputs_f32(s, 8000 + i) for i, s in enumerate(specs)]
    x = data[0][0]
    xd = G.dev(x)
    dev_w = [(G.dev(w), G.dev(b)) for (_, w, b) in data]
    tuples = [(G.desc_of(s), w, b, s.act, s.add) for s, (w, b) in zip(specs, dev_w)]
    outs = []
    for upto in (1, 2, 3):
        arr = glowmi.seq_layers(tuples[:upto])
        arena = torch.empty(glowmi.seq_arena_bytes(arr, False), dtype=torch.uint8, device="cuda:0")
        s = specs[upto - 1]
        y = G.poison((n, s.oh, s.ow, s.k), torch.float32)
        if upto == 1 or upto == 2:
            glowmi.seq_conv2d(xd, arr, y, arena)
        else:
            glowmi.seq_conv2d(xd, arr, y, arena)
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    prev = x
    for i, s in enumerate(specs):
        _, w, b = data[i]
        ref = oracle.conv2d_f32_add(prev, w, b, x if s.add else None, (1, 1), (s.pad,) * 4, 1, act=s.act)
        G.assert_close_f32(outs[i], ref, f"sequence layer {i}")
        prev = outs[i]
    # graph replays, with eager work and synchronisation in between, each checked against eager
    arr = glowmi.seq_layers(tuples)
    arena = torch.empty(glowmi.seq_arena_bytes(arr, False), dtype=torch.uint8, device="cuda:0")
    y = G.poison(outs[2].shape, torch.float32)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        glowmi.seq_conv2d(xd, arr, y, arena, side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            glowmi.seq_conv2d(xd, arr, y, arena, side)
    torch.cuda.synchronize()
    for rep in range(3):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), outs[2], err_msg=f"graph replay {rep}")
        scratch = torch.empty(1 << 16, device="cuda:0").normal_()      # the program's own eager work
        float(scratch.sum())


@pytest.mark.parametrize("n,hw,c,mid", [(2, 9, 32, 16), (3, 14, 256, 64), (1, 28, 128, 64)])
def test_sequence_int8_bottleneck(n, hw, c, mid, knobs):
    """Integer arithmetic end to end: the whole block must match the oracle's chain bit for bit."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", "1")
    specs = _block_layers(n, hw, c, mid)
    data = [wl.conv_inputs_q(s, 8100 + i) for i, s in enumerate(specs)]
    xq = data[0][0]
    qps = [d[3] for d in data]
    # a layer's input type is the previous layer's output type
    in_q = [(qps[0].x_scale, qps[0].x_off)] + [(qps[i].y_scale, qps[i].y_off) for i in range(2)]
    xd = G.dev(xq)
    tuples, keep = [], []
    for i, s in enumerate(specs):
        _, w, b, qp = data[i]
        wd, bd = G.dev(w), G.dev(b)
        keep.append((wd, bd))
        tuples.append((G.desc_of(s), wd, bd, s.act, s.add, glowmi.QParam(qp.w_scale, qp.w_off),
                       glowmi.QParam(qp.y_scale, qp.y_off)))
    arr = glowmi.seq_layers(tuples)
    arena = torch.empty(glowmi.seq_arena_bytes(arr, True), dtype=torch.uint8, device="cuda:0")
    last = specs[-1]
    y = G.poison((n, last.oh, last.ow, last.k), torch.int8)
    glowmi.seq_qconv2d(xd, glowmi.QParam(*in_q[0]), arr, y, arena)
    torch.cuda.synchronize()
    prev = xq
    for i, s in enumerate(specs):
        _, w, b, qp = data[i]
        prev = oracle.qconv2d_add(prev, in_q[i][0], in_q[i][1], w, qp.w_scale, qp.w_off, b,
                                  xq if s.add else None, in_q[0][0], in_q[0][1], qp.y_scale, qp.y_off,
                                  (1, 1), (s.pad,) * 4, 1, act=s.act)
    G.assert_equal_i8(y.cpu().numpy(), prev, "int8 bottleneck sequence")
    assert 0.02 < np.mean((prev > -128) & (prev < 127)), "almost everything saturates"
