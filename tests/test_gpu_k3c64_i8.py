"""The int8 kernel for 3x3 filters over 64 input channels (filter resident in LDS; at stride 1 a block's
input patch staged once per wavefront, at other strides one gathered chunk per filter row) through the C
ABI against the CPU oracle, bit-exact: strides,
every kind of padding, ragged pixel counts and channel counts, several filter slices, both requantize
forms, the tensor-add link, and the planner's own choice at a size where it takes this kernel.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  k  stride  pads(t,l,b,r)
K3_SHAPES = [
    (1, 8, 8, 64, (1, 1), (1, 1, 1, 1)),          # two pixel blocks, every border kind
    (2, 13, 11, 64, (1, 1), (1, 1, 1, 1)),        # ragged last block, blocks that span rows and images
    (1, 9, 9, 64, (1, 1), (0, 0, 0, 0)),          # unpadded: 7x7 outputs
    (3, 15, 17, 64, (2, 2), (1, 1, 1, 1)),        # stride 2
    (1, 14, 14, 64, (2, 1), (0, 1, 1, 0)),        # mixed strides, one-sided padding
    (1, 6, 6, 64, (1, 1), (2, 2, 2, 2)),          # padding as wide as the filter allows: whole windows outside
    (2, 10, 12, 16, (1, 1), (1, 1, 1, 1)),        # one run of 16 output channels
    (1, 12, 12, 80, (1, 1), (1, 1, 1, 1)),        # two slices, the second with a single run of 16
    (1, 7, 23, 208, (1, 1), (1, 1, 1, 1)),        # four slices, ragged
    (1, 1, 1, 64, (1, 1), (1, 1, 1, 1)),          # one pixel: only the centre tap inside
    (5, 3, 40, 128, (1, 2), (1, 0, 1, 1)),        # wide short images
    (1, 70, 70, 64, (1, 1), (1, 1, 1, 1)),        # more blocks than one workgroup's wavefronts: several per wavefront on few CUs
    (2, 5, 9, 64, (1, 1), (1, 1, 1, 1)),          # 5 x 9 outputs: a 4 x 8 block grid ragged by one row and one column
    (3, 4, 8, 32, (1, 1), (1, 1, 1, 1)),          # exactly one block per image
    (1, 11, 30, 64, (1, 1), (0, 2, 2, 0)),        # one-sided padding at stride 1, 11 x 30 outputs
]


# "gather" forced only where the planner would not take it anyway (stride 1)
K3_CASES = [(i, form) for i in range(len(K3_SHAPES)) for form in ("2d", "gather")
            if form == "2d" or K3_SHAPES[i][4] == (1, 1)]


@pytest.mark.parametrize("i,form", K3_CASES)
@pytest.mark.parametrize("dist,x_off", [("normal", None), ("uniform", -9)])
@pytest.mark.parametrize("waves", ["8", "16"])
def test_qconv2d_k3c64(i, form, dist, x_off, waves, knobs):
    """form "2d": the planner's own choice (at stride 1 the form that stages a block's input patch once);
    "gather": the form that gathers per filter row, which the planner takes for other strides only."""
    G = _gpu()
    knobs.set("I8_K3_MIN_BLOCKS", "1")     # take this kernel at any size
    knobs.set("I8_K3_WAVES", waves)
    n, h, w, k, st, pd = K3_SHAPES[i]
    if form == "gather":
        knobs.set("I8_K3_GATHER", "1")
    want_2d = form == "2d" and st == (1, 1)
    layer = wl.ConvLayer(f"k3_{i}", n, h, w, 64, k, 3, 3, 1, 0, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9500 + i, dist=dist, w_off=0)
    if x_off is not None:
        qp = wl.QParams(qp.x_scale, x_off, qp.w_scale, qp.w_off, qp.y_scale, qp.y_off)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, 1)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                             st, pd, 1, act=act)
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, act)
        assert variant.startswith("conv_k3c64_i8_w" + waves) and ("_2d" in variant) == want_2d, variant
        G.assert_equal_i8(got, ref, f"k3c64 {K3_SHAPES[i]} {dist} act {act} [{variant}]")
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, None, qp.y_scale, qp.y_off,
                         st, pd, 1, act=wl.ACT_NONE)
    got, _ = G.gpu_qconv2d(xq, wq, None, qp, desc, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"k3c64 {K3_SHAPES[i]} without bias")


@pytest.mark.parametrize("i", [1, 3, 7, 12])
@pytest.mark.parametrize("gather", [False, True])
def test_qconv2d_chain_k3c64(i, gather, knobs):
    """Tensor-add link of the element-wise chain behind this kernel (both forms), out of place and in place."""
    G = _gpu()
    knobs.set("I8_K3_MIN_BLOCKS", "1")
    if gather:
        knobs.set("I8_K3_GATHER", "1")
    n, h, w, k, st, pd = K3_SHAPES[i]
    layer = wl.ConvLayer(f"k3_{i}", n, h, w, 64, k, 3, 3, 1, 0, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9600 + i, dist="normal", w_off=0)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, 1)
    oh, ow = oracle.out_dim(h, 3, st[0], pd[0], pd[2]), oracle.out_dim(w, 3, st[1], pd[1], pd[3])
    rq = np.random.default_rng(9600 + i).integers(-128, 128, size=(n, oh, ow, k), dtype=np.int8)
    r_scale, r_off = float(np.float32(qp.y_scale * 0.7)), 9
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d_add(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, rq, r_scale, r_off,
                                 qp.y_scale, qp.y_off, st, pd, 1, act=act)
        for in_place in (False, True):
            got, variant = G.gpu_qconv2d_chain(xq, wq, bq, qp, rq, r_scale, r_off, desc, act, in_place=in_place)
            assert variant.startswith("conv_k3c64_i8") and variant.endswith("_add"), variant
            G.assert_equal_i8(got, ref, f"k3c64 chain {i} act {act} in-place {in_place} [{variant}]")


@pytest.mark.parametrize("mr_exp", [-1, 1, -3, -8])
def test_qconv2d_k3c64_multipliers(mr_exp, knobs):
    """Both requantize forms (64-bit for multipliers from 1/4 up, multiply-high below)."""
    G = _gpu()
    knobs.set("I8_K3_MIN_BLOCKS", "1")
    rng = np.random.default_rng(9700 + mr_exp)
    xq = rng.integers(-4, 5, size=(2, 9, 9, 64), dtype=np.int8)
    wq = rng.integers(-4, 5, size=(48, 3, 3, 64), dtype=np.int8)
    bq = rng.integers(-50, 50, size=(48,), dtype=np.int32)
    qp = wl.QParams(0.8, 1, float(2.0 ** mr_exp), 0, 1.0, -3)
    pd = (1, 1, 1, 1)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.make_desc(xq.shape, wq.shape, (1, 1), pd, 1), wl.ACT_RELU)
    assert variant.startswith("conv_k3c64_i8"), variant
    G.assert_equal_i8(got, ref, f"k3c64 multiplier 0.8*2^{mr_exp}")


def test_k3c64_not_taken_with_filter_offset_and_taken_by_the_planner(knobs):
    G = _gpu()
    pd = (1, 1, 1, 1)
    # planner's own choice: 2 x 128 x 128 pixels = 1024 blocks of 32
    layer = wl.ConvLayer("k3_big", 2, 128, 128, 64, 64, 3, 3, 1, 1, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9800, dist="normal", w_off=0)
    desc = G.make_desc(xq.shape, wq.shape, (1, 1), pd, 1)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, wl.ACT_RELU)
    assert variant.startswith("conv_k3c64_i8"), variant
    G.assert_equal_i8(got, ref, "planner-chosen k3c64")
    # a filter offset other than 0 takes the generic kernels
    knobs.set("I8_K3_MIN_BLOCKS", "1")
    layer = wl.ConvLayer("k3_off", 1, 9, 9, 64, 64, 3, 3, 1, 1, 1)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9801, dist="normal", w_off=5)
    desc = G.make_desc(xq.shape, wq.shape, (1, 1), pd, 1)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), pd, 1, act=wl.ACT_RELU)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, wl.ACT_RELU)
    assert not variant.startswith("conv_k3c64_i8"), variant
    G.assert_equal_i8(got, ref, "3x3 c64 int8 with a filter offset")
