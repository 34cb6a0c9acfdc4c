"""Depthwise 3x3 convolution (groups == channels, one filter per channel), fp32 and int8, through the C ABI
against the CPU oracle element by element: fp32 within 1e-5 + 1e-4 |oracle|, int8 bit-exact.  Strides 1 and 2,
every kind of padding, output widths that are not a multiple of the four-pixel runs the kernel walks, channel
counts from one quad to more than a wavefront's worth, a batch, no bias, both requantize forms, a filter offset,
uniformly drawn codes (saturation), and every layer bench.py times at its full size.  Shapes the kernel does not take
(channels not a multiple of four, another filter size, a tensor operand behind the layer, groups of more than
one channel) must still be right on the generic kernels.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  c  stride  pads (top, left, bottom, right)
SHAPES = [
    (1, 8, 8, 4, 1, (1, 1, 1, 1)),          # one channel quad
    (2, 13, 17, 8, 1, (1, 1, 1, 1)),        # ragged runs (17 = 4 * 4 + 1), a batch
    (1, 9, 22, 64, 1, (0, 0, 0, 0)),        # no padding, 20 output columns
    (3, 14, 15, 132, 1, (1, 0, 0, 1)),      # asymmetric padding, 33 quads: wavefronts straddle pixels
    (1, 5, 6, 256, 1, (2, 2, 2, 2)),        # padding wider than the filter needs
    (2, 16, 19, 32, 2, (1, 1, 1, 1)),       # stride 2, odd width
    (1, 15, 15, 96, 2, (0, 1, 1, 0)),       # stride 2, asymmetric padding
    (1, 3, 3, 16, 1, (0, 0, 0, 0)),         # a single output pixel
    (4, 28, 28, 128, 1, (1, 1, 1, 1)),      # more runs than one pass of the grid's threads per quad on small chips
    (1, 112, 112, 64, 2, (1, 1, 1, 1)),     # a network's first depthwise stage
]


def _layer(i):
    n, h, w, c, st, pd = SHAPES[i]
    return n, h, w, c, st, pd


ROW_FORMS = [1, 2, 3]      # knob DW: the planner's choice, one output row per run, two


@pytest.mark.parametrize("i", range(len(SHAPES)))
@pytest.mark.parametrize("rows", ROW_FORMS)
def test_depthwise_f32(i, rows, knobs):
    G = _gpu()
    knobs.set("DW", rows)
    n, h, w, c, st, pd = _layer(i)
    rng = np.random.default_rng(38000 + i)
    x = rng.standard_normal(size=(n, h, w, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(c, 3, 3, 1)) / 3).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(c,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, (st, st), pd, c)
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.conv2d_f32(x, wt, bias, (st, st), pd, c, act=act)
        got, variant = G.gpu_conv2d_f32(x, wt, bias, desc, act)
        assert variant == f"conv_dw_f32_3x3s{st}", variant
        G.assert_close_f32(got, ref, f"depthwise fp32 {SHAPES[i]} act {act}")
        got, variant = G.gpu_conv2d_f32(x, wt, bias, desc, act, use_workspace=False)
        assert variant == f"conv_dw_f32_3x3s{st}", variant
        G.assert_close_f32(got, ref, f"depthwise fp32 {SHAPES[i]} act {act} without a workspace")


@pytest.mark.parametrize("i", range(len(SHAPES)))
@pytest.mark.parametrize("dist,w_off", [("normal", 0), ("uniform", -7)])
@pytest.mark.parametrize("rows", ROW_FORMS)
def test_depthwise_int8(i, dist, w_off, rows, knobs):
    G = _gpu()
    knobs.set("DW", rows)
    n, h, w, c, st, pd = _layer(i)
    layer = wl.ConvLayer(f"dw{i}", n, h, w, c, c, 3, 3, st, 1, c)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 38100 + i, dist=dist, w_off=w_off)
    desc = G.make_desc(xq.shape, wq.shape, (st, st), pd, c)
    for act, bias in ((wl.ACT_RELU, bq), (wl.ACT_NONE, None)):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bias, qp.y_scale, qp.y_off,
                             (st, st), pd, c, act=act)
        got, variant = G.gpu_qconv2d(xq, wq, bias, qp, desc, act)
        assert variant == f"conv_dw_i8_3x3s{st}", variant
        G.assert_equal_i8(got, ref, f"depthwise int8 {SHAPES[i]} {dist} act {act}")


@pytest.mark.parametrize("y_scale_factor", [2.0, 64.0, 2.0 ** 26])
@pytest.mark.parametrize("w_off", [0, 3])
def test_depthwise_int8_every_requantize_form(y_scale_factor, w_off):
    """Multipliers of 1/4 and more take the 64-bit form, smaller ones the multiply-high, which without a filter
    offset has the rounding constant and the output offset folded into one addend down to multipliers of 2^-24;
    below that the unfolded form again."""
    G = _gpu()
    layer = wl.ConvLayer("dwq", 2, 12, 14, 24, 24, 3, 3, 1, 1, 24)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 38200, dist="normal", w_off=w_off)
    qp = wl.QParams(qp.x_scale, qp.x_off, qp.w_scale, qp.w_off, qp.x_scale * qp.w_scale * y_scale_factor, qp.y_off)
    desc = G.make_desc(xq.shape, wq.shape, (1, 1), (1, 1, 1, 1), 24)
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         (1, 1), (1, 1, 1, 1), 24, act=wl.ACT_NONE)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, wl.ACT_NONE)
    assert variant == "conv_dw_i8_3x3s1", variant
    G.assert_equal_i8(got, ref, f"depthwise int8, multiplier 1/{y_scale_factor}")


def test_shapes_the_depthwise_kernel_leaves_to_the_generic_ones(knobs):
    G = _gpu()
    rng = np.random.default_rng(38300)
    cases = [
        (6, 6, 3, 1),       # channels not a multiple of four
        (8, 8, 5, 1),       # 5 x 5 filter
        (16, 4, 3, 1),      # four groups of four channels: not depthwise
        (8, 8, 3, 3),       # stride 3
    ]
    for c, groups, r, st in cases:
        x = rng.standard_normal(size=(2, 11, 13, c)).astype(np.float32)
        wt = (rng.standard_normal(size=(c, r, r, c // groups)) / r).astype(np.float32)
        b = rng.uniform(-0.1, 0.1, size=(c,)).astype(np.float32)
        pd = (r // 2,) * 4
        desc = G.make_desc(x.shape, wt.shape, (st, st), pd, groups)
        ref = oracle.conv2d_f32(x, wt, b, (st, st), pd, groups, act=wl.ACT_RELU)
        got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
        assert not variant.startswith("conv_dw"), (variant, c, groups, r, st)
        G.assert_close_f32(got, ref, f"generic path c {c} groups {groups} filter {r} stride {st}")
    # a tensor operand behind a depthwise layer: the generic kernels' chain
    c = 16
    x = rng.standard_normal(size=(1, 9, 9, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(c, 3, 3, 1)) / 3).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(c,)).astype(np.float32)
    add = rng.standard_normal(size=(1, 9, 9, c)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), (1, 1, 1, 1), c)
    ref = oracle.conv2d_f32_add(x, wt, b, add, (1, 1), (1, 1, 1, 1), c, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32_chain(x, wt, b, add, desc, wl.ACT_RELU)
    assert not variant.startswith("conv_dw"), variant
    G.assert_close_f32(got, ref, "depthwise with a tensor add behind it")
    # the knob at 0: the generic kernels on a shape the depthwise kernel would take
    knobs.set("DW", 0)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), c, act=wl.ACT_RELU)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_RELU)
    assert not variant.startswith("conv_dw"), variant
    G.assert_close_f32(got, ref, "depthwise on the generic kernels")


@pytest.mark.parametrize("i", range(9))
def test_depthwise_layers_bench_times_fp32_and_int8(i):
    """Each of the nine layers of bench.py's depthwise workloads at batch 32, with the seeds bench.py uses: every
    output element, int8 into two differently pre-filled outputs."""
    G = _gpu()
    layer = wl.depthwise_layers(32)[i]
    st, pd = (layer.stride, layer.stride), (layer.pad,) * 4
    x, wt, b = wl.conv_inputs_f32(layer, wl.layer_seed(7, i))
    desc = G.desc_of(layer)
    ref = oracle.conv2d_f32(x, wt, b, st, pd, layer.groups, act=layer.act)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, layer.act)
    assert variant == f"conv_dw_f32_3x3s{layer.stride}", variant
    G.assert_close_f32(got, ref, f"{layer.name} fp32")
    xq, wq, bq, qp = wl.conv_inputs_q(layer, wl.layer_seed(7, i))
    ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                         st, pd, layer.groups, act=layer.act)
    for fill in (77, -5):
        got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, layer.act, fill=fill)
        assert variant == f"conv_dw_i8_3x3s{layer.stride}", variant
        G.assert_equal_i8(got, ref, f"{layer.name} int8 (output pre-filled with {fill})")


# ---------------------------------------------------------------------------------------------------
# a depthwise-separable block as one sequence out of one arena: depthwise 3x3 + Relu -> pointwise 1x1 + Relu
# ---------------------------------------------------------------------------------------------------
def _separable_layers(n, hw, c, k, stride):
    dw = wl.ConvLayer("s1", n, hw, hw, c, c, 3, 3, stride, 1, groups=c)
    return [dw, wl.ConvLayer("s2", n, dw.oh, dw.ow, c, k, 1, 1, 1, 0)]


@pytest.mark.parametrize("n,hw,c,k,stride", [(2, 14, 32, 64, 1), (1, 15, 64, 128, 2), (3, 9, 8, 24, 1)])
def test_separable_block_f32_sequence(n, hw, c, k, stride):
    """Each layer of the sequence against the oracle fed with the GPU's own previous activation, and a captured
    graph of the sequence replayed against the eager result (no memset nodes, default-priority stream)."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    specs = _separable_layers(n, hw, c, k, stride)
    data = [wl.conv_inputs_f32(s, 38500 + i) for i, s in enumerate(specs)]
    x = data[0][0]
    xd = G.dev(x)
    dev_w = [(G.dev(w), G.dev(b)) for (_, w, b) in data]
    tuples = [(G.desc_of(s), w, b, s.act, s.add) for s, (w, b) in zip(specs, dev_w)]
    outs = []
    for upto in (1, 2):
        arr = glowmi.seq_layers(tuples[:upto])
        arena = torch.empty(max(glowmi.seq_arena_bytes(arr, False), 16), dtype=torch.uint8, device="cuda:0")
        s = specs[upto - 1]
        y = G.poison((n, s.oh, s.ow, s.k), torch.float32)
        glowmi.seq_conv2d(xd, arr, y, arena)
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    prev = x
    for i, s in enumerate(specs):
        _, w, b = data[i]
        ref = oracle.conv2d_f32(prev, w, b, (s.stride, s.stride), (s.pad,) * 4, s.groups, act=s.act)
        G.assert_close_f32(outs[i], ref, f"separable block layer {i}")
        prev = outs[i]
    arr = glowmi.seq_layers(tuples)
    arena = torch.empty(max(glowmi.seq_arena_bytes(arr, False), 16), dtype=torch.uint8, device="cuda:0")
    y = G.poison(outs[1].shape, torch.float32)
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
        np.testing.assert_array_equal(y.cpu().numpy(), outs[1], err_msg=f"graph replay {rep}")
        scratch = torch.empty(1 << 16, device="cuda:0").normal_()      # the program's own eager work
        float(scratch.sum())


@pytest.mark.parametrize("n,hw,c,k,stride", [(2, 14, 32, 64, 1), (1, 15, 64, 128, 2), (3, 9, 8, 24, 1)])
def test_separable_block_int8_sequence(n, hw, c, k, stride):
    """Integer arithmetic end to end: the block must match the oracle's two layers bit for bit."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    specs = _separable_layers(n, hw, c, k, stride)
    data = [wl.conv_inputs_q(s, 38600 + i) for i, s in enumerate(specs)]
    xq = data[0][0]
    qps = [d[3] for d in data]
    in_q = [(qps[0].x_scale, qps[0].x_off), (qps[0].y_scale, qps[0].y_off)]     # a layer reads its predecessor's type
    xd = G.dev(xq)
    tuples, keep = [], []
    for i, s in enumerate(specs):
        _, w, b, qp = data[i]
        wd, bd = G.dev(w), G.dev(b)
        keep.append((wd, bd))
        tuples.append((G.desc_of(s), wd, bd, s.act, s.add, glowmi.QParam(qp.w_scale, qp.w_off),
                       glowmi.QParam(qp.y_scale, qp.y_off)))
    arr = glowmi.seq_layers(tuples)
    arena = torch.empty(max(glowmi.seq_arena_bytes(arr, True), 16), dtype=torch.uint8, device="cuda:0")
    last = specs[-1]
    y = G.poison((n, last.oh, last.ow, last.k), torch.int8)
    glowmi.seq_qconv2d(xd, glowmi.QParam(*in_q[0]), arr, y, arena)
    torch.cuda.synchronize()
    prev = xq
    for i, s in enumerate(specs):
        _, w, b, qp = data[i]
        prev = oracle.qconv2d(prev, in_q[i][0], in_q[i][1], w, qp.w_scale, qp.w_off, b, qp.y_scale, qp.y_off,
                              (s.stride, s.stride), (s.pad,) * 4, s.groups, act=s.act)
    G.assert_equal_i8(y.cpu().numpy(), prev, "int8 separable block sequence")
    assert 0.02 < np.mean((prev > -128) & (prev < 127)), "almost everything saturates"
