"""Degenerate and extreme shapes through the C ABI against the CPU oracle: single pixels, single
channels, filters larger than the (padded) map allows for more than one output, strides beyond the
filter, one-element FullyConnected, the deepest reduction the quantized path accepts, saturation at
both rails, and a launch on a stream of the caller's.  fp32: |gpu - oracle| <= 1e-5 + 1e-4 |oracle|;
int8: bit-exact.
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
EDGE_CONV = [
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0, 0, 0), 1),            # one pixel, one channel, one tap
    (1, 1, 1, 5, 3, 3, 3, (1, 1), (1, 1, 1, 1), 1),            # 1x1 map under a 3x3 filter: only the centre tap is inside
    (2, 3, 3, 4, 4, 3, 3, (1, 1), (0, 0, 0, 0), 1),            # filter = map: one output pixel per image
    (1, 2, 9, 3, 2, 2, 2, (5, 4), (0, 0, 0, 0), 1),            # stride larger than the filter: input columns skipped
    (1, 5, 1, 8, 8, 5, 1, (1, 1), (2, 0, 2, 0), 1),            # one column: 5x1 filter, padding only above and below
    (1, 1, 7, 8, 8, 1, 7, (1, 1), (0, 3, 0, 3), 1),            # one row: 1x7 filter
    (3, 4, 4, 6, 6, 1, 1, (1, 1), (0, 0, 0, 0), 6),            # depthwise: 6 groups of one channel
    (1, 6, 6, 4, 12, 3, 3, (1, 1), (1, 1, 1, 1), 4),           # groups with one input channel and three outputs each
    (1, 4, 4, 1, 70, 3, 3, (1, 1), (1, 1, 1, 1), 1),           # one input channel, more outputs than one tile is wide
    (7, 2, 2, 2, 2, 2, 2, (1, 1), (1, 1, 1, 1), 1),            # every window touches padding
    (1, 9, 9, 16, 16, 3, 3, (1, 1), (0, 0, 5, 7), 1),          # padding on the bottom / right only, wider than the filter
]


@pytest.mark.parametrize("i", range(len(EDGE_CONV)))
def test_edge_conv_f32(i):
    G = _gpu()
    n, h, w, c, k, r, s, st, pd, g = EDGE_CONV[i]
    rng = np.random.default_rng(9000 + i)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = rng.uniform(-1, 1, size=(k, r, s, c // g)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.conv2d_f32(x, wt, b, st, pd, g, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_conv2d_f32(x, wt, b, desc, act, use_workspace=use_ws)
            G.assert_close_f32(got, ref, f"edge conv {i} act {act} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("i", range(len(EDGE_CONV)))
@pytest.mark.parametrize("w_off", [0, 9])
def test_edge_conv_int8(i, w_off):
    G = _gpu()
    n, h, w, c, k, r, s, st, pd, g = EDGE_CONV[i]
    layer = wl.ConvLayer(f"edge{i}", n, h, w, c, k, r, s, 1, 0, g)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 9100 + i, dist="uniform", w_off=w_off)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, g)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off,
                             st, pd, g, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_qconv2d(xq, wq, bq, qp, desc, act, use_workspace=use_ws)
            G.assert_equal_i8(got, ref, f"edge qconv {i} w_off {w_off} act {act} ws {use_ws} [{variant}]")


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 4, 4), (16, 4, 4), (17, 4, 4), (1, 3, 1), (2, 1, 5), (1, 65535, 4)],
                         ids=lambda s: "x".join(map(str, s)))
def test_edge_fc(shape):
    """One-element and one-row FullyConnected, 16 / 17 rows (either side of the skinny kernel's limit),
    and the deepest reduction the quantized path accepts (65535)."""
    G = _gpu()
    M, K, N = shape
    rng = np.random.default_rng(9200 + M + K + N)
    a = rng.uniform(-1, 1, size=(M, K)).astype(np.float32)
    w = (rng.uniform(-1, 1, size=(K, N)) / np.sqrt(K)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(N,)).astype(np.float32)
    ref = oracle.fc_f32(a, w, b, act=wl.ACT_RELU)
    for use_ws in (True, False):
        got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_RELU, use_workspace=use_ws)
        G.assert_close_f32(got, ref, f"edge fc {shape} ws {use_ws} [{variant}]")
    layer = wl.FcLayer("edge", M, K, N)
    aq, wq, bq, qp = wl.fc_inputs_q(layer, 9300 + M + K + N, dist="uniform", w_off=-3)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=wl.ACT_RELU)
    for use_ws in (True, False):
        got, variant = G.gpu_qfc(aq, wq, bq, qp, wl.ACT_RELU, use_workspace=use_ws)
        G.assert_equal_i8(got, ref, f"edge qfc {shape} ws {use_ws} [{variant}]")


def test_int8_saturates_at_both_rails():
    """All codes at the extremes: accumulators of the largest magnitude a reduction of this depth can
    produce, requantized with a multiplier near one, must clamp to -128 and 127 exactly as the oracle."""
    G = _gpu()
    K, N = 4608, 64
    aq = np.full((4, K), 127, np.int8)
    aq[1] = -128
    aq[2, ::2] = -128
    wq = np.full((K, N), 127, np.int8)
    wq[:, ::3] = -128
    bq = np.zeros((N,), np.int32)
    bq[::5] = 2 ** 30
    qp = wl.QParams(1.0, 0, 0.9, 0, 1.0, 0)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=wl.ACT_NONE)
    assert (ref == 127).any() and (ref == -128).any()
    got, variant = G.gpu_qfc(aq, wq, bq, qp, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"saturation [{variant}]")


def test_launch_on_a_caller_stream_and_back_to_back():
    """Two different layers queued on a non-default stream without synchronising in between; results
    only read after the stream has drained."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    rng = np.random.default_rng(9400)
    x = rng.uniform(-1, 1, size=(2, 12, 12, 16)).astype(np.float32)
    w1 = (rng.uniform(-1, 1, size=(32, 3, 3, 16)) / 12).astype(np.float32)
    b1 = rng.uniform(-0.1, 0.1, size=(32,)).astype(np.float32)
    w2 = (rng.uniform(-1, 1, size=(24, 1, 1, 32)) / 6).astype(np.float32)
    b2 = rng.uniform(-0.1, 0.1, size=(24,)).astype(np.float32)
    d1 = G.make_desc(x.shape, w1.shape, (1, 1), (1, 1, 1, 1), 1)
    d2 = G.make_desc((2, 12, 12, 32), w2.shape, (1, 1), (0, 0, 0, 0), 1)
    stream = torch.cuda.Stream()
    xd, w1d, b1d, w2d, b2d = G.dev(x), G.dev(w1), G.dev(b1), G.dev(w2), G.dev(b2)
    y1 = G.poison((2, 12, 12, 32), torch.float32)
    y2 = G.poison((2, 12, 12, 24), torch.float32)
    torch.cuda.synchronize()
    glowmi.conv2d(xd, w1d, b1d, y1, d1, wl.ACT_RELU, None, stream)
    glowmi.conv2d(y1, w2d, b2d, y2, d2, wl.ACT_NONE, None, stream)
    stream.synchronize()
    r1 = oracle.conv2d_f32(x, w1, b1, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_RELU)
    G.assert_close_f32(y1.cpu().numpy(), r1, "first layer on a caller stream")
    r2 = oracle.conv2d_f32(y1.cpu().numpy(), w2, b2, (1, 1), (0, 0, 0, 0), 1, act=wl.ACT_NONE)
    G.assert_close_f32(y2.cpu().numpy(), r2, "second layer on a caller stream")


@pytest.mark.parametrize("case", ["fc_skinny16", "conv_small", "conv_tiled_split", "fc_tiled"])
def test_bias_at_a_four_byte_address(case):
    """The ABI asks only 4-byte alignment of the bias: every kernel family reads it correctly from an
    address 4 bytes past a 16-byte boundary."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    rng = np.random.default_rng(9500)

    def shifted(b):
        pad = torch.zeros(b.size + 1, dtype=torch.float32, device="cuda:0")
        pad[1:] = torch.from_numpy(b)
        view = pad[1:]
        assert view.data_ptr() % 16 == 4
        return view

    if case in ("fc_skinny16", "fc_tiled"):
        M, K, N = (8, 512, 264) if case == "fc_skinny16" else (70, 4096, 96)
        a = rng.uniform(-1, 1, size=(M, K)).astype(np.float32)
        w = (rng.uniform(-1, 1, size=(K, N)) / np.sqrt(K)).astype(np.float32)
        b = rng.uniform(-0.1, 0.1, size=(N,)).astype(np.float32)
        y = G.poison((M, N), torch.float32)
        glowmi.fc(G.dev(a), G.dev(w), shifted(b), y, M, K, N, wl.ACT_RELU, G.workspace(glowmi.fc_workspace_bytes(M, K, N)))
        torch.cuda.synchronize()
        variant = glowmi.last_variant()
        assert ("skinny16" in variant) == (case == "fc_skinny16"), variant
        G.assert_close_f32(y.cpu().numpy(), oracle.fc_f32(a, w, b, act=wl.ACT_RELU), f"{case} [{variant}]")
        return
    if case == "conv_small":
        shape, wshape, pd = (1, 14, 14, 64), (64, 3, 3, 64), (1, 1, 1, 1)
    else:
        shape, wshape, pd = (1, 7, 7, 512), (96, 3, 3, 512), (1, 1, 1, 1)
    x = rng.uniform(-1, 1, size=shape).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=wshape) / np.sqrt(np.prod(wshape[1:]))).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(wshape[0],)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), pd, 1)
    oh, ow = glowmi.conv_out_shape(desc)
    y = G.poison((shape[0], oh, ow, wshape[0]), torch.float32)
    glowmi.conv2d(G.dev(x), G.dev(wt), shifted(b), y, desc, wl.ACT_RELU, G.workspace(glowmi.conv2d_workspace_bytes(desc)))
    torch.cuda.synchronize()
    variant = glowmi.last_variant()
    G.assert_close_f32(y.cpu().numpy(), oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_RELU), f"{case} [{variant}]")
