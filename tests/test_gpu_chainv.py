"""General element-wise chains behind the contraction (glowmi_conv2d_chainv / glowmi_qconv2d_chainv)
through the C ABI against the CPU oracle, element by element: op lists of every kind and order, with
one and two added tensors, in place, with and without a workspace (split reduction + finishing
kernel), ragged shapes, groups, scalar and vector gathers.  fp32: |gpu - oracle| <= 1e-5 + 1e-4 |oracle|;
int8: bit-exact.  Lists that are one of the fixed shapes must give the fixed entry points' kernels.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# n  h  w  c  k  r  s  stride  pads  groups
SHAPES = [
    (2, 9, 9, 8, 12, 3, 3, (1, 1), (1, 1, 1, 1), 1),          # ragged tile, vector gathers
    (1, 17, 13, 3, 70, 3, 3, (2, 1), (1, 0, 1, 2), 1),        # scalar gathers, two column tiles
    (3, 12, 12, 16, 16, 1, 1, (1, 1), (0, 0, 0, 0), 2),       # pointwise, groups
    (1, 7, 7, 512, 96, 3, 3, (1, 1), (1, 1, 1, 1), 1),        # deep reduction on few pixels: split + finishing kernel
    (1, 6, 6, 2080, 32, 1, 1, (1, 1), (0, 0, 0, 0), 1),       # reduction beyond 32 slabs (second accumulator set)
    (2, 20, 20, 32, 64, 3, 3, (1, 1), (1, 1, 1, 1), 1),       # several full tiles
]


def _lists_f32(rng, yshape):
    t1 = rng.uniform(-1, 1, size=yshape).astype(np.float32)
    t2 = rng.uniform(-1, 1, size=yshape).astype(np.float32)
    return [
        [("mul", 0.5)],
        [("clip", -0.25, 0.4)],
        [("max", 0.125), ("add", t1)],
        [("add", t1), ("mul", -1.5), ("add", t2), ("max", -0.1)],
        [("mul", 2.0), ("add", t1), ("clip", -1.0, 1.5)],
        [("clip", -0.5, 0.5), ("mul", 3.0), ("clip", -1.0, 1.25), ("add", t2)],
        [("max", 0.0), ("max", 0.5)],
    ]


@pytest.mark.parametrize("si", range(len(SHAPES)))
def test_conv2d_chainv_f32(si):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    n, h, w, c, k, r, s, st, pd, g = SHAPES[si]
    rng = np.random.default_rng(11000 + si)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.uniform(-1, 1, size=(k, r, s, c // g)) / np.sqrt(r * s * c // g)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    desc = G.make_desc(x.shape, wt.shape, st, pd, g)
    oh, ow = glowmi.conv_out_shape(desc)
    yshape = (n, oh, ow, k)
    xd, wd, bd = G.dev(x), G.dev(wt), G.dev(b)
    for li, ops in enumerate(_lists_f32(rng, yshape)):
        ref = oracle.conv2d_f32_chain(x, wt, b, ops, st, pd, g)
        dev_ops = [(o[0], G.dev(o[1])) if o[0] == "add" else o for o in ops]
        need = glowmi.conv2d_chainv_workspace_bytes(desc, dev_ops)
        for use_ws in (True, False):
            whole, y = G.guarded(yshape, torch.float32)
            glowmi.conv2d_chainv(xd, wd, bd, y, desc, dev_ops, G.workspace(need) if use_ws else None)
            torch.cuda.synchronize()
            variant = glowmi.last_variant()
            assert G.guards_intact(whole, torch.float32), "write outside the output tensor"
            assert variant.endswith("_chainv"), variant
            G.assert_close_f32(y.cpu().numpy(), ref, f"shape {si} list {li} ws {use_ws} [{variant}]")
        if si == 3:
            assert need > 0, "this shape is meant to exercise the split reduction"
    # in place: the output buffer holds the first added tensor
    ops = _lists_f32(rng, yshape)[4]
    ref = oracle.conv2d_f32_chain(x, wt, b, ops, st, pd, g)
    whole, y = G.guarded(yshape, torch.float32)
    y.copy_(torch.from_numpy(ops[1][1]))
    glowmi.conv2d_chainv(xd, wd, bd, y, desc, [ops[0], ("add", y), ops[2]],
                         G.workspace(glowmi.conv2d_chainv_workspace_bytes(desc, [ops[0], ("add", y), ops[2]])))
    torch.cuda.synchronize()
    G.assert_close_f32(y.cpu().numpy(), ref, f"shape {si} in place [{glowmi.last_variant()}]")
    # without bias
    ref = oracle.conv2d_f32_chain(x, wt, None, [("mul", 0.75), ("clip", -0.3, 0.3)], st, pd, g)
    whole, y = G.guarded(yshape, torch.float32)
    glowmi.conv2d_chainv(xd, wd, None, y, desc, [("mul", 0.75), ("clip", -0.3, 0.3)])
    torch.cuda.synchronize()
    G.assert_close_f32(y.cpu().numpy(), ref, f"shape {si} without bias")


def test_chainv_fixed_shapes_take_the_fixed_kernels(knobs):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    knobs.set("F32_PW_MIN_ITEMS", 1)          # the pointwise kernel at this small size
    layer = wl.ConvLayer("pw", 8, 28, 28, 64, 128, 1, 1, 1, 0)
    x, wt, b = wl.conv_inputs_f32(layer, 11100)
    t = wl.addend_f32(layer, 11100)
    desc = G.desc_of(layer)
    xd, wd, bd, td = G.dev(x), G.dev(wt), G.dev(b), G.dev(t)
    for ops, ref in (([], oracle.conv2d_f32(x, wt, b)),
                     ([("max", 0.0)], oracle.conv2d_f32(x, wt, b, act=wl.ACT_RELU)),
                     ([("add", td)], oracle.conv2d_f32_add(x, wt, b, t)),
                     ([("add", td), ("max", 0.0)], oracle.conv2d_f32_add(x, wt, b, t, act=wl.ACT_RELU))):
        y = G.poison((8, 28, 28, 128), torch.float32)
        glowmi.conv2d_chainv(xd, wd, bd, y, desc, ops, G.workspace(glowmi.conv2d_chainv_workspace_bytes(desc, ops)))
        torch.cuda.synchronize()
        assert not glowmi.last_variant().endswith("_chainv"), glowmi.last_variant()
        G.assert_close_f32(y.cpu().numpy(), ref, f"fixed shape {[o[0] for o in ops]} [{glowmi.last_variant()}]")
    assert glowmi.last_variant().startswith("conv_pw_f32"), glowmi.last_variant()


def _lists_i8(rng, yshape, span, sy):
    t1 = rng.integers(-128, 128, size=yshape, dtype=np.int8)
    t2 = rng.integers(-128, 128, size=yshape, dtype=np.int8)
    q1 = (float(np.float32(sy * 0.7)), 9)
    q2 = (float(np.float32(sy * 1.9)), -31)
    lo, hi = float(np.float32(-0.3 * span)), float(np.float32(0.45 * span))
    return [
        [("mul", 0.5)],
        [("mul", 1.37)],
        [("clip", lo, hi)],
        [("max", lo), ("add", t1) + q1],
        [("add", t1) + q1, ("clip", lo, hi)],
        [("mul", 4.0), ("add", t1) + q1, ("max", float(np.float32(0.1 * span)))],
        [("add", t1) + q1, ("mul", 0.5), ("add", t2) + q2, ("clip", lo, hi)],
        [("mul", 0.7321), ("max", 0.0), ("add", t2) + q2],
    ]


@pytest.mark.parametrize("si", range(len(SHAPES)))
@pytest.mark.parametrize("w_off", [0, -7])
def test_qconv2d_chainv(si, w_off):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    n, h, w, c, k, r, s, st, pd, g = SHAPES[si]
    layer = wl.ConvLayer(f"cv{si}", n, h, w, c, k, r, s, 1, 0, g)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 11200 + si, dist="normal", w_off=w_off)
    desc = G.make_desc(xq.shape, wq.shape, st, pd, g)
    oh, ow = glowmi.conv_out_shape(desc)
    yshape = (n, oh, ow, k)
    _, acc = oracle.qconv2d(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, st, pd, g,
                            return_acc=True)
    span = float(np.abs(acc).max()) * qp.x_scale * qp.w_scale
    rng = np.random.default_rng(11300 + si)
    xd, wd, bd = G.dev(xq), G.dev(wq), G.dev(bq)
    xp, wp, yp = G.qparams(qp)
    for li, ops in enumerate(_lists_i8(rng, yshape, span, qp.y_scale)):
        ref = oracle.qconv2d_chain(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, ops, qp.y_scale, qp.y_off,
                                   st, pd, g)
        dev_ops = [("add", G.dev(o[1]), glowmi.QParam(o[2], o[3])) if o[0] == "add" else o for o in ops]
        need = glowmi.qconv2d_chainv_workspace_bytes(desc, dev_ops)
        for use_ws in (True, False):
            whole, y = G.guarded(yshape, torch.int8)
            glowmi.qconv2d_chainv(xd, xp, wd, wp, bd, y, yp, desc, dev_ops, G.workspace(need) if use_ws else None)
            torch.cuda.synchronize()
            variant = glowmi.last_variant()
            assert G.guards_intact(whole, torch.int8), "write outside the output tensor"
            assert variant.endswith("_chainv"), variant
            G.assert_equal_i8(y.cpu().numpy(), ref, f"shape {si} list {li} w_off {w_off} ws {use_ws} [{variant}]")
        if li == 2:
            assert 0.02 < np.mean((ref > -128) & (ref < 127)), "almost everything saturates"
    # in place: the output buffer holds the added tensor
    ops = _lists_i8(rng, yshape, span, qp.y_scale)[4]
    ref = oracle.qconv2d_chain(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, ops, qp.y_scale, qp.y_off, st, pd, g)
    whole, y = G.guarded(yshape, torch.int8)
    y.copy_(torch.from_numpy(ops[0][1]))
    dev_ops = [("add", y, glowmi.QParam(ops[0][2], ops[0][3])), ops[1]]
    glowmi.qconv2d_chainv(xd, xp, wd, wp, bd, y, yp, desc, dev_ops, G.workspace(glowmi.qconv2d_chainv_workspace_bytes(desc, dev_ops)))
    torch.cuda.synchronize()
    G.assert_equal_i8(y.cpu().numpy(), ref, f"shape {si} in place [{glowmi.last_variant()}]")


def test_qchainv_fixed_shapes_take_the_fixed_kernels(knobs):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    knobs.set("I8_PW_MIN_ITEMS", 1)
    layer = wl.ConvLayer("pw", 8, 28, 28, 64, 128, 1, 1, 1, 0)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, 11400)
    rq, r_scale, r_off = wl.addend_q(layer, 11400, qp.y_scale)
    desc = G.desc_of(layer)
    xd, wd, bd, rd = G.dev(xq), G.dev(wq), G.dev(bq), G.dev(rq)
    xp, wp, yp = G.qparams(qp)
    add = ("add", rd, glowmi.QParam(r_scale, r_off))
    args = (xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq)
    for ops, ref in (([], oracle.qconv2d(*args, qp.y_scale, qp.y_off)),
                     ([("max", 0.0)], oracle.qconv2d(*args, qp.y_scale, qp.y_off, act=wl.ACT_RELU)),
                     ([add], oracle.qconv2d_add(*args, rq, r_scale, r_off, qp.y_scale, qp.y_off)),
                     ([add, ("max", 0.0)], oracle.qconv2d_add(*args, rq, r_scale, r_off, qp.y_scale, qp.y_off, act=wl.ACT_RELU))):
        y = G.poison((8, 28, 28, 128), torch.int8)
        glowmi.qconv2d_chainv(xd, xp, wd, wp, bd, y, yp, desc, ops, G.workspace(glowmi.qconv2d_chainv_workspace_bytes(desc, ops)))
        torch.cuda.synchronize()
        assert not glowmi.last_variant().endswith("_chainv"), glowmi.last_variant()
        G.assert_equal_i8(y.cpu().numpy(), ref, f"fixed shape {[o[0] for o in ops]} [{glowmi.last_variant()}]")
    assert glowmi.last_variant().startswith("conv_pw_i8"), glowmi.last_variant()
