"""Helpers for the GPU parity tests: run the HIP path through the C ABI from numpy inputs.

torch is used only to hold device memory and to name the stream; every step of the computation is
done by libglowmi.so.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_1805_00907_amd as glowmi
from paper_1805_00907_amd.workloads import ConvLayer, FcLayer

DEV = "cuda:0"


def desc_of(layer: ConvLayer) -> glowmi.ConvDesc:
    return glowmi.ConvDesc(layer.n, layer.h, layer.w, layer.c, layer.k, layer.r, layer.s, layer.stride,
                           layer.stride, layer.pad, layer.pad, layer.pad, layer.pad, layer.groups)


def make_desc(x_shape, w_shape, stride, pads, groups) -> glowmi.ConvDesc:
    n, h, w, c = x_shape
    k, r, s, _ = w_shape
    return glowmi.ConvDesc(n, h, w, c, k, r, s, stride[0], stride[1], pads[0], pads[1], pads[2], pads[3], groups)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def workspace(nbytes: int):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV) if nbytes else None


def poison(shape, dtype, fill=77):
    """Output buffer pre-filled with a value no test expects (NaN for float, the code `fill` for
    int8), so unwritten elements are caught."""
    if dtype == torch.float32:
        return torch.full(shape, float("nan"), dtype=dtype, device=DEV)
    return torch.full(shape, fill, dtype=dtype, device=DEV)


GUARD = 4096   # elements of untouched poison kept on either side of a guarded output


def guarded(shape, dtype, fill=77):
    """A poisoned output inside a larger poisoned allocation: (whole buffer, view of the output)."""
    count = int(np.prod(shape))
    whole = poison((count + 2 * GUARD,), dtype, fill)
    return whole, whole[GUARD:GUARD + count].view(shape)


def guards_intact(whole, dtype, fill=77):
    lo, hi = whole[:GUARD], whole[-GUARD:]
    if dtype == torch.float32:
        return bool(torch.isnan(lo).all() and torch.isnan(hi).all())
    return bool((lo == fill).all() and (hi == fill).all())


def gpu_conv2d_f32(x, w, b, desc, act, use_workspace=True):
    oh, ow = glowmi.conv_out_shape(desc)
    xd, wd, bd = dev(x), dev(w), dev(b)
    whole, y = guarded((desc.n, oh, ow, desc.k), torch.float32)
    ws = workspace(glowmi.conv2d_workspace_bytes(desc)) if use_workspace else None
    glowmi.conv2d(xd, wd, bd, y, desc, act, ws)
    torch.cuda.synchronize()
    assert guards_intact(whole, torch.float32), "write outside the output tensor"
    return y.cpu().numpy(), glowmi.last_variant()


def gpu_conv2d_f32_chain(x, w, b, addend, desc, act, use_workspace=True, in_place=False):
    """conv + bias + addend + act through glowmi_conv2d_chain; in_place: the output buffer holds the addend."""
    oh, ow = glowmi.conv_out_shape(desc)
    xd, wd, bd = dev(x), dev(w), dev(b)
    whole, y = guarded((desc.n, oh, ow, desc.k), torch.float32)
    if in_place:
        y.copy_(torch.from_numpy(np.ascontiguousarray(addend)))
        ad = y
    else:
        ad = dev(addend)
    ws = workspace(glowmi.conv2d_workspace_bytes(desc)) if use_workspace else None
    glowmi.conv2d_chain(xd, wd, bd, y, desc, addend=ad, act=act, workspace=ws)
    torch.cuda.synchronize()
    assert guards_intact(whole, torch.float32), "write outside the output tensor"
    return y.cpu().numpy(), glowmi.last_variant()


def gpu_qconv2d_chain(xq, wq, bq, qp, addend_q, r_scale, r_off, desc, act, use_workspace=True, in_place=False,
                      fill=77):
    oh, ow = glowmi.conv_out_shape(desc)
    xd, wd, bd = dev(xq), dev(wq), dev(bq)
    whole, y = guarded((desc.n, oh, ow, desc.k), torch.int8, fill)
    if in_place:
        y.copy_(torch.from_numpy(np.ascontiguousarray(addend_q)))
        ad = y
    else:
        ad = dev(addend_q)
    ws = workspace(glowmi.qconv2d_workspace_bytes(desc)) if use_workspace else None
    xp, wp, yp = qparams(qp)
    glowmi.qconv2d_chain(xd, xp, wd, wp, bd, y, yp, desc, addend=ad, addend_q=glowmi.QParam(r_scale, r_off),
                         act=act, workspace=ws)
    torch.cuda.synchronize()
    assert guards_intact(whole, torch.int8, fill), "write outside the output tensor"
    return y.cpu().numpy(), glowmi.last_variant()


def gpu_fc_f32(a, w, b, act, use_workspace=True):
    M, K = a.shape
    N = w.shape[1]
    ad, wd, bd = dev(a), dev(w), dev(b)
    y = poison((M, N), torch.float32)
    ws = workspace(glowmi.fc_workspace_bytes(M, K, N)) if use_workspace else None
    glowmi.fc(ad, wd, bd, y, M, K, N, act, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy(), glowmi.last_variant()


def qparams(qp):
    return (glowmi.QParam(qp.x_scale, qp.x_off), glowmi.QParam(qp.w_scale, qp.w_off),
            glowmi.QParam(qp.y_scale, qp.y_off))


def gpu_qconv2d(xq, wq, bq, qp, desc, act, use_workspace=True, fill=77):
    oh, ow = glowmi.conv_out_shape(desc)
    xd, wd, bd = dev(xq), dev(wq), dev(bq)
    whole, y = guarded((desc.n, oh, ow, desc.k), torch.int8, fill)
    ws = workspace(glowmi.qconv2d_workspace_bytes(desc)) if use_workspace else None
    xp, wp, yp = qparams(qp)
    glowmi.qconv2d(xd, xp, wd, wp, bd, y, yp, desc, act, ws)
    torch.cuda.synchronize()
    assert guards_intact(whole, torch.int8, fill), "write outside the output tensor"
    return y.cpu().numpy(), glowmi.last_variant()


def gpu_qfc(aq, wq, bq, qp, act, use_workspace=True, fill=77):
    M, K = aq.shape
    N = wq.shape[1]
    ad, wd, bd = dev(aq), dev(wq), dev(bq)
    y = poison((M, N), torch.int8, fill)
    ws = workspace(glowmi.qfc_workspace_bytes(M, K, N)) if use_workspace else None
    xp, wp, yp = qparams(qp)
    glowmi.qfc(ad, xp, wd, wp, bd, y, yp, M, K, N, act, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy(), glowmi.last_variant()


RTOL, ATOL = 1e-4, 1e-5     # |gpu - oracle| <= ATOL + RTOL * |oracle|, element-wise


def assert_close_f32(got, ref, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite or unwritten outputs"
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    bad = err > bound
    if bad.any():
        i = np.argmax(err - bound)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst at flat {i}: "
                             f"gpu {got.flat[i]!r} oracle {ref.flat[i]!r}")
    return float((err / bound).max())


def assert_equal_i8(got, ref, what=""):
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape and got.dtype == np.int8, (what, got.shape, got.dtype)
    bad = got != ref
    if bad.any():
        i = int(np.flatnonzero(bad.reshape(-1))[0])
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} codes differ; first at flat {i}: "
                             f"gpu {got.flat[i]} oracle {ref.flat[i]}")
