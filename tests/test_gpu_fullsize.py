"""Parity at the full sizes of the baseline configs, in the launch configuration bench.py times
(workspace supplied).  Convolutions are checked on sampled outputs the oracle computes one by one
(all border pixels of the first and last image plus 20000 random outputs); FC layers are compared
in full.  fp32: |gpu - oracle| <= 1e-5 + 1e-4 |oracle|.  int8: bit-exact.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


def _conv_f32_sampled(layer, seed):
    G = _gpu()
    x, w, b = wl.conv_inputs_f32(layer, seed)
    got, variant = G.gpu_conv2d_f32(x, w, b, G.desc_of(layer), layer.act)
    idx = wl.sample_output_indices(layer, seed)
    ref = oracle.conv2d_f32_points(x, w, b, idx, (layer.stride,) * 2, (layer.pad,) * 4, layer.groups, act=layer.act)
    assert np.all(np.isfinite(got)), f"{layer.name}: unwritten or non-finite outputs"
    G.assert_close_f32(got.reshape(-1)[idx], ref, f"{layer.name} [{variant}]")


@pytest.mark.parametrize("li", range(5))
def test_resnet50_fp32_batch32(li):
    _conv_f32_sampled(wl.resnet50_layers(32)[li], wl.layer_seed(1, 5 + li))


@pytest.mark.parametrize("li", range(5))
def test_vgg19_fp32_conv_batch16(li):
    _conv_f32_sampled(wl.vgg19_conv_layers(16)[li], wl.layer_seed(2, li))


@pytest.mark.parametrize("li", range(3))
def test_vgg19_fp32_fc(li):
    G = _gpu()
    layer = wl.vgg19_fc_layers(16)[li]
    a, w, b = wl.fc_inputs_f32(layer, wl.layer_seed(2, 5 + li))
    ref = oracle.fc_f32(a, w, b, act=layer.act)
    got, variant = G.gpu_fc_f32(a, w, b, layer.act)
    G.assert_close_f32(got, ref, f"{layer.name} [{variant}]")
    got, variant = G.gpu_fc_f32(a, w, b, layer.act, use_workspace=False)
    G.assert_close_f32(got, ref, f"{layer.name} without workspace [{variant}]")


@pytest.mark.parametrize("li", range(5))
@pytest.mark.parametrize("dist", ["normal", "uniform"])
def test_resnet50_int8_batch32(li, dist):
    G = _gpu()
    layer = wl.resnet50_layers(32)[li]
    seed = wl.layer_seed(3, li)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, seed, dist=dist)
    got, variant = G.gpu_qconv2d(xq, wq, bq, qp, G.desc_of(layer), layer.act)
    idx = wl.sample_output_indices(layer, seed)
    ref = oracle.qconv2d_points(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, idx,
                                (layer.stride,) * 2, (layer.pad,) * 4, layer.groups, act=layer.act)
    G.assert_equal_i8(got.reshape(-1)[idx], ref, f"{layer.name} {dist} [{variant}]")
    if dist == "normal":   # the recipe is meant to exercise the unsaturated range too
        assert 0.02 < np.mean((ref > -128) & (ref < 127)), "almost everything saturates"


@pytest.mark.parametrize("li", range(4))
def test_fc_sweep_fp32(li):
    G = _gpu()
    layer = wl.fc_sweep_layers()[li]
    a, w, b = wl.fc_inputs_f32(layer, wl.layer_seed(4, li), dist="uniform_fan_in")
    ref = oracle.fc_f32(a, w, b, act=layer.act)
    got, variant = G.gpu_fc_f32(a, w, b, layer.act)
    G.assert_close_f32(got, ref, f"{layer.name} [{variant}]")


def test_fc_fp32_unscaled_weights_backward_error():
    """Weights drawn U(-1,1) without the fan-in scaling make outputs of magnitude sqrt(K)/3 that
    cancel to near zero in places; no fp32-accumulating kernel can hold an absolute 1e-5 there.
    The bound that does hold for any sound fp32 contraction is componentwise in |A||W|:
    |gpu - exact| <= 1e-6 * sum_k |a_mk| |w_kn|  (the textbook bound is K * 2^-24 times that sum)."""
    G = _gpu()
    layer = wl.fc_sweep_layers()[2]          # (256, 4096, 4096)
    a, w, b = wl.fc_inputs_f32(layer, wl.layer_seed(4, 20), dist="uniform")
    ref = oracle.fc_f32(a, w, b, act=wl.ACT_NONE).astype(np.float64)
    got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_NONE)
    mag = np.abs(a).astype(np.float64) @ np.abs(w).astype(np.float64) + np.abs(b)
    err = np.abs(got.astype(np.float64) - ref)
    # the oracle itself rounds once to float32: allow that half ulp as well
    assert np.all(err <= 1e-6 * mag + 2.0 ** -24 * np.abs(ref)), f"[{variant}] max ratio {(err / mag).max():.3e}"


@pytest.mark.parametrize("li", range(4))
def test_fc_sweep_int8(li):
    G = _gpu()
    layer = wl.fc_sweep_layers()[li]
    aq, wq, bq, qp = wl.fc_inputs_q(layer, wl.layer_seed(4, 10 + li))
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=layer.act)
    got, variant = G.gpu_qfc(aq, wq, bq, qp, layer.act)
    G.assert_equal_i8(got, ref, f"{layer.name} [{variant}]")


@pytest.mark.parametrize("li", range(4))
def test_resnet50_block_tails_fp32(li):
    """1x1 expand convolution + residual add + Relu in one kernel, at batch 32."""
    G = _gpu()
    layer = wl.resnet50_block_tails(32)[li]
    seed = wl.layer_seed(5, li)
    x, w, b = wl.conv_inputs_f32(layer, seed)
    add = wl.addend_f32(layer, seed)
    got, variant = G.gpu_conv2d_f32_chain(x, w, b, add, G.desc_of(layer), layer.act)
    idx = wl.sample_output_indices(layer, seed)
    ref = oracle.conv2d_f32_add_points(x, w, b, add, idx, (1, 1), (0, 0, 0, 0), 1, act=layer.act)
    assert np.all(np.isfinite(got)), f"{layer.name}: unwritten or non-finite outputs"
    G.assert_close_f32(got.reshape(-1)[idx], ref, f"{layer.name} [{variant}]")
    assert 0.2 < np.mean(ref > 0) < 0.8        # the add and the Relu both matter on these inputs


@pytest.mark.parametrize("li", range(4))
def test_resnet50_block_tails_int8(li):
    G = _gpu()
    layer = wl.resnet50_block_tails(32)[li]
    seed = wl.layer_seed(5, li)
    xq, wq, bq, qp = wl.conv_inputs_q(layer, seed)
    rq, r_scale, r_off = wl.addend_q(layer, seed, qp.y_scale)
    got, variant = G.gpu_qconv2d_chain(xq, wq, bq, qp, rq, r_scale, r_off, G.desc_of(layer), layer.act)
    idx = wl.sample_output_indices(layer, seed)
    ref = oracle.qconv2d_add_points(xq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, rq, r_scale, r_off,
                                    qp.y_scale, qp.y_off, idx, (1, 1), (0, 0, 0, 0), 1, act=layer.act)
    G.assert_equal_i8(got.reshape(-1)[idx], ref, f"{layer.name} [{variant}]")
    assert 0.02 < np.mean((ref > -128) & (ref < 127)), "almost everything saturates"
