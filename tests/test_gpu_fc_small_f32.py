"""The single-launch fp32 FullyConnected kernel for few rows (reduction split over the wavefronts of a
workgroup, summed through LDS) through the C ABI against the CPU oracle, element by element:
every strip width, ragged K (not a multiple of the 16-row step), N not a multiple of the strip,
several row blocks with a ragged last one, with and without bias / Relu, bias at a 4-byte address.
|gpu - oracle| <= 1e-5 + 1e-4 |oracle|.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


SHAPES = [(1, 64, 16), (1, 2048, 1000), (16, 4096, 1000), (64, 2048, 1000), (3, 100, 7), (17, 260, 34),
          (5, 68, 130), (33, 1028, 196), (16, 4096, 4096), (2, 8192, 64), (64, 64, 64), (48, 516, 1001)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("vw", [0, 1, 2, 4])
def test_fc_small_f32(shape, vw, knobs):
    G = _gpu()
    M, K, N = shape
    if vw and N % vw:
        pytest.skip("strip width needs N to be a multiple of the vector width")
    if vw:
        knobs.set("F32_FC_SMALL_VW", vw)
    knobs.set("F32_FC_SMALL_MAX_KB", 1 << 20)        # take this kernel at any size (the planner stops at 8.5 MB)
    knobs.set("F32_FC_SMALL_MIN_M", 1)               # and for any number of rows (the planner starts at 17)
    layer = wl.FcLayer("fs", M, K, N)
    a, w, b = wl.fc_inputs_f32(layer, 12000 + M + K + N, dist="uniform_fan_in")
    for act, bias in ((wl.ACT_RELU, b), (wl.ACT_NONE, None)):
        ref = oracle.fc_f32(a, w, bias, act=act)
        got, variant = G.gpu_fc_f32(a, w, bias, act)
        assert variant.startswith("fc_small_f32"), variant
        if vw:
            assert variant.endswith(f"_w{16 * vw}"), variant
        G.assert_close_f32(got, ref, f"fc_small_f32 {shape} vw {vw} act {act} [{variant}]")


def test_fc_small_f32_bias_at_a_four_byte_address_and_output_guards():
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    M, K, N = 7, 520, 100
    layer = wl.FcLayer("fs", M, K, N)
    a, w, b = wl.fc_inputs_f32(layer, 12100, dist="uniform_fan_in")
    ad, wd = G.dev(a), G.dev(w)
    bpad = torch.zeros(N + 1, dtype=torch.float32, device="cuda:0")
    bpad[1:] = torch.from_numpy(b)
    bias = bpad[1:]                                   # 4 bytes past a 16-byte boundary
    assert bias.data_ptr() % 16 == 4
    glowmi.tuning_set("F32_FC_SMALL_MIN_M", 1)
    whole, y = G.guarded((M, N), torch.float32)
    glowmi.fc(ad, wd, bias, y, M, K, N, wl.ACT_RELU)
    torch.cuda.synchronize()
    assert glowmi.last_variant().startswith("fc_small_f32")
    glowmi.tuning_reset()
    assert G.guards_intact(whole, torch.float32), "write outside the output tensor"
    G.assert_close_f32(y.cpu().numpy(), oracle.fc_f32(a, w, b, act=wl.ACT_RELU), "bias at a 4-byte address")


def test_fc_small_f32_is_the_planners_choice_from_17_rows_and_can_be_switched_off(knobs):
    G = _gpu()
    layer = wl.FcLayer("fs", 40, 256, 64)
    a, w, b = wl.fc_inputs_f32(layer, 12200)
    got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_RELU)
    assert variant.startswith("fc_small_f32"), variant
    G.assert_close_f32(got, oracle.fc_f32(a, w, b, act=wl.ACT_RELU), f"[{variant}]")
    a16, w16, b16 = wl.fc_inputs_f32(wl.FcLayer("fs", 16, 256, 64), 12201)
    got, variant = G.gpu_fc_f32(a16, w16, b16, wl.ACT_RELU)
    assert variant == "fc_skinny16_f32", variant
    knobs.set("F32_FC_SMALL_OFF", 1)
    got, variant = G.gpu_fc_f32(a, w, b, wl.ACT_RELU)
    assert not variant.startswith("fc_small_f32"), variant
    G.assert_close_f32(got, oracle.fc_f32(a, w, b, act=wl.ACT_RELU), f"[{variant}]")
