"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, validates arguments before launching anything, and derives the same integer
requantization multiplier as the oracle's independent implementation."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1805_00907_amd as glowmi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000   # aligned, never dereferenced: validation fails before any launch


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "glowmi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(glowmi_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = glowmi.library()
    names = _declared_symbols()
    assert {"glowmi_conv2d", "glowmi_fc", "glowmi_qconv2d", "glowmi_qfc"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/glowmi.h but not exported"


def _desc(**kw):
    base = dict(n=1, h=8, w=8, c=4, k=4, r=3, s=3, stride_h=1, stride_w=1, pad_t=1, pad_l=1, pad_b=1, pad_r=1, groups=1)
    base.update(kw)
    return glowmi.ConvDesc(**base)


def test_out_shape_follows_the_paper_examples():
    d = glowmi.ConvDesc(8, 28, 28, 1, 16, 5, 5, 1, 1, 2, 2, 2, 2, 1)       # Section 3.5 listing
    assert glowmi.conv_out_shape(d) == (28, 28)
    d = glowmi.ConvDesc(8, 28, 28, 16, 16, 3, 3, 3, 3, 0, 0, 0, 0, 1)      # its pool geometry: floor
    assert glowmi.conv_out_shape(d) == (9, 9)


@pytest.mark.parametrize("kw,status", [
    (dict(n=0), 2), (dict(c=-1), 2), (dict(stride_h=0), 2), (dict(pad_l=-1), 2),
    (dict(groups=3), 2), (dict(groups=0), 2), (dict(r=11, pad_t=0, pad_b=0), 2),
    (dict(n=1 << 20, h=1 << 10, w=1 << 10), 3),
])
def test_conv_descriptor_errors(kw, status):
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.conv2d(FAKE, FAKE, None, FAKE, _desc(**kw), stream=0)
    assert e.value.status == status
    assert glowmi.library().glowmi_last_error()


def test_pointer_errors():
    d = _desc()
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.conv2d(None, FAKE, None, FAKE, d, stream=0)
    assert e.value.status == 1
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.conv2d(FAKE, FAKE + 4, None, FAKE, d, stream=0)
    assert e.value.status == 4
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.conv2d(FAKE, FAKE, FAKE + 2, FAKE, d, stream=0)
    assert e.value.status == 4
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.fc(FAKE, FAKE, None, None, 4, 4, 4, stream=0)
    assert e.value.status == 1
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.fc(FAKE, FAKE, None, FAKE, 4, 0, 4, stream=0)
    assert e.value.status == 2
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.conv2d(FAKE, FAKE, None, FAKE, d, act=7, stream=0)
    assert e.value.status == 3


def test_quant_errors():
    d = _desc()
    ok = glowmi.QParam(0.1, 0)
    for bad in (glowmi.QParam(0.0, 0), glowmi.QParam(-1.0, 0), glowmi.QParam(float("nan"), 0),
                glowmi.QParam(float("inf"), 0), glowmi.QParam(0.1, 128), glowmi.QParam(0.1, -129)):
        for pos in range(3):
            q = [ok, ok, ok]
            q[pos] = bad
            with pytest.raises(glowmi.GlowmiError) as e:
                glowmi.qconv2d(FAKE, q[0], FAKE, q[1], None, FAKE, q[2], d, stream=0)
            assert e.value.status == 5
    with pytest.raises(glowmi.GlowmiError) as e:     # multiplier far outside the representable range
        glowmi.qfc(FAKE, glowmi.QParam(1e30, 0), FAKE, glowmi.QParam(1e30, 0), None, FAKE, glowmi.QParam(1e-30, 0),
                   4, 4, 4, stream=0)
    assert e.value.status == 5
    with pytest.raises(glowmi.GlowmiError) as e:     # reduction too deep for an int32 accumulator
        glowmi.qfc(FAKE, ok, FAKE, ok, None, FAKE, ok, 4, 70000, 4, stream=0)
    assert e.value.status == 3


def test_accumulator_bound_counts_the_offsets():
    """|x - x_off| reaches 128 + |x_off| and |w - w_off| reaches 128 + |w_off| (Section 4.1: codes and offsets
    in [-128, 127]), so the depth an int32 accumulator can take depends on both offsets."""
    ok = glowmi.QParam(0.1, 0)

    def status(K, x_off, w_off):
        try:
            glowmi.qfc(FAKE, glowmi.QParam(0.1, x_off), FAKE, glowmi.QParam(0.1, w_off), None, FAKE, ok, 4, K, 4, stream=0)
        except glowmi.GlowmiError as e:
            return e.status, str(e)
        return 0, ""

    # symmetric filter, small activation offset: the deepest supported reduction is accepted (the call
    # then fails at the launch, there is no GPU behind the fake pointers, or succeeds in validation)
    assert status(65535, 20, 0)[0] in (0, 6)
    # extreme offsets: 255 * 255 * K must stay below 2^31 - 2^27
    limit = ((1 << 31) - (1 << 27)) // (255 * 255)
    assert status(limit, 127, 127)[0] in (0, 6)
    st, msg = status(limit + 1, 127, 127)
    assert st == 3 and "int32 accumulator" in msg
    st, msg = status(33026, -127, 127)              # the depth from which 255 * 255 * K can pass 2^31
    assert st == 3
    st, msg = status(40000, 0, -128)                # 128 * 256 * 40000 = 1.3e9: fine
    assert st in (0, 6)
    st, msg = status(65535, 127, 0)                 # 255 * 128 * 65535 = 2.139e9 > 2^31 - 2^27
    assert st == 3


def test_addend_multiplier_is_bounded():
    """A rescaled addend term must fit the accumulator: multipliers of 2^19 and above are rejected."""
    d = _desc()
    x, w = glowmi.QParam(2.0 ** -10, 0), glowmi.QParam(2.0 ** -10, 0)        # accumulator scale 2^-20
    y = glowmi.QParam(0.1, 0)
    for r_scale, want in ((2.0 ** -2, (0, 6)), (0.9, (5,))):                 # multipliers 2^18 and 0.9 * 2^20
        try:
            glowmi.qconv2d_chain(FAKE, x, FAKE, w, None, FAKE, y, d, addend=FAKE + (1 << 20),
                                 addend_q=glowmi.QParam(r_scale, 0), stream=0)
            st = 0
        except glowmi.GlowmiError as e:
            st = e.status
        assert st in want, (r_scale, st)


def test_tuning_knobs():
    glowmi.tuning_reset()
    base = glowmi.fc_workspace_bytes(64, 4096, 4096)
    glowmi.tuning_set("F32_TILE", 2)
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.tuning_set("NO_SUCH_KNOB", 1)
    assert e.value.status == 3
    # a forced split beyond what the slabs allow is clamped, and the workspace query follows the knob
    glowmi.tuning_set("F32_TILE", 0)
    glowmi.tuning_set("F32_SPLIT", 1000000)
    forced = glowmi.fc_workspace_bytes(64, 4096, 4096)
    assert forced > 0 and forced <= 256 * 64 * 4096 * 4
    glowmi.tuning_reset()
    assert glowmi.fc_workspace_bytes(64, 4096, 4096) == base


def test_fc_noalloc_rejects_what_its_scratch_cannot_hold():
    cap = glowmi.fc_noalloc_max_scratch_bytes()
    assert cap == 8 << 20
    M, K, N = 64, 25088, 4096
    assert glowmi.fc_workspace_bytes(M, K, N) > cap
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.fc_noalloc(FAKE, FAKE, None, FAKE, M, K, N, stream=0)
    assert e.value.status == 3 and "scratch" in str(e.value)
    with pytest.raises(glowmi.GlowmiError) as e:      # the usual validation comes first
        glowmi.fc_noalloc(FAKE, FAKE + 4, None, FAKE, 4, 4, 4, stream=0)
    assert e.value.status == 4


def test_binding_checks_tensors_before_the_call():
    """A tensor on the wrong device, of the wrong type, non-contiguous or too small never reaches the library."""
    import torch
    d = _desc()
    x = torch.zeros(1 * 8 * 8 * 4)
    with pytest.raises(ValueError, match="device tensor"):
        glowmi.conv2d(x, FAKE, None, FAKE, d, stream=0)


def test_requant_params_match_oracle():
    rng = np.random.default_rng(6)
    for _ in range(2000):
        sx, sw, sy = (float(np.float32(v)) for v in rng.uniform(0.001, 0.3, size=3))
        assert glowmi.requant_params(sx, sw, sy) == oracle.requant_params(sx, sw, sy)
    assert glowmi.requant_params(1.0 + 2.0 ** -17, 1.0 - 2.0 ** -17, 1.0) == (1 << 30, 30)   # carry case
    assert glowmi.requant_params(0.5, 0.5, 1.0) == (1 << 30, 32)


def test_rescale_params_match_oracle():
    rng = np.random.default_rng(7)
    for _ in range(2000):
        sr, sx, sw = (float(np.float32(v)) for v in rng.uniform(0.001, 0.3, size=3))
        assert glowmi.rescale_params(sr, sx, sw) == oracle.rescale_params(sr, sx, sw)
    assert glowmi.rescale_params(0.25, 0.5, 0.5) == (1 << 30, 30)
    with pytest.raises(glowmi.GlowmiError) as e:
        glowmi.rescale_params(1e30, 1e-30, 1e-30)
    assert e.value.status == 5


def test_chain_errors():
    d = _desc()
    ok = glowmi.QParam(0.1, 0)
    oh, ow = glowmi.conv_out_shape(d)
    y_bytes = d.n * oh * ow * d.k * 4
    with pytest.raises(glowmi.GlowmiError) as e:      # misaligned addend
        glowmi.conv2d_chain(FAKE, FAKE, None, FAKE, d, addend=FAKE + 4, stream=0)
    assert e.value.status == 4
    with pytest.raises(glowmi.GlowmiError) as e:      # overlaps the output without being it
        glowmi.conv2d_chain(FAKE, FAKE, None, FAKE + 4096, d, addend=FAKE + 4096 + 16, stream=0)
    assert e.value.status == 3 and y_bytes > 16
    with pytest.raises(glowmi.GlowmiError) as e:      # addend offset out of range
        glowmi.qconv2d_chain(FAKE, ok, FAKE, ok, None, FAKE, ok, d, addend=FAKE + (1 << 20),
                             addend_q=glowmi.QParam(0.1, 200), stream=0)
    assert e.value.status == 5
    with pytest.raises(glowmi.GlowmiError) as e:      # addend scale unusable
        glowmi.qconv2d_chain(FAKE, ok, FAKE, ok, None, FAKE, ok, d, addend=FAKE + (1 << 20),
                             addend_q=glowmi.QParam(0.0, 0), stream=0)
    assert e.value.status == 5
    import ctypes
    status = glowmi.library().glowmi_conv2d_chain(FAKE, FAKE, None, FAKE, ctypes.byref(d), None, None, 0, 0)
    assert status == 1                                # NULL chain


def test_chainv_errors():
    d = _desc()
    ok = glowmi.QParam(0.1, 0)
    far = FAKE + (1 << 20)

    def f32(ops):
        try:
            glowmi.conv2d_chainv(FAKE, FAKE, None, FAKE, d, ops, stream=0)
        except glowmi.GlowmiError as e:
            return e.status
        return 0

    def q(ops):
        try:
            glowmi.qconv2d_chainv(FAKE, ok, FAKE, ok, None, FAKE, ok, d, ops, stream=0)
        except glowmi.GlowmiError as e:
            return e.status
        return 0

    assert f32([("mul", 1.0)] * 5) == 3                           # too many ops
    assert f32([("mul", 2.0), ("add", None)]) == 1                # NULL tensor
    assert f32([("mul", 2.0), ("add", far + 4)]) == 4             # misaligned tensor
    assert f32([("mul", 2.0), ("add", FAKE + 16)]) == 3           # overlaps the output without being it
    assert f32([("clip", 1.0, -1.0)]) == 2
    assert f32([("mul", float("nan"))]) == 2
    assert q([("mul", 0.0)]) == 5 and q([("mul", -1.0)]) == 5 and q([("mul", float("inf"))]) == 5
    assert q([("clip", 1.0, -1.0)]) == 5
    assert q([("mul", 2.0), ("add", far, glowmi.QParam(0.0, 0))]) == 5
    assert q([("mul", 2.0), ("add", far, glowmi.QParam(0.1, 300))]) == 5
    assert q([("mul", 2.0), ("add", far, glowmi.QParam(1e9, 0))]) == 5       # multiplier far too large
    lib = glowmi.library()
    bad_kind = (glowmi.ChainOp * 1)(glowmi.ChainOp(9, 0.0, 0.0, None, ok))
    assert lib.glowmi_conv2d_chainv(FAKE, FAKE, None, FAKE, ctypes.byref(d), bad_kind, 1, None, 0, 0) == 3
    assert lib.glowmi_conv2d_chainv(FAKE, FAKE, None, FAKE, ctypes.byref(d), None, 2, None, 0, 0) == 1
    # workspace query follows the list: a fixed shape asks for what the fixed entry point asks
    big = glowmi.ConvDesc(1, 7, 7, 512, 512, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    assert glowmi.conv2d_chainv_workspace_bytes(big, [("max", 0.0)]) == glowmi.conv2d_workspace_bytes(big)
    assert glowmi.conv2d_chainv_workspace_bytes(big, [("mul", 2.0)]) > 0


def test_fold_batchnorm_matches_oracle():
    """Host-only entry point: runs without a GPU.  Same double arithmetic, so bit-identical."""
    rng = np.random.default_rng(8)
    for k, shape in ((5, (5, 3, 3, 4)), (64, (64, 7, 7, 3)), (1, (1, 1, 1, 9))):
        w = rng.standard_normal(size=shape).astype(np.float32)
        b = rng.standard_normal(size=k).astype(np.float32)
        gamma = rng.uniform(0.5, 1.5, size=k).astype(np.float32)
        beta, mean = (rng.standard_normal(size=k).astype(np.float32) for _ in range(2))
        var = rng.uniform(0.05, 3.0, size=k).astype(np.float32)
        for bias in (b, None):
            got_w, got_b = glowmi.fold_batchnorm(w, bias, gamma, beta, mean, var, 1e-5)
            ref_w, ref_b = oracle.fold_batchnorm(w, bias, gamma, beta, mean, var, 1e-5)
            np.testing.assert_array_equal(got_w, ref_w)
            np.testing.assert_array_equal(got_b, ref_b)
    with pytest.raises(glowmi.GlowmiError) as e:      # variance + eps not positive
        glowmi.fold_batchnorm(w, b, gamma, beta, mean, np.zeros(1, np.float32), 0.0)
    assert e.value.status == 2


def test_elementwise_errors():
    ok = glowmi.QParam(0.1, 0)
    lib = glowmi.library()
    assert lib.glowmi_quantize(None, FAKE, 16, ok, 0) == 1
    assert lib.glowmi_quantize(FAKE, FAKE + (1 << 20), 0, ok, 0) == 2
    assert lib.glowmi_quantize(FAKE, FAKE + 4, 16, ok, 0) == 4
    assert lib.glowmi_quantize(FAKE, FAKE + 32, 16, ok, 0) == 3                      # overlap
    assert lib.glowmi_dequantize(FAKE, FAKE + (1 << 20), 16, glowmi.QParam(0.0, 0), 0) == 5
    assert lib.glowmi_rescale(FAKE, ok, FAKE + 16, ok, 64, 0) == 3                   # partial overlap
    assert lib.glowmi_rescale(FAKE, ok, FAKE + (1 << 20), glowmi.QParam(0.1, 300), 64, 0) == 5


def test_sequence_planning_and_errors():
    """Arena planning is host code: two alternating activation regions + the largest workspace."""
    d1 = glowmi.ConvDesc(2, 8, 8, 16, 8, 1, 1, 1, 1, 0, 0, 0, 0, 1)      # -> 2x8x8x8
    d2 = glowmi.ConvDesc(2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, 1)       # -> 2x8x8x8
    d3 = glowmi.ConvDesc(2, 8, 8, 8, 16, 1, 1, 1, 1, 0, 0, 0, 0, 1)      # -> 2x8x8x16 (+ shortcut)
    arr = glowmi.seq_layers([(d1, FAKE, None, 1, False), (d2, FAKE, None, 1, False), (d3, FAKE, None, 1, True)])
    act_bytes = 2 * 8 * 8 * 8 * 4
    need = glowmi.seq_arena_bytes(arr, False)
    assert need >= 2 * act_bytes and need % 256 == 0
    assert glowmi.seq_arena_bytes(arr, True) >= 2 * (act_bytes // 4)
    lib = glowmi.library()
    assert lib.glowmi_seq_conv2d(FAKE, arr, 3, FAKE, FAKE, need - 256, 0) == 4          # arena too small
    bad = glowmi.seq_layers([(d1, FAKE, None, 1, False), (d3, FAKE, None, 1, False), (d2, FAKE, None, 1, False)])
    assert glowmi.seq_arena_bytes(bad, False) == 0
    assert lib.glowmi_seq_conv2d(FAKE, bad, 3, FAKE, FAKE, 1 << 20, 0) == 2             # shapes do not chain
    short = glowmi.seq_layers([(d1, FAKE, None, 1, True)])                              # shortcut shape mismatch
    assert lib.glowmi_seq_conv2d(FAKE, short, 1, FAKE, FAKE, 1 << 20, 0) == 2
    assert lib.glowmi_seq_conv2d(None, arr, 3, FAKE, FAKE, need, 0) == 1
    assert lib.glowmi_last_error()                                                      # planning errors leave a message
    # a bad layer in the middle is found before anything is launched: the status is the validation
    # error (5), not a launch failure on the fake pointers (6)
    okq, badq = glowmi.QParam(0.1, 0), glowmi.QParam(-1.0, 0)
    arrq = glowmi.seq_layers([(d1, FAKE, None, 1, False, okq, okq), (d2, FAKE, None, 1, False, badq, okq),
                              (d3, FAKE, None, 1, True, okq, okq)])
    needq = glowmi.seq_arena_bytes(arrq, True)
    assert lib.glowmi_seq_qconv2d(FAKE, okq, arrq, 3, FAKE, FAKE, needq, 0) == 5
    assert b"scale" in lib.glowmi_last_error()
    misaligned = glowmi.seq_layers([(d1, FAKE, None, 1, False), (d2, FAKE + 4, None, 1, False), (d3, FAKE, None, 1, True)])
    assert lib.glowmi_seq_conv2d(FAKE, misaligned, 3, FAKE, FAKE, need, 0) == 4


def test_workspace_queries_are_pure():
    assert glowmi.fc_workspace_bytes(16, 25088, 4096) > 0
    # the query plans with the operand sizes the call will see: a matrix too large for the single-launch
    # kernel gets the split-reduction workspace, a small one needs none
    assert glowmi.fc_workspace_bytes(16, 4096, 4096) > 0
    assert glowmi.fc_workspace_bytes(40, 2048, 1000) == 0
    assert glowmi.fc_workspace_bytes(0, 1, 1) == 0
    # a large contraction asks for room to repack both operands as two fp16 planes (4 bytes per element, each
    # operand's planes rounded up to 256 bytes, plus a 4 KB trailer: the largest magnitude and the partial maxima
    # it was taken from); with that kernel switched off, plenty of tiles: no split
    up = lambda v: (v + 255) // 256 * 256
    planes_of = lambda elems: up(4 * elems) + 4096
    big = glowmi.ConvDesc(16, 14, 14, 512, 512, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    x_elems, w_elems, y_elems = 16 * 14 * 14 * 512, 512 * 3 * 3 * 512, 16 * 14 * 14 * 512
    need = glowmi.conv2d_workspace_bytes(big)
    planes = planes_of(x_elems) + planes_of(w_elems)
    assert need >= planes and (need - planes) % (4 * y_elems) == 0    # + the partial sums of a split reduction
    glowmi.tuning_set("F32_P3", 0)
    try:
        assert glowmi.conv2d_workspace_bytes(big) % (4 * y_elems) == 0     # partial sums only
    finally:
        glowmi.tuning_reset()
    # 3x3 stride 1 on maps that tile into 16 x 16 blocks: only the filter is repacked
    vgg2 = glowmi.ConvDesc(16, 112, 112, 128, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    assert glowmi.conv2d_workspace_bytes(vgg2) == planes_of(128 * 3 * 3 * 128)
    # 3x3 over 64 channels on many pixels: only the filter is repacked
    c64 = glowmi.ConvDesc(16, 224, 224, 64, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    assert glowmi.conv2d_workspace_bytes(c64) == planes_of(64 * 3 * 3 * 64)
    # a FullyConnected too small to pay for the repacking never asks for it
    assert glowmi.fc_workspace_bytes(128, 4096, 4096) < 4 * (128 * 4096 + 4096 * 4096)


def test_packed_filter_queries_and_errors():
    """Filters transformed ahead of time: sizes, and every refusal happens before a launch."""
    up = lambda v: (v + 255) // 256 * 256
    planes_of = lambda elems: up(4 * elems) + 4096                    # two fp16 planes and the trailer
    vgg2 = glowmi.ConvDesc(16, 112, 112, 128, 128, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    assert glowmi.conv2d_filter_planes_bytes(vgg2) == planes_of(128 * 3 * 3 * 128)
    assert glowmi.conv2d_packed_workspace_bytes(vgg2) == 0            # the tile kernel needs nothing else
    big = glowmi.ConvDesc(32, 7, 7, 512, 512, 3, 3, 1, 1, 1, 1, 1, 1, 1)
    planes = glowmi.conv2d_filter_planes_bytes(big)
    assert planes == planes_of(512 * 3 * 3 * 512)
    assert glowmi.conv2d_packed_workspace_bytes(big) == glowmi.conv2d_workspace_bytes(big) - planes
    first = glowmi.ConvDesc(1, 224, 224, 3, 64, 7, 7, 2, 2, 3, 3, 3, 3, 1)       # 3 channels: no plane form
    assert glowmi.conv2d_filter_planes_bytes(first) == 0
    assert glowmi.conv2d_packed_workspace_bytes(first) == glowmi.conv2d_workspace_bytes(first)
    assert glowmi.conv2d_filter_planes_bytes(glowmi.ConvDesc(1, 4, 4, 8, 8, 5, 5, 1, 1, 0, 0, 0, 0, 1)) == 0   # bad desc
    assert glowmi.fc_filter_planes_bytes(4096, 1000) == planes_of(4096 * 1000)
    assert glowmi.fc_filter_planes_bytes(4100, 4096) == 0             # K not a multiple of 8
    assert glowmi.fc_filter_planes_bytes(0, 8) == 0
    # with the weights' planes given, a FullyConnected of 256 rows is worth the kernel over planes: room for the input's planes
    assert glowmi.fc_packed_workspace_bytes(256, 4096, 4096) >= planes_of(256 * 4096)
    assert glowmi.fc_packed_workspace_bytes(1024, 9216, 4096) == \
        glowmi.fc_workspace_bytes(1024, 9216, 4096) - glowmi.fc_filter_planes_bytes(9216, 4096)
    lib = glowmi.library()
    import ctypes
    chain = glowmi.Chain(None, glowmi.QParam(1.0, 0), 0)
    args = lambda d, planes_ptr, w=FAKE: (FAKE, w, planes_ptr, None, FAKE, ctypes.byref(d), ctypes.byref(chain), None, 0, 0)
    assert lib.glowmi_conv2d_packed(*args(first, FAKE)) == 3          # planes for a shape without a plane form
    assert "plane form" in lib.glowmi_last_error().decode()
    assert lib.glowmi_conv2d_packed(*args(vgg2, FAKE + 8)) == 4       # misaligned planes
    assert lib.glowmi_conv2d_packed(*args(vgg2, FAKE, FAKE + 4)) == 4  # the usual checks still apply
    assert lib.glowmi_conv2d_packed(FAKE, FAKE, FAKE, None, FAKE, ctypes.byref(vgg2), None, None, 0, 0) == 1   # chain NULL
    assert lib.glowmi_fc_packed(FAKE, FAKE, FAKE, None, FAKE, 64, 4100, 64, 0, None, 0, 0) == 3
    assert lib.glowmi_fc_packed(FAKE, FAKE, FAKE + 2, None, FAKE, 64, 4096, 64, 0, None, 0, 0) == 4
    assert lib.glowmi_conv2d_pack_filter(FAKE, ctypes.byref(first), FAKE, 1 << 20, 0) == 3
    assert lib.glowmi_conv2d_pack_filter(FAKE, ctypes.byref(vgg2), FAKE, planes_of(128 * 9 * 128) - 1, 0) == 2   # buffer too small
    assert lib.glowmi_conv2d_pack_filter(None, ctypes.byref(vgg2), FAKE, 1 << 30, 0) == 1
    assert lib.glowmi_conv2d_pack_filter(FAKE, ctypes.byref(vgg2), FAKE + 4, 1 << 30, 0) == 4
    assert lib.glowmi_fc_pack_filter(FAKE, 4100, 64, FAKE, 1 << 30, 0) == 3
    assert lib.glowmi_fc_pack_filter(FAKE, 4096, 64, FAKE, 100, 0) == 2
    assert lib.glowmi_fc_pack_filter(FAKE, 0, 64, FAKE, 100, 0) == 2


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1805_00907_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "glow_oracle" not in text, f
