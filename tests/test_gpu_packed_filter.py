"""Filters transformed ahead of time (glowmi_*_pack_filter + glowmi_*_packed) through the C ABI.

The planes themselves are checked against what they are defined to be: the tensor scaled by the power of two
that brings its largest magnitude below 2^15, every scaled weight cut into h1 = fp16(v) and
H2 = fp16((v - h1) * 2^11) (round to nearest even; below fp16's normal range H2 alone carries the value), a
convolution filter in its own order and a FullyConnected weight transposed, the largest magnitude's bits in the
trailer.  The *_packed calls are checked
against the CPU oracle element by element at |gpu - oracle| <= 1e-5 + 1e-4 |oracle| on each kernel that
reads planes (the contraction over planes, both 3x3 tile kernels), with and without a workspace, with the
tensor-add link, a split reduction and a ragged FullyConnected; and against the plain call on the same
kernel, whose result they must reproduce bit for bit.  A layer whose kernel reads no planes ignores them.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


def _planes_layout(elems):
    """(bytes of the two planes, offset of the trailer, total bytes)."""
    padded = (4 * elems + 255) // 256 * 256
    return 4 * elems, padded, padded + 4096


def _check_planes(host_bytes, w_in_plane_order):
    """host_bytes: the plane buffer; the weights in the order the planes keep them."""
    w = np.ascontiguousarray(w_in_plane_order)
    plane_bytes, trailer_at, total = _planes_layout(w.size)
    assert host_bytes.size == total
    planes = host_bytes[:plane_bytes].view(np.float16).reshape((2,) + w.shape)
    max_bits = int((w.view(np.uint32) & 0x7FFFFFFF).max())
    assert int(host_bytes[trailer_at:trailer_at + 4].view(np.uint32)[0]) == max_bits
    se = 141 - max((max_bits >> 23) & 0xFF, 1)
    v = np.ldexp(w, se).astype(np.float32)                      # exact: a power of two
    assert np.abs(v).max() < 2.0 ** 15
    h1 = v.astype(np.float16)
    h1[np.abs(v) < 2.0 ** -14] = 0
    r = v - h1.astype(np.float32)                               # exact in fp32
    h2 = (r * np.float32(2048)).astype(np.float16)
    assert np.array_equal(planes[0].view(np.uint16), h1.view(np.uint16))
    assert np.array_equal(planes[1].view(np.uint16), h2.view(np.uint16))
    # what the pieces stand for: within 2^-22 of the value (11 significant bits each, round to nearest); under fp16's
    # normal range (the second piece alone) within 2^-11 of it, or 2^-36 absolute once the second piece is subnormal too
    back = planes[0].astype(np.float64) + planes[1].astype(np.float64) / 2048.0
    v64 = np.abs(v.astype(np.float64))
    err = np.abs(back - v.astype(np.float64))
    rel = np.where(v64 < 2.0 ** -14, 2.0 ** -11, 2.0 ** -22)
    assert np.all(err <= np.maximum(rel * v64, 2.0 ** -36))


def test_conv_filter_planes_are_the_two_piece_cut():
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    rng = np.random.default_rng(36000)
    k, r, s, c = 72, 3, 3, 40
    w = (rng.standard_normal(size=(k, r, s, c)) * np.exp2(rng.integers(-20, 20, size=(k, r, s, c)))).astype(np.float32)
    w[::5, 1, 2, ::3] = 0.0
    w[1::7, 0, 0, 1::4] = np.exp2(rng.integers(-8, 8, size=w[1::7, 0, 0, 1::4].shape)).astype(np.float32)
    desc = glowmi.ConvDesc(1, 8, 8, c, k, r, s, 1, 1, 1, 1, 1, 1, 1)
    nbytes = glowmi.conv2d_filter_planes_bytes(desc)
    assert nbytes == _planes_layout(w.size)[2]
    buf = torch.full((nbytes + 512,), 0x5A, dtype=torch.uint8, device="cuda:0")
    glowmi.conv2d_pack_filter(G.dev(w), desc, buf[256:256 + nbytes])
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:256] == 0x5A).all() and (host[256 + nbytes:] == 0x5A).all(), "write outside the plane buffer"
    _check_planes(host[256:256 + nbytes], w)


@pytest.mark.parametrize("K,N", [(64, 32), (136, 200), (4104, 130), (8, 1000)])
def test_fc_filter_planes_are_the_transposed_cut(K, N):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    rng = np.random.default_rng(36100 + K + N)
    w = (rng.uniform(-1, 1, size=(K, N)) * np.exp2(rng.integers(-12, 12, size=(K, N)))).astype(np.float32)
    nbytes = glowmi.fc_filter_planes_bytes(K, N)
    buf = torch.full((nbytes + 512,), 0x5A, dtype=torch.uint8, device="cuda:0")
    glowmi.fc_pack_filter(G.dev(w), K, N, buf[256:256 + nbytes])
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:256] == 0x5A).all() and (host[256 + nbytes:] == 0x5A).all(), "write outside the plane buffer"
    _check_planes(host[256:256 + nbytes], np.ascontiguousarray(w.T))


def _conv_both_ways(x, wt, b, desc, act, addend=None, use_workspace=True):
    """(plain call's output and variant, packed call's output and variant) on fresh guarded outputs."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    oh, ow = glowmi.conv_out_shape(desc)
    xd, wd, bd, ad = G.dev(x), G.dev(wt), G.dev(b), G.dev(addend)
    planes = torch.empty(glowmi.conv2d_filter_planes_bytes(desc), dtype=torch.uint8, device="cuda:0")
    glowmi.conv2d_pack_filter(wd, desc, planes)
    out = []
    for packed in (False, True):
        whole, y = G.guarded((desc.n, oh, ow, desc.k), torch.float32)
        need = glowmi.conv2d_packed_workspace_bytes(desc) if packed else glowmi.conv2d_workspace_bytes(desc)
        ws = G.workspace(need) if use_workspace else None
        if packed:
            glowmi.conv2d_packed(xd, wd, planes, bd, y, desc, addend=ad, act=act, workspace=ws)
        else:
            glowmi.conv2d_chain(xd, wd, bd, y, desc, addend=ad, act=act, workspace=ws)
        torch.cuda.synchronize()
        assert G.guards_intact(whole, torch.float32), "write outside the output tensor"
        out.append((y.cpu().numpy(), glowmi.last_variant()))
    return out


def _conv_inputs(seed, n, h, w, c, k, r, s, groups=1):
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, size=(n, h, w, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(k, r, s, c // groups)) / np.sqrt(r * s * c // groups)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b


# n  h  w  c  k  r  s  stride  pad  groups  split
P3_SHAPES = [
    (2, 14, 14, 64, 128, 3, 3, 1, 1, 1, 0),
    (1, 19, 17, 32, 200, 3, 3, 1, 1, 1, 0),
    (2, 15, 15, 72, 136, 5, 5, 2, 2, 1, 3),     # split reduction + finishing kernel
    (1, 16, 16, 64, 192, 3, 3, 1, 1, 2, 0),     # two groups
    (3, 9, 11, 128, 72, 1, 1, 1, 0, 1, 0),      # pointwise
    (1, 7, 7, 512, 256, 3, 3, 1, 1, 1, 4),
]


@pytest.mark.parametrize("i", range(len(P3_SHAPES)))
def test_conv_packed_contraction_over_planes(i, knobs):
    G = _gpu()
    n, h, w, c, k, r, s, st, pd, g, split = P3_SHAPES[i]
    knobs.set("F32_P3_MIN_M", 1)
    knobs.set("F32_P3_RATIO", 0)
    knobs.set("F32_K3", 0)
    knobs.set("F32_K3C64", 0)
    if split:
        knobs.set("F32_SPLIT", split)
    x, wt, b = _conv_inputs(36200 + i, n, h, w, c, k, r, s, g)
    desc = G.make_desc(x.shape, wt.shape, (st, st), (pd, pd, pd, pd), g)
    ref = oracle.conv2d_f32(x, wt, b, (st, st), (pd, pd, pd, pd), g, act=wl.ACT_RELU)
    (plain, v_plain), (packed, v_packed) = _conv_both_ways(x, wt, b, desc, wl.ACT_RELU)
    assert v_plain.startswith("igemm_f32_p3") and v_packed == v_plain, (v_plain, v_packed)
    G.assert_close_f32(packed, ref, f"packed conv case {i} [{v_packed}]")
    assert np.array_equal(packed, plain), "the packed call must reproduce the plain call bit for bit"


# n  h  w  c  k
K3_SHAPES = [
    (2, 20, 37, 96, 128),      # 16 x 16 x 128 tiles, three chunks, ragged
    (1, 18, 18, 128, 200),
    (2, 21, 45, 96, 64),       # 16 x 32 x 64 tiles
    (9, 56, 56, 64, 128),      # 144 tiles
]


@pytest.mark.parametrize("i", range(len(K3_SHAPES)))
@pytest.mark.parametrize("use_workspace", [True, False])
def test_conv_packed_3x3_tile_kernel(i, use_workspace, knobs):
    G = _gpu()
    n, h, w, c, k = K3_SHAPES[i]
    knobs.set("F32_K3_ANY", 1)
    knobs.set("F32_K3C64", 0)
    x, wt, b = _conv_inputs(36300 + i, n, h, w, c, k, 3, 3)
    rng = np.random.default_rng(36350 + i)
    add = rng.uniform(-1, 1, size=(n, h, w, k)).astype(np.float32) if i % 2 else None
    desc = G.make_desc(x.shape, wt.shape, (1, 1), (1, 1, 1, 1), 1)
    if add is None:
        ref = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_RELU)
    else:
        ref = oracle.conv2d_f32_add(x, wt, b, add, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_RELU)
    (plain, v_plain), (packed, v_packed) = _conv_both_ways(x, wt, b, desc, wl.ACT_RELU, addend=add,
                                                           use_workspace=use_workspace)
    # with the planes given the tile kernel needs no workspace at all; the plain call without one cannot take it
    assert v_packed.startswith("conv_k3_f32_f16x3"), v_packed
    assert v_plain.startswith("conv_k3_f32_f16x3") == use_workspace, v_plain
    G.assert_close_f32(packed, ref, f"packed 3x3 case {i} [{v_packed}]")
    G.assert_close_f32(plain, ref, f"plain 3x3 case {i} [{v_plain}]")
    if use_workspace:
        assert v_packed == v_plain and np.array_equal(packed, plain)


@pytest.mark.parametrize("shape", [(2, 40, 40, 64), (3, 33, 50, 200), (1, 224, 224, 64)],
                         ids=lambda s: "x".join(map(str, s)))
def test_conv_packed_3x3_c64_kernel(shape, knobs):
    G = _gpu()
    n, h, w, k = shape
    knobs.set("F32_K3C64_MIN_TILES", 1)
    x, wt, b = _conv_inputs(36400 + h, n, h, w, 64, k, 3, 3)
    desc = G.make_desc(x.shape, wt.shape, (1, 1), (1, 1, 1, 1), 1)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_NONE)
    (plain, v_plain), (packed, v_packed) = _conv_both_ways(x, wt, b, desc, wl.ACT_NONE)
    assert v_packed.startswith("conv_k3c64_f32_f16x3") and v_packed == v_plain, (v_plain, v_packed)
    G.assert_close_f32(packed, ref, f"packed 3x3 c64 {shape} [{v_packed}]")
    assert np.array_equal(packed, plain)


def test_conv_packed_planes_are_ignored_by_kernels_that_read_none(knobs):
    """A pointwise layer and a tiny one take kernels that read the fp32 filter: the planes given may hold anything."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    for seed, (n, h, w, c, k, r) in enumerate([(2, 28, 28, 64, 256, 1), (1, 6, 6, 16, 24, 3)]):
        x, wt, b = _conv_inputs(36500 + seed, n, h, w, c, k, r, r)
        pd = r // 2
        desc = G.make_desc(x.shape, wt.shape, (1, 1), (pd, pd, pd, pd), 1)
        ref = oracle.conv2d_f32(x, wt, b, (1, 1), (pd, pd, pd, pd), 1, act=wl.ACT_RELU)
        garbage = torch.full((glowmi.conv2d_filter_planes_bytes(desc),), 0xFF, dtype=torch.uint8, device="cuda:0")
        y = G.poison(ref.shape, torch.float32)
        ws = G.workspace(glowmi.conv2d_packed_workspace_bytes(desc))
        glowmi.conv2d_packed(G.dev(x), G.dev(wt), garbage, G.dev(b), y, desc, act=wl.ACT_RELU, workspace=ws)
        torch.cuda.synchronize()
        variant = glowmi.last_variant()
        assert "f16x3" not in variant, variant
        assert not variant.startswith("igemm_f32_p3"), variant
        G.assert_close_f32(y.cpu().numpy(), ref, f"planes ignored [{variant}]")


FC_SHAPES = [(300, 512, 256), (129, 72, 200), (257, 1032, 65), (64, 40, 1000), (130, 4104, 130)]


@pytest.mark.parametrize("shape", FC_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("split", [0, 3])
def test_fc_packed(shape, split, knobs):
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    knobs.set("F32_P3_MIN_M", 1)
    knobs.set("F32_P3_RATIO", 0)
    if split:
        knobs.set("F32_SPLIT", split)
    M, K, N = shape
    a, w, b = wl.fc_inputs_f32(wl.FcLayer("packed", M, K, N), 36600 + M + K + N, dist="uniform_fan_in")
    ref = oracle.fc_f32(a, w, b, act=wl.ACT_RELU)
    ad, wd, bd = G.dev(a), G.dev(w), G.dev(b)
    planes = torch.empty(glowmi.fc_filter_planes_bytes(K, N), dtype=torch.uint8, device="cuda:0")
    glowmi.fc_pack_filter(wd, K, N, planes)
    y = G.poison((M, N), torch.float32)
    glowmi.fc_packed(ad, wd, planes, bd, y, M, K, N, wl.ACT_RELU, G.workspace(glowmi.fc_packed_workspace_bytes(M, K, N)))
    torch.cuda.synchronize()
    variant = glowmi.last_variant()
    assert variant.startswith("igemm_f32_p3"), variant
    got = y.cpu().numpy()
    G.assert_close_f32(got, ref, f"packed fc {shape} split {split} [{variant}]")
    plain, v_plain = G.gpu_fc_f32(a, w, b, wl.ACT_RELU)
    assert v_plain == variant and np.array_equal(got, plain)


def test_fc_packed_takes_the_plane_kernel_where_the_plain_call_does_not():
    """256 x 8192 x 512 with the default planner: 341 flops per operand element when the call has to cut 4 M weights
    as well, less than the kernel over planes needs to pay for the cutting, so the plain call stays on the fp32 matrix
    cores; with the planes given only the input is cut and the call moves."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    M, K, N = 256, 8192, 512
    a, w, b = wl.fc_inputs_f32(wl.FcLayer("packed", M, K, N), 36700, dist="uniform_fan_in")
    ref = oracle.fc_f32(a, w, b, act=wl.ACT_NONE)
    plain, v_plain = G.gpu_fc_f32(a, w, b, wl.ACT_NONE)
    assert not v_plain.startswith("igemm_f32_p3"), v_plain
    ad, wd, bd = G.dev(a), G.dev(w), G.dev(b)
    planes = torch.empty(glowmi.fc_filter_planes_bytes(K, N), dtype=torch.uint8, device="cuda:0")
    glowmi.fc_pack_filter(wd, K, N, planes)
    y = G.poison((M, N), torch.float32)
    glowmi.fc_packed(ad, wd, planes, bd, y, M, K, N, wl.ACT_NONE, G.workspace(glowmi.fc_packed_workspace_bytes(M, K, N)))
    torch.cuda.synchronize()
    assert glowmi.last_variant().startswith("igemm_f32_p3"), glowmi.last_variant()
    G.assert_close_f32(y.cpu().numpy(), ref, "packed fc 256x8192x512")
    G.assert_close_f32(plain, ref, "plain fc 256x8192x512")
    # without a workspace for the input's planes the packed call falls back like the plain one
    y2 = G.poison((M, N), torch.float32)
    glowmi.fc_packed(ad, wd, planes, bd, y2, M, K, N, wl.ACT_NONE, None)
    torch.cuda.synchronize()
    assert not glowmi.last_variant().startswith("igemm_f32_p3")
    G.assert_close_f32(y2.cpu().numpy(), ref, "packed fc without a workspace")


@pytest.mark.parametrize("kind", ["planes_split", "tile_kernel"])
def test_packed_calls_replay_from_a_hip_graph(kind, knobs):
    """The packed calls launch only kernels (cutting the input, the contraction, the finishing kernel of a split
    reduction): captured once, every replay - with the program's own eager work and synchronisation in between -
    must reproduce the eager result bit for bit."""
    import torch
    import paper_1805_00907_amd as glowmi
    G = _gpu()
    if kind == "planes_split":
        knobs.set("F32_P3_MIN_M", 1)
        knobs.set("F32_P3_RATIO", 0)
        knobs.set("F32_K3", 0)
        knobs.set("F32_SPLIT", 3)
        x, wt, b = _conv_inputs(36800, 2, 15, 15, 72, 136, 5, 5)
        st, pd, prefix = 2, 2, "igemm_f32_p3"
    else:
        knobs.set("F32_K3_ANY", 1)
        knobs.set("F32_K3C64", 0)
        x, wt, b = _conv_inputs(36801, 2, 28, 28, 96, 160, 3, 3)
        st, pd, prefix = 1, 1, "conv_k3_f32_f16x3"
    desc = G.make_desc(x.shape, wt.shape, (st, st), (pd, pd, pd, pd), 1)
    ref = oracle.conv2d_f32(x, wt, b, (st, st), (pd, pd, pd, pd), 1, act=wl.ACT_RELU)
    xd, wd, bd = G.dev(x), G.dev(wt), G.dev(b)
    planes = torch.empty(glowmi.conv2d_filter_planes_bytes(desc), dtype=torch.uint8, device="cuda:0")
    glowmi.conv2d_pack_filter(wd, desc, planes)
    ws = G.workspace(glowmi.conv2d_packed_workspace_bytes(desc))
    y = G.poison(ref.shape, torch.float32)
    glowmi.conv2d_packed(xd, wd, planes, bd, y, desc, act=wl.ACT_RELU, workspace=ws)
    torch.cuda.synchronize()
    assert glowmi.last_variant().startswith(prefix), glowmi.last_variant()
    eager = y.cpu().numpy()
    G.assert_close_f32(eager, ref, f"eager [{glowmi.last_variant()}]")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        glowmi.conv2d_packed(xd, wd, planes, bd, y, desc, act=wl.ACT_RELU, workspace=ws, stream=side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            glowmi.conv2d_packed(xd, wd, planes, bd, y, desc, act=wl.ACT_RELU, workspace=ws, stream=side)
    torch.cuda.synchronize()
    for rep in range(3):
        y.fill_(float("nan"))
        if ws is not None:
            ws.fill_(0x5A)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y.cpu().numpy(), eager, err_msg=f"graph replay {rep}")
        scratch = torch.empty(1 << 16, device="cuda:0").normal_()      # the program's own eager work
        float(scratch.sum())
