"""What the fp32 kernels on the fp16 matrix cores promise about accuracy, through the C ABI, on each of the four
kernels that read planes (the contraction over planes, the fixed-tile, shaped-tile and 64-channel 3x3 kernels).

Every operand tensor (for the input of the 3x3 tile kernels: every patch a workgroup stages) is scaled by a power
of two taken from its own largest magnitude and cut into two fp16 pieces; a product is three piece products
accumulated in fp32.  From that follow, and are checked here:
  * scaling an operand by a power of two scales the result by it and changes nothing else: bit for bit, wherever
    the tensors sit in fp32's range (largest magnitudes from 2^-100 to 2^100);
  * componentwise fp32-level accuracy, |gpu - exact| <= 4 * 2^-22 * (|A||W| + |b|), for tensors whose elements
    spread over 24 binades;
  * elements more than 2^28 below their tensor's largest magnitude keep 11 significant bits, and the product of two
    such elements (one from each operand, below 2^-56 of the largest product) is dropped: the error all of this
    adds stays below 2^-38 of (largest |x|) * (largest |w|) * (reduction length);
  * all-zero operands, and an input whose largest element is an fp32 subnormal, give the bias;
  * an infinity or NaN in an operand makes the outputs it reaches non-finite and every other output right or NaN.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


KERNELS = ["planes", "k3_fixed", "k3_shaped", "k3c64"]


def _select(kind, knobs):
    """Knobs that route a small 3x3 layer to the kernel, the layer's (c, k), and the variant prefix expected."""
    if kind == "planes":
        knobs.set("F32_P3_MIN_M", 1)
        knobs.set("F32_P3_RATIO", 0)
        knobs.set("F32_K3", 0)
        knobs.set("F32_K3C64", 0)
        return 96, 136, "igemm_f32_p3"
    if kind == "k3c64":
        knobs.set("F32_K3C64_MIN_TILES", 1)
        return 64, 72, "conv_k3c64_f32_f16x3"
    knobs.set("F32_K3_ANY", 1)
    knobs.set("F32_K3C64", 0)
    knobs.set("F32_K3V", 1 if kind == "k3_shaped" else 0)
    return 96, 136, "conv_k3_f32_f16x3"


def _layer(kind, knobs, seed):
    c, k, prefix = _select(kind, knobs)
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, size=(2, 19, 21, c)).astype(np.float32)
    wt = (rng.standard_normal(size=(k, 3, 3, c)) / np.sqrt(9 * c)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(k,)).astype(np.float32)
    return x, wt, b, prefix


def _run(x, wt, b, prefix, act=None):
    G = _gpu()
    desc = G.make_desc(x.shape, wt.shape, (1, 1), (1, 1, 1, 1), 1)
    got, variant = G.gpu_conv2d_f32(x, wt, b, desc, wl.ACT_NONE if act is None else act)
    assert variant.startswith(prefix), variant
    return got


def _exact_and_scale(x, wt, b):
    """The oracle's result (the fp64 sum rounded once to fp32: within 2^-24 of the exact value) as float64, and the
    componentwise scale |A||W| + |b| (the oracle on the magnitudes)."""
    pd = (1, 1, 1, 1)
    exact = oracle.conv2d_f32(x, wt, b, (1, 1), pd, 1, act=wl.ACT_NONE).astype(np.float64)
    scale = oracle.conv2d_f32(np.abs(x), np.abs(wt), np.abs(b), (1, 1), pd, 1, act=wl.ACT_NONE).astype(np.float64)
    return exact, scale


@pytest.mark.parametrize("kind", KERNELS)
@pytest.mark.parametrize("ex,ew", [(80, -90), (-100, 40), (100, -90), (-50, -50), (13, 0)])
def test_power_of_two_scaling_changes_only_the_scale(kind, ex, ew, knobs):
    x, wt, b, prefix = _layer(kind, knobs, 37000)
    base = _run(x, wt, b, prefix)
    xs = np.ldexp(x, ex).astype(np.float32)
    ws = np.ldexp(wt, ew).astype(np.float32)
    bs = np.ldexp(b, ex + ew).astype(np.float32)
    assert np.array_equal(np.ldexp(xs, -ex), x) and np.array_equal(np.ldexp(ws, -ew), wt)   # nothing lost on the way
    got = _run(xs, ws, bs, prefix)
    assert np.all(np.isfinite(got))
    assert np.array_equal(np.ldexp(got.astype(np.float64), -(ex + ew)), base.astype(np.float64)), \
        np.abs(np.ldexp(got.astype(np.float64), -(ex + ew)) - base).max()


@pytest.mark.parametrize("kind", KERNELS)
def test_wide_value_range_is_held_to_fp32_accuracy(kind, knobs):
    """Magnitudes over 24 binades inside each tensor, exact powers of two and zeros among them."""
    x, wt, b, prefix = _layer(kind, knobs, 37100)
    rng = np.random.default_rng(37101)
    x = (x * np.exp2(rng.integers(-12, 12, size=x.shape))).astype(np.float32)
    wt = (wt * np.exp2(rng.integers(-12, 12, size=wt.shape))).astype(np.float32)
    x[:, ::3, ::5, ::7] = np.exp2(rng.integers(-10, 10, size=x[:, ::3, ::5, ::7].shape)).astype(np.float32)
    wt[::3, :, :, ::11] = 0.0
    got = _run(x, wt, b, prefix)
    exact, scale = _exact_and_scale(x, wt, b)
    err = np.abs(got.astype(np.float64) - exact)
    assert np.all(np.isfinite(got))
    worst = float((err / scale).max())
    assert worst <= 4 * 2.0 ** -22 + 2.0 ** -24, worst


@pytest.mark.parametrize("kind", KERNELS)
@pytest.mark.parametrize("where", ["input", "filter", "both"])
def test_elements_far_below_the_largest_keep_eleven_bits(kind, where, knobs):
    """One huge element in a tensor pushes the others more than 2^28 below the largest magnitude: they are carried
    by the second piece alone (11 bits).  With such elements in one operand the results keep about ten bits
    componentwise; with them in both operands their mutual products are dropped, and the error is bounded
    against the tensors' largest magnitudes only."""
    x, wt, b, prefix = _layer(kind, knobs, 37200)
    big_x, big_w = 2.0 ** 33, 2.0 ** 31
    if where in ("input", "both"):
        x[0, 0, 0, 0] = np.float32(big_x)
    if where in ("filter", "both"):
        wt[0, 0, 0, 0] = np.float32(big_w)
    got = _run(x, wt, b, prefix)
    exact, scale = _exact_and_scale(x, wt, b)
    kred = 9 * x.shape[3]
    bound = (4 * 2.0 ** -22 + 2.0 ** -24) * scale + 2.0 ** -38 * float(np.abs(x).max()) * float(np.abs(wt).max()) * kred
    err = np.abs(got.astype(np.float64) - exact)
    assert np.all(np.isfinite(got))
    assert np.all(err <= bound), float((err / bound).max())
    if where != "both":
        assert float((err / scale).max()) <= 2.0 ** -9


@pytest.mark.parametrize("kind", KERNELS)
def test_zero_and_subnormal_operands(kind, knobs):
    x, wt, b, prefix = _layer(kind, knobs, 37300)
    pd = (1, 1, 1, 1)
    zero_x = np.zeros_like(x)
    got = _run(zero_x, wt, b, prefix)
    assert np.array_equal(got, np.broadcast_to(b, got.shape))
    zero_w = np.zeros_like(wt)
    got = _run(x, zero_w, b, prefix)
    assert np.array_equal(got, np.broadcast_to(b, got.shape))
    tiny = (x * np.float32(2.0 ** -140)).astype(np.float32)          # every element an fp32 subnormal or zero
    got = _run(tiny, wt, b, prefix)
    ref = oracle.conv2d_f32(tiny, wt, b, (1, 1), pd, 1, act=wl.ACT_NONE)
    _gpu().assert_close_f32(got, ref, "subnormal input")


@pytest.mark.parametrize("kind", KERNELS)
@pytest.mark.parametrize("what", ["inf_in_input", "nan_in_filter"])
def test_a_non_finite_operand_never_gives_wrong_finite_values(kind, what, knobs):
    """No power of two scales a tensor (or a staged patch) that holds an infinity or a NaN.  Every output such an
    element reaches is non-finite, as in exact arithmetic; any other output is either right or NaN (all of them
    NaN where the scale is the whole tensor's), never a finite number that is wrong."""
    x, wt, b, prefix = _layer(kind, knobs, 37400)
    if what == "inf_in_input":
        x[1, 7, 9, 3] = np.inf
    else:
        wt[5, 1, 1, 2] = np.nan
    got = _run(x, wt, b, prefix)
    ref = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), 1, act=wl.ACT_NONE)
    reached = ~np.isfinite(ref)
    assert reached.any() and not reached.all()
    assert not np.isfinite(got[reached]).any()
    rest = ~reached & ~np.isnan(got)
    assert np.all(np.isfinite(got[rest]))
    assert np.all(np.abs(got[rest] - ref[rest]) <= 1e-5 + 1e-4 * np.abs(ref[rest]))
    if kind == "planes" or what == "nan_in_filter":
        assert np.all(np.isnan(got))                      # the scale of a whole tensor
