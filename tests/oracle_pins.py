"""Pins for the CPU oracle: checks against things the paper and the mathematics fix.

None of the expected values here is produced by the oracle.  They come from: the shape examples the
paper prints, hand-evaluated cases (tests/golden/), an explicit im2col matrix multiplied with numpy
in float64 (the equivalence the paper's Section 7 relies on when it contrasts im2col+GEMM with
direct convolution), closed forms, algebraic identities, and exact rational arithmetic.

Every pin is a plain function that raises AssertionError.  test_oracle_pins.py runs each of them
against the real oracle; test_oracle_mutants.py re-runs them against builds of the oracle with one
planted mistake each and requires a failure.
"""
from __future__ import annotations

import math
import os
from fractions import Fraction

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                out.append(line.split())
    return out


# ---------------------------------------------------------------------------------------------------
# independent reference: explicit im2col matrix + numpy float64 matmul
# ---------------------------------------------------------------------------------------------------

def im2col_matmul(x, w, bias, stride, pads, groups, pad_value=0.0):
    """Direct construction of the patch matrix, then one float64 matmul per group."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    n, h, wd, c = x.shape
    k, r, s, cg = w.shape
    sh, sw = stride
    pt, pl, pb, pr = pads
    xp = np.full((n, h + pt + pb, wd + pl + pr, c), pad_value, dtype=np.float64)
    xp[:, pt:pt + h, pl:pl + wd, :] = x
    oh = (h + pt + pb - r) // sh + 1
    ow = (wd + pl + pr - s) // sw + 1
    kg = k // groups
    y = np.zeros((n, oh, ow, k), dtype=np.float64)
    for g in range(groups):
        cols = np.empty((n, oh, ow, r, s, cg), dtype=np.float64)
        for i in range(oh):
            for j in range(ow):
                cols[:, i, j] = xp[:, i * sh:i * sh + r, j * sw:j * sw + s, g * cg:(g + 1) * cg]
        a = cols.reshape(n * oh * ow, r * s * cg)
        b = w[g * kg:(g + 1) * kg].reshape(kg, r * s * cg).T
        y[..., g * kg:(g + 1) * kg] = (a @ b).reshape(n, oh, ow, kg)
    if bias is not None:
        y += np.asarray(bias, dtype=np.float64)
    return y


TINY_SHAPES = [
    # n  h  w  c  k  r  s  stride   pads(t,l,b,r)  groups
    (1, 5, 5, 1, 1, 3, 3, (1, 1), (1, 1, 1, 1), 1),
    (2, 7, 6, 3, 4, 3, 2, (1, 1), (0, 0, 0, 0), 1),
    (2, 9, 8, 4, 6, 3, 3, (2, 2), (1, 1, 1, 1), 1),
    (1, 8, 11, 2, 3, 5, 3, (2, 1), (2, 0, 1, 2), 1),
    (3, 6, 6, 4, 6, 3, 3, (1, 2), (1, 2, 0, 1), 2),
    (1, 10, 10, 6, 9, 1, 1, (1, 1), (0, 0, 0, 0), 3),
    (2, 12, 12, 3, 5, 7, 7, (2, 2), (3, 3, 3, 3), 1),
    (1, 4, 4, 8, 8, 4, 4, (1, 1), (0, 0, 0, 0), 8),
]


def _rand(rng, shape):
    return rng.uniform(-1, 1, size=shape).astype(np.float32)


def pin_shape_examples():
    for in_, k, s, p, out in _rows("paper_shape_examples.txt"):
        assert oracle.out_dim(int(in_), int(k), int(s), int(p), int(p)) == int(out)
    # the listing's convolution end to end: 8x28x28x1 with 16x5x5x1, [5 1 2 16] -> 8x28x28x16
    x = np.zeros((8, 28, 28, 1), np.float32)
    w = np.zeros((16, 5, 5, 1), np.float32)
    y = oracle.conv2d_f32(x, w, np.zeros(16, np.float32), (1, 1), (2, 2, 2, 2))
    assert y.shape == (8, 28, 28, 16)
    assert oracle.out_dim(4, 5, 1, 0, 0) == 0          # kernel larger than the padded input
    assert oracle.out_dim(7, 3, 2, 0, 1) == 3          # floor((7+1-3)/2)+1


def pin_conv_vs_im2col():
    rng = np.random.default_rng(11)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES:
        x = _rand(rng, (n, h, w, c)); wt = _rand(rng, (k, r, s, c // g)); b = _rand(rng, (k,))
        ref = im2col_matmul(x, wt, b, st, pd, g)
        got = oracle.conv2d_f32(x, wt, b, st, pd, g)
        assert got.shape == ref.shape
        # the oracle rounds a float64 sum once to float32
        np.testing.assert_allclose(got.astype(np.float64), ref, rtol=1e-6, atol=1e-6)
        ref_relu = np.maximum(ref, 0.0)
        got_relu = oracle.conv2d_f32(x, wt, b, st, pd, g, act=oracle.ACT_RELU)
        np.testing.assert_allclose(got_relu.astype(np.float64), ref_relu, rtol=1e-6, atol=1e-6)
        # no bias
        got_nb = oracle.conv2d_f32(x, wt, None, st, pd, g)
        np.testing.assert_allclose(got_nb.astype(np.float64), im2col_matmul(x, wt, None, st, pd, g),
                                   rtol=1e-6, atol=1e-6)


def pin_conv_points_match_definition():
    rng = np.random.default_rng(12)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[2:5]:
        x = _rand(rng, (n, h, w, c)); wt = _rand(rng, (k, r, s, c // g)); b = _rand(rng, (k,))
        ref = np.maximum(im2col_matmul(x, wt, b, st, pd, g), 0.0).reshape(-1)
        idx = rng.permutation(ref.size)[: max(1, ref.size // 3)].astype(np.int64)
        got = oracle.conv2d_f32_points(x, wt, b, idx, st, pd, g, act=oracle.ACT_RELU)
        np.testing.assert_allclose(got.astype(np.float64), ref[idx], rtol=1e-6, atol=1e-6)


def pin_identity_and_delta_filters():
    rng = np.random.default_rng(13)
    x = _rand(rng, (2, 6, 7, 5))
    b = _rand(rng, (5,))
    # 1x1 identity filter: Y = X + b (exactly representable sums of two floats rounded once)
    eye = np.eye(5, dtype=np.float32).reshape(5, 1, 1, 5)
    y = oracle.conv2d_f32(x, eye, b)
    np.testing.assert_array_equal(y, (x.astype(np.float64) + b.astype(np.float64)).astype(np.float32))
    # centred delta 3x3 with pad 1: Y = X
    d = np.zeros((5, 3, 3, 5), np.float32)
    for ch in range(5):
        d[ch, 1, 1, ch] = 1.0
    np.testing.assert_array_equal(oracle.conv2d_f32(x, d, None, (1, 1), (1, 1, 1, 1)), x)
    # delta at filter position (r=0, s=2): Y[oh,ow] = X[oh-1, ow+1], zero outside -> no filter flip
    d = np.zeros((5, 3, 3, 5), np.float32)
    for ch in range(5):
        d[ch, 0, 2, ch] = 1.0
    y = oracle.conv2d_f32(x, d, None, (1, 1), (1, 1, 1, 1))
    exp = np.zeros_like(x)
    exp[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    np.testing.assert_array_equal(y, exp)
    # asymmetric hand example, one channel: x = [[1,2],[3,4]], w = [[10,20],[30,40]], no pad -> 300
    x2 = np.array([1, 2, 3, 4], np.float32).reshape(1, 2, 2, 1)
    w2 = np.array([10, 20, 30, 40], np.float32).reshape(1, 2, 2, 1)
    assert float(oracle.conv2d_f32(x2, w2)[0, 0, 0, 0]) == 1 * 10 + 2 * 20 + 3 * 30 + 4 * 40
    # filter index order [k][r][s][c]: r walks rows (H), s walks columns (W)
    x3 = np.arange(12, dtype=np.float32).reshape(1, 3, 4, 1)
    w3 = np.zeros((1, 2, 3, 1), np.float32); w3[0, 1, 2, 0] = 1.0
    y3 = oracle.conv2d_f32(x3, w3)
    np.testing.assert_array_equal(y3[0, :, :, 0], x3[0, 1:3, 2:4, 0])


def pin_linearity_in_filter():
    rng = np.random.default_rng(14)
    # small integers: every product and sum is exact in double, so linearity must hold exactly
    x = rng.integers(-8, 9, size=(2, 7, 7, 4)).astype(np.float32)
    w1 = rng.integers(-8, 9, size=(6, 3, 3, 2)).astype(np.float32)
    w2 = rng.integers(-8, 9, size=(6, 3, 3, 2)).astype(np.float32)
    args = dict(stride=(2, 1), pads=(1, 1, 1, 1), groups=2)
    y1 = oracle.conv2d_f32(x, w1, None, **args).astype(np.float64)
    y2 = oracle.conv2d_f32(x, w2, None, **args).astype(np.float64)
    y12 = oracle.conv2d_f32(x, 3 * w1 - 2 * w2, None, **args).astype(np.float64)
    np.testing.assert_array_equal(y12, 3 * y1 - 2 * y2)


def pin_all_ones_closed_form():
    n, h, w, c, k, r, s = 1, 6, 5, 3, 2, 3, 3
    x = np.ones((n, h, w, c), np.float32); wt = np.ones((k, r, s, c), np.float32)
    y = oracle.conv2d_f32(x, wt, None, (1, 1), (1, 1, 1, 1))
    rows = np.array([min(i + 1, h - 1) - max(i - 1, 0) + 1 for i in range(h)])
    cols = np.array([min(j + 1, w - 1) - max(j - 1, 0) + 1 for j in range(w)])
    exp = (rows[:, None] * cols[None, :] * c).astype(np.float32)
    for kk in range(k):
        np.testing.assert_array_equal(y[0, :, :, kk], exp)
    assert y[0, 0, 0, 0] == 4 * c and y[0, 2, 2, 0] == 9 * c and y[0, 0, 2, 1] == 6 * c


def pin_pointwise_is_matmul():
    rng = np.random.default_rng(15)
    x = _rand(rng, (2, 5, 4, 16)); wt = _rand(rng, (24, 1, 1, 16)); b = _rand(rng, (24,))
    ref = x.reshape(-1, 16).astype(np.float64) @ wt.reshape(24, 16).astype(np.float64).T + b
    np.testing.assert_allclose(oracle.conv2d_f32(x, wt, b).reshape(-1, 24), ref, rtol=1e-6, atol=1e-6)


def pin_fc():
    rng = np.random.default_rng(16)
    a = _rand(rng, (5, 37)); w = _rand(rng, (37, 11)); b = _rand(rng, (11,))
    ref = a.astype(np.float64) @ w.astype(np.float64) + b.astype(np.float64)
    np.testing.assert_allclose(oracle.fc_f32(a, w, b), ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(oracle.fc_f32(a, w, None), ref - b, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(oracle.fc_f32(a, w, b, act=oracle.ACT_RELU), np.maximum(ref, 0), rtol=1e-6,
                               atol=1e-6)
    # FC equals a 1x1 convolution on a 1x1 map with the filter being the transposed weight
    yc = oracle.conv2d_f32(a.reshape(5, 1, 1, 37), np.ascontiguousarray(w.T).reshape(11, 1, 1, 37), b)
    np.testing.assert_array_equal(yc.reshape(5, 11), oracle.fc_f32(a, w, b))
    # non-square operands with distinct integer entries catch a transposed operand exactly
    a2 = np.arange(6, dtype=np.float32).reshape(2, 3)
    w2 = np.arange(12, dtype=np.float32).reshape(3, 4) - 5
    np.testing.assert_array_equal(oracle.fc_f32(a2, w2, None), (a2.astype(np.float64) @ w2).astype(np.float32))


def pin_relu_sign_pattern():
    rng = np.random.default_rng(17)
    x = _rand(rng, (1, 6, 6, 3)); wt = _rand(rng, (4, 3, 3, 3)); b = _rand(rng, (4,))
    pre = im2col_matmul(x, wt, b, (1, 1), (1, 1, 1, 1), 1)
    y = oracle.conv2d_f32(x, wt, b, (1, 1), (1, 1, 1, 1), act=oracle.ACT_RELU)
    neg = pre < 0
    assert neg.any() and (~neg).any()
    assert np.all(y[neg] == 0.0) and not np.any(np.signbit(y[neg]))
    np.testing.assert_allclose(y[~neg], pre[~neg], rtol=1e-6, atol=1e-6)


def pin_dequantize_hand_cases():
    for scale, off, q, val in _rows("dequantize_hand_cases.txt"):
        got = oracle.dequantize(np.array([int(q)], np.int8), float(scale), int(off))[0]
        assert got == float(val), (scale, off, q, val, got)


def pin_quantize_round_trip():
    codes = np.arange(-128, 128).astype(np.int8)
    for scale, off in [(0.5, -3), (0.0123, 17), (0.1, -128), (0.07, 127), (3.0, 0)]:
        v = oracle.dequantize(codes, scale, off)
        np.testing.assert_array_equal(oracle.quantize(v, scale, off), codes)
    # saturation and ties-to-even of the helper
    q = oracle.quantize(np.array([1000.0, -1000.0, 0.25, 0.75, 1.25]), 0.5, 0)
    np.testing.assert_array_equal(q, np.array([127, -128, 0, 2, 2], np.int8))
    # a NaN takes the code of the real value zero (reading), infinities saturate
    q = oracle.quantize(np.array([float("nan"), float("inf"), float("-inf")]), 0.5, -7)
    np.testing.assert_array_equal(q, np.array([-7, 127, -128], np.int8))


def pin_int_accumulator_vs_real_domain():
    """Dequantize everything, convolve in float64 (im2col reference), divide by sx*sw: must equal
    the integer accumulator exactly (small integers times a power-of-two scale are exact)."""
    rng = np.random.default_rng(18)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[1:6]:
        xq = rng.integers(-128, 128, size=(n, h, w, c), dtype=np.int8)
        wq = rng.integers(-128, 128, size=(k, r, s, c // g), dtype=np.int8)
        bq = rng.integers(-5000, 5000, size=(k,), dtype=np.int32)
        sx, x_off, sw, w_off = 0.25, int(rng.integers(-20, 21)), 0.125, int(rng.integers(-5, 6))
        xr = (xq.astype(np.float64) - x_off) * sx
        wr = (wq.astype(np.float64) - w_off) * sw
        real = im2col_matmul(xr, wr, bq.astype(np.float64) * sx * sw, st, pd, g)   # zero padding, real domain
        acc_ref = real / (sx * sw)
        assert np.all(acc_ref == np.rint(acc_ref))
        _, acc = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, 1.0, 0, st, pd, g, return_acc=True)
        np.testing.assert_array_equal(acc.astype(np.float64), acc_ref)
    # FC
    aq = rng.integers(-128, 128, size=(4, 19), dtype=np.int8)
    wq = rng.integers(-128, 128, size=(19, 7), dtype=np.int8)
    bq = rng.integers(-5000, 5000, size=(7,), dtype=np.int32)
    _, acc = oracle.qfc(aq, 0.5, 3, wq, 0.25, -2, bq, 1.0, 0, return_acc=True)
    ref = (aq.astype(np.int64) - 3) @ (wq.astype(np.int64) + 2) + bq
    np.testing.assert_array_equal(acc, ref)


def _exact_requant(acc, mant, shift, y_off, lo):
    """Exact rational arithmetic: floor(acc*mant/2^shift + 1/2) + y_off, saturated."""
    q = math.floor(Fraction(acc * mant, 1 << shift) + Fraction(1, 2)) + y_off
    return max(lo, min(127, q))


def pin_requantize_hand_cases():
    for sx, sw, sy, acc, y_off, lo, exp in _rows("requantize_hand_cases.txt"):
        m, sh = oracle.requant_params(float(sx), float(sw), float(sy))
        got = oracle.requantize(int(acc), m, sh, int(y_off), int(lo))
        assert got == int(exp), (sx, sw, sy, acc, y_off, lo, exp, got)


def pin_requant_params():
    # powers of two: mantissa 2^30, shift = 30 + k   (Mr = 2^-k)
    for k in range(0, 20):
        m, sh = oracle.requant_params(2.0 ** -k, 1.0, 1.0)
        assert (m, sh) == (1 << 30, 30 + k), (k, m, sh)
    # general: m * 2^-sh within 2^-31 relative of the double product, m in [2^30, 2^31)
    rng = np.random.default_rng(19)
    for _ in range(2000):
        sx, sw, sy = (float(np.float32(v)) for v in rng.uniform(0.001, 0.2, size=3))
        m, sh = oracle.requant_params(sx, sw, sy)
        mr = Fraction(sx) * Fraction(sw) / Fraction(sy)
        assert (1 << 30) <= m < (1 << 31)
        assert abs(Fraction(m, 1 << sh) - mr) <= mr / (1 << 31)
    # just below a power of two, mantissa still representable: f = 1 - 2^-24, no carry
    below = float(np.nextafter(np.float32(0.5), np.float32(0)))   # 0.5 - 2^-25
    m, sh = oracle.requant_params(below, 1.0, 1.0)
    assert Fraction(m, 1 << sh) == Fraction(below), (m, sh)
    assert m == (1 << 31) - (1 << 7) and sh == 32, (m, sh)
    # carry case: (1 + 2^-17)(1 - 2^-17) = 1 - 2^-34 is exact in double; f * 2^31 = 2^31 - 1/8 rounds
    # to 2^31, which must be renormalised to 2^30 with the exponent bumped -> the same as Mr = 1
    m, sh = oracle.requant_params(1.0 + 2.0 ** -17, 1.0 - 2.0 ** -17, 1.0)
    assert (m, sh) == (1 << 30, 30), (m, sh)
    m, sh = oracle.requant_params(0.125 * (1.0 + 2.0 ** -17), 1.0 - 2.0 ** -17, 1.0)
    assert (m, sh) == (1 << 30, 33), (m, sh)
    for bad in [(0.0, 1.0, 1.0), (-1.0, 1.0, 1.0), (1.0, float("nan"), 1.0), (1.0, 1.0, float("inf")),
                (1e30, 1e30, 1e-30), (1e-30, 1e-30, 1e30)]:
        try:
            oracle.requant_params(*bad)
        except oracle.OracleError as e:
            assert e.code == oracle.BAD_QUANT
        else:
            raise AssertionError(f"accepted {bad}")


def pin_requantize_exact_rational():
    rng = np.random.default_rng(20)
    edge = [0, 1, -1, 2, -2, 2**31 - 1, -2**31, 2**30, -2**30]
    for _ in range(60):
        sx, sw, sy = (float(np.float32(v)) for v in rng.uniform(0.001, 0.3, size=3))
        m, sh = oracle.requant_params(sx, sw, sy)
        y_off = int(rng.integers(-128, 128))
        lo = int(rng.choice([-128, max(-128, y_off)]))
        accs = edge + [1 << (sh - 1 - 30) if sh > 31 else 1, -(1 << max(0, sh - 31))]
        accs += [int(v) for v in rng.integers(-2**31, 2**31, size=300)]
        accs += [int(v) for v in rng.integers(-40000, 40000, size=1300)]
        for a in accs:
            assert oracle.requantize(a, m, sh, y_off, lo) == _exact_requant(a, m, sh, y_off, lo), (a, m, sh)
    # exact ties with an odd power-of-two multiplier: acc = (2j+1) * 2^(k-1) -> j+1 (half up), both signs
    for k in (1, 3, 7):
        m, sh = oracle.requant_params(2.0 ** -k, 1.0, 1.0)
        for j in range(-40, 40):
            acc = (2 * j + 1) << (k - 1)
            assert oracle.requantize(acc, m, sh, 0, -128) == j + 1
            assert oracle.requantize(acc, m, sh, 0, -128) == math.floor((acc + (1 << (k - 1))) / (1 << k))


def pin_requantize_vs_real_formula():
    """Within one half code (plus the 2^-31 mantissa error) of the real-valued rule of Section 4.1,
    monotone in the accumulator, saturating at both rails."""
    rng = np.random.default_rng(21)
    for _ in range(40):
        sx, sw, sy = (float(np.float32(v)) for v in rng.uniform(0.002, 0.2, size=3))
        m, sh = oracle.requant_params(sx, sw, sy)
        mr = sx * sw / sy
        y_off = int(rng.integers(-20, 21))
        span = int(200 / mr)
        accs = np.sort(rng.integers(-span, span, size=400))
        prev = -129
        for a in accs:
            q = oracle.requantize(int(a), m, sh, y_off, -128)
            real = a * mr + y_off
            if -128 < real < 127:
                assert abs(q - real) <= 0.5 + 2.0 ** -30 * abs(a * mr) + 1e-9
            assert q >= prev
            prev = q
        assert oracle.requantize(2**31 - 1, m, sh, y_off, -128) == 127 or (2**31 - 1) * mr + y_off < 127.5
        assert oracle.requantize(10 * span, m, sh, y_off, -128) == 127
        assert oracle.requantize(-10 * span, m, sh, y_off, -128) == -128


def pin_quantized_relu():
    rng = np.random.default_rng(22)
    xq = rng.integers(-128, 128, size=(1, 6, 6, 4), dtype=np.int8)
    wq = rng.integers(-127, 128, size=(5, 3, 3, 4), dtype=np.int8)
    bq = rng.integers(-300, 300, size=(5,), dtype=np.int32)
    for y_off in (-128, -20, 0, 20, 127):
        args = (xq, 0.05, 3, wq, 0.01, 0, bq, 0.4, y_off, (1, 1), (1, 1, 1, 1), 1)
        plain = oracle.qconv2d(*args, act=oracle.ACT_NONE).astype(np.int32)
        relu = oracle.qconv2d(*args, act=oracle.ACT_RELU).astype(np.int32)
        # max on same-scale operands is a plain integer compare against the code of real zero
        np.testing.assert_array_equal(relu, np.maximum(plain, max(-128, y_off)))
        assert relu.min() >= max(-128, y_off)
        if y_off in (-20, 0, 20):
            assert (plain < y_off).any() and (plain > y_off).any()


def pin_zero_point_and_padding():
    """Input constantly equal to its offset is the real value 0 everywhere, padding included, so
    every output is requantize(bias)."""
    rng = np.random.default_rng(23)
    x_off, w_off = 7, -4
    xq = np.full((2, 5, 6, 3), x_off, np.int8)
    wq = rng.integers(-128, 128, size=(4, 3, 3, 3), dtype=np.int8)
    bq = np.array([100, -250, 0, 77], np.int32)
    sx, sw, sy, y_off = 0.5, 0.25, 1.0, -3          # multiplier 1/8
    y, acc = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, (1, 1), (1, 1, 1, 1), 1,
                            return_acc=True)
    exp = np.array([math.floor(b / 8 + 0.5) + y_off for b in bq])
    assert np.all(acc == bq.reshape(1, 1, 1, 4))
    assert np.all(y == exp.reshape(1, 1, 1, 4))
    # and a non-constant input: full pipeline against integer numpy + exact rational requantize
    xq = rng.integers(-128, 128, size=(2, 5, 6, 3), dtype=np.int8)
    sx, sw, sy = 0.043, 0.0071, 0.09
    m, sh = oracle.requant_params(sx, sw, sy)
    xr = xq.astype(np.float64) - x_off
    wr = wq.astype(np.float64) - w_off
    acc_ref = im2col_matmul(xr, wr, bq.astype(np.float64), (2, 1), (1, 0, 1, 2), 1).astype(np.int64)
    y = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, (2, 1), (1, 0, 1, 2), 1, act=oracle.ACT_RELU)
    exp = np.vectorize(lambda a: _exact_requant(int(a), m, sh, y_off, y_off))(acc_ref)
    np.testing.assert_array_equal(y.astype(np.int64), exp)
    idx = np.arange(0, y.size, 3, dtype=np.int64)
    pts = oracle.qconv2d_points(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, idx, (2, 1), (1, 0, 1, 2), 1,
                                act=oracle.ACT_RELU)
    np.testing.assert_array_equal(pts.astype(np.int64), exp.reshape(-1)[idx])


def pin_qfc_full():
    rng = np.random.default_rng(24)
    aq = rng.integers(-128, 128, size=(3, 50), dtype=np.int8)
    wq = rng.integers(-128, 128, size=(50, 9), dtype=np.int8)
    bq = rng.integers(-3000, 3000, size=(9,), dtype=np.int32)
    sa, a_off, sw, w_off, sy, y_off = 0.031, -11, 0.0093, 5, 0.27, 9
    m, sh = oracle.requant_params(sa, sw, sy)
    acc = (aq.astype(np.int64) - a_off) @ (wq.astype(np.int64) - w_off) + bq
    for act, lo in ((oracle.ACT_NONE, -128), (oracle.ACT_RELU, y_off)):
        exp = np.vectorize(lambda a: _exact_requant(int(a), m, sh, y_off, lo))(acc)
        got = oracle.qfc(aq, sa, a_off, wq, sw, w_off, bq, sy, y_off, act=act)
        np.testing.assert_array_equal(got.astype(np.int64), exp)


def pin_accumulator_overflow_is_reported():
    aq = np.full((1, 140000), 127, np.int8)
    wq = np.full((140000, 1), 127, np.int8)
    try:
        oracle.qfc(aq, 0.1, 0, wq, 0.1, 0, None, 1.0, 0)     # 140000 * 16129 > 2^31
    except oracle.OracleError as e:
        assert e.code == oracle.ACC_OVERFLOW
    else:
        raise AssertionError("overflow not reported")


# ---------------------------------------------------------------------------------------------------
# the element-wise chain with a tensor add (Section 5.2 stacking; fused Add + max of Section 5.3)
# ---------------------------------------------------------------------------------------------------

def pin_conv_add_f32():
    """act(conv + bias + addend) against the im2col reference plus the addend, in float64; the addend
    enters before the activation (cases where it flips the sign in both directions exist)."""
    rng = np.random.default_rng(31)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES:
        x = _rand(rng, (n, h, w, c)); wt = _rand(rng, (k, r, s, c // g)); b = _rand(rng, (k,))
        pre = im2col_matmul(x, wt, b, st, pd, g)
        add = (2.0 * _rand(rng, pre.shape)).astype(np.float32)
        ref = pre + add.astype(np.float64)
        got = oracle.conv2d_f32_add(x, wt, b, add, st, pd, g)
        np.testing.assert_allclose(got.astype(np.float64), ref, rtol=1e-6, atol=1e-6)
        got_relu = oracle.conv2d_f32_add(x, wt, b, add, st, pd, g, act=oracle.ACT_RELU)
        np.testing.assert_allclose(got_relu.astype(np.float64), np.maximum(ref, 0.0), rtol=1e-6, atol=1e-6)
        if pre.size > 50:
            assert ((pre < -1e-3) & (ref > 1e-3)).any() and ((pre > 1e-3) & (ref < -1e-3)).any()
        assert np.all(got_relu[ref < -1e-6] == 0.0)
        # without an addend it is the plain operator, bit for bit
        np.testing.assert_array_equal(oracle.conv2d_f32_add(x, wt, b, None, st, pd, g),
                                      oracle.conv2d_f32(x, wt, b, st, pd, g))
        idx = rng.permutation(ref.size)[: max(1, ref.size // 3)].astype(np.int64)
        pts = oracle.conv2d_f32_add_points(x, wt, b, add, idx, st, pd, g, act=oracle.ACT_RELU)
        np.testing.assert_allclose(pts.astype(np.float64), np.maximum(ref, 0.0).reshape(-1)[idx],
                                   rtol=1e-6, atol=1e-6)
    # closed form: 1x1 identity filter -> Y = X + b + addend
    x = _rand(rng, (2, 5, 4, 6)); b = _rand(rng, (6,)); add = _rand(rng, (2, 5, 4, 6))
    eye = np.eye(6, dtype=np.float32).reshape(6, 1, 1, 6)
    got = oracle.conv2d_f32_add(x, eye, b, add)
    np.testing.assert_allclose(got.astype(np.float64),
                               x.astype(np.float64) + b.astype(np.float64) + add.astype(np.float64),
                               rtol=1e-7, atol=1e-7)


def pin_rescale_node():
    """The stand-alone rescale: exact rationals for every code, identity on equal types, and the
    real-valued rule (same real value on the new scale) within one code."""
    rng = np.random.default_rng(34)
    codes = np.arange(-128, 128, dtype=np.int8)
    for _ in range(200):
        s_in, s_out = (float(np.float32(v)) for v in rng.uniform(0.01, 0.3, size=2))
        o_in, o_out = (int(v) for v in rng.integers(-128, 128, size=2))
        got = oracle.rescale(codes, s_in, o_in, s_out, o_out)
        m, sh = oracle.requant_params(s_in, 1.0, s_out)
        exp = np.array([_exact_requant(int(c) - o_in, m, sh, o_out, -128) for c in codes], dtype=np.int64)
        np.testing.assert_array_equal(got.astype(np.int64), exp)
        real = (codes.astype(np.float64) - o_in) * s_in / s_out + o_out
        inside = (real > -127) & (real < 126)
        assert np.all(np.abs(got.astype(np.float64) - real)[inside] <= 0.5 + 1e-6)
    np.testing.assert_array_equal(oracle.rescale(codes, 0.125, 7, 0.125, 7), codes)
    # halving the scale doubles the distance from the offset (until saturation)
    got = oracle.rescale(codes, 0.25, 0, 0.125, 0).astype(np.int64)
    np.testing.assert_array_equal(got, np.clip(2 * codes.astype(np.int64), -128, 127))
    # float tensors: quantize(dequantize(q)) == q through the float32 wrappers as well
    for scale, off in ((0.5, -3), (0.0123, 17)):
        np.testing.assert_array_equal(oracle.quantize_f32(oracle.dequantize_f32(codes, scale, off), scale, off), codes)
    assert oracle.dequantize_f32(np.array([-128, -3, 127], np.int8), 0.5, -3).tolist() == [-62.5, 0.0, 65.0]


def pin_fold_batchnorm():
    """Convolution with the folded filter equals batch normalization applied to the convolution,
    the latter written out from the definition on the float64 im2col reference."""
    rng = np.random.default_rng(35)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[1:6]:
        x = _rand(rng, (n, h, w, c)); wt = _rand(rng, (k, r, s, c // g)); b = _rand(rng, (k,))
        gamma = rng.uniform(0.5, 1.5, size=k).astype(np.float32); beta = _rand(rng, (k,))
        mean = _rand(rng, (k,)); var = rng.uniform(0.1, 2.0, size=k).astype(np.float32)
        eps = 1e-3
        conv = im2col_matmul(x, wt, b, st, pd, g)
        ref = gamma.astype(np.float64) * (conv - mean.astype(np.float64)) / np.sqrt(var.astype(np.float64) + eps) \
            + beta.astype(np.float64)
        wf, bf = oracle.fold_batchnorm(wt, b, gamma, beta, mean, var, eps)
        got = oracle.conv2d_f32(x, wf, bf, st, pd, g)
        np.testing.assert_allclose(got.astype(np.float64), ref, rtol=2e-5, atol=2e-5)
    # identity statistics leave the layer alone
    wf, bf = oracle.fold_batchnorm(wt, b, np.ones(k), np.zeros(k), np.zeros(k), np.ones(k), 0.0)
    np.testing.assert_array_equal(wf, wt); np.testing.assert_array_equal(bf, b)
    # no bias: b' = -mean * scale + beta
    wf, bf = oracle.fold_batchnorm(wt, None, gamma, beta, mean, var, 0.0)
    np.testing.assert_allclose(bf, -mean / np.sqrt(var) * gamma + beta, rtol=1e-6, atol=1e-6)


def _exact_rescale(d, mant, shift):
    return math.floor(Fraction(d * mant, 1 << shift) + Fraction(1, 2))


def pin_rescale_params_and_term():
    # ratio 2^k: mantissa 2^30, shift 30 - k
    for k in range(-10, 12):
        m, sh = oracle.rescale_params(2.0 ** k, 1.0, 1.0)
        assert (m, sh) == (1 << 30, 30 - k), (k, m, sh)
        m, sh = oracle.rescale_params(1.0, 2.0 ** -k, 1.0)
        assert (m, sh) == (1 << 30, 30 - k), (k, m, sh)
    rng = np.random.default_rng(32)
    for _ in range(500):
        sr, sx, sw = (float(np.float32(v)) for v in rng.uniform(0.002, 0.3, size=3))
        m, sh = oracle.rescale_params(sr, sx, sw)
        ratio = Fraction(sr) / (Fraction(sx) * Fraction(sw))
        assert (1 << 30) <= m < (1 << 31)
        # the double product sx*sw is rounded once before the division: 2^-52 on top of the mantissa's 2^-31
        assert abs(Fraction(m, 1 << sh) - ratio) <= ratio / (1 << 30)
        for d in list(range(-255, 256, 7)) + [-255, -1, 0, 1, 255]:
            assert oracle.rescale_term(d, m, sh) == _exact_rescale(d, m, sh), (d, m, sh)
    # ratio 1: the term is the code difference itself; ratio 1/2: ties go up, both signs
    m, sh = oracle.rescale_params(0.25, 0.5, 0.5)
    assert [oracle.rescale_term(d, m, sh) for d in (-255, -3, 0, 4, 255)] == [-255, -3, 0, 4, 255]
    m, sh = oracle.rescale_params(0.125, 0.5, 0.5)
    assert [oracle.rescale_term(d, m, sh) for d in (-3, -2, -1, 0, 1, 2, 3)] == [-1, -1, 0, 0, 1, 1, 2]
    for bad in [(0.0, 1.0, 1.0), (1.0, -1.0, 1.0), (float("nan"), 1.0, 1.0), (1e30, 1e-30, 1e-30)]:
        try:
            oracle.rescale_params(*bad)
        except oracle.OracleError as e:
            assert e.code == oracle.BAD_QUANT
        else:
            raise AssertionError(f"accepted {bad}")


def pin_qconv_add():
    """Composition from parts pinned elsewhere: plain accumulator (integer/real-domain pin) + exact
    rational rescale of the addend, then the exact rational requantize; and the real-valued rule."""
    rng = np.random.default_rng(33)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[1:7]:
        xq = rng.integers(-128, 128, size=(n, h, w, c), dtype=np.int8)
        wq = rng.integers(-40, 41, size=(k, r, s, c // g), dtype=np.int8)
        bq = rng.integers(-3000, 3000, size=(k,), dtype=np.int32)
        sx, sw, sy, sr = (float(np.float32(v)) for v in (0.05, 0.01, 0.9 * r * s, rng.uniform(0.02, 0.2)))
        x_off, w_off, y_off, r_off = (int(v) for v in rng.integers(-20, 21, size=4))
        _, acc = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g, return_acc=True)
        rq = rng.integers(-128, 128, size=acc.shape, dtype=np.int8)
        m, sh = oracle.requant_params(sx, sw, sy)
        rm, rsh = oracle.rescale_params(sr, sx, sw)
        for act in (oracle.ACT_NONE, oracle.ACT_RELU):
            lo = max(-128, y_off) if act == oracle.ACT_RELU else -128
            got, acc_add = oracle.qconv2d_add(xq, sx, x_off, wq, sw, w_off, bq, rq, sr, r_off, sy, y_off,
                                              st, pd, g, act=act, return_acc=True)
            exp_acc = np.array([int(a) + _exact_rescale(int(q) - r_off, rm, rsh)
                                for a, q in zip(acc.reshape(-1), rq.reshape(-1))], dtype=np.int64)
            np.testing.assert_array_equal(acc_add.reshape(-1).astype(np.int64), exp_acc)
            exp = np.array([_exact_requant(int(a), m, sh, y_off, lo) for a in exp_acc], dtype=np.int64)
            np.testing.assert_array_equal(got.reshape(-1).astype(np.int64), exp)
            # real-valued rule of Section 4.1: (conv + addend) / sy + y_off, within one code
            real = (acc.astype(np.float64) * sx * sw + (rq.astype(np.float64) - r_off) * sr) / sy + y_off
            inside = (real > lo + 1) & (real < 126)
            assert inside.any()
            assert np.all(np.abs(got.astype(np.float64) - real)[inside] <= 1.0 + 1e-6)
            idx = rng.permutation(got.size)[: max(1, got.size // 3)].astype(np.int64)
            pts = oracle.qconv2d_add_points(xq, sx, x_off, wq, sw, w_off, bq, rq, sr, r_off, sy, y_off, idx,
                                            st, pd, g, act=act)
            np.testing.assert_array_equal(pts, got.reshape(-1)[idx])
        # an addend constantly at its offset is the real value 0: the plain operator
        same = oracle.qconv2d_add(xq, sx, x_off, wq, sw, w_off, bq, np.full(acc.shape, r_off, np.int8), sr,
                                  r_off, sy, y_off, st, pd, g)
        np.testing.assert_array_equal(same, oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g))



# ---------------------------------------------------------------------------------------------------
# general element-wise chains behind the contraction (Section 5.2: any run of data-parallel operators)
# ---------------------------------------------------------------------------------------------------

def _apply_chain_real(v, ops):
    """The op list on a float64 array, in order (add tensors are float64 arrays of v's shape)."""
    v = np.array(v, dtype=np.float64)
    for op in ops:
        if op[0] == "add":
            v = v + np.asarray(op[1], dtype=np.float64)
        elif op[0] == "mul":
            v = v * float(np.float32(op[1]))
        elif op[0] == "max":
            v = np.maximum(v, float(np.float32(op[1])))
        elif op[0] == "clip":
            v = np.minimum(np.maximum(v, float(np.float32(op[1]))), float(np.float32(op[2])))
    return v


def pin_conv_chain_f32():
    """chain(conv + bias) against the im2col reference with the same ops applied in numpy float64; the
    order of the ops matters and is respected; degenerate lists reduce to operators pinned above."""
    rng = np.random.default_rng(41)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[:7]:
        x = _rand(rng, (n, h, w, c)); wt = _rand(rng, (k, r, s, c // g)); b = _rand(rng, (k,))
        pre = im2col_matmul(x, wt, b, st, pd, g)
        t1 = (2.0 * _rand(rng, pre.shape)).astype(np.float32); t2 = _rand(rng, pre.shape)
        lists = [
            [],
            [("max", 0.0)],
            [("add", t1)],
            [("add", t1), ("max", 0.0)],
            [("max", 0.0), ("add", t1)],                                  # the other order: a different result
            [("mul", 0.37), ("add", t1), ("clip", -0.25, 0.6)],
            [("add", t1), ("mul", -1.5), ("add", t2), ("max", -0.1)],      # fp32 chains take any factor, two tensors
            [("clip", -0.5, 0.5), ("mul", 3.0), ("clip", -1.0, 1.25), ("add", t2)],
        ]
        outs = []
        for ops in lists:
            got = oracle.conv2d_f32_chain(x, wt, b, ops, st, pd, g).astype(np.float64)
            np.testing.assert_allclose(got, _apply_chain_real(pre, ops), rtol=1e-6, atol=1e-6, err_msg=str([o[0] for o in ops]))
            outs.append(got)
        if pre.size > 50:
            assert np.abs(outs[3] - outs[4]).max() > 0.1               # order is not ignored
        # special cases that reduce to the pinned plain operators, bit for bit
        np.testing.assert_array_equal(oracle.conv2d_f32_chain(x, wt, b, [], st, pd, g), oracle.conv2d_f32(x, wt, b, st, pd, g))
        np.testing.assert_array_equal(oracle.conv2d_f32_chain(x, wt, b, [("max", 0.0)], st, pd, g),
                                      oracle.conv2d_f32(x, wt, b, st, pd, g, act=oracle.ACT_RELU))
        np.testing.assert_array_equal(oracle.conv2d_f32_chain(x, wt, b, [("add", t1), ("max", 0.0)], st, pd, g),
                                      oracle.conv2d_f32_add(x, wt, b, t1, st, pd, g, act=oracle.ACT_RELU))
        # no bias
        got = oracle.conv2d_f32_chain(x, wt, None, [("mul", 2.0)], st, pd, g).astype(np.float64)
        np.testing.assert_allclose(got, 2.0 * im2col_matmul(x, wt, None, st, pd, g), rtol=1e-6, atol=1e-6)
    # closed forms: 1x1 identity filter, y = clip(2 * (x + b) + t, lo, hi); multiply by zero wipes the contraction
    x = _rand(rng, (2, 4, 3, 5)); b = _rand(rng, (5,)); t = _rand(rng, (2, 4, 3, 5))
    eye = np.eye(5, dtype=np.float32).reshape(5, 1, 1, 5)
    got = oracle.conv2d_f32_chain(x, eye, b, [("mul", 2.0), ("add", t), ("clip", -1.0, 1.5)])
    exp = np.clip(2.0 * (x.astype(np.float64) + b) + t, -1.0, 1.5)
    np.testing.assert_allclose(got.astype(np.float64), exp, rtol=1e-7, atol=1e-7)
    got = oracle.conv2d_f32_chain(x, eye, b, [("mul", 0.0), ("add", t)])
    np.testing.assert_array_equal(got, t)
    for bad in ([("clip", 1.0, -1.0)],):
        try:
            oracle.conv2d_f32_chain(x, eye, b, bad)
        except oracle.OracleError as e:
            assert e.code == oracle.BAD_SHAPE
        else:
            raise AssertionError("inverted clip bounds accepted")


def _exact_threshold(v, s):
    """floor(v / s + 1/2) in exact rationals (v a float32 value, s a double)."""
    return math.floor(Fraction(float(np.float32(v))) / Fraction(s) + Fraction(1, 2))


def pin_chain_threshold():
    # hand cases on a power-of-two grid: ties go up, both signs
    assert [oracle.chain_threshold(v, 0.125) for v in (0.3125, -0.3125, 0.25, -0.25, 0.0, 0.06, -0.07)] == \
        [3, -2, 2, -2, 0, 0, -1]
    assert oracle.chain_threshold(1e30, 1e-6) == 2**31 - 1 and oracle.chain_threshold(-1e30, 1e-6) == -2**31
    rng = np.random.default_rng(42)
    for _ in range(2000):
        v = float(np.float32(rng.uniform(-50, 50)))
        s = float(rng.uniform(1e-5, 0.3))
        exact = _exact_threshold(v, s)
        got = oracle.chain_threshold(v, s)
        # the double quotient is rounded once: it can differ from the exact rule only within 2^-40 of a tie
        frac = Fraction(v) / Fraction(s) + Fraction(1, 2)
        near_tie = abs(frac - round(frac)) < Fraction(1, 1 << 40)
        assert got == exact or near_tie, (v, s, got, exact)


def pin_qconv_chain():
    """The quantized chain composed from parts pinned elsewhere (plain accumulator; exact-rational
    rescale terms, thresholds and requantize), its special cases that are operators pinned above, and
    the real-valued rule within one code."""
    rng = np.random.default_rng(43)
    for (n, h, w, c, k, r, s, st, pd, g) in TINY_SHAPES[1:7]:
        xq = rng.integers(-128, 128, size=(n, h, w, c), dtype=np.int8)
        wq = rng.integers(-40, 41, size=(k, r, s, c // g), dtype=np.int8)
        bq = rng.integers(-3000, 3000, size=(k,), dtype=np.int32)
        sx, sw, sy = (float(np.float32(v)) for v in (0.05, 0.01, 0.9 * r * s))
        sr, sr2 = (float(np.float32(v)) for v in rng.uniform(0.02, 0.2, size=2))
        x_off, w_off, y_off, r_off, r2_off = (int(v) for v in rng.integers(-20, 21, size=5))
        _, acc = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g, return_acc=True)
        rq = rng.integers(-128, 128, size=acc.shape, dtype=np.int8)
        rq2 = rng.integers(-128, 128, size=acc.shape, dtype=np.int8)
        s0 = float(np.float64(sx) * np.float64(sw))          # the accumulator's scale, formed in double
        real0 = acc.astype(np.float64) * sx * sw
        span = float(np.abs(real0).max())

        # ---- special cases: operators pinned above, bit for bit
        np.testing.assert_array_equal(oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, [], sy, y_off, st, pd, g),
                                      oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g))
        np.testing.assert_array_equal(
            oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, [("max", 0.0)], sy, y_off, st, pd, g),
            oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g, act=oracle.ACT_RELU))
        for tail, act in (([], oracle.ACT_NONE), ([("max", 0.0)], oracle.ACT_RELU)):
            np.testing.assert_array_equal(
                oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, [("add", rq, sr, r_off)] + tail, sy, y_off, st, pd, g),
                oracle.qconv2d_add(xq, sx, x_off, wq, sw, w_off, bq, rq, sr, r_off, sy, y_off, st, pd, g, act=act))
        # a multiply by 2^j is the same operator with the output scale divided by 2^j (exact in float)
        for j in (-2, 1, 3):
            np.testing.assert_array_equal(
                oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, [("mul", 2.0 ** j)], sy, y_off, st, pd, g),
                oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, float(np.float32(sy * 2.0 ** -j)), y_off, st, pd, g))

        # ---- general lists against exact rationals; multipliers with power-of-two factors are exact,
        # others are held to the tolerance of a 31-bit mantissa
        lo_v, hi_v = float(np.float32(-0.3 * span)), float(np.float32(0.45 * span))
        lists = [
            [("max", lo_v)],
            [("clip", lo_v, hi_v)],
            [("add", rq, sr, r_off), ("clip", lo_v, hi_v)],
            [("clip", lo_v, hi_v), ("add", rq, sr, r_off)],                               # the other order
            [("mul", 4.0), ("add", rq, sr, r_off), ("max", float(np.float32(0.1 * span)))],
            [("add", rq, sr, r_off), ("mul", 0.5), ("add", rq2, sr2, r2_off), ("clip", lo_v, hi_v)],
            [("mul", 0.7321), ("max", 0.0), ("add", rq2, sr2, r2_off)],
        ]
        m_plain, sh_plain = oracle.requant_params(sx, sw, sy)
        outs, accs = [], []
        for ops in lists:
            got, acc_after = oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, ops, sy, y_off, st, pd, g,
                                                  return_acc=True)
            outs.append(got)
            accs.append(acc_after)
            exp_acc = acc.astype(object).reshape(-1).copy()      # python ints
            s_cur, pow2, exact = s0, 0, True
            real = real0.copy().reshape(-1)
            for op in ops:
                if op[0] == "mul":
                    cval = float(np.float32(op[1]))
                    s_cur = float(np.float64(s_cur) * np.float64(cval))
                    real = real * cval
                    if cval in (0.5, 4.0):
                        pow2 += int(math.log2(cval))
                    else:
                        exact = False
                elif op[0] == "add":
                    t, ts, toff = op[1].reshape(-1), op[2], op[3]
                    real = real + (t.astype(np.float64) - toff) * ts
                    ratio = Fraction(ts) / Fraction(s_cur)
                    if exact:
                        rm, rsh = oracle.rescale_params(ts, sx, sw)   # pinned; a factor 2^pow2 only moves the shift
                        rsh += pow2
                        assert abs(Fraction(rm, 1 << rsh) - ratio) <= ratio / (1 << 30)
                        exp_acc = np.array([int(a) + _exact_rescale(int(q) - toff, rm, rsh) for a, q in zip(exp_acc, t)],
                                           dtype=object)
                    else:
                        exp_acc = None
                elif op[0] in ("max", "clip"):
                    bounds = [float(np.float32(b)) for b in op[1:]]
                    real = np.maximum(real, bounds[0])
                    if len(bounds) > 1:
                        real = np.minimum(real, bounds[1])
                    if exp_acc is not None:
                        ts_ = [_exact_threshold(b, s_cur) for b in bounds]
                        exp_acc = np.array([max(int(a), ts_[0]) for a in exp_acc], dtype=object)
                        if len(ts_) > 1:
                            exp_acc = np.array([min(int(a), ts_[1]) for a in exp_acc], dtype=object)
            if exp_acc is not None:
                np.testing.assert_array_equal(acc_after.reshape(-1).astype(object), exp_acc, err_msg=str([o[0] for o in ops]))
                if exact:      # final multiplier = the plain one times 2^pow2
                    exp = np.array([_exact_requant(int(a), m_plain, sh_plain - pow2, y_off, -128) for a in exp_acc],
                                   dtype=np.int64)
                    np.testing.assert_array_equal(got.reshape(-1).astype(np.int64), exp)
            # the real-valued rule of Section 4.1 on the chain evaluated in real numbers, within one code
            # (each rescaled tensor term is off by at most half an accumulator step, each bound likewise)
            realq = real / sy + y_off
            inside = (realq > -126) & (realq < 126)
            assert inside.any()
            assert np.all(np.abs(got.reshape(-1).astype(np.float64) - realq)[inside] <= 1.0 + 1e-6), [o[0] for o in ops]
        assert (accs[2] != accs[3]).any()                               # order is not ignored
        # a clipped result lies between the codes of its bounds and equals the unclipped one inside them
        plain = oracle.qconv2d(xq, sx, x_off, wq, sw, w_off, bq, sy, y_off, st, pd, g).astype(np.int64)
        clipped = outs[1].astype(np.int64)
        lo_c = _exact_requant(_exact_threshold(lo_v, s0), m_plain, sh_plain, y_off, -128)
        hi_c = _exact_requant(_exact_threshold(hi_v, s0), m_plain, sh_plain, y_off, -128)
        assert clipped.min() >= lo_c and clipped.max() <= hi_c and (clipped == lo_c).any() and (clipped == hi_c).any()
        inner = (plain > lo_c) & (plain < hi_c)
        np.testing.assert_array_equal(clipped[inner], plain[inner])
    for bad_ops, code in (([("mul", 0.0)], oracle.BAD_QUANT), ([("mul", -2.0)], oracle.BAD_QUANT),
                          ([("clip", 1.0, -1.0)], oracle.BAD_QUANT), ([("add", rq, 0.0, 0)], oracle.BAD_QUANT),
                          ([("add", rq, 0.1, 200)], oracle.BAD_QUANT)):
        try:
            oracle.qconv2d_chain(xq, sx, x_off, wq, sw, w_off, bq, bad_ops, sy, y_off, st, pd, g)
        except oracle.OracleError as e:
            assert e.code == code, (bad_ops[0][0], e.code)
        else:
            raise AssertionError(f"accepted {bad_ops[0][0]}")

ALL_PINS = [
    pin_shape_examples,
    pin_conv_vs_im2col,
    pin_conv_points_match_definition,
    pin_identity_and_delta_filters,
    pin_linearity_in_filter,
    pin_all_ones_closed_form,
    pin_pointwise_is_matmul,
    pin_fc,
    pin_relu_sign_pattern,
    pin_dequantize_hand_cases,
    pin_quantize_round_trip,
    pin_int_accumulator_vs_real_domain,
    pin_requantize_hand_cases,
    pin_requant_params,
    pin_requantize_exact_rational,
    pin_requantize_vs_real_formula,
    pin_quantized_relu,
    pin_zero_point_and_padding,
    pin_qfc_full,
    pin_accumulator_overflow_is_reported,
    pin_conv_add_f32,
    pin_rescale_params_and_term,
    pin_qconv_add,
    pin_conv_chain_f32,
    pin_chain_threshold,
    pin_qconv_chain,
    pin_rescale_node,
    pin_fold_batchnorm,
]
