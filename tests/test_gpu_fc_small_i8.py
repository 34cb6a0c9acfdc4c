"""The single-launch int8 FullyConnected kernel for at most 64 rows through the C ABI against the CPU
oracle, bit-exact: 1..64 rows on either side of the 32-row block, reductions shorter than one
wavefront's slice, not a multiple of it, and longer than one pass, column counts that are not
multiples of 16 or 32 (the last 16-byte run of the weight tensor is then fetched shifted), all four
combinations of zero / non-zero input and filter offsets, both requantize forms, no bias; and the
shapes just outside its range fall to the other kernels.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_1805_00907_amd import workloads as wl


def _gpu():
    import gpu_util
    return gpu_util


# M  K  N
SMALL_FC = [
    (1, 2048, 1000),      # the batch-1 classifier; last strip with 8 columns: the last run is fetched shifted by two dwords
    (64, 2048, 1000),     # two row blocks, N = 31 strips + 8 columns
    (1, 16, 4),           # the smallest the kernel takes: one 16-code run, one column group
    (5, 48, 36),          # reduction shorter than one step of 32, one strip + 4 columns
    (31, 272, 64),        # one wavefront's slice + 16
    (32, 2064, 100),      # eight slices + 16: the first wavefront's second pass holds 16 codes
    (33, 4096, 20),       # two passes, second row block with a single row
    (64, 8192, 44),       # four passes (the longest reduction the kernel takes)
    (17, 1024, 1004),     # last strip with 12 columns: the tensor's last 16-byte run is fetched shifted by one dword
    (2, 256, 1008),       # last strip with 16 columns: its second run lies wholly past the row (no straddle)
    (9, 512, 1012),       # last strip with 20 columns: second run straddles by three dwords
]


@pytest.mark.parametrize("shape", SMALL_FC, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dist,x_off,w_off", [("normal", None, 0), ("uniform", -7, 0), ("uniform", 0, 5), ("normal", 11, -3)])
def test_qfc_small(shape, dist, x_off, w_off):
    G = _gpu()
    M, K, N = shape
    layer = wl.FcLayer("small", M, K, N)
    aq, wq, bq, qp = wl.fc_inputs_q(layer, 9900 + M + K + N, dist=dist, w_off=w_off)
    if x_off is not None:
        qp = wl.QParams(qp.x_scale, x_off, qp.w_scale, qp.w_off, qp.y_scale, qp.y_off)
    for act in (wl.ACT_RELU, wl.ACT_NONE):
        ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=act)
        for use_ws in (True, False):
            got, variant = G.gpu_qfc(aq, wq, bq, qp, act, use_workspace=use_ws)
            assert variant.startswith("fc_small_i8"), variant
            G.assert_equal_i8(got, ref, f"small qfc {shape} {dist} x_off {x_off} w_off {w_off} act {act} [{variant}]")
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, None, qp.y_scale, qp.y_off, act=wl.ACT_NONE)
    got, _ = G.gpu_qfc(aq, wq, None, qp, wl.ACT_NONE)
    G.assert_equal_i8(got, ref, f"small qfc {shape} without bias")


@pytest.mark.parametrize("mr_exp", [-1, 1, -3, -8])
def test_qfc_small_multipliers(mr_exp):
    """Both requantize forms (64-bit for multipliers from 1/4 up, multiply-high below)."""
    G = _gpu()
    rng = np.random.default_rng(9990 + mr_exp)
    aq = rng.integers(-4, 5, size=(40, 192), dtype=np.int8)
    wf = rng.integers(-4, 5, size=(192, 52), dtype=np.int8)
    bf = rng.integers(-20, 20, size=(52,), dtype=np.int32)
    qp = wl.QParams(0.8, 1, float(2.0 ** mr_exp), 0, 1.0, -3)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wf, qp.w_scale, qp.w_off, bf, qp.y_scale, qp.y_off, act=wl.ACT_RELU)
    got, variant = G.gpu_qfc(aq, wf, bf, qp, wl.ACT_RELU)
    assert variant.startswith("fc_small_i8"), variant
    G.assert_equal_i8(got, ref, f"small qfc multiplier 0.8*2^{mr_exp}")


@pytest.mark.parametrize("shape", [(65, 2048, 1000), (8, 2040, 64), (8, 2048, 62), (4, 8208, 32)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qfc_just_outside_the_small_kernel(shape):
    """65 rows, a reduction that is no multiple of 16, a column count that is no multiple of 4, a
    reduction above 8192: other kernels, same results."""
    G = _gpu()
    M, K, N = shape
    layer = wl.FcLayer("outside", M, K, N)
    aq, wq, bq, qp = wl.fc_inputs_q(layer, 9995 + M + K + N, dist="uniform", w_off=2)
    ref = oracle.qfc(aq, qp.x_scale, qp.x_off, wq, qp.w_scale, qp.w_off, bq, qp.y_scale, qp.y_off, act=wl.ACT_RELU)
    got, variant = G.gpu_qfc(aq, wq, bq, qp, wl.ACT_RELU)
    assert not variant.startswith("fc_small_i8"), variant
    G.assert_equal_i8(got, ref, f"qfc {shape} [{variant}]")
