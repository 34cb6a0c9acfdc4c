"""numpy front end of the CPU oracle (``glow_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's ``cpu_baseline`` leg use
it; the product package never imports it.  The wrappers only marshal numpy arrays into the C
functions; every piece of arithmetic lives in the C file, next to the citation of the passage of
the paper (arXiv 1805.00907) it follows.

Layouts (Section 3.5 listing; filter-layout figure of Section 5.2):
  x  [N][H][W][C]      w  [K][R][S][C/groups]      bias [K]      y  [N][OH][OW][K]
  FC (Section 3.4): a [M][K], w [K][N], bias [N], y [M][N].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "glow_oracle.c")
_SO = os.path.join(_HERE, "libgloworacle.so")

ACT_NONE = 0
ACT_RELU = 1

OK, BAD_SHAPE, BAD_QUANT, ACC_OVERFLOW = 0, 1, 2, 3

# kinds of a general chain's ops (Section 5.2: any run of data-parallel operators is stacked)
OP_ADD_TENSOR, OP_MUL_SCALAR, OP_MAX_SCALAR, OP_CLIP = 1, 2, 3, 4


class ChainOp(ctypes.Structure):
    """oracle_chain_op: kind; a, b scalars; tensor pointer; the tensor's scale/offset (quantized add)."""
    _fields_ = [("kind", ctypes.c_int32), ("a", ctypes.c_float), ("b", ctypes.c_float),
                ("tensor", ctypes.c_void_p), ("t_scale", ctypes.c_float), ("t_offset", ctypes.c_int32)]


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: oracle status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over the outer loops; no fast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def _bind(path: str) -> ctypes.CDLL:
    L = ctypes.CDLL(path)
    i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
    L.oracle_num_threads.restype = ctypes.c_int
    L.oracle_out_dim.restype = i64
    L.oracle_out_dim.argtypes = [i64] * 5
    L.oracle_conv2d_f32.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int]
    L.oracle_conv2d_f32_points.argtypes = [vp, vp, vp, vp, ctypes.c_int, vp, i64, vp]
    L.oracle_conv2d_f32_add.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int]
    L.oracle_conv2d_f32_add_points.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, vp, i64, vp]
    L.oracle_rescale.argtypes = [vp, i64, f32, i32, f32, i32, vp]
    L.oracle_rescale_params.argtypes = [f32, f32, f32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.oracle_rescale_term.argtypes = [i32, i32, i32]
    L.oracle_rescale_term.restype = i64
    L.oracle_qconv2d_add.argtypes = [vp, f32, i32, vp, f32, i32, vp, vp, f32, i32, vp, f32, i32, vp,
                                     ctypes.c_int, vp]
    L.oracle_qconv2d_add_points.argtypes = [vp, f32, i32, vp, f32, i32, vp, vp, f32, i32, f32, i32, vp,
                                            ctypes.c_int, vp, i64, vp]
    L.oracle_fc_f32.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.c_int]
    L.oracle_dequantize.argtypes = [vp, i64, f32, i32, vp]
    L.oracle_dequantize.restype = None
    L.oracle_quantize.argtypes = [vp, i64, f32, i32, vp]
    L.oracle_quantize.restype = None
    L.oracle_requant_params.argtypes = [f32, f32, f32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.oracle_requantize.argtypes = [i32] * 5
    L.oracle_requantize.restype = i32
    L.oracle_qconv2d.argtypes = [vp, f32, i32, vp, f32, i32, vp, vp, f32, i32, vp, ctypes.c_int, vp]
    L.oracle_qconv2d_points.argtypes = [vp, f32, i32, vp, f32, i32, vp, f32, i32, vp, ctypes.c_int,
                                        vp, i64, vp]
    L.oracle_qfc.argtypes = [vp, f32, i32, vp, f32, i32, vp, vp, f32, i32, i64, i64, i64,
                             ctypes.c_int, vp]
    cp = ctypes.POINTER(ChainOp)
    L.oracle_conv2d_f32_chain.argtypes = [vp, vp, vp, cp, i32, vp, vp]
    L.oracle_qconv2d_chain.argtypes = [vp, f32, i32, vp, f32, i32, vp, cp, i32, vp, f32, i32, vp, vp]
    L.oracle_chain_threshold.argtypes = [f32, ctypes.c_double]
    L.oracle_chain_threshold.restype = i32
    L.oracle_fold_batchnorm.argtypes = [vp] * 6 + [f32, i64, i64, vp, vp]
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_SO)
    return _lib


class use_library:
    """Context manager for the oracle's own mutation tests: route every wrapper through another
    build of the C file (one with a planted mistake) and restore the real one afterwards."""

    def __init__(self, path: str):
        self._path = path
        self._saved = None

    def __enter__(self):
        global _lib
        self._saved = lib()
        _lib = _bind(self._path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self._saved
        return False


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dtype, shape=None) -> np.ndarray:
    out = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(out.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(out.shape)}")
    return out


def out_dim(inp: int, kernel: int, stride: int, pad_lo: int, pad_hi: int) -> int:
    return int(lib().oracle_out_dim(inp, kernel, stride, pad_lo, pad_hi))


def _conv_params(x_shape, w_shape, stride, pads, groups) -> Tuple[np.ndarray, Tuple[int, ...]]:
    n, h, w_, c = (int(v) for v in x_shape)
    k, r, s, cg = (int(v) for v in w_shape)
    sh, sw = (int(v) for v in stride)
    pt, pl, pb, pr = (int(v) for v in pads)
    if groups <= 0 or c % groups or cg != c // groups:
        raise OracleError(BAD_SHAPE, "conv params")
    p = np.array([n, h, w_, c, k, r, s, sh, sw, pt, pl, pb, pr, groups], dtype=np.int64)
    oh = out_dim(h, r, sh, pt, pb)
    ow = out_dim(w_, s, sw, pl, pr)
    return p, (n, oh, ow, k)


def conv2d_f32(x, w, bias=None, stride=(1, 1), pads=(0, 0, 0, 0), groups=1, act=ACT_NONE) -> np.ndarray:
    x = _arr(x, np.float32); w = _arr(w, np.float32)
    p, yshape = _conv_params(x.shape, w.shape, stride, pads, groups)
    b = None if bias is None else _arr(bias, np.float32, (w.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "conv2d_f32")
    y = np.empty(yshape, dtype=np.float32)
    rc = lib().oracle_conv2d_f32(_ptr(x), _ptr(w), _ptr(b), _ptr(y), _ptr(p), act)
    if rc:
        raise OracleError(rc, "conv2d_f32")
    return y


def conv2d_f32_points(x, w, bias, flat_idx, stride=(1, 1), pads=(0, 0, 0, 0), groups=1,
                      act=ACT_NONE) -> np.ndarray:
    x = _arr(x, np.float32); w = _arr(w, np.float32)
    p, _ = _conv_params(x.shape, w.shape, stride, pads, groups)
    b = None if bias is None else _arr(bias, np.float32, (w.shape[0],))
    idx = _arr(flat_idx, np.int64)
    out = np.empty(idx.shape, dtype=np.float32)
    rc = lib().oracle_conv2d_f32_points(_ptr(x), _ptr(w), _ptr(b), _ptr(p), act, _ptr(idx), idx.size,
                                        _ptr(out))
    if rc:
        raise OracleError(rc, "conv2d_f32_points")
    return out


def conv2d_f32_add(x, w, bias, addend, stride=(1, 1), pads=(0, 0, 0, 0), groups=1, act=ACT_NONE) -> np.ndarray:
    """act(conv + bias + addend): the contraction with a tensor add stacked before the activation."""
    x = _arr(x, np.float32); w = _arr(w, np.float32)
    p, yshape = _conv_params(x.shape, w.shape, stride, pads, groups)
    b = None if bias is None else _arr(bias, np.float32, (w.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "conv2d_f32_add")
    r = None if addend is None else _arr(addend, np.float32, yshape)
    y = np.empty(yshape, dtype=np.float32)
    rc = lib().oracle_conv2d_f32_add(_ptr(x), _ptr(w), _ptr(b), _ptr(r), _ptr(y), _ptr(p), act)
    if rc:
        raise OracleError(rc, "conv2d_f32_add")
    return y


def conv2d_f32_add_points(x, w, bias, addend, flat_idx, stride=(1, 1), pads=(0, 0, 0, 0), groups=1,
                          act=ACT_NONE) -> np.ndarray:
    x = _arr(x, np.float32); w = _arr(w, np.float32)
    p, yshape = _conv_params(x.shape, w.shape, stride, pads, groups)
    b = None if bias is None else _arr(bias, np.float32, (w.shape[0],))
    r = None if addend is None else _arr(addend, np.float32, yshape)
    idx = _arr(flat_idx, np.int64)
    out = np.empty(idx.shape, dtype=np.float32)
    rc = lib().oracle_conv2d_f32_add_points(_ptr(x), _ptr(w), _ptr(b), _ptr(r), _ptr(p), act, _ptr(idx),
                                            idx.size, _ptr(out))
    if rc:
        raise OracleError(rc, "conv2d_f32_add_points")
    return out


def fc_f32(a, w, bias=None, act=ACT_NONE) -> np.ndarray:
    a = _arr(a, np.float32); w = _arr(w, np.float32)
    M, K = a.shape
    K2, N = w.shape
    if K != K2:
        raise OracleError(BAD_SHAPE, "fc_f32")
    b = None if bias is None else _arr(bias, np.float32, (N,))
    y = np.empty((M, N), dtype=np.float32)
    rc = lib().oracle_fc_f32(_ptr(a), _ptr(w), _ptr(b), _ptr(y), M, K, N, act)
    if rc:
        raise OracleError(rc, "fc_f32")
    return y


def dequantize(q, scale: float, offset: int) -> np.ndarray:
    q = _arr(q, np.int8)
    v = np.empty(q.shape, dtype=np.float64)
    lib().oracle_dequantize(_ptr(q), q.size, scale, offset, _ptr(v))
    return v


def quantize(value, scale: float, offset: int) -> np.ndarray:
    v = _arr(value, np.float64)
    q = np.empty(v.shape, dtype=np.int8)
    lib().oracle_quantize(_ptr(v), v.size, scale, offset, _ptr(q))
    return q


def requant_params(sx: float, sw: float, sy: float) -> Tuple[int, int]:
    m, sh = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().oracle_requant_params(sx, sw, sy, ctypes.byref(m), ctypes.byref(sh))
    if rc:
        raise OracleError(rc, "requant_params")
    return int(m.value), int(sh.value)


def requantize(acc: int, mant: int, shift: int, y_offset: int, lo: int = -128) -> int:
    return int(lib().oracle_requantize(int(acc), int(mant), int(shift), int(y_offset), int(lo)))


def quantize_f32(x, scale: float, offset: int) -> np.ndarray:
    """Codes of a float32 tensor: the float values are exact in double, then `quantize`."""
    return quantize(np.asarray(x, dtype=np.float32).astype(np.float64), scale, offset)


def dequantize_f32(q, scale: float, offset: int) -> np.ndarray:
    """Values of a quantized tensor rounded once to float32 ((q - offset) * scale is exact in double)."""
    return dequantize(q, scale, offset).astype(np.float32)


def rescale(q, s_in: float, in_offset: int, s_out: float, out_offset: int) -> np.ndarray:
    q = _arr(q, np.int8)
    out = np.empty(q.shape, dtype=np.int8)
    rc = lib().oracle_rescale(_ptr(q), q.size, s_in, in_offset, s_out, out_offset, _ptr(out))
    if rc:
        raise OracleError(rc, "rescale")
    return out


def rescale_params(sr: float, sx: float, sw: float) -> Tuple[int, int]:
    """(mant, shift) of the multiplier sr / (sx*sw) that brings an addend to the accumulator's scale."""
    m, s = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().oracle_rescale_params(sr, sx, sw, ctypes.byref(m), ctypes.byref(s))
    if rc:
        raise OracleError(rc, "rescale_params")
    return int(m.value), int(s.value)


def rescale_term(d: int, mant: int, shift: int) -> int:
    return int(lib().oracle_rescale_term(int(d), int(mant), int(shift)))


def qconv2d_add(xq, x_scale, x_off, wq, w_scale, w_off, bias_q, addend_q, r_scale, r_off, y_scale, y_off,
                stride=(1, 1), pads=(0, 0, 0, 0), groups=1, act=ACT_NONE, return_acc=False):
    xq = _arr(xq, np.int8); wq = _arr(wq, np.int8)
    p, yshape = _conv_params(xq.shape, wq.shape, stride, pads, groups)
    b = None if bias_q is None else _arr(bias_q, np.int32, (wq.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "qconv2d_add")
    r = None if addend_q is None else _arr(addend_q, np.int8, yshape)
    y = np.empty(yshape, dtype=np.int8)
    acc = np.empty(yshape, dtype=np.int32) if return_acc else None
    rc = lib().oracle_qconv2d_add(_ptr(xq), x_scale, x_off, _ptr(wq), w_scale, w_off, _ptr(b), _ptr(r),
                                  r_scale, r_off, _ptr(y), y_scale, y_off, _ptr(p), act, _ptr(acc))
    if rc:
        raise OracleError(rc, "qconv2d_add")
    return (y, acc) if return_acc else y


def qconv2d_add_points(xq, x_scale, x_off, wq, w_scale, w_off, bias_q, addend_q, r_scale, r_off, y_scale,
                       y_off, flat_idx, stride=(1, 1), pads=(0, 0, 0, 0), groups=1, act=ACT_NONE) -> np.ndarray:
    xq = _arr(xq, np.int8); wq = _arr(wq, np.int8)
    p, yshape = _conv_params(xq.shape, wq.shape, stride, pads, groups)
    b = None if bias_q is None else _arr(bias_q, np.int32, (wq.shape[0],))
    r = None if addend_q is None else _arr(addend_q, np.int8, yshape)
    idx = _arr(flat_idx, np.int64)
    out = np.empty(idx.shape, dtype=np.int8)
    rc = lib().oracle_qconv2d_add_points(_ptr(xq), x_scale, x_off, _ptr(wq), w_scale, w_off, _ptr(b),
                                         _ptr(r), r_scale, r_off, y_scale, y_off, _ptr(p), act, _ptr(idx),
                                         idx.size, _ptr(out))
    if rc:
        raise OracleError(rc, "qconv2d_add_points")
    return out


def qconv2d(xq, x_scale, x_off, wq, w_scale, w_off, bias_q, y_scale, y_off, stride=(1, 1),
            pads=(0, 0, 0, 0), groups=1, act=ACT_NONE, return_acc=False):
    xq = _arr(xq, np.int8); wq = _arr(wq, np.int8)
    p, yshape = _conv_params(xq.shape, wq.shape, stride, pads, groups)
    b = None if bias_q is None else _arr(bias_q, np.int32, (wq.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "qconv2d")
    y = np.empty(yshape, dtype=np.int8)
    acc = np.empty(yshape, dtype=np.int32) if return_acc else None
    rc = lib().oracle_qconv2d(_ptr(xq), x_scale, x_off, _ptr(wq), w_scale, w_off, _ptr(b), _ptr(y),
                              y_scale, y_off, _ptr(p), act, _ptr(acc))
    if rc:
        raise OracleError(rc, "qconv2d")
    return (y, acc) if return_acc else y


def qconv2d_points(xq, x_scale, x_off, wq, w_scale, w_off, bias_q, y_scale, y_off, flat_idx,
                   stride=(1, 1), pads=(0, 0, 0, 0), groups=1, act=ACT_NONE) -> np.ndarray:
    xq = _arr(xq, np.int8); wq = _arr(wq, np.int8)
    p, _ = _conv_params(xq.shape, wq.shape, stride, pads, groups)
    b = None if bias_q is None else _arr(bias_q, np.int32, (wq.shape[0],))
    idx = _arr(flat_idx, np.int64)
    out = np.empty(idx.shape, dtype=np.int8)
    rc = lib().oracle_qconv2d_points(_ptr(xq), x_scale, x_off, _ptr(wq), w_scale, w_off, _ptr(b),
                                     y_scale, y_off, _ptr(p), act, _ptr(idx), idx.size, _ptr(out))
    if rc:
        raise OracleError(rc, "qconv2d_points")
    return out


def qfc(aq, a_scale, a_off, wq, w_scale, w_off, bias_q, y_scale, y_off, act=ACT_NONE, return_acc=False):
    aq = _arr(aq, np.int8); wq = _arr(wq, np.int8)
    M, K = aq.shape
    K2, N = wq.shape
    if K != K2:
        raise OracleError(BAD_SHAPE, "qfc")
    b = None if bias_q is None else _arr(bias_q, np.int32, (N,))
    y = np.empty((M, N), dtype=np.int8)
    acc = np.empty((M, N), dtype=np.int32) if return_acc else None
    rc = lib().oracle_qfc(_ptr(aq), a_scale, a_off, _ptr(wq), w_scale, w_off, _ptr(b), _ptr(y), y_scale,
                          y_off, M, K, N, act, _ptr(acc))
    if rc:
        raise OracleError(rc, "qfc")
    return (y, acc) if return_acc else y


def fold_batchnorm(w, bias, gamma, beta, mean, var, eps: float):
    """Batch normalization merged into the preceding convolution (the paper does this before code
    generation, Section 5.3).  -> (w', b'), float32; the arithmetic is in the C file."""
    w = _arr(w, np.float32)
    k = w.shape[0]
    per = w.size // k
    g, bt, mu, vr = (_arr(np.asarray(a, dtype=np.float32).reshape(k), np.float32) for a in (gamma, beta, mean, var))
    b = None if bias is None else _arr(np.asarray(bias, dtype=np.float32).reshape(k), np.float32)
    w_out, b_out = np.empty_like(w), np.empty((k,), dtype=np.float32)
    rc = lib().oracle_fold_batchnorm(_ptr(w), _ptr(b), _ptr(g), _ptr(bt), _ptr(mu), _ptr(vr), eps, k, per,
                                     _ptr(w_out), _ptr(b_out))
    if rc:
        raise OracleError(rc, "fold_batchnorm")
    return w_out, b_out


def _chain_ops(ops, yshape, tensor_dtype):
    """ops: list of ("add", tensor[, scale, offset]) | ("mul", c) | ("max", v) | ("clip", lo, hi).
    -> (ctypes array, list of arrays kept alive)."""
    arr = (ChainOp * max(1, len(ops)))()
    keep = []
    for i, op in enumerate(ops):
        kind = op[0]
        if kind == "add":
            t = _arr(op[1], tensor_dtype, yshape)
            keep.append(t)
            scale, offset = (op[2], op[3]) if len(op) > 2 else (1.0, 0)
            arr[i] = ChainOp(OP_ADD_TENSOR, 0.0, 0.0, t.ctypes.data, scale, offset)
        elif kind == "mul":
            arr[i] = ChainOp(OP_MUL_SCALAR, op[1], 0.0, None, 1.0, 0)
        elif kind == "max":
            arr[i] = ChainOp(OP_MAX_SCALAR, op[1], 0.0, None, 1.0, 0)
        elif kind == "clip":
            arr[i] = ChainOp(OP_CLIP, op[1], op[2], None, 1.0, 0)
        else:
            raise ValueError(kind)
    return arr, keep


def conv2d_f32_chain(x, w, bias, ops, stride=(1, 1), pads=(0, 0, 0, 0), groups=1) -> np.ndarray:
    """chain(conv + bias): the ops applied in order to every output element (Section 5.2 stacking)."""
    x = _arr(x, np.float32); w = _arr(w, np.float32)
    p, yshape = _conv_params(x.shape, w.shape, stride, pads, groups)
    b = None if bias is None else _arr(bias, np.float32, (w.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "conv2d_f32_chain")
    arr, keep = _chain_ops(ops, yshape, np.float32)
    y = np.empty(yshape, dtype=np.float32)
    rc = lib().oracle_conv2d_f32_chain(_ptr(x), _ptr(w), _ptr(b), arr, len(ops), _ptr(y), _ptr(p))
    if rc:
        raise OracleError(rc, "conv2d_f32_chain")
    return y


def qconv2d_chain(xq, x_scale, x_off, wq, w_scale, w_off, bias_q, ops, y_scale, y_off, stride=(1, 1),
                  pads=(0, 0, 0, 0), groups=1, return_acc=False):
    """The quantized chain: ops on the int32 accumulator in order, then one requantize."""
    xq = _arr(xq, np.int8); wq = _arr(wq, np.int8)
    p, yshape = _conv_params(xq.shape, wq.shape, stride, pads, groups)
    b = None if bias_q is None else _arr(bias_q, np.int32, (wq.shape[0],))
    if min(yshape) <= 0:
        raise OracleError(BAD_SHAPE, "qconv2d_chain")
    arr, keep = _chain_ops(ops, yshape, np.int8)
    y = np.empty(yshape, dtype=np.int8)
    acc = np.empty(yshape, dtype=np.int32) if return_acc else None
    rc = lib().oracle_qconv2d_chain(_ptr(xq), x_scale, x_off, _ptr(wq), w_scale, w_off, _ptr(b), arr, len(ops),
                                    _ptr(y), y_scale, y_off, _ptr(p), _ptr(acc))
    if rc:
        raise OracleError(rc, "qconv2d_chain")
    return (y, acc) if return_acc else y


def chain_threshold(v: float, s: float) -> int:
    """A real max/clip bound v on an accumulator grid of step s: floor(v / s + 0.5), saturated to int32."""
    return int(lib().oracle_chain_threshold(v, s))
