"""ctypes binding of libglowmi.so with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

ACT_NONE = 0
ACT_RELU = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libglowmi.so")

STATUS_NAMES = {0: "GLOWMI_OK", 1: "GLOWMI_ERR_NULL", 2: "GLOWMI_ERR_SHAPE", 3: "GLOWMI_ERR_UNSUPPORTED",
                4: "GLOWMI_ERR_ALIGN", 5: "GLOWMI_ERR_QUANT", 6: "GLOWMI_ERR_HIP"}


class ConvDesc(ctypes.Structure):
    """glowmi_conv_desc: input n,h,w,c; filter k,r,s; strides; pads (top, left, bottom, right); groups."""
    _fields_ = [(name, ctypes.c_int32) for name in
                ("n", "h", "w", "c", "k", "r", "s", "stride_h", "stride_w",
                 "pad_t", "pad_l", "pad_b", "pad_r", "groups")]


class QParam(ctypes.Structure):
    """glowmi_qparam: value = (q - offset) * scale."""
    _fields_ = [("scale", ctypes.c_float), ("offset", ctypes.c_int32)]


class Chain(ctypes.Structure):
    """glowmi_chain: bias add -> + addend (optional tensor of y's shape) -> act."""
    _fields_ = [("addend", ctypes.c_void_p), ("addend_q", QParam), ("act", ctypes.c_int)]


OP_ADD_TENSOR, OP_MUL_SCALAR, OP_MAX_SCALAR, OP_CLIP = 1, 2, 3, 4
MAX_CHAIN_OPS = 4


class ChainOp(ctypes.Structure):
    """glowmi_chain_op: kind; scalars a, b; tensor operand and (quantized form) its scale/offset."""
    _fields_ = [("kind", ctypes.c_int), ("a", ctypes.c_float), ("b", ctypes.c_float), ("tensor", ctypes.c_void_p),
                ("tensor_q", QParam)]


class SeqLayer(ctypes.Structure):
    """glowmi_seq_layer: one layer of a back-to-back sequence."""
    _fields_ = [("desc", ConvDesc), ("w", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("wq", QParam),
                ("yq", QParam), ("act", ctypes.c_int), ("add_input", ctypes.c_int32)]


class GlowmiError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def library_path() -> str:
    return _LIB_PATH


def library() -> ctypes.CDLL:
    """Load libglowmi.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_1805_00907_amd.build` "
                          "(glowmi has no CPU or PyTorch fallback)")
    # torch ships its own HIP runtime; import it first so that this library binds to the same
    # runtime instance that owns the device memory and streams handed to it.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(ConvDesc)
    L.glowmi_conv_out_shape.argtypes = [dp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.glowmi_conv2d.argtypes = [vp, vp, vp, vp, dp, ctypes.c_int, vp, sz, vp]
    L.glowmi_conv2d_workspace_bytes.argtypes = [dp]
    L.glowmi_conv2d_workspace_bytes.restype = sz
    L.glowmi_fc.argtypes = [vp, vp, vp, vp, i32, i32, i32, ctypes.c_int, vp, sz, vp]
    L.glowmi_fc_workspace_bytes.argtypes = [i32, i32, i32]
    L.glowmi_fc_workspace_bytes.restype = sz
    L.glowmi_fc_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, i32, ctypes.c_int, vp]
    L.glowmi_conv2d_filter_planes_bytes.argtypes = [dp]
    L.glowmi_conv2d_filter_planes_bytes.restype = sz
    L.glowmi_conv2d_pack_filter.argtypes = [vp, dp, vp, sz, vp]
    L.glowmi_conv2d_packed_workspace_bytes.argtypes = [dp]
    L.glowmi_conv2d_packed_workspace_bytes.restype = sz
    L.glowmi_fc_filter_planes_bytes.argtypes = [i32, i32]
    L.glowmi_fc_filter_planes_bytes.restype = sz
    L.glowmi_fc_pack_filter.argtypes = [vp, i32, i32, vp, sz, vp]
    L.glowmi_fc_packed_workspace_bytes.argtypes = [i32, i32, i32]
    L.glowmi_fc_packed_workspace_bytes.restype = sz
    L.glowmi_fc_packed.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, ctypes.c_int, vp, sz, vp]
    L.glowmi_fc_noalloc_max_scratch_bytes.argtypes = []
    L.glowmi_fc_noalloc_max_scratch_bytes.restype = sz
    L.glowmi_tuning_set.argtypes = [ctypes.c_char_p, i32]
    L.glowmi_tuning_reset.argtypes = []
    L.glowmi_tuning_reset.restype = None
    L.glowmi_qconv2d.argtypes = [vp, QParam, vp, QParam, vp, vp, QParam, dp, ctypes.c_int, vp, sz, vp]
    L.glowmi_qconv2d_workspace_bytes.argtypes = [dp]
    L.glowmi_qconv2d_workspace_bytes.restype = sz
    L.glowmi_qfc.argtypes = [vp, QParam, vp, QParam, vp, vp, QParam, i32, i32, i32, ctypes.c_int, vp, sz, vp]
    L.glowmi_qfc_workspace_bytes.argtypes = [i32, i32, i32]
    L.glowmi_qfc_workspace_bytes.restype = sz
    cp = ctypes.POINTER(Chain)
    L.glowmi_conv2d_chain.argtypes = [vp, vp, vp, vp, dp, cp, vp, sz, vp]
    L.glowmi_qconv2d_chain.argtypes = [vp, QParam, vp, QParam, vp, vp, QParam, dp, cp, vp, sz, vp]
    L.glowmi_conv2d_packed.argtypes = [vp, vp, vp, vp, vp, dp, cp, vp, sz, vp]
    op = ctypes.POINTER(ChainOp)
    L.glowmi_conv2d_chainv.argtypes = [vp, vp, vp, vp, dp, op, i32, vp, sz, vp]
    L.glowmi_conv2d_chainv_workspace_bytes.argtypes = [dp, op, i32]
    L.glowmi_conv2d_chainv_workspace_bytes.restype = sz
    L.glowmi_qconv2d_chainv.argtypes = [vp, QParam, vp, QParam, vp, vp, QParam, dp, op, i32, vp, sz, vp]
    L.glowmi_qconv2d_chainv_workspace_bytes.argtypes = [dp, op, i32]
    L.glowmi_qconv2d_chainv_workspace_bytes.restype = sz
    sp = ctypes.POINTER(SeqLayer)
    L.glowmi_seq_arena_bytes.argtypes = [sp, i32, i32]
    L.glowmi_seq_arena_bytes.restype = sz
    L.glowmi_seq_conv2d.argtypes = [vp, sp, i32, vp, vp, sz, vp]
    L.glowmi_seq_qconv2d.argtypes = [vp, QParam, sp, i32, vp, vp, sz, vp]
    L.glowmi_quantize.argtypes = [vp, vp, sz, QParam, vp]
    L.glowmi_dequantize.argtypes = [vp, vp, sz, QParam, vp]
    L.glowmi_rescale.argtypes = [vp, QParam, vp, QParam, sz, vp]
    L.glowmi_fold_batchnorm.argtypes = [vp] * 6 + [ctypes.c_float, i32, ctypes.c_int64, vp, vp]
    L.glowmi_requant_params.argtypes = [ctypes.c_float] * 3 + [ctypes.POINTER(i32)] * 2
    L.glowmi_rescale_params.argtypes = [ctypes.c_float] * 3 + [ctypes.POINTER(i32)] * 2
    L.glowmi_status_string.argtypes = [ctypes.c_int]
    L.glowmi_status_string.restype = ctypes.c_char_p
    L.glowmi_last_error.restype = ctypes.c_char_p
    L.glowmi_last_variant.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status: int) -> None:
    if status != 0:
        raise GlowmiError(status, library().glowmi_last_error().decode())


def last_variant() -> str:
    return library().glowmi_last_variant().decode()


def _ptr(t, dtype: Optional[str] = None, count: Optional[int] = None, what: str = "tensor") -> Optional[int]:
    """Device address of a torch tensor (None -> NULL); a raw integer address is passed through.

    For a tensor, the facts the C side cannot see are checked here, because a mismatch would become
    an out-of-bounds access on the device: it must live on a GPU, be contiguous, have the element
    type `dtype` ("float32", "int8", "int32") and hold at least `count` elements."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError(f"{what}: expected a device tensor, got one on {t.device}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor is not contiguous")
    if dtype is not None and str(t.dtype) != "torch." + dtype:
        raise ValueError(f"{what}: expected {dtype}, got {t.dtype}")
    if count is not None and t.numel() < count:
        raise ValueError(f"{what}: {t.numel()} elements, the call needs {count}")
    return t.data_ptr()


def _conv_counts(desc: ConvDesc) -> Tuple[int, int, int]:
    """(input, filter, output) element counts of a descriptor; zeros when the library will reject it."""
    oh, ow = ctypes.c_int32(0), ctypes.c_int32(0)
    if library().glowmi_conv_out_shape(ctypes.byref(desc), ctypes.byref(oh), ctypes.byref(ow)) != 0:
        return 0, 0, 0
    return (desc.n * desc.h * desc.w * desc.c, desc.k * desc.r * desc.s * (desc.c // desc.groups),
            desc.n * oh.value * ow.value * desc.k)


def _ws(workspace) -> Tuple[Optional[int], int]:
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace: expected a contiguous device tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _stream(stream) -> Optional[int]:
    """hipStream_t handle: a torch stream, a raw handle, or torch's current stream when None."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def conv_out_shape(desc: ConvDesc) -> Tuple[int, int]:
    oh, ow = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(library().glowmi_conv_out_shape(ctypes.byref(desc), ctypes.byref(oh), ctypes.byref(ow)))
    return oh.value, ow.value


def conv2d_workspace_bytes(desc: ConvDesc) -> int:
    return int(library().glowmi_conv2d_workspace_bytes(ctypes.byref(desc)))


def conv2d(x, w, bias, y, desc: ConvDesc, act: int = ACT_NONE, workspace=None, stream=None) -> None:
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    _check(library().glowmi_conv2d(_ptr(x, "float32", nx, "x"), _ptr(w, "float32", nw, "w"),
                                   _ptr(bias, "float32", desc.k, "bias"), _ptr(y, "float32", ny, "y"),
                                   ctypes.byref(desc), act, wp, wb, _stream(stream)))


def fc_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(library().glowmi_fc_workspace_bytes(M, K, N))


def fc(a, w, bias, y, M: int, K: int, N: int, act: int = ACT_NONE, workspace=None, stream=None) -> None:
    wp, wb = _ws(workspace)
    _check(library().glowmi_fc(_ptr(a, "float32", M * K, "a"), _ptr(w, "float32", K * N, "w"),
                               _ptr(bias, "float32", N, "bias"), _ptr(y, "float32", M * N, "y"), M, K, N, act, wp,
                               wb, _stream(stream)))


def fc_noalloc(a, w, bias, y, M: int, K: int, N: int, act: int = ACT_NONE, stream=None) -> None:
    """glowmi_fc without a workspace argument and without any allocation (library-owned static scratch)."""
    _check(library().glowmi_fc_noalloc(_ptr(a, "float32", M * K, "a"), _ptr(w, "float32", K * N, "w"),
                                       _ptr(bias, "float32", N, "bias"), _ptr(y, "float32", M * N, "y"), M, K, N,
                                       act, _stream(stream)))


def fc_noalloc_max_scratch_bytes() -> int:
    return int(library().glowmi_fc_noalloc_max_scratch_bytes())


def tuning_set(name: str, value: int) -> None:
    """Set a tuning knob (experiments and tests), e.g. tuning_set("F32_TILE", 2)."""
    _check(library().glowmi_tuning_set(name.encode(), int(value)))


def tuning_reset() -> None:
    """Every knob back to the planner's own choice."""
    library().glowmi_tuning_reset()


def qconv2d_workspace_bytes(desc: ConvDesc) -> int:
    return int(library().glowmi_qconv2d_workspace_bytes(ctypes.byref(desc)))


def qconv2d(x, xq: QParam, w, wq: QParam, bias, y, yq: QParam, desc: ConvDesc, act: int = ACT_NONE,
            workspace=None, stream=None) -> None:
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    _check(library().glowmi_qconv2d(_ptr(x, "int8", nx, "x"), xq, _ptr(w, "int8", nw, "w"), wq,
                                    _ptr(bias, "int32", desc.k, "bias"), _ptr(y, "int8", ny, "y"), yq,
                                    ctypes.byref(desc), act, wp, wb, _stream(stream)))


def conv2d_chain(x, w, bias, y, desc: ConvDesc, addend=None, act: int = ACT_NONE, workspace=None,
                 stream=None) -> None:
    """y = act(conv + bias + addend); addend is a float tensor of y's shape (may be y) or None."""
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    chain = Chain(_ptr(addend, "float32", ny, "addend"), QParam(1.0, 0), act)
    _check(library().glowmi_conv2d_chain(_ptr(x, "float32", nx, "x"), _ptr(w, "float32", nw, "w"),
                                         _ptr(bias, "float32", desc.k, "bias"), _ptr(y, "float32", ny, "y"),
                                         ctypes.byref(desc), ctypes.byref(chain), wp, wb, _stream(stream)))


def _planes(planes, need: int) -> Tuple[Optional[int], int]:
    """Address and size of a plane buffer (any element type); it must hold `need` bytes when that is known."""
    if planes is None:
        return None, 0
    if not planes.is_cuda or not planes.is_contiguous():
        raise ValueError("planes: expected a contiguous device tensor")
    have = planes.numel() * planes.element_size()
    if need and have < need:
        raise ValueError(f"planes: {have} bytes, the filter's planes take {need}")
    return planes.data_ptr(), have


def conv2d_filter_planes_bytes(desc: ConvDesc) -> int:
    return int(library().glowmi_conv2d_filter_planes_bytes(ctypes.byref(desc)))


def conv2d_pack_filter(w, desc: ConvDesc, planes, stream=None) -> None:
    """Writes the fp16 planes of the filter `w` (made once, ahead of the calls that use them) to `planes`."""
    _, nw, _ = _conv_counts(desc)
    pp, pb = _planes(planes, 0)
    _check(library().glowmi_conv2d_pack_filter(_ptr(w, "float32", nw, "w"), ctypes.byref(desc), pp, pb,
                                               _stream(stream)))


def conv2d_packed_workspace_bytes(desc: ConvDesc) -> int:
    return int(library().glowmi_conv2d_packed_workspace_bytes(ctypes.byref(desc)))


def conv2d_packed(x, w, w_planes, bias, y, desc: ConvDesc, addend=None, act: int = ACT_NONE, workspace=None,
                  stream=None) -> None:
    """conv2d_chain with the filter's planes from conv2d_pack_filter (None: the plain call)."""
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    pp, _ = _planes(w_planes, conv2d_filter_planes_bytes(desc))
    chain = Chain(_ptr(addend, "float32", ny, "addend"), QParam(1.0, 0), act)
    _check(library().glowmi_conv2d_packed(_ptr(x, "float32", nx, "x"), _ptr(w, "float32", nw, "w"), pp,
                                          _ptr(bias, "float32", desc.k, "bias"), _ptr(y, "float32", ny, "y"),
                                          ctypes.byref(desc), ctypes.byref(chain), wp, wb, _stream(stream)))


def fc_filter_planes_bytes(K: int, N: int) -> int:
    return int(library().glowmi_fc_filter_planes_bytes(K, N))


def fc_pack_filter(w, K: int, N: int, planes, stream=None) -> None:
    """Writes the fp16 planes of the [K][N] weight `w` (transposed to [N][K]) to `planes`."""
    pp, pb = _planes(planes, 0)
    _check(library().glowmi_fc_pack_filter(_ptr(w, "float32", K * N, "w"), K, N, pp, pb, _stream(stream)))


def fc_packed_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(library().glowmi_fc_packed_workspace_bytes(M, K, N))


def fc_packed(a, w, w_planes, bias, y, M: int, K: int, N: int, act: int = ACT_NONE, workspace=None,
              stream=None) -> None:
    """fc with the weight's planes from fc_pack_filter (None: the plain call)."""
    wp, wb = _ws(workspace)
    pp, _ = _planes(w_planes, fc_filter_planes_bytes(K, N))
    _check(library().glowmi_fc_packed(_ptr(a, "float32", M * K, "a"), _ptr(w, "float32", K * N, "w"), pp,
                                      _ptr(bias, "float32", N, "bias"), _ptr(y, "float32", M * N, "y"), M, K, N,
                                      act, wp, wb, _stream(stream)))


def qconv2d_chain(x, xq: QParam, w, wq: QParam, bias, y, yq: QParam, desc: ConvDesc, addend=None,
                  addend_q: Optional[QParam] = None, act: int = ACT_NONE, workspace=None, stream=None) -> None:
    """Quantized form: addend is an int8 tensor of y's shape with scale/offset addend_q."""
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    chain = Chain(_ptr(addend, "int8", ny, "addend"), addend_q if addend_q is not None else QParam(1.0, 0), act)
    _check(library().glowmi_qconv2d_chain(_ptr(x, "int8", nx, "x"), xq, _ptr(w, "int8", nw, "w"), wq,
                                          _ptr(bias, "int32", desc.k, "bias"), _ptr(y, "int8", ny, "y"), yq,
                                          ctypes.byref(desc), ctypes.byref(chain), wp, wb, _stream(stream)))


def chain_ops(ops, dtype: str = "float32", count: Optional[int] = None):
    """ctypes array of ChainOp from a list of ("add", tensor[, QParam]) | ("mul", a) | ("max", a) |
    ("clip", a, b).  Tensors are device tensors of the output's element type (or raw addresses)."""
    arr = (ChainOp * max(1, len(ops)))()
    for i, o in enumerate(ops):
        if o[0] == "add":
            q = o[2] if len(o) > 2 else QParam(1.0, 0)
            arr[i] = ChainOp(OP_ADD_TENSOR, 0.0, 0.0, _ptr(o[1], dtype, count, f"op {i} tensor"), q)
        elif o[0] == "mul":
            arr[i] = ChainOp(OP_MUL_SCALAR, o[1], 0.0, None, QParam(1.0, 0))
        elif o[0] == "max":
            arr[i] = ChainOp(OP_MAX_SCALAR, o[1], 0.0, None, QParam(1.0, 0))
        elif o[0] == "clip":
            arr[i] = ChainOp(OP_CLIP, o[1], o[2], None, QParam(1.0, 0))
        else:
            raise ValueError(f"unknown chain op {o[0]!r}")
    return arr


def conv2d_chainv_workspace_bytes(desc: ConvDesc, ops) -> int:
    arr = chain_ops(ops)
    return int(library().glowmi_conv2d_chainv_workspace_bytes(ctypes.byref(desc), arr, len(ops)))


def conv2d_chainv(x, w, bias, y, desc: ConvDesc, ops, workspace=None, stream=None) -> None:
    """y = ops applied in order to (conv + bias): a general stack of data-parallel operators."""
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    arr = chain_ops(ops, "float32", ny)
    _check(library().glowmi_conv2d_chainv(_ptr(x, "float32", nx, "x"), _ptr(w, "float32", nw, "w"),
                                          _ptr(bias, "float32", desc.k, "bias"), _ptr(y, "float32", ny, "y"),
                                          ctypes.byref(desc), arr, len(ops), wp, wb, _stream(stream)))


def qconv2d_chainv_workspace_bytes(desc: ConvDesc, ops) -> int:
    arr = chain_ops(ops, "int8")
    return int(library().glowmi_qconv2d_chainv_workspace_bytes(ctypes.byref(desc), arr, len(ops)))


def qconv2d_chainv(x, xq: QParam, w, wq: QParam, bias, y, yq: QParam, desc: ConvDesc, ops, workspace=None,
                   stream=None) -> None:
    """Quantized general chain: the ops act on the int32 accumulator, then one requantize."""
    wp, wb = _ws(workspace)
    nx, nw, ny = _conv_counts(desc)
    arr = chain_ops(ops, "int8", ny)
    _check(library().glowmi_qconv2d_chainv(_ptr(x, "int8", nx, "x"), xq, _ptr(w, "int8", nw, "w"), wq,
                                           _ptr(bias, "int32", desc.k, "bias"), _ptr(y, "int8", ny, "y"), yq,
                                           ctypes.byref(desc), arr, len(ops), wp, wb, _stream(stream)))


def qfc_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(library().glowmi_qfc_workspace_bytes(M, K, N))


def qfc(a, aq: QParam, w, wq: QParam, bias, y, yq: QParam, M: int, K: int, N: int, act: int = ACT_NONE,
        workspace=None, stream=None) -> None:
    wp, wb = _ws(workspace)
    _check(library().glowmi_qfc(_ptr(a, "int8", M * K, "a"), aq, _ptr(w, "int8", K * N, "w"), wq,
                                _ptr(bias, "int32", N, "bias"), _ptr(y, "int8", M * N, "y"), yq, M, K, N, act, wp,
                                wb, _stream(stream)))


def requant_params(x_scale: float, w_scale: float, y_scale: float) -> Tuple[int, int]:
    m, s = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(library().glowmi_requant_params(x_scale, w_scale, y_scale, ctypes.byref(m), ctypes.byref(s)))
    return m.value, s.value


def rescale_params(r_scale: float, x_scale: float, w_scale: float) -> Tuple[int, int]:
    m, s = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(library().glowmi_rescale_params(r_scale, x_scale, w_scale, ctypes.byref(m), ctypes.byref(s)))
    return m.value, s.value


def quantize(x, q, qp: QParam, count: Optional[int] = None, stream=None) -> None:
    """float32 device tensor x -> int8 device tensor q with scale/offset qp."""
    n = x.numel() if count is None else count
    _check(library().glowmi_quantize(_ptr(x, "float32", n, "x"), _ptr(q, "int8", n, "q"), n, qp, _stream(stream)))


def dequantize(q, x, qp: QParam, count: Optional[int] = None, stream=None) -> None:
    n = q.numel() if count is None else count
    _check(library().glowmi_dequantize(_ptr(q, "int8", n, "q"), _ptr(x, "float32", n, "x"), n, qp, _stream(stream)))


def rescale(q_in, from_q: QParam, q_out, to_q: QParam, count: Optional[int] = None, stream=None) -> None:
    """The same real values on another scale/offset; q_out may be q_in."""
    n = q_in.numel() if count is None else count
    _check(library().glowmi_rescale(_ptr(q_in, "int8", n, "q_in"), from_q, _ptr(q_out, "int8", n, "q_out"), to_q, n,
                                    _stream(stream)))


def fold_batchnorm(w, bias, gamma, beta, mean, var, eps: float):
    """Host arrays (numpy float32): -> (w_folded, bias_folded) with batch normalization merged in."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    k = w.shape[0]
    per = w.size // k
    arrs = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in (bias, gamma, beta, mean, var)]
    w_out, b_out = np.empty_like(w), np.empty((k,), dtype=np.float32)
    hp = lambda a: None if a is None else a.ctypes.data
    _check(library().glowmi_fold_batchnorm(hp(w), hp(arrs[0]), hp(arrs[1]), hp(arrs[2]), hp(arrs[3]), hp(arrs[4]),
                                           eps, k, per, hp(w_out), hp(b_out)))
    return w_out, b_out


def seq_layers(layers) -> "ctypes.Array":
    """ctypes array of SeqLayer from (desc, w, bias, act, add_input[, wq, yq]) tuples of device tensors."""
    arr = (SeqLayer * len(layers))()
    for i, l in enumerate(layers):
        desc, w, bias, act, add_input = l[:5]
        quantized = len(l) > 5
        wq, yq = (l[5], l[6]) if quantized else (QParam(1.0, 0), QParam(1.0, 0))
        _, nw, _ = _conv_counts(desc)
        arr[i] = SeqLayer(desc, _ptr(w, "int8" if quantized else "float32", nw, f"layer {i} w"),
                          _ptr(bias, "int32" if quantized else "float32", desc.k, f"layer {i} bias"), wq, yq, act,
                          1 if add_input else 0)
    return arr


def seq_arena_bytes(arr, quantized: bool) -> int:
    return int(library().glowmi_seq_arena_bytes(arr, len(arr), 1 if quantized else 0))


def seq_conv2d(x, arr, y, arena, stream=None) -> None:
    ap, ab = _ws(arena)
    nx, _, _ = _conv_counts(arr[0].desc)
    _, _, ny = _conv_counts(arr[len(arr) - 1].desc)
    st = library().glowmi_seq_conv2d(_ptr(x, "float32", nx, "x"), arr, len(arr), _ptr(y, "float32", ny, "y"), ap, ab,
                                     _stream(stream))
    if st != 0:
        raise GlowmiError(st, library().glowmi_last_error().decode() or "sequence rejected")


def seq_qconv2d(x, xq: QParam, arr, y, arena, stream=None) -> None:
    ap, ab = _ws(arena)
    nx, _, _ = _conv_counts(arr[0].desc)
    _, _, ny = _conv_counts(arr[len(arr) - 1].desc)
    st = library().glowmi_seq_qconv2d(_ptr(x, "int8", nx, "x"), xq, arr, len(arr), _ptr(y, "int8", ny, "y"), ap, ab,
                                      _stream(stream))
    if st != 0:
        raise GlowmiError(st, library().glowmi_last_error().decode() or "sequence rejected")
