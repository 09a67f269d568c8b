"""ctypes binding of libcct.so (include/cct.h).  Argument marshalling only.

Every function here has the name of the C entry point it calls.  Tensors are
torch tensors on the GPU (contiguous fp32); the binding passes their
``data_ptr()`` and the current HIP stream.  Nothing is computed in Python and
there is no fallback: importing this module raises if libcct.so is missing.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcct.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libcct.so has not been built (run `python -m paper_1504_04343_amd.build` or "
        "`__graft_entry__.build()`); there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

LOWER_AUTO, LOWER_TYPE1, LOWER_TYPE2, LOWER_TYPE3, LOWER_FUSED = 0, 1, 2, 3, 4
PREC_F32, PREC_BF16_IN_F32_ACC = 0, 1
PASS_FORWARD, PASS_BACKWARD_DATA, PASS_BACKWARD_WEIGHTS = 0, 1, 2
OK, EINVAL, EWORKSPACE, EUNSUPPORTED, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = [
    "cct_strerror", "cct_last_hip_error", "cct_conv_output_dims", "cct_lowered_shape",
    "cct_pick_lowering", "cct_lowering_cost", "cct_conv_workspace_bytes",
    "cct_conv_workspace_bytes_for_chunk", "cct_conv_forward", "cct_conv_backward_data",
    "cct_conv_backward_weights", "cct_lowered_ld", "cct_lower", "cct_profile_enable",
    "cct_profile_read", "cct_calibration_copy", "cct_conv_forward_static",
    "cct_relu_forward", "cct_relu_backward", "cct_pool_output_dims", "cct_maxpool_forward",
    "cct_maxpool_backward", "cct_lrn_forward", "cct_lrn_backward",
    "cct_dropout_forward", "cct_dropout_backward", "cct_softmax_loss_forward",
    "cct_softmax_loss_backward",
]


class ConvDesc(ctypes.Structure):
    """cct_conv_desc_t."""
    _fields_ = [(k, ctypes.c_int32) for k in
                ("N", "C", "H", "W", "O", "K", "stride", "pad", "groups", "lowering", "precision")]


class CctError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (code %d)" % (where, strerror(code), code))


_vp, _sz, _i32, _i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
_dp = ctypes.POINTER(ConvDesc)
_lib.cct_strerror.restype = ctypes.c_char_p
_lib.cct_strerror.argtypes = [ctypes.c_int]
_lib.cct_last_hip_error.restype = ctypes.c_int
_lib.cct_last_hip_error.argtypes = []
_lib.cct_conv_output_dims.argtypes = [_dp, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
_lib.cct_lowered_shape.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(_i64), ctypes.POINTER(_i64),
                                   ctypes.POINTER(_i64)]
_lib.cct_lowered_ld.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(_i64)]
_lib.cct_pick_lowering.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
_lib.cct_lowering_cost.argtypes = [_dp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
_lib.cct_conv_workspace_bytes.argtypes = [_dp, ctypes.c_int, ctypes.POINTER(_sz)]
_lib.cct_conv_workspace_bytes_for_chunk.argtypes = [_dp, ctypes.c_int, _i32, ctypes.POINTER(_sz)]
_lib.cct_conv_forward.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.cct_conv_forward_static.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp]
_lib.cct_conv_backward_data.argtypes = [_dp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.cct_conv_backward_weights.argtypes = [_dp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.cct_lower.argtypes = [_dp, ctypes.c_int, _vp, _vp, _vp]


class PoolDesc(ctypes.Structure):
    """cct_pool_desc_t."""
    _fields_ = [(k, ctypes.c_int32) for k in ("N", "C", "H", "W", "K", "stride", "pad")]


class LrnDesc(ctypes.Structure):
    """cct_lrn_desc_t."""
    _fields_ = [(k, ctypes.c_int32) for k in ("N", "C", "H", "W", "size")] + \
               [(k, ctypes.c_float) for k in ("alpha", "beta", "k")]


_pp = ctypes.POINTER(PoolDesc)
_lib.cct_relu_forward.argtypes = [_vp, _vp, _i64, _vp]
_lib.cct_relu_backward.argtypes = [_vp, _vp, _vp, _i64, _vp]
_lib.cct_pool_output_dims.argtypes = [_pp, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]
_lib.cct_maxpool_forward.argtypes = [_pp, _vp, _vp, _vp, _vp]
_lib.cct_maxpool_backward.argtypes = [_pp, _vp, _vp, _vp, _vp]
_lib.cct_lrn_forward.argtypes = [ctypes.POINTER(LrnDesc), _vp, _vp, _vp]
_lib.cct_lrn_backward.argtypes = [ctypes.POINTER(LrnDesc), _vp, _vp, _vp, _vp]
_lib.cct_dropout_forward.argtypes = [_vp, _vp, ctypes.c_float, _vp, _i64, _vp]
_lib.cct_dropout_backward.argtypes = [_vp, _vp, ctypes.c_float, _vp, _i64, _vp]
_lib.cct_softmax_loss_forward.argtypes = [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.cct_softmax_loss_backward.argtypes = [_i32, _i32, _vp, _vp, _vp, _vp]


class ProfileEntry(ctypes.Structure):
    """cct_profile_entry_t."""
    _fields_ = [("name", ctypes.c_char * 96), ("launches", _i64), ("total_ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


_lib.cct_calibration_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.cct_profile_enable.argtypes = [ctypes.c_int]
_lib.cct_profile_read.argtypes = [ctypes.POINTER(ProfileEntry), _i32, ctypes.POINTER(_i32)]
for _name in EXPORTS:
    if _name not in ("cct_strerror",):
        getattr(_lib, _name).restype = ctypes.c_int


def make_desc(N, C, H, W, O, K, stride=1, pad=0, groups=1, lowering=LOWER_AUTO,
              precision=PREC_F32) -> ConvDesc:
    return ConvDesc(N, C, H, W, O, K, stride, pad, groups, lowering, precision)


def strerror(code: int) -> str:
    return _lib.cct_strerror(int(code)).decode()


def _check(rc, where):
    if rc != OK:
        raise CctError(rc, where)


def cct_last_hip_error() -> int:
    return int(_lib.cct_last_hip_error())


def cct_conv_output_dims(desc: ConvDesc):
    ho, wo = _i32(), _i32()
    _check(_lib.cct_conv_output_dims(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo)),
           "cct_conv_output_dims")
    return ho.value, wo.value


def cct_lowered_shape(desc: ConvDesc, lowering: int):
    r, c, rc_ = _i64(), _i64(), _i64()
    _check(_lib.cct_lowered_shape(ctypes.byref(desc), int(lowering), ctypes.byref(r),
                                  ctypes.byref(c), ctypes.byref(rc_)), "cct_lowered_shape")
    return r.value, c.value, rc_.value


def cct_lowered_ld(desc: ConvDesc, lowering: int) -> int:
    ld = _i64()
    _check(_lib.cct_lowered_ld(ctypes.byref(desc), int(lowering), ctypes.byref(ld)),
           "cct_lowered_ld")
    return ld.value


def cct_pick_lowering(desc: ConvDesc, pass_: int = PASS_FORWARD) -> int:
    out = ctypes.c_int()
    _check(_lib.cct_pick_lowering(ctypes.byref(desc), int(pass_), ctypes.byref(out)),
           "cct_pick_lowering")
    return out.value


def cct_lowering_cost(desc: ConvDesc, pass_: int, lowering: int) -> float:
    out = ctypes.c_double()
    _check(_lib.cct_lowering_cost(ctypes.byref(desc), int(pass_), int(lowering), ctypes.byref(out)),
           "cct_lowering_cost")
    return out.value


def cct_conv_workspace_bytes(desc: ConvDesc, pass_: int) -> int:
    out = _sz()
    _check(_lib.cct_conv_workspace_bytes(ctypes.byref(desc), int(pass_), ctypes.byref(out)),
           "cct_conv_workspace_bytes")
    return out.value


def cct_conv_workspace_bytes_for_chunk(desc: ConvDesc, pass_: int, images_per_chunk: int) -> int:
    out = _sz()
    _check(_lib.cct_conv_workspace_bytes_for_chunk(ctypes.byref(desc), int(pass_),
                                                   int(images_per_chunk), ctypes.byref(out)),
           "cct_conv_workspace_bytes_for_chunk")
    return out.value


def cct_profile_enable(on: bool) -> None:
    _check(_lib.cct_profile_enable(1 if on else 0), "cct_profile_enable")


def cct_profile_read(max_entries: int = 64):
    """List of dicts (name, launches, total_ms, flops, bytes), one per kernel name."""
    arr = (ProfileEntry * max_entries)()
    n = _i32()
    _check(_lib.cct_profile_read(arr, max_entries, ctypes.byref(n)), "cct_profile_read")
    return [dict(name=arr[i].name.decode(), launches=int(arr[i].launches),
                 total_ms=float(arr[i].total_ms), flops=float(arr[i].flops),
                 bytes=float(arr[i].bytes)) for i in range(n.value)]


def cct_calibration_copy(src, dst) -> None:
    """Plain device copy of src into dst (same-size contiguous GPU tensors)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise ValueError("src and dst must be GPU tensors of the same byte size")
    _check(_lib.cct_calibration_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()),
           "cct_calibration_copy")


# ---- device entry points -----------------------------------------------------------------

def _ptr(t, name, shape=None, optional=False):
    import torch
    if t is None:
        if optional:
            return None
        raise ValueError("%s is required" % name)
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch tensor on the GPU" % name)
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be contiguous fp32" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ws(workspace):
    import torch
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or \
            workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous uint8 torch tensor on the GPU")
    return workspace.data_ptr(), workspace.numel()


def alloc_workspace(desc: ConvDesc, pass_: int, images_per_chunk: int | None = None):
    """Caller-side helper: a uint8 device tensor of the queried size."""
    import torch
    n = cct_conv_workspace_bytes(desc, pass_) if images_per_chunk is None else \
        cct_conv_workspace_bytes_for_chunk(desc, pass_, images_per_chunk)
    return torch.empty(n, dtype=torch.uint8, device="cuda")


def _shapes(desc: ConvDesc):
    ho, wo = cct_conv_output_dims(desc)
    return ((desc.N, desc.C, desc.H, desc.W), (desc.O, desc.C // desc.groups, desc.K, desc.K),
            (desc.N, desc.O, ho, wo))


def cct_conv_forward(desc: ConvDesc, x, w, bias, y, workspace) -> None:
    xs, ws_, ys = _shapes(desc)
    wp, wn = _ws(workspace)
    _check(_lib.cct_conv_forward(ctypes.byref(desc), _ptr(x, "x", xs), _ptr(w, "w", ws_),
                                 _ptr(bias, "bias", (desc.O,), optional=True), _ptr(y, "y", ys),
                                 wp, wn, _stream()), "cct_conv_forward")


def cct_conv_forward_static(desc: ConvDesc, x, w, bias, y) -> None:
    xs, ws_, ys = _shapes(desc)
    _check(_lib.cct_conv_forward_static(ctypes.byref(desc), _ptr(x, "x", xs), _ptr(w, "w", ws_),
                                        _ptr(bias, "bias", (desc.O,), optional=True),
                                        _ptr(y, "y", ys), _stream()), "cct_conv_forward_static")


def cct_conv_backward_data(desc: ConvDesc, w, dy, dx, workspace) -> None:
    xs, ws_, ys = _shapes(desc)
    wp, wn = _ws(workspace)
    _check(_lib.cct_conv_backward_data(ctypes.byref(desc), _ptr(w, "w", ws_), _ptr(dy, "dy", ys),
                                       _ptr(dx, "dx", xs), wp, wn, _stream()),
           "cct_conv_backward_data")


def cct_conv_backward_weights(desc: ConvDesc, x, dy, dw, dbias, workspace) -> None:
    xs, ws_, ys = _shapes(desc)
    wp, wn = _ws(workspace)
    _check(_lib.cct_conv_backward_weights(ctypes.byref(desc), _ptr(x, "x", xs), _ptr(dy, "dy", ys),
                                          _ptr(dw, "dw", ws_),
                                          _ptr(dbias, "dbias", (desc.O,), optional=True), wp, wn,
                                          _stream()), "cct_conv_backward_weights")


def cct_lower(desc: ConvDesc, lowering: int, x, dhat) -> None:
    xs, _, _ = _shapes(desc)
    _, cols, _ = cct_lowered_shape(desc, lowering)
    ld = cct_lowered_ld(desc, lowering)
    _check(_lib.cct_lower(ctypes.byref(desc), int(lowering), _ptr(x, "x", xs),
                          _ptr(dhat, "dhat", (desc.groups * cols, ld)), _stream()), "cct_lower")


# ---- ReLU and max pooling -------------------------------------------------------------------

def make_pool_desc(N, C, H, W, K, stride, pad=0) -> PoolDesc:
    return PoolDesc(N, C, H, W, K, stride, pad)


def cct_pool_output_dims(desc: PoolDesc):
    ho, wo = _i32(), _i32()
    _check(_lib.cct_pool_output_dims(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo)),
           "cct_pool_output_dims")
    return ho.value, wo.value


def cct_relu_forward(x, y) -> None:
    _check(_lib.cct_relu_forward(_ptr(x, "x"), _ptr(y, "y", x.shape), x.numel(), _stream()),
           "cct_relu_forward")


def cct_relu_backward(x, dy, dx) -> None:
    _check(_lib.cct_relu_backward(_ptr(x, "x"), _ptr(dy, "dy", x.shape), _ptr(dx, "dx", x.shape),
                                  x.numel(), _stream()), "cct_relu_backward")


def _iptr(t, name, shape):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.int32 or \
            not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise TypeError("%s must be a contiguous int32 GPU tensor of shape %s" % (name, tuple(shape)))
    return t.data_ptr()


def cct_maxpool_forward(desc: PoolDesc, x, y, argmax=None) -> None:
    ho, wo = cct_pool_output_dims(desc)
    ys = (desc.N, desc.C, ho, wo)
    _check(_lib.cct_maxpool_forward(ctypes.byref(desc), _ptr(x, "x", (desc.N, desc.C, desc.H, desc.W)),
                                    _ptr(y, "y", ys),
                                    None if argmax is None else _iptr(argmax, "argmax", ys),
                                    _stream()), "cct_maxpool_forward")


def cct_maxpool_backward(desc: PoolDesc, dy, argmax, dx) -> None:
    ho, wo = cct_pool_output_dims(desc)
    ys = (desc.N, desc.C, ho, wo)
    _check(_lib.cct_maxpool_backward(ctypes.byref(desc), _ptr(dy, "dy", ys), _iptr(argmax, "argmax", ys),
                                     _ptr(dx, "dx", (desc.N, desc.C, desc.H, desc.W)), _stream()),
           "cct_maxpool_backward")


def make_lrn_desc(N, C, H, W, size=5, alpha=1e-4, beta=0.75, k=1.0) -> LrnDesc:
    return LrnDesc(N, C, H, W, size, alpha, beta, k)


def cct_lrn_forward(desc: LrnDesc, x, y) -> None:
    shape = (desc.N, desc.C, desc.H, desc.W)
    _check(_lib.cct_lrn_forward(ctypes.byref(desc), _ptr(x, "x", shape), _ptr(y, "y", shape), _stream()),
           "cct_lrn_forward")


def cct_lrn_backward(desc: LrnDesc, x, dy, dx) -> None:
    shape = (desc.N, desc.C, desc.H, desc.W)
    _check(_lib.cct_lrn_backward(ctypes.byref(desc), _ptr(x, "x", shape), _ptr(dy, "dy", shape),
                                 _ptr(dx, "dx", shape), _stream()), "cct_lrn_backward")


def _u8ptr(t, name, shape):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.uint8 or \
            not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise TypeError("%s must be a contiguous uint8 GPU tensor of shape %s" % (name, tuple(shape)))
    return t.data_ptr()


def cct_dropout_forward(x, mask, scale, y) -> None:
    _check(_lib.cct_dropout_forward(_ptr(x, "x"), _u8ptr(mask, "mask", x.shape), scale,
                                    _ptr(y, "y", x.shape), x.numel(), _stream()), "cct_dropout_forward")


def cct_dropout_backward(dy, mask, scale, dx) -> None:
    _check(_lib.cct_dropout_backward(_ptr(dy, "dy"), _u8ptr(mask, "mask", dy.shape), scale,
                                     _ptr(dx, "dx", dy.shape), dy.numel(), _stream()),
           "cct_dropout_backward")


def cct_softmax_loss_forward(x, label, prob, image_loss, loss) -> None:
    """x, prob: [N, C] fp32; label: [N] int32; image_loss: [N] fp32; loss: [1] fp32."""
    N, C = x.shape
    _check(_lib.cct_softmax_loss_forward(N, C, _ptr(x, "x"), _iptr(label, "label", (N,)),
                                         _ptr(prob, "prob", (N, C)), _ptr(image_loss, "image_loss", (N,)),
                                         _ptr(loss, "loss", (1,)), _stream()), "cct_softmax_loss_forward")


def cct_softmax_loss_backward(prob, label, dx) -> None:
    N, C = prob.shape
    _check(_lib.cct_softmax_loss_backward(N, C, _ptr(prob, "prob"), _iptr(label, "label", (N,)),
                                          _ptr(dx, "dx", (N, C)), _stream()), "cct_softmax_loss_backward")
