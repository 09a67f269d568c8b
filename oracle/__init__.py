"""CPU oracle for the lowering-based convolutional layer (TEST INFRASTRUCTURE ONLY).

Thin ctypes binding over ``conv_oracle.c`` (plain C, fp64 accumulation).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product path never does, and this
package imports nothing from the HIP path.

``layers_oracle.c`` holds the rectified linear unit, max pooling and local response normalisation
(Caffe's definitions), the layers between CaffeNet's convolutions.

Part A is the direct definition (eq. (1) of the paper plus Caffe-style stride /
pad / groups / bias) and its two adjoints; Part B is the paper's three lowerings
(Sec. 2.1) executed as lower -> multiply -> lift.  See the header of
``conv_oracle.c`` for conventions and for the list of pins.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "conv_oracle.c"), os.path.join(_HERE, "layers_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile conv_oracle.c and layers_oracle.c with gcc (-O2 -fopenmp) into liboracle.so."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB] + _SRCS
        subprocess.run(cmd, check=True)
    return _LIB


class _Dims(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "C", "H", "W", "O", "K", "stride", "pad", "groups")]


@dataclass(frozen=True)
class Dims:
    """Problem shape: NCHW input, O x (C/groups) x K x K kernels."""
    N: int
    C: int
    H: int
    W: int
    O: int
    K: int
    stride: int = 1
    pad: int = 0
    groups: int = 1

    def _c(self) -> _Dims:
        return _Dims(self.N, self.C, self.H, self.W, self.O, self.K, self.stride, self.pad,
                     self.groups)


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are fp32 (the bytes the GPU sees), got %s" % a.dtype)
    return a


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (rc=%d)" % (what, rc))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def output_dims(d: Dims):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    _check(_load().oracle_output_dims(ctypes.byref(d._c()), ctypes.byref(ho), ctypes.byref(wo)),
           "output_dims")
    return ho.value, wo.value


def _expect(a, shape, name):
    if tuple(a.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(a.shape), tuple(shape)))


def conv_forward(d: Dims, x, w, bias=None) -> np.ndarray:
    """y (fp64, N x O x Hout x Wout) from the direct definition."""
    x, w = _f32(x), _f32(w)
    ho, wo = output_dims(d)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    _expect(w, (d.O, d.C // d.groups, d.K, d.K), "w")
    b = None if bias is None else _f32(bias)
    if b is not None:
        _expect(b, (d.O,), "bias")
    y = np.empty((d.N, d.O, ho, wo), np.float64)
    _check(_load().oracle_conv_forward(ctypes.byref(d._c()), _p(x, ctypes.c_float),
                                       _p(w, ctypes.c_float), _p(b, ctypes.c_float),
                                       _p(y, ctypes.c_double)), "conv_forward")
    return y


def conv_forward_at(d: Dims, x, w, bias, idx) -> np.ndarray:
    """Forward at sampled linear indices of y."""
    x, w = _f32(x), _f32(w)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    _expect(w, (d.O, d.C // d.groups, d.K, d.K), "w")
    b = None if bias is None else _f32(bias)
    idx = np.ascontiguousarray(idx, np.int64)
    out = np.empty(idx.shape, np.float64)
    _check(_load().oracle_conv_forward_at(ctypes.byref(d._c()), _p(x, ctypes.c_float),
                                          _p(w, ctypes.c_float), _p(b, ctypes.c_float),
                                          _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                          _p(out, ctypes.c_double)), "conv_forward_at")
    return out


def conv_backward_data(d: Dims, w, dy) -> np.ndarray:
    """dx (fp64, N x C x H x W): adjoint of the forward map in x."""
    w, dy = _f32(w), _f32(dy)
    ho, wo = output_dims(d)
    _expect(w, (d.O, d.C // d.groups, d.K, d.K), "w")
    _expect(dy, (d.N, d.O, ho, wo), "dy")
    dx = np.empty((d.N, d.C, d.H, d.W), np.float64)
    _check(_load().oracle_conv_backward_data(ctypes.byref(d._c()), _p(w, ctypes.c_float),
                                             _p(dy, ctypes.c_float), _p(dx, ctypes.c_double)),
           "conv_backward_data")
    return dx


def conv_backward_data_at(d: Dims, w, dy, idx) -> np.ndarray:
    w, dy = _f32(w), _f32(dy)
    ho, wo = output_dims(d)
    _expect(w, (d.O, d.C // d.groups, d.K, d.K), "w")
    _expect(dy, (d.N, d.O, ho, wo), "dy")
    idx = np.ascontiguousarray(idx, np.int64)
    out = np.empty(idx.shape, np.float64)
    _check(_load().oracle_conv_backward_data_at(ctypes.byref(d._c()), _p(w, ctypes.c_float),
                                                _p(dy, ctypes.c_float), _p(idx, ctypes.c_int64),
                                                ctypes.c_int64(idx.size),
                                                _p(out, ctypes.c_double)),
           "conv_backward_data_at")
    return out


def conv_backward_weights(d: Dims, x, dy, want_dbias: bool = True):
    """(dw, dbias) in fp64: adjoint of the forward map in w, and the plain sum of dy."""
    x, dy = _f32(x), _f32(dy)
    ho, wo = output_dims(d)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    _expect(dy, (d.N, d.O, ho, wo), "dy")
    dw = np.empty((d.O, d.C // d.groups, d.K, d.K), np.float64)
    db = np.empty((d.O,), np.float64) if want_dbias else None
    _check(_load().oracle_conv_backward_weights(ctypes.byref(d._c()), _p(x, ctypes.c_float),
                                                _p(dy, ctypes.c_float), _p(dw, ctypes.c_double),
                                                _p(db, ctypes.c_double)),
           "conv_backward_weights")
    return dw, db


def conv_backward_weights_at(d: Dims, x, dy, idx) -> np.ndarray:
    x, dy = _f32(x), _f32(dy)
    ho, wo = output_dims(d)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    _expect(dy, (d.N, d.O, ho, wo), "dy")
    idx = np.ascontiguousarray(idx, np.int64)
    out = np.empty(idx.shape, np.float64)
    _check(_load().oracle_conv_backward_weights_at(ctypes.byref(d._c()), _p(x, ctypes.c_float),
                                                   _p(dy, ctypes.c_float),
                                                   _p(idx, ctypes.c_int64),
                                                   ctypes.c_int64(idx.size),
                                                   _p(out, ctypes.c_double)),
           "conv_backward_weights_at")
    return out


# ---- Part B: the paper's three lowerings -------------------------------------------------

def lowered_shape(d: Dims, lowering: int):
    """(rows, cols, rcols) per group: D^ is rows x cols, K^ is cols x rcols, R^ is rows x rcols."""
    r, c, rc = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_load().oracle_lowered_shape(ctypes.byref(d._c()), int(lowering), ctypes.byref(r),
                                        ctypes.byref(c), ctypes.byref(rc)), "lowered_shape")
    return r.value, c.value, rc.value


def lower_data(d: Dims, lowering: int, x) -> np.ndarray:
    """D^ as fp32 array (groups, rows, cols); a pure copy of x entries and zeros."""
    x = _f32(x)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    rows, cols, _ = lowered_shape(d, lowering)
    dhat = np.empty((d.groups, rows, cols), np.float32)
    _check(_load().oracle_lower_data(ctypes.byref(d._c()), int(lowering), _p(x, ctypes.c_float),
                                     _p(dhat, ctypes.c_float)), "lower_data")
    return dhat


def lower_kernel(d: Dims, lowering: int, w) -> np.ndarray:
    """K^ as fp32 array (groups, cols, rcols)."""
    w = _f32(w)
    _expect(w, (d.O, d.C // d.groups, d.K, d.K), "w")
    _, cols, rcols = lowered_shape(d, lowering)
    khat = np.empty((d.groups, cols, rcols), np.float32)
    _check(_load().oracle_lower_kernel(ctypes.byref(d._c()), int(lowering), _p(w, ctypes.c_float),
                                       _p(khat, ctypes.c_float)), "lower_kernel")
    return khat


def multiply(d: Dims, lowering: int, dhat, khat) -> np.ndarray:
    """R^ = D^ K^ per group, fp64, shape (groups, rows, rcols)."""
    dhat, khat = _f32(dhat), _f32(khat)
    rows, cols, rcols = lowered_shape(d, lowering)
    _expect(dhat, (d.groups, rows, cols), "dhat")
    _expect(khat, (d.groups, cols, rcols), "khat")
    rhat = np.empty((d.groups, rows, rcols), np.float64)
    _check(_load().oracle_multiply(ctypes.byref(d._c()), int(lowering), _p(dhat, ctypes.c_float),
                                   _p(khat, ctypes.c_float), _p(rhat, ctypes.c_double)),
           "multiply")
    return rhat


def lift(d: Dims, lowering: int, rhat, bias=None) -> np.ndarray:
    """Lifting phase (+ bias): R^ -> y (fp64, NCHW)."""
    rhat = np.ascontiguousarray(rhat, np.float64)
    rows, _, rcols = lowered_shape(d, lowering)
    _expect(rhat, (d.groups, rows, rcols), "rhat")
    b = None if bias is None else _f32(bias)
    ho, wo = output_dims(d)
    y = np.empty((d.N, d.O, ho, wo), np.float64)
    _check(_load().oracle_lift(ctypes.byref(d._c()), int(lowering), _p(rhat, ctypes.c_double),
                               _p(b, ctypes.c_float), _p(y, ctypes.c_double)), "lift")
    return y


def conv_forward_lowered(d: Dims, lowering: int, x, w, bias=None) -> np.ndarray:
    """The paper's route: lower, multiply, lift."""
    return lift(d, lowering, multiply(d, lowering, lower_data(d, lowering, x),
                                      lower_kernel(d, lowering, w)), bias)


# ---- the layers between the convolutions: ReLU and max pooling (layers_oracle.c) ----------

class _Pool(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in ("N", "C", "H", "W", "K", "stride", "pad")]


@dataclass(frozen=True)
class PoolDims:
    """Max pooling over K x K windows of an N x C x H x W tensor (Caffe's output-size rule)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    stride: int
    pad: int = 0

    def _c(self) -> _Pool:
        return _Pool(self.N, self.C, self.H, self.W, self.K, self.stride, self.pad)


def pool_output_dims(d: PoolDims):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    _check(_load().oracle_pool_output_dims(ctypes.byref(d._c()), ctypes.byref(ho), ctypes.byref(wo)),
           "pool_output_dims")
    return ho.value, wo.value


def relu_forward(x) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    _check(_load().oracle_relu_forward(_p(x, ctypes.c_float), _p(y, ctypes.c_float),
                                       ctypes.c_int64(x.size)), "relu_forward")
    return y


def relu_backward(x, dy) -> np.ndarray:
    x, dy = _f32(x), _f32(dy)
    _expect(dy, x.shape, "dy")
    dx = np.empty_like(x)
    _check(_load().oracle_relu_backward(_p(x, ctypes.c_float), _p(dy, ctypes.c_float),
                                        _p(dx, ctypes.c_float), ctypes.c_int64(x.size)), "relu_backward")
    return dx


def maxpool_forward(d: PoolDims, x):
    """(y, argmax): fp32 values and int32 plane indices h*W + w of the chosen pixels."""
    x = _f32(x)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    ho, wo = pool_output_dims(d)
    y = np.empty((d.N, d.C, ho, wo), np.float32)
    am = np.empty((d.N, d.C, ho, wo), np.int32)
    _check(_load().oracle_maxpool_forward(ctypes.byref(d._c()), _p(x, ctypes.c_float),
                                          _p(y, ctypes.c_float), _p(am, ctypes.c_int32)), "maxpool_forward")
    return y, am


def maxpool_backward(d: PoolDims, dy, argmax) -> np.ndarray:
    dy = _f32(dy)
    argmax = np.ascontiguousarray(argmax, np.int32)
    ho, wo = pool_output_dims(d)
    _expect(dy, (d.N, d.C, ho, wo), "dy")
    _expect(argmax, (d.N, d.C, ho, wo), "argmax")
    dx = np.empty((d.N, d.C, d.H, d.W), np.float32)
    _check(_load().oracle_maxpool_backward(ctypes.byref(d._c()), _p(dy, ctypes.c_float),
                                           _p(argmax, ctypes.c_int32), _p(dx, ctypes.c_float)),
           "maxpool_backward")
    return dx


class _Lrn(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in ("N", "C", "H", "W", "size")] + \
               [(k, ctypes.c_double) for k in ("alpha", "beta", "k")]


@dataclass(frozen=True)
class LrnDims:
    """Local response normalisation across `size` channels of an N x C x H x W tensor."""
    N: int
    C: int
    H: int
    W: int
    size: int = 5
    alpha: float = 1e-4
    beta: float = 0.75
    k: float = 1.0

    def _c(self) -> _Lrn:
        return _Lrn(self.N, self.C, self.H, self.W, self.size, self.alpha, self.beta, self.k)


def lrn_forward(d: LrnDims, x) -> np.ndarray:
    x = _f32(x)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    y = np.empty_like(x)
    _check(_load().oracle_lrn_forward(ctypes.byref(d._c()), _p(x, ctypes.c_float), _p(y, ctypes.c_float)),
           "lrn_forward")
    return y


def lrn_backward(d: LrnDims, x, dy) -> np.ndarray:
    x, dy = _f32(x), _f32(dy)
    _expect(x, (d.N, d.C, d.H, d.W), "x")
    _expect(dy, x.shape, "dy")
    dx = np.empty_like(x)
    _check(_load().oracle_lrn_backward(ctypes.byref(d._c()), _p(x, ctypes.c_float), _p(dy, ctypes.c_float),
                                       _p(dx, ctypes.c_float)), "lrn_backward")
    return dx


def dropout(x, mask, scale) -> np.ndarray:
    """y = x * mask * scale (forward), or dx from dy (backward: the same map)."""
    x = _f32(x)
    mask = np.ascontiguousarray(mask, np.uint8)
    _expect(mask, x.shape, "mask")
    y = np.empty_like(x)
    _check(_load().oracle_dropout(_p(x, ctypes.c_float), _p(mask, ctypes.c_uint8), ctypes.c_double(scale),
                                  _p(y, ctypes.c_float), ctypes.c_int64(x.size)), "dropout")
    return y


def softmax_loss_forward(x, label):
    """(prob fp32 [N, C], loss as a Python float): softmax over the C scores of each image and the
    mean negative log-likelihood of the labels."""
    x = _f32(x)
    label = np.ascontiguousarray(label, np.int32)
    N, C = x.shape
    _expect(label, (N,), "label")
    prob = np.empty_like(x)
    loss = ctypes.c_double()
    _check(_load().oracle_softmax_loss_forward(N, C, _p(x, ctypes.c_float), _p(label, ctypes.c_int32),
                                               _p(prob, ctypes.c_float), ctypes.byref(loss)),
           "softmax_loss_forward")
    return prob, loss.value


def softmax_loss_backward(prob, label) -> np.ndarray:
    prob = _f32(prob)
    label = np.ascontiguousarray(label, np.int32)
    N, C = prob.shape
    _expect(label, (N,), "label")
    dx = np.empty_like(prob)
    _check(_load().oracle_softmax_loss_backward(N, C, _p(prob, ctypes.c_float), _p(label, ctypes.c_int32),
                                                _p(dx, ctypes.c_float)), "softmax_loss_backward")
    return dx
