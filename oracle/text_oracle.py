"""ctypes front end of the extension oracle (``text_oracle.c``): zero padding, the layer epilogue (bias, folded
batch-norm affine, residual add) and the half-precision contract.

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.  It never imports the HIP package and shares nothing with it; the arithmetic lives in the C file
(paper Sec. 3.1 / 3.3 operators, App. A.1.1 unfold formulation for the padding, App. A.2 and Sec. 5 for the epilogue).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "text_oracle.c")
_LIB = os.path.join(_HERE, "libtext_oracle.so")

MODES = {"max": 0, "min": 1, "compound": 2, "parallel": 3}


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "C_in", "H", "W", "C_out", "KH", "KW",
        "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


@dataclass(frozen=True)
class Shape:
    N: int
    C_in: int
    H: int
    W: int
    C_out: int
    KH: int
    KW: int
    stride: int = 1
    pad: int = 0
    dil: int = 1

    def c(self) -> _Shape:
        return _Shape(self.N, self.C_in, self.H, self.W, self.C_out, self.KH, self.KW,
                      self.stride, self.stride, self.pad, self.pad, self.dil, self.dil)

    @property
    def out_hw(self):
        ho = (self.H + 2 * self.pad - self.dil * (self.KH - 1) - 1) // self.stride + 1
        wo = (self.W + 2 * self.pad - self.dil * (self.KW - 1) - 1) // self.stride + 1
        return ho, wo


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-Wall",
               "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P, S = ctypes.c_void_p, ctypes.POINTER(_Shape)
        lib.text_forward.argtypes = [S, ctypes.c_int, ctypes.c_int] + [P] * 14
        lib.text_backward.argtypes = [S, ctypes.c_int] + [P] * 8
        lib.text_backward_bias.argtypes = [S, P, P]
        lib.text_forward_f16.argtypes = [S, ctypes.c_int, ctypes.c_int] + [P] * 10
        lib.text_double_to_half.argtypes = [ctypes.c_double]
        lib.text_double_to_half.restype = ctypes.c_uint16
        lib.text_half_to_double.argtypes = [ctypes.c_uint16]
        lib.text_half_to_double.restype = ctypes.c_double
        _lib = lib
    return _lib


def _arr(a, dt, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=dt)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def double_to_half(v: float) -> int:
    return int(_load().text_double_to_half(float(v)))


def half_to_double(h: int) -> float:
    return float(_load().text_half_to_double(int(h)))


def forward(s: Shape, mode: str, x, w_min=None, w_max=None, alpha=None, beta=None, pad_zero=False, bias=None,
            scale=None, shift=None, residual=None):
    """dict(y, y_min, y_max, idx_min, idx_max); y carries the epilogue, the branch outputs and indices do not."""
    ho, wo = s.out_hw
    oshape, wshape = (s.N, s.C_out, ho, wo), (s.C_out, s.C_in, s.KH, s.KW)
    x = _arr(x, np.float32, (s.N, s.C_in, s.H, s.W))
    w_min, w_max = _arr(w_min, np.float32, wshape), _arr(w_max, np.float32, wshape)
    vec = lambda a: _arr(a, np.float32, (s.C_out,))
    alpha, beta, bias, scale, shift = vec(alpha), vec(beta), vec(bias), vec(scale), vec(shift)
    residual = _arr(residual, np.float32, oshape)
    do_min, do_max = mode != "max", mode != "min"
    y = np.empty(oshape, np.float32)
    y_min = np.empty(oshape, np.float32) if do_min else None
    y_max = np.empty(oshape, np.float32) if do_max else None
    idx_min = np.empty(oshape, np.int32) if do_min else None
    idx_max = np.empty(oshape, np.int32) if do_max else None
    cs = s.c()
    rc = _load().text_forward(ctypes.byref(cs), MODES[mode], int(bool(pad_zero)), _p(x), _p(w_min), _p(w_max),
                              _p(alpha), _p(beta), _p(bias), _p(scale), _p(shift), _p(residual), _p(y), _p(y_min),
                              _p(y_max), _p(idx_min), _p(idx_max))
    if rc != 0:
        raise ValueError(f"text_forward rejected the arguments (rc={rc})")
    return dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)


def backward(s: Shape, mode: str, gy, idx_min=None, idx_max=None, alpha=None, beta=None):
    """dict(grad_x, grad_w_min, grad_w_max) as float64; winners in the padding feed the kernel gradient only."""
    ho, wo = s.out_hw
    oshape, wshape = (s.N, s.C_out, ho, wo), (s.C_out, s.C_in, s.KH, s.KW)
    gy = _arr(gy, np.float32, oshape)
    idx_min, idx_max = _arr(idx_min, np.int32, oshape), _arr(idx_max, np.int32, oshape)
    alpha, beta = _arr(alpha, np.float32, (s.C_out,)), _arr(beta, np.float32, (s.C_out,))
    gx = np.empty((s.N, s.C_in, s.H, s.W), np.float64)
    g_min = np.empty(wshape, np.float64) if mode != "max" else None
    g_max = np.empty(wshape, np.float64) if mode in ("max", "parallel") else None
    cs = s.c()
    rc = _load().text_backward(ctypes.byref(cs), MODES[mode], _p(gy), _p(alpha), _p(beta), _p(idx_min), _p(idx_max),
                               _p(gx), _p(g_min), _p(g_max))
    if rc != 0:
        raise ValueError(f"text_backward rejected the arguments (rc={rc})")
    return dict(grad_x=gx, grad_w_min=g_min, grad_w_max=g_max)


def backward_bias(s: Shape, gy):
    ho, wo = s.out_hw
    gy = _arr(gy, np.float32, (s.N, s.C_out, ho, wo))
    gb = np.empty((s.C_out,), np.float64)
    cs = s.c()
    if _load().text_backward_bias(ctypes.byref(cs), _p(gy), _p(gb)) != 0:
        raise ValueError("text_backward_bias rejected the arguments")
    return gb


def forward_f16(s: Shape, mode: str, x, w_min=None, w_max=None, alpha=None, beta=None, pad_zero=False):
    """Half-precision contract.  x and the kernels are numpy float16 arrays (or anything exactly representable);
    returns float16 arrays y, y_min, y_max and int32 indices."""
    ho, wo = s.out_hw
    oshape, wshape = (s.N, s.C_out, ho, wo), (s.C_out, s.C_in, s.KH, s.KW)
    h = lambda a, shp: None if a is None else np.ascontiguousarray(np.asarray(a, np.float16).reshape(shp))
    x, w_min, w_max = h(x, (s.N, s.C_in, s.H, s.W)), h(w_min, wshape), h(w_max, wshape)
    alpha, beta = _arr(alpha, np.float32, (s.C_out,)), _arr(beta, np.float32, (s.C_out,))
    do_min, do_max = mode != "max", mode != "min"
    y = np.empty(oshape, np.float16)
    y_min = np.empty(oshape, np.float16) if do_min else None
    y_max = np.empty(oshape, np.float16) if do_max else None
    idx_min = np.empty(oshape, np.int32) if do_min else None
    idx_max = np.empty(oshape, np.int32) if do_max else None
    cs = s.c()
    rc = _load().text_forward_f16(ctypes.byref(cs), MODES[mode], int(bool(pad_zero)), _p(x), _p(w_min), _p(w_max),
                                  _p(alpha), _p(beta), _p(y), _p(y_min), _p(y_max), _p(idx_min), _p(idx_max))
    if rc != 0:
        raise ValueError(f"text_forward_f16 rejected the arguments (rc={rc})")
    return dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
