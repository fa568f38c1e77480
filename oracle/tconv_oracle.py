"""ctypes front end of the CPU oracle (``tconv_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this module.  It never imports the
HIP package and shares nothing with it.

The arithmetic lives in the C file; this module only builds it with gcc,
marshals numpy arrays and allocates the outputs.  Operator definitions: paper
Sec. 3.1 (base operators, layers (iv) and (v)) and Sec. 3.3 (compound and
parallel definitions).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tconv_oracle.c")
_LIB = os.path.join(_HERE, "libtconv_oracle.so")

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
    stride_w: Optional[int] = None
    pad_w: Optional[int] = None
    dil_w: Optional[int] = None

    def c(self) -> _Shape:
        sw = self.stride if self.stride_w is None else self.stride_w
        pw = self.pad if self.pad_w is None else self.pad_w
        dw = self.dil if self.dil_w is None else self.dil_w
        return _Shape(self.N, self.C_in, self.H, self.W, self.C_out, self.KH, self.KW,
                      self.stride, sw, self.pad, pw, self.dil, dw)

    @property
    def K(self) -> int:
        return self.C_in * self.KH * self.KW


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no contraction, OpenMP).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.oracle_out_shape.argtypes = [ctypes.POINTER(_Shape), ctypes.POINTER(ctypes.c_int32),
                                         ctypes.POINTER(ctypes.c_int32)]
        lib.oracle_tconv_forward.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 10 + [ctypes.c_int]
        lib.oracle_tconv_backward_input.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 6
        lib.oracle_tconv_backward_weight.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 7
        lib.oracle_tconv_forward_mixed.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 4 + [ctypes.c_int]
        lib.oracle_tconv_backward_alpha_beta.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 5
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def out_shape(s: Shape):
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    cs = s.c()
    if _load().oracle_out_shape(ctypes.byref(cs), ctypes.byref(ho), ctypes.byref(wo)) != 0:
        raise ValueError("kernel larger than the padded input")
    return int(ho.value), int(wo.value)


def _f32(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _i32(a, shape):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.int32)
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def forward(s: Shape, mode: str, x, w_min=None, w_max=None, alpha=None, beta=None, out_bf16=False):
    """Returns dict(y, y_min, y_max, idx_min, idx_max); entries of a dead branch are None."""
    m = MODES[mode]
    ho, wo = out_shape(s)
    x = _f32(x, (s.N, s.C_in, s.H, s.W))
    wshape = (s.C_out, s.C_in, s.KH, s.KW)
    w_min, w_max = _f32(w_min, wshape), _f32(w_max, wshape)
    alpha, beta = _f32(alpha, (s.C_out,)), _f32(beta, (s.C_out,))
    oshape = (s.N, s.C_out, ho, wo)
    do_min, do_max = mode != "max", mode != "min"
    y = np.empty(oshape, np.float32)
    y_min = np.empty(oshape, np.float32) if do_min else None
    y_max = np.empty(oshape, np.float32) if do_max else None
    idx_min = np.empty(oshape, np.int32) if do_min else None
    idx_max = np.empty(oshape, np.int32) if do_max else None
    cs = s.c()
    rc = _load().oracle_tconv_forward(ctypes.byref(cs), m, _p(x), _p(w_min), _p(w_max), _p(alpha),
                                      _p(beta), _p(y), _p(y_min), _p(y_max), _p(idx_min),
                                      _p(idx_max), int(bool(out_bf16)))
    if rc != 0:
        raise ValueError(f"oracle_tconv_forward rejected the arguments (rc={rc})")
    return dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)


def backward_input(s: Shape, mode: str, gy, idx_min=None, idx_max=None, alpha=None, beta=None):
    """grad_x as float64 [N, C_in, H, W]."""
    ho, wo = out_shape(s)
    oshape = (s.N, s.C_out, ho, wo)
    gy = _f32(gy, oshape)
    idx_min, idx_max = _i32(idx_min, oshape), _i32(idx_max, oshape)
    alpha, beta = _f32(alpha, (s.C_out,)), _f32(beta, (s.C_out,))
    gx = np.empty((s.N, s.C_in, s.H, s.W), np.float64)
    cs = s.c()
    rc = _load().oracle_tconv_backward_input(ctypes.byref(cs), MODES[mode], _p(gy), _p(alpha),
                                             _p(beta), _p(idx_min), _p(idx_max), _p(gx))
    if rc != 0:
        raise ValueError(f"oracle_tconv_backward_input rejected the arguments (rc={rc})")
    return gx


def backward_weight(s: Shape, mode: str, gy, idx_min=None, idx_max=None, alpha=None, beta=None):
    """(grad_w_min, grad_w_max) as float64 OIHW; compound returns (grad_w, None); a dead branch is None."""
    ho, wo = out_shape(s)
    oshape = (s.N, s.C_out, ho, wo)
    gy = _f32(gy, oshape)
    idx_min, idx_max = _i32(idx_min, oshape), _i32(idx_max, oshape)
    alpha, beta = _f32(alpha, (s.C_out,)), _f32(beta, (s.C_out,))
    wshape = (s.C_out, s.C_in, s.KH, s.KW)
    g_min = np.empty(wshape, np.float64) if mode != "max" else None
    g_max = np.empty(wshape, np.float64) if mode in ("max", "parallel") else None
    cs = s.c()
    rc = _load().oracle_tconv_backward_weight(ctypes.byref(cs), MODES[mode], _p(gy), _p(alpha),
                                              _p(beta), _p(idx_min), _p(idx_max), _p(g_min),
                                              _p(g_max))
    if rc != 0:
        raise ValueError(f"oracle_tconv_backward_weight rejected the arguments (rc={rc})")
    return g_min, g_max


def backward_alpha_beta(s: Shape, mode: str, gy, y_min, y_max):
    """(grad_alpha, grad_beta) as float64 [C_out]: sums of gy*y_min and gy*y_max over (n, oh, ow)."""
    ho, wo = out_shape(s)
    oshape = (s.N, s.C_out, ho, wo)
    gy, y_min, y_max = _f32(gy, oshape), _f32(y_min, oshape), _f32(y_max, oshape)
    ga = np.empty((s.C_out,), np.float64)
    gb = np.empty((s.C_out,), np.float64)
    cs = s.c()
    rc = _load().oracle_tconv_backward_alpha_beta(ctypes.byref(cs), MODES[mode], _p(gy), _p(y_min),
                                                  _p(y_max), _p(ga), _p(gb))
    if rc != 0:
        raise ValueError(f"oracle_tconv_backward_alpha_beta rejected the arguments (rc={rc})")
    return ga, gb


def forward_mixed(s: Shape, layer: str, x, w, out_bf16: bool = False):
    """Mixed layers of Sec. 3.1: layer "minplus_max" = (iii), "maxplus_min" = (vi).
    Returns dict(y, idx) with idx the flattened winning tap k."""
    ho, wo = out_shape(s)
    x = _f32(x, (s.N, s.C_in, s.H, s.W))
    w = _f32(w, (s.C_out, s.C_in, s.KH, s.KW))
    y = np.empty((s.N, s.C_out, ho, wo), np.float32)
    idx = np.empty((s.N, s.C_out, ho, wo), np.int32)
    cs = s.c()
    outer_max = {"minplus_max": 1, "maxplus_min": 0}[layer]
    rc = _load().oracle_tconv_forward_mixed(ctypes.byref(cs), outer_max, _p(x), _p(w), _p(y), _p(idx),
                                            1 if out_bf16 else 0)
    if rc != 0:
        raise ValueError(f"oracle_tconv_forward_mixed rejected the arguments (rc={rc})")
    return dict(y=y, idx=idx)
