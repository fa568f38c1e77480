"""ctypes front end of the CPU oracle of the depthwise tropical layer (``tdw_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module.  It never imports the HIP package and shares nothing with it.
The arithmetic lives in the C file; this module builds it with gcc, marshals numpy arrays and allocates
the outputs.  Layer definition: paper Sec. 3.1 base operators applied per channel, combined as in
Sec. 3.5 / 3.6; used by the MobileNetV2 variants of Sec. 5.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .tconv_oracle import MODES, Shape, _Shape

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tdw_oracle.c")
_LIB = os.path.join(_HERE, "libtdw_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no contraction, OpenMP).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.oracle_tdw_forward.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 8
        lib.oracle_tdw_backward.argtypes = [ctypes.POINTER(_Shape), ctypes.c_int] + [P] * 11
        lib.oracle_tdw_forward.restype = ctypes.c_int
        lib.oracle_tdw_backward.restype = ctypes.c_int
        _lib = lib
    return _lib


def _arr(a, shape, dt=np.float32):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dt)
    assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def out_hw(s: Shape):
    c = s.c()
    ho = (s.H + 2 * c.pad_h - c.dil_h * (s.KH - 1) - 1) // c.stride_h + 1
    wo = (s.W + 2 * c.pad_w - c.dil_w * (s.KW - 1) - 1) // c.stride_w + 1
    return ho, wo


def forward(s: Shape, mode: str, x, w_min=None, w_max=None, alpha=None, beta=None, taps: bool = False):
    """y [N, C_out, H_out, W_out] fp32.  Kernels [C_out, 1, KH, KW]; alpha, beta [C_out] or None (ones).
    taps=True: returns (y, tap_min, tap_max), the winning taps t = i*KW + j (int32; None for a dead branch)."""
    ho, wo = out_hw(s)
    wshape = (s.C_out, 1, s.KH, s.KW)
    x = _arr(x, (s.N, s.C_in, s.H, s.W))
    w_min, w_max = _arr(w_min, wshape), _arr(w_max, wshape)
    alpha, beta = _arr(alpha, (s.C_out,)), _arr(beta, (s.C_out,))
    y = np.empty((s.N, s.C_out, ho, wo), np.float32)
    tmin = np.empty(y.shape, np.int32) if (taps and mode != "max") else None
    tmax = np.empty(y.shape, np.int32) if (taps and mode != "min") else None
    cs = s.c()
    rc = _load().oracle_tdw_forward(ctypes.byref(cs), MODES[mode], _p(x), _p(w_min), _p(w_max),
                                    _p(alpha), _p(beta), _p(y), _p(tmin), _p(tmax))
    if rc != 0:
        raise ValueError(f"oracle_tdw_forward rejected the arguments (rc={rc})")
    return (y, tmin, tmax) if taps else y


def backward(s: Shape, mode: str, x, gy, w_min=None, w_max=None, alpha=None, beta=None):
    """dict of float64 gradients: grad_x, grad_w_min, grad_w_max (compound: grad_w_min holds the one tensor,
    grad_w_max is None), grad_alpha, grad_beta (None in the max / min layers)."""
    ho, wo = out_hw(s)
    wshape = (s.C_out, 1, s.KH, s.KW)
    x = _arr(x, (s.N, s.C_in, s.H, s.W))
    gy = _arr(gy, (s.N, s.C_out, ho, wo))
    w_min, w_max = _arr(w_min, wshape), _arr(w_max, wshape)
    alpha, beta = _arr(alpha, (s.C_out,)), _arr(beta, (s.C_out,))
    two = mode in ("compound", "parallel")
    gx = np.empty(x.shape, np.float64)
    g1 = np.empty(wshape, np.float64) if mode != "max" else None
    g2 = np.empty(wshape, np.float64) if mode in ("max", "parallel") else None
    ga = np.empty((s.C_out,), np.float64) if two else None
    gb = np.empty((s.C_out,), np.float64) if two else None
    cs = s.c()
    rc = _load().oracle_tdw_backward(ctypes.byref(cs), MODES[mode], _p(x), _p(w_min), _p(w_max),
                                     _p(alpha), _p(beta), _p(gy), _p(gx), _p(g1), _p(g2), _p(ga), _p(gb))
    if rc != 0:
        raise ValueError(f"oracle_tdw_backward rejected the arguments (rc={rc})")
    return dict(grad_x=gx, grad_w_min=g1, grad_w_max=g2, grad_alpha=ga, grad_beta=gb)
