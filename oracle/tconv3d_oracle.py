"""ctypes front end of the CPU oracle of the three-dimensional layers (``tconv3d_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg
may import this module.  It never imports the HIP package and shares nothing with it.  Layer definitions:
paper Sec. 3.2, three-dimensional base operators and layers (iii) - (vi); Sec. 3.3 compound / parallel.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tconv3d_oracle.c")
_LIB = os.path.join(_HERE, "libtconv3d_oracle.so")

MODES = {"max": 0, "min": 1, "compound": 2, "parallel": 3, "minplus_max": 4, "maxplus_min": 5}


class _Shape3d(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C_in", "D", "H", "W", "C_out", "KD", "KH", "KW")] + \
               [("stride", ctypes.c_int32 * 3), ("pad", ctypes.c_int32 * 3), ("dil", ctypes.c_int32 * 3)]


@dataclass(frozen=True)
class Shape3d:
    N: int
    C_in: int
    D: int
    H: int
    W: int
    C_out: int
    KD: int
    KH: int
    KW: int
    stride: Tuple[int, int, int] = (1, 1, 1)
    pad: Tuple[int, int, int] = (0, 0, 0)
    dil: Tuple[int, int, int] = (1, 1, 1)

    def c(self) -> _Shape3d:
        a3 = ctypes.c_int32 * 3
        return _Shape3d(self.N, self.C_in, self.D, self.H, self.W, self.C_out, self.KD, self.KH, self.KW,
                        a3(*self.stride), a3(*self.pad), a3(*self.dil))

    @property
    def out(self):
        return tuple((n + 2 * p - d * (k - 1) - 1) // s + 1 for n, k, s, p, d in
                     zip((self.D, self.H, self.W), (self.KD, self.KH, self.KW), self.stride, self.pad, self.dil))


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
        lib.oracle_tconv3d_forward.argtypes = [ctypes.POINTER(_Shape3d), ctypes.c_int] + [P] * 10
        lib.oracle_tconv3d_backward.argtypes = [ctypes.POINTER(_Shape3d), ctypes.c_int] + [P] * 8
        lib.oracle_tconv3d_forward.restype = ctypes.c_int
        lib.oracle_tconv3d_backward.restype = ctypes.c_int
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


def _sides(mode):
    return mode not in ("max", "maxplus_min"), mode not in ("min", "minplus_max")


def forward(s: Shape3d, mode: str, x, w_min=None, w_max=None, alpha=None, beta=None):
    """dict(y, y_min, y_max, idx_min, idx_max); entries of a side the mode does not have are None."""
    do_min, do_max = _sides(mode)
    oshape, wshape = (s.N, s.C_out) + s.out, (s.C_out, s.C_in, s.KD, s.KH, s.KW)
    x = _arr(x, (s.N, s.C_in, s.D, s.H, s.W))
    w_min, w_max = _arr(w_min, wshape), _arr(w_max, wshape)
    alpha, beta = _arr(alpha, (s.C_out,)), _arr(beta, (s.C_out,))
    y = np.empty(oshape, np.float32)
    ymn = np.empty(oshape, np.float32) if do_min else None
    ymx = np.empty(oshape, np.float32) if do_max else None
    imn = np.empty(oshape, np.int32) if do_min else None
    imx = np.empty(oshape, np.int32) if do_max else None
    cs = s.c()
    rc = _load().oracle_tconv3d_forward(ctypes.byref(cs), MODES[mode], _p(x), _p(w_min), _p(w_max), _p(alpha),
                                        _p(beta), _p(y), _p(ymn), _p(ymx), _p(imn), _p(imx))
    if rc != 0:
        raise ValueError(f"oracle_tconv3d_forward rejected the arguments (rc={rc})")
    return dict(y=y, y_min=ymn, y_max=ymx, idx_min=imn, idx_max=imx)


def backward(s: Shape3d, mode: str, gy, idx_min=None, idx_max=None, alpha=None, beta=None):
    """dict of float64 gradients grad_x, grad_w_min, grad_w_max (compound: grad_w_min holds the one tensor)."""
    do_min, do_max = _sides(mode)
    oshape, wshape = (s.N, s.C_out) + s.out, (s.C_out, s.C_in, s.KD, s.KH, s.KW)
    gy = _arr(gy, oshape)
    idx_min, idx_max = _arr(idx_min, oshape, np.int32), _arr(idx_max, oshape, np.int32)
    alpha, beta = _arr(alpha, (s.C_out,)), _arr(beta, (s.C_out,))
    gx = np.empty((s.N, s.C_in, s.D, s.H, s.W), np.float64)
    g1 = np.empty(wshape, np.float64) if do_min else None
    g2 = np.empty(wshape, np.float64) if (do_max and mode != "compound") else None
    cs = s.c()
    rc = _load().oracle_tconv3d_backward(ctypes.byref(cs), MODES[mode], _p(gy), _p(alpha), _p(beta), _p(idx_min),
                                         _p(idx_max), _p(gx), _p(g1), _p(g2))
    if rc != 0:
        raise ValueError(f"oracle_tconv3d_backward rejected the arguments (rc={rc})")
    return dict(grad_x=gx, grad_w_min=g1, grad_w_max=g2)
