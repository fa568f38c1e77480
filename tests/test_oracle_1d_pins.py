"""Pins for the CPU oracle of the one-dimensional layers (oracle/tconv1d_oracle.c; paper Sec. 3.2, 1-D base
operators and layers (iii) - (vi), Sec. 3.3 compound / parallel), none of which re-types its loops: a
sliding-window formulation with numpy (windows materialised by stride tricks, numpy's first-occurrence argmin /
argmax), the already pinned two-dimensional oracle on the same data viewed as an H = 1 image, closed forms
(K = 1, zero kernels = library pooling), and invariants.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F
from numpy.lib.stride_tricks import sliding_window_view

from oracle import tconv1d_oracle as o1
from oracle import tconv_oracle as orc

MODES = ["max", "min", "compound", "parallel", "minplus_max", "maxplus_min"]
GEOS = [(3, 1, 1, 1), (3, 2, 1, 1), (5, 1, 2, 1), (3, 1, 2, 2), (8, 4, 3, 1), (1, 1, 0, 1), (4, 3, 0, 2)]  # K, stride, pad, dil


def _layer(seed, N=2, C=3, L=23, CO=4, K=3, stride=1, pad=1, dil=1, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        draw = lambda shape: rng.integers(-3, 4, shape).astype(np.float32)
    else:
        draw = lambda shape: rng.standard_normal(shape).astype(np.float32)
    s = o1.Shape1d(N, C, L, CO, K, stride, pad, dil)
    return s, draw((N, C, L)), draw((CO, C, K)), draw((CO, C, K)), rng


def _kernels(mode, w1, w2):
    if mode in ("max", "maxplus_min"):
        return None, w2
    if mode in ("min", "minplus_max"):
        return w1, None
    return (w1, w1) if mode == "compound" else (w1, w2)


def _windows(s, x, fill):
    """[N, C, L_out, K]: the K values under every output position, padding = fill."""
    xp = np.pad(x, ((0, 0), (0, 0), (s.pad, s.pad)), constant_values=fill)
    span = s.dil * (s.K - 1) + 1
    return sliding_window_view(xp, span, axis=2)[:, :, ::s.stride, ::s.dil]


def _reference(s, mode, x, w_min, w_max, alpha, beta):
    res = {}
    for side, w, inner_max in (("min", w_min, False), ("max", w_max, True)):
        if w is None:
            continue
        win = _windows(s, x, -np.inf if inner_max else np.inf)                      # [N, C, Lo, K]
        sums = win[:, None].astype(np.float32) + w[None, :, :, None, :]             # [N, CO, C, Lo, K]
        sums = np.ascontiguousarray(sums.transpose(0, 1, 3, 2, 4))                  # [N, CO, Lo, C, K]
        outer_max = (mode == "minplus_max") if side == "min" else (mode != "maxplus_min")
        if outer_max == inner_max:      # one extremum over all C*K taps, first occurrence = lowest k
            flat = sums.reshape(*sums.shape[:3], -1)
            k = flat.argmax(-1) if inner_max else flat.argmin(-1)
            v = np.take_along_axis(flat, k[..., None], -1)[..., 0]
        else:                           # mixed: taps first, then channels
            t = sums.argmax(-1) if inner_max else sums.argmin(-1)                   # [N, CO, Lo, C]
            vc = np.take_along_axis(sums, t[..., None], -1)[..., 0]
            c = vc.argmax(-1) if outer_max else vc.argmin(-1)
            v = np.take_along_axis(vc, c[..., None], -1)[..., 0]
            k = c * s.K + np.take_along_axis(t, c[..., None], -1)[..., 0]
        res["y_" + side], res["idx_" + side] = v.astype(np.float32), k.astype(np.int32)
    if "y_min" in res and "y_max" in res:
        a = np.ones(s.C_out, np.float32) if alpha is None else alpha
        b = np.ones(s.C_out, np.float32) if beta is None else beta
        res["y"] = ((a[None, :, None] * res["y_min"]).astype(np.float32)
                    + (b[None, :, None] * res["y_max"]).astype(np.float32)).astype(np.float32)
    else:
        res["y"] = res.get("y_min", res.get("y_max"))
    return res


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("K,stride,pad,dil", GEOS)
def test_sliding_window_formulation(mode, integer, K, stride, pad, dil):
    s, x, w1, w2, rng = _layer(3 + K, K=K, stride=stride, pad=pad, dil=dil, integer=integer)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    a = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    b = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    r = o1.forward(s, mode, x, wmn, wmx, a, b)
    ref = _reference(s, mode, x, wmn, wmx, a, b)
    for k, v in ref.items():
        assert np.array_equal(r[k], v), k


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("K,stride,pad,dil", GEOS)
def test_equals_two_dimensional_oracle_on_a_one_row_image(mode, K, stride, pad, dil):
    """x [N, C, L] viewed as [N, C, 1, L] with a 1 x K kernel is the same layer: values, winners (the flattened
    tap k = c*K + i is the same number) and gradients."""
    s, x, w1, w2, rng = _layer(11, K=K, stride=stride, pad=pad, dil=dil, integer=True)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    a = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    b = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    r = o1.forward(s, mode, x, wmn, wmx, a, b)
    s2 = orc.Shape(s.N, s.C_in, 1, s.L, s.C_out, 1, K, stride=1, pad=0, dil=1, stride_w=stride, pad_w=pad, dil_w=dil)
    x2 = x[:, :, None, :]
    k2 = lambda w: None if w is None else w[:, :, None, :]
    gy = rng.standard_normal(r["y"].shape).astype(np.float32)
    if mode in ("minplus_max", "maxplus_min"):
        side = "min" if mode == "minplus_max" else "max"
        f = orc.forward_mixed(s2, mode, x2, k2(wmn if side == "min" else wmx))
        assert np.array_equal(r["y"], f["y"][:, :, 0]) and np.array_equal(r["idx_" + side], f["idx"][:, :, 0])
        bmode, kw = side, {"idx_" + side: f["idx"]}
    else:
        f = orc.forward(s2, mode, x2, w_min=k2(wmn), w_max=k2(wmx), alpha=a, beta=b)
        for k in ("y", "y_min", "y_max", "idx_min", "idx_max"):
            assert (r[k] is None and f[k] is None) or np.array_equal(r[k], f[k][:, :, 0]), k
        bmode, kw = mode, dict(idx_min=f["idx_min"], idx_max=f["idx_max"], alpha=a, beta=b)
    g = o1.backward(s, mode, gy, r["idx_min"], r["idx_max"], a, b)
    gx = orc.backward_input(s2, bmode, gy[:, :, None, :], **kw)
    g1, g2 = orc.backward_weight(s2, bmode, gy[:, :, None, :], **kw)
    assert np.allclose(g["grad_x"], gx[:, :, 0], rtol=0, atol=1e-12)
    if g["grad_w_min"] is not None:
        assert np.allclose(g["grad_w_min"], g1[:, :, 0], rtol=0, atol=1e-12)
    if g["grad_w_max"] is not None:
        assert np.allclose(g["grad_w_max"], g2[:, :, 0], rtol=0, atol=1e-12)


def test_zero_kernel_is_pooling_then_channel_reduction():
    s, x, _, _, _ = _layer(5, C=4, L=30, K=3, stride=2, pad=1)
    z = np.zeros((s.C_out, s.C_in, 3), np.float32)
    xt = torch.from_numpy(x)
    mx = F.max_pool1d(xt, 3, stride=2, padding=1)
    mn = -F.max_pool1d(-xt, 3, stride=2, padding=1)
    for mode, ref in (("max", mx.amax(1)), ("min", mn.amin(1)), ("minplus_max", mn.amax(1)), ("maxplus_min", mx.amin(1))):
        wmn, wmx = _kernels(mode, z, z)
        y = o1.forward(s, mode, x, wmn, wmx)["y"]
        for co in range(s.C_out):
            assert np.array_equal(y[:, co], ref.numpy()), mode


def test_invariants():
    s, x, w1, w2, rng = _layer(9, integer=False, K=5, pad=2)
    # duality: min-layer(x, w) = -max-layer(-x, -w), winners included
    a = o1.forward(s, "min", x, w1, None)
    b = o1.forward(s, "max", -x, None, -w1)
    assert np.array_equal(a["y"], -b["y"]) and np.array_equal(a["idx_min"], b["idx_max"])
    # every index points into the window and reproduces the value
    r = o1.forward(s, "max", x, None, w2)
    c, i = np.divmod(r["idx_max"], s.K)
    pos = np.arange(s.L_out)[None, None, :] * s.stride - s.pad + i * s.dil
    assert (pos >= 0).all() and (pos < s.L).all()
    n_i = np.arange(s.N)[:, None, None]
    co_i = np.arange(s.C_out)[None, :, None]
    assert np.array_equal(r["y"], x[n_i, c, pos] + w2[co_i, c, i])
    # gradient mass: each branch deposits its scaled gradient exactly once
    al, be = rng.uniform(-1, 1, s.C_out).astype(np.float32), rng.uniform(-1, 1, s.C_out).astype(np.float32)
    p = o1.forward(s, "parallel", x, w1, w2, al, be)
    gy = rng.standard_normal(p["y"].shape).astype(np.float32)
    g = o1.backward(s, "parallel", gy, p["idx_min"], p["idx_max"], al, be)
    tot = ((al.astype(np.float64) + be.astype(np.float64))[None, :, None] * gy).sum()
    assert abs(g["grad_x"].sum() - tot) < 1e-9
    assert abs(g["grad_w_min"].sum() - (al.astype(np.float64)[None, :, None] * gy).sum()) < 1e-9


def test_rejects_window_in_padding():
    with pytest.raises(ValueError):
        o1.forward(o1.Shape1d(1, 1, 8, 1, 3, 1, 3, 1), "max", np.zeros((1, 1, 8), np.float32), None,
                   np.zeros((1, 1, 3), np.float32))
