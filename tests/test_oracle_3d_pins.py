"""Pins for the CPU oracle of the three-dimensional layers (oracle/tconv3d_oracle.c; paper Sec. 3.2, 3-D base
operators and layers (iii) - (vi), Sec. 3.3 compound / parallel), none of which re-types its loops: a
sliding-window formulation with numpy stride tricks, the already pinned two-dimensional oracle on volumes of
depth 1 and on volumes whose whole depth is one window (depth taps become channels), library pooling for zero
kernels, and invariants.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F
from numpy.lib.stride_tricks import sliding_window_view

from oracle import tconv3d_oracle as o3
from oracle import tconv_oracle as orc

MODES = ["max", "min", "compound", "parallel", "minplus_max", "maxplus_min"]
# (KD, KH, KW), stride, pad, dil
GEOS = [((3, 3, 3), (1, 1, 1), (1, 1, 1), (1, 1, 1)), ((3, 3, 3), (2, 2, 2), (1, 1, 1), (1, 1, 1)),
        ((2, 3, 1), (1, 2, 1), (1, 0, 0), (1, 1, 1)), ((3, 2, 3), (1, 1, 2), (2, 1, 2), (2, 1, 2)),
        ((1, 1, 1), (1, 1, 1), (0, 0, 0), (1, 1, 1))]


def _layer(seed, N=2, C=3, D=6, H=7, W=8, CO=3, k=(3, 3, 3), stride=(1, 1, 1), pad=(1, 1, 1), dil=(1, 1, 1), integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        draw = lambda shape: rng.integers(-3, 4, shape).astype(np.float32)
    else:
        draw = lambda shape: rng.standard_normal(shape).astype(np.float32)
    s = o3.Shape3d(N, C, D, H, W, CO, k[0], k[1], k[2], stride, pad, dil)
    return s, draw((N, C, D, H, W)), draw((CO, C) + tuple(k)), draw((CO, C) + tuple(k)), rng


def _kernels(mode, w1, w2):
    if mode in ("max", "maxplus_min"):
        return None, w2
    if mode in ("min", "minplus_max"):
        return w1, None
    return (w1, w1) if mode == "compound" else (w1, w2)


def _windows(s, x, fill):
    """[N, C, Do, Ho, Wo, KD*KH*KW]: the values under every output position in tap order, padding = fill."""
    pd, ph, pw = s.pad
    xp = np.pad(x, ((0, 0), (0, 0), (pd, pd), (ph, ph), (pw, pw)), constant_values=fill)
    span = tuple(d * (k - 1) + 1 for d, k in zip(s.dil, (s.KD, s.KH, s.KW)))
    v = sliding_window_view(xp, span, axis=(2, 3, 4))
    v = v[:, :, ::s.stride[0], ::s.stride[1], ::s.stride[2], ::s.dil[0], ::s.dil[1], ::s.dil[2]]
    return np.ascontiguousarray(v).reshape(*v.shape[:5], -1)


def _reference(s, mode, x, w_min, w_max, alpha, beta):
    res = {}
    KK = s.KD * s.KH * s.KW
    for side, w, inner_max in (("min", w_min, False), ("max", w_max, True)):
        if w is None:
            continue
        win = _windows(s, x, -np.inf if inner_max else np.inf)                              # [N, C, Do, Ho, Wo, KK]
        sums = win[:, None].astype(np.float32) + w.reshape(1, s.C_out, s.C_in, 1, 1, 1, KK)  # [N, CO, C, Do, Ho, Wo, KK]
        sums = np.ascontiguousarray(np.moveaxis(sums, 2, 5))                                 # [N, CO, Do, Ho, Wo, C, KK]
        outer_max = (mode == "minplus_max") if side == "min" else (mode != "maxplus_min")
        if outer_max == inner_max:
            flat = sums.reshape(*sums.shape[:5], -1)
            k = flat.argmax(-1) if inner_max else flat.argmin(-1)
            v = np.take_along_axis(flat, k[..., None], -1)[..., 0]
        else:
            t = sums.argmax(-1) if inner_max else sums.argmin(-1)
            vc = np.take_along_axis(sums, t[..., None], -1)[..., 0]
            c = vc.argmax(-1) if outer_max else vc.argmin(-1)
            v = np.take_along_axis(vc, c[..., None], -1)[..., 0]
            k = c * KK + np.take_along_axis(t, c[..., None], -1)[..., 0]
        res["y_" + side], res["idx_" + side] = v.astype(np.float32), k.astype(np.int32)
    if "y_min" in res and "y_max" in res:
        a = np.ones(s.C_out, np.float32) if alpha is None else alpha
        b = np.ones(s.C_out, np.float32) if beta is None else beta
        e = (None, slice(None), None, None, None)
        res["y"] = ((a[e] * res["y_min"]).astype(np.float32) + (b[e] * res["y_max"]).astype(np.float32)).astype(np.float32)
    else:
        res["y"] = res.get("y_min", res.get("y_max"))
    return res


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("k,stride,pad,dil", GEOS)
def test_sliding_window_formulation(mode, integer, k, stride, pad, dil):
    s, x, w1, w2, rng = _layer(3, k=k, stride=stride, pad=pad, dil=dil, integer=integer)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    a = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    b = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    r = o3.forward(s, mode, x, wmn, wmx, a, b)
    ref = _reference(s, mode, x, wmn, wmx, a, b)
    for key, v in ref.items():
        assert np.array_equal(r[key], v), key


@pytest.mark.parametrize("mode", MODES)
def test_depth_one_is_the_two_dimensional_layer(mode):
    """D = KD = 1: the pinned two-dimensional oracle, winners and gradients included."""
    s, x, w1, w2, rng = _layer(5, D=1, k=(1, 3, 3), stride=(1, 2, 1), pad=(0, 1, 1), integer=True)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    a = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    b = rng.uniform(-1, 1, s.C_out).astype(np.float32) if two else None
    r = o3.forward(s, mode, x, wmn, wmx, a, b)
    s2 = orc.Shape(s.N, s.C_in, s.H, s.W, s.C_out, 3, 3, stride=2, pad=1, dil=1, stride_w=1, pad_w=1, dil_w=1)
    sq = lambda v: None if v is None else v[:, :, 0]
    gy = rng.standard_normal(r["y"].shape).astype(np.float32)
    if mode in ("minplus_max", "maxplus_min"):
        side = "min" if mode == "minplus_max" else "max"
        f = orc.forward_mixed(s2, mode, sq(x), sq(wmn if side == "min" else wmx))
        assert np.array_equal(sq(r["y"]), f["y"]) and np.array_equal(sq(r["idx_" + side]), f["idx"])
        bmode, kw = side, {"idx_" + side: f["idx"]}
    else:
        f = orc.forward(s2, mode, sq(x), w_min=sq(wmn), w_max=sq(wmx), alpha=a, beta=b)
        for key in ("y", "y_min", "y_max", "idx_min", "idx_max"):
            assert (r[key] is None and f[key] is None) or np.array_equal(sq(r[key]), f[key]), key
        bmode, kw = mode, dict(idx_min=f["idx_min"], idx_max=f["idx_max"], alpha=a, beta=b)
    g = o3.backward(s, mode, gy, r["idx_min"], r["idx_max"], a, b)
    gx = orc.backward_input(s2, bmode, sq(gy), **kw)
    g1, g2 = orc.backward_weight(s2, bmode, sq(gy), **kw)
    assert np.allclose(sq(g["grad_x"]), gx, rtol=0, atol=1e-12)
    if g["grad_w_min"] is not None:
        assert np.allclose(sq(g["grad_w_min"]), g1, rtol=0, atol=1e-12)
    if g["grad_w_max"] is not None:
        assert np.allclose(sq(g["grad_w_max"]), g2, rtol=0, atol=1e-12)


@pytest.mark.parametrize("mode", ["max", "min", "compound", "parallel"])
def test_full_depth_window_folds_depth_into_channels(mode):
    """KD = D without depth padding: one output depth, and the taps (c, a) of a full-window layer are the
    C_in*D channels of a two-dimensional layer on x viewed as [N, C_in*D, H, W] - same flattened k."""
    s, x, w1, w2, rng = _layer(7, D=3, k=(3, 3, 3), pad=(0, 1, 1))
    wmn, wmx = _kernels(mode, w1, w2)
    r = o3.forward(s, mode, x, wmn, wmx)
    s2 = orc.Shape(s.N, s.C_in * 3, s.H, s.W, s.C_out, 3, 3, stride=1, pad=1, dil=1)
    fold = lambda v: None if v is None else v.reshape(v.shape[0], -1, *v.shape[3:])
    f = orc.forward(s2, mode, fold(x), w_min=fold(wmn), w_max=fold(wmx))
    for key in ("y", "idx_min", "idx_max"):
        assert (r[key] is None and f[key] is None) or np.array_equal(r[key][:, :, 0], f[key]), key


def test_zero_kernel_is_pooling_then_channel_reduction():
    s, x, _, _, _ = _layer(9, C=4, stride=(2, 1, 2))
    z = np.zeros((s.C_out, s.C_in, 3, 3, 3), np.float32)
    xt = torch.from_numpy(x)
    mx = F.max_pool3d(xt, 3, stride=(2, 1, 2), padding=1)
    mn = -F.max_pool3d(-xt, 3, stride=(2, 1, 2), padding=1)
    for mode, ref in (("max", mx.amax(1)), ("min", mn.amin(1)), ("minplus_max", mn.amax(1)), ("maxplus_min", mx.amin(1))):
        wmn, wmx = _kernels(mode, z, z)
        y = o3.forward(s, mode, x, wmn, wmx)["y"]
        for co in range(s.C_out):
            assert np.array_equal(y[:, co], ref.numpy()), mode


def test_invariants():
    s, x, w1, w2, rng = _layer(11, stride=(1, 2, 1), pad=(1, 1, 0))
    a = o3.forward(s, "min", x, w1, None)
    b = o3.forward(s, "max", -x, None, -w1)
    assert np.array_equal(a["y"], -b["y"]) and np.array_equal(a["idx_min"], b["idx_max"])
    al, be = rng.uniform(-1, 1, s.C_out).astype(np.float32), rng.uniform(-1, 1, s.C_out).astype(np.float32)
    p = o3.forward(s, "parallel", x, w1, w2, al, be)
    gy = rng.standard_normal(p["y"].shape).astype(np.float32)
    g = o3.backward(s, "parallel", gy, p["idx_min"], p["idx_max"], al, be)
    e = (None, slice(None), None, None, None)
    tot = ((al.astype(np.float64) + be.astype(np.float64))[e] * gy).sum()
    assert abs(g["grad_x"].sum() - tot) < 1e-9
    assert abs(g["grad_w_max"].sum() - (be.astype(np.float64)[e] * gy).sum()) < 1e-9
    # the winner reproduces the value
    r = o3.forward(s, "max", x, None, w2)
    KK = 27
    c, t = np.divmod(r["idx_max"], KK)
    ta, ti, tj = t // 9, (t // 3) % 3, t % 3
    Do, Ho, Wo = s.out
    od, oh, ow = np.meshgrid(np.arange(Do), np.arange(Ho), np.arange(Wo), indexing="ij")
    idd, ihh, iww = od[None, None] * 1 - 1 + ta, oh[None, None] * 2 - 1 + ti, ow[None, None] * 1 - 0 + tj
    n_i = np.arange(s.N)[:, None, None, None, None]
    co_i = np.arange(s.C_out)[None, :, None, None, None]
    assert np.array_equal(r["y"], x[n_i, c, idd, ihh, iww] + w2[co_i, c, ta, ti, tj])


def test_rejects_window_in_padding():
    with pytest.raises(ValueError):
        o3.forward(o3.Shape3d(1, 1, 4, 4, 4, 1, 3, 3, 3, (1, 1, 1), (3, 1, 1), (1, 1, 1)), "max",
                   np.zeros((1, 1, 4, 4, 4), np.float32), None, np.zeros((1, 1, 3, 3, 3), np.float32))
