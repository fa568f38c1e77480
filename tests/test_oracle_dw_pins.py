"""Pins for the CPU oracle of the depthwise tropical layer (oracle/tdw_oracle.c), none of which re-types its
loops: the per-channel slices against the already pinned full-window oracle (a depthwise layer is that layer
with one input channel, paper Sec. 3.1 base operators; Sec. 5 MobileNetV2 variants), the pinned Sum-channel
oracle with coefficients that are zero off the channel's own group, an unfold formulation with torch ops,
zero kernels = library pooling, the hand-worked all-ties winners, invariants and finite differences.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tconv_oracle as orc
from oracle import tdw_oracle as odw
from oracle import tsum_oracle as osum

MODES = ["max", "min", "compound", "parallel"]
GEOS = [(1, 1, 1, 3), (2, 1, 1, 3), (1, 2, 2, 3), (1, 0, 1, 2), (2, 2, 1, 5)]


def _layer(seed, N=2, C=3, mult=1, H=7, W=6, k=3, stride=1, pad=1, dil=1, integer=False):
    rng = np.random.default_rng(seed)
    CO = C * mult
    if integer:
        draw = lambda shape: rng.integers(-4, 5, shape).astype(np.float32)
        coef = lambda: rng.integers(-2, 3, CO).astype(np.float32)
    else:
        draw = lambda shape: rng.standard_normal(shape).astype(np.float32)
        coef = lambda: rng.uniform(-1, 1, CO).astype(np.float32)
    x, w1, w2 = draw((N, C, H, W)), draw((CO, 1, k, k)), draw((CO, 1, k, k))
    return orc.Shape(N, C, H, W, CO, k, k, stride, pad, dil), x, w1, w2, coef(), coef(), rng


def _kernels(mode, w1, w2):
    if mode == "max":
        return None, w2
    if mode == "min":
        return w1, None
    if mode == "compound":
        return w1, w1
    return w1, w2


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("mult", [1, 2])
@pytest.mark.parametrize("stride,pad,dil,k", GEOS)
def test_channel_slices_are_the_full_window_layer(mode, mult, stride, pad, dil, k):
    """Output channel co of a depthwise layer is the full-window layer with C_in = C_out = 1 on input channel
    co // mult: values bit for bit, all gradients up to the rounding of double sums."""
    s, x, w1, w2, a, b, rng = _layer(3 + k, mult=mult, k=k, stride=stride, pad=pad, dil=dil, H=9, W=8)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    y, tmin, tmax = odw.forward(s, mode, x, wmn, wmx, a if two else None, b if two else None, taps=True)
    gy = rng.standard_normal(y.shape).astype(np.float32)
    g = odw.backward(s, mode, x, gy, wmn, wmx, a if two else None, b if two else None)
    s1 = orc.Shape(s.N, 1, s.H, s.W, 1, k, k, stride, pad, dil)
    gx = np.zeros(x.shape, np.float64)
    for co in range(s.C_out):
        c = co // mult
        kw = dict(w_min=None if wmn is None else wmn[co:co + 1], w_max=None if wmx is None else wmx[co:co + 1])
        ab = dict(alpha=a[co:co + 1], beta=b[co:co + 1]) if two else {}
        r = orc.forward(s1, mode, x[:, c:c + 1], **kw, **ab)
        assert np.array_equal(y[:, co:co + 1], r["y"])
        if mode != "max":   # one input channel: the flattened winner k of the full-window layer is the tap
            assert np.array_equal(tmin[:, co:co + 1], r["idx_min"])
        if mode != "min":
            assert np.array_equal(tmax[:, co:co + 1], r["idx_max"])
        ikw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"], **ab)
        gx[:, c:c + 1] += orc.backward_input(s1, mode, gy[:, co:co + 1], **ikw)
        g1, g2 = orc.backward_weight(s1, mode, gy[:, co:co + 1], **ikw)
        if mode != "max":
            assert np.allclose(g["grad_w_min"][co:co + 1], g1, rtol=0, atol=1e-12)
        if mode in ("max", "parallel"):
            assert np.allclose(g["grad_w_max"][co:co + 1], g2, rtol=0, atol=1e-12)
        if two:
            ga, gb = orc.backward_alpha_beta(s1, mode, gy[:, co:co + 1], r["y_min"], r["y_max"])
            assert np.allclose(g["grad_alpha"][co], ga[0], rtol=0, atol=1e-12)
            assert np.allclose(g["grad_beta"][co], gb[0], rtol=0, atol=1e-12)
    assert np.allclose(g["grad_x"], gx, rtol=0, atol=1e-12)


@pytest.mark.parametrize("mode", ["compound", "parallel"])
def test_equals_sum_channel_layer_with_block_diagonal_coefficients(mode):
    """The Sum-channel layer with alpha[c, co] = beta[c, co] = 0 unless c == co // mult, and kernels that carry
    the depthwise kernel in that channel's slot, is the depthwise layer (the other terms add +-0)."""
    s, x, w1, w2, a, b, _ = _layer(12, C=3, mult=2, stride=2, integer=True)
    wmn, wmx = _kernels(mode, w1, w2)
    A = np.zeros((s.C_in, s.C_out), np.float32)
    B = np.zeros((s.C_in, s.C_out), np.float32)
    W1 = np.zeros((s.C_out, s.C_in, 3, 3), np.float32)
    W2 = np.zeros((s.C_out, s.C_in, 3, 3), np.float32)
    for co in range(s.C_out):
        A[co // 2, co], B[co // 2, co] = a[co], b[co]
        W1[co, co // 2], W2[co, co // 2] = wmn[co, 0], wmx[co, 0]
    y = odw.forward(s, mode, x, wmn, wmx, a, b)
    ys = osum.forward(s, mode, x, W1, W2, A, B)
    assert np.array_equal(y, ys)   # integers: exact; +0 and -0 compare equal


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("stride,pad,dil,k", GEOS)
def test_unfold_formulation(mode, stride, pad, dil, k):
    s, x, w1, w2, a, b, _ = _layer(5, C=4, mult=2, k=k, stride=stride, pad=pad, dil=dil, H=9, W=8)
    wmn, wmx = _kernels(mode, w1, w2)
    ho, wo = odw.out_hw(s)
    xt = torch.from_numpy(x)

    def base(w, want_max):
        xp = F.pad(xt, (pad,) * 4, value=float("-inf") if want_max else float("inf"))
        cols = F.unfold(xp, (k, k), dilation=dil, stride=stride).view(s.N, s.C_in, k * k, ho * wo)
        cols = cols.repeat_interleave(2, dim=1)                       # channel co reads input channel co // 2
        sums = cols + torch.from_numpy(w).view(1, s.C_out, k * k, 1)
        return sums.amax(dim=2) if want_max else sums.amin(dim=2)

    if mode == "max":
        ref = base(wmx, True)
    elif mode == "min":
        ref = base(wmn, False)
    else:
        ref = torch.from_numpy(a).view(1, -1, 1) * base(wmn, False) + torch.from_numpy(b).view(1, -1, 1) * base(wmx, True)
    two = mode in ("compound", "parallel")
    y = odw.forward(s, mode, x, wmn, wmx, a if two else None, b if two else None)
    assert np.array_equal(y, ref.view(s.N, s.C_out, ho, wo).numpy())


def test_zero_kernel_is_pooling():
    s, x, _, _, a, b, _ = _layer(6, C=5, H=10, W=9, stride=2)
    z = np.zeros((s.C_out, 1, 3, 3), np.float32)
    xt = torch.from_numpy(x)
    mx = F.max_pool2d(xt, 3, stride=2, padding=1).numpy()
    mn = (-F.max_pool2d(-xt, 3, stride=2, padding=1)).numpy()
    assert np.array_equal(odw.forward(s, "max", x, None, z), mx)
    assert np.array_equal(odw.forward(s, "min", x, z, None), mn)
    ref = (a[None, :, None, None] * mn).astype(np.float32) + (b[None, :, None, None] * mx).astype(np.float32)
    assert np.array_equal(odw.forward(s, "compound", x, z, z, a, b), ref)
    assert np.array_equal(odw.forward(s, "parallel", x, z, z), mn + mx)   # NULL coefficients are ones


def test_all_ties_pick_the_lowest_valid_tap():
    """x == 1, w == 0 on a 3x3 map with pad 1: every tap ties, the winner is the lowest valid tap.  By hand the
    winners of the 9 windows are [[4,3,3],[1,0,0],[1,0,0]]; with gy == 1 a branch sends grad_w = counts of the
    taps and grad_x = [[4,2,0],[2,1,0],[0,0,0]]."""
    s = orc.Shape(1, 1, 3, 3, 1, 3, 3, 1, 1, 1)
    x = np.ones((1, 1, 3, 3), np.float32)
    z = np.zeros((1, 1, 3, 3), np.float32)
    gy = np.ones((1, 1, 3, 3), np.float32)
    for mode, scale in (("max", 1), ("min", 1), ("compound", 2)):
        wmn, wmx = _kernels(mode, z, z)
        g = odw.backward(s, mode, x, gy, wmn, wmx)
        assert np.array_equal(g["grad_x"][0, 0], scale * np.array([[4, 2, 0], [2, 1, 0], [0, 0, 0]], np.float64))
        gw = g["grad_w_max"] if mode == "max" else g["grad_w_min"]
        assert np.array_equal(gw.reshape(9), scale * np.array([4, 2, 0, 2, 1, 0, 0, 0, 0], np.float64))
    g = odw.backward(s, "parallel", x, gy, z, z, np.array([2.0], np.float32), np.array([-3.0], np.float32))
    assert np.array_equal(g["grad_x"][0, 0], -1.0 * np.array([[4, 2, 0], [2, 1, 0], [0, 0, 0]], np.float64))
    assert g["grad_alpha"][0] == 9.0 and g["grad_beta"][0] == 9.0


@pytest.mark.parametrize("integer", [False, True])
def test_invariants(integer):
    s, x, w1, w2, a, b, rng = _layer(9, C=4, mult=2, integer=integer)
    # duality: min-layer(x, w) = -max-layer(-x, -w)
    assert np.array_equal(odw.forward(s, "min", x, w1, None), -odw.forward(s, "max", -x, None, -w1))
    # compound with alpha = 1, beta = 0 is the min layer; parallel with alpha = 0, beta = 1 the max layer
    one, zero = np.ones(s.C_out, np.float32), np.zeros(s.C_out, np.float32)
    ymin, ymax = odw.forward(s, "min", x, w1, None), odw.forward(s, "max", x, None, w2)
    assert np.array_equal(odw.forward(s, "compound", x, w1, w1, one, zero), ymin + np.float32(0))
    assert np.array_equal(odw.forward(s, "parallel", x, w1, w2, zero, one), ymax + np.float32(0))
    # gradient mass: every branch of every output deposits its scaled gradient exactly once
    gy = rng.standard_normal(ymin.shape).astype(np.float32)
    g = odw.backward(s, "parallel", x, gy, w1, w2, a, b)
    tot = ((a.astype(np.float64) + b.astype(np.float64))[None, :, None, None] * gy.astype(np.float64)).sum()
    ta = (a.astype(np.float64)[None, :, None, None] * gy).sum()
    assert abs(g["grad_x"].sum() - tot) < 1e-9 and abs(g["grad_w_min"].sum() - ta) < 1e-9
    # the coefficient gradients are correlations of gy with the branch outputs
    assert np.allclose(g["grad_alpha"], (gy.astype(np.float64) * ymin).sum((0, 2, 3)), rtol=0, atol=1e-10)
    assert np.allclose(g["grad_beta"], (gy.astype(np.float64) * ymax).sum((0, 2, 3)), rtol=0, atol=1e-10)


@pytest.mark.parametrize("mode", MODES)
def test_backward_against_finite_differences(mode):
    """L = sum(gy * y) evaluated in fp64 with numpy (windows materialised by slicing); the central difference is
    exact wherever no winner changes within +-h."""
    s, x, w1, w2, a, b, rng = _layer(31, N=1, C=2, mult=2, H=5, W=5)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    y = odw.forward(s, mode, x, wmn, wmx, a if two else None, b if two else None)
    gyf = rng.standard_normal(y.shape).astype(np.float32)
    gy = gyf.astype(np.float64)
    g = odw.backward(s, mode, x, gyf, wmn, wmx, a if two else None, b if two else None)

    def loss(xv, wmnv, wmxv, av, bv):
        tot, sig = 0.0, []
        for want_max, wv, cv in ((False, wmnv, av), (True, wmxv, bv)):
            if wv is None:
                continue
            xp = np.pad(xv, ((0, 0), (0, 0), (1, 1), (1, 1)), constant_values=-np.inf if want_max else np.inf)
            win = np.stack([xp[:, :, i:i + 5, j:j + 5] for i in range(3) for j in range(3)], axis=2)  # [N,C,9,5,5]
            sums = np.repeat(win, 2, axis=1) + wv.reshape(1, s.C_out, 9, 1, 1)
            v = sums.max(axis=2) if want_max else sums.min(axis=2)
            sig.append(sums.argmax(axis=2) if want_max else sums.argmin(axis=2))
            coef = cv.reshape(1, -1, 1, 1) if two else 1.0
            tot += (gy * coef * v).sum()
        return tot, np.stack(sig)

    h = 2.0 ** -10
    x64 = x.astype(np.float64)
    w64 = {k: (None if v is None else v.astype(np.float64)) for k, v in (("mn", wmn), ("mx", wmx))}
    a64, b64 = a.astype(np.float64), b.astype(np.float64)

    def check(make, ref, need):
        ok = 0
        for pos, args_p, args_m in make():
            (lp, sp), (lm, sm) = loss(*args_p), loss(*args_m)
            if np.array_equal(sp, sm):
                assert abs((lp - lm) / (2 * h) - ref[pos]) < 1e-6, pos
                ok += 1
        assert ok >= need

    def vary_x():
        for pos in itertools.product(range(1), range(2), range(5), range(5)):
            p, m = x64.copy(), x64.copy()
            p[pos] += h
            m[pos] -= h
            yield pos, (p, w64["mn"], w64["mx"], a64, b64), (m, w64["mn"], w64["mx"], a64, b64)

    def vary_w(which):
        def gen():
            for pos in itertools.product(range(4), range(1), range(3), range(3)):
                p, m = w64[which].copy(), w64[which].copy()
                p[pos] += h
                m[pos] -= h
                if mode == "compound":
                    yield pos, (x64, p, p, a64, b64), (x64, m, m, a64, b64)
                elif which == "mn":
                    yield pos, (x64, p, w64["mx"], a64, b64), (x64, m, w64["mx"], a64, b64)
                else:
                    yield pos, (x64, w64["mn"], p, a64, b64), (x64, w64["mn"], m, a64, b64)
        return gen

    check(vary_x, g["grad_x"], 25)
    if mode != "max":
        check(vary_w("mn"), g["grad_w_min"], 18)
    if mode in ("max", "parallel"):
        check(vary_w("mx"), g["grad_w_max"], 18)
    if two:
        for name, idx in (("grad_alpha", 3), ("grad_beta", 4)):
            for co in range(s.C_out):
                args_p = [x64, w64["mn"], w64["mx"], a64.copy(), b64.copy()]
                args_m = [x64, w64["mn"], w64["mx"], a64.copy(), b64.copy()]
                args_p[idx][co] += h
                args_m[idx][co] -= h
                assert abs((loss(*args_p)[0] - loss(*args_m)[0]) / (2 * h) - g[name][co]) < 1e-6


def test_rejects_bad_shapes():
    x = np.zeros((1, 2, 4, 4), np.float32)
    with pytest.raises(ValueError):   # C_out must be a multiple of C_in
        odw.forward(orc.Shape(1, 2, 4, 4, 3, 3, 3, 1, 1, 1), "max", x, None, np.zeros((3, 1, 3, 3), np.float32))
    with pytest.raises(ValueError):   # a window could be all padding
        odw.forward(orc.Shape(1, 2, 4, 4, 2, 3, 3, 1, 3, 1), "max", x, None, np.zeros((2, 1, 3, 3), np.float32))
