"""Pins for the CPU oracle of the Sum-channel layers (oracle/tsum_oracle.c), none of which re-types its loops:
closed forms (1x1 kernels, zero kernels = pooling through a library routine), the single-input-channel
case that reduces to the already pinned full-window oracle, an unfold formulation with torch ops, the
hand-worked all-ties winners of a 3x3 map, algebraic invariants of the layer equations (paper Sec. 3.1
layers (i), (ii); Sec. 3.5 / 3.6 two-parameter layers), and finite differences for every gradient.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tconv_oracle as orc
from oracle import tsum_oracle as osum

MODES = ["max", "min", "compound", "parallel"]


def _layer(seed, N=2, C=3, H=7, W=6, CO=4, k=3, stride=1, pad=1, dil=1, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        draw = lambda shape: rng.integers(-4, 5, shape).astype(np.float32)
    else:
        draw = lambda shape: rng.standard_normal(shape).astype(np.float32)
    x, w1, w2 = draw((N, C, H, W)), draw((CO, C, k, k)), draw((CO, C, k, k))
    if integer:
        a, b = rng.integers(-2, 3, (C, CO)).astype(np.float32), rng.integers(-2, 3, (C, CO)).astype(np.float32)
    else:
        a, b = rng.uniform(-1, 1, (C, CO)).astype(np.float32), rng.uniform(-1, 1, (C, CO)).astype(np.float32)
    return orc.Shape(N, C, H, W, CO, k, k, stride, pad, dil), x, w1, w2, a, b, rng


def _kernels(mode, w1, w2):
    """(w_min, w_max) as the layer of that mode takes them."""
    if mode == "max":
        return None, w2
    if mode == "min":
        return w1, None
    if mode == "compound":
        return w1, w1
    return w1, w2


def _unfold_reference(s, mode, x, w_min, w_max, alpha, beta, dtype=torch.float32):
    """The layer equations with torch ops: pad with the semiring identity, unfold each channel's windows,
    add the kernel, amin / amax over the taps, then the weighted channel sum in ascending c_in."""
    c = s.c()
    xt = torch.from_numpy(x).to(dtype)
    ho, wo = osum.out_hw(s)
    two = mode in ("compound", "parallel")

    def base(w, want_max):
        fill = float("-inf") if want_max else float("inf")
        xp = F.pad(xt, (c.pad_w, c.pad_w, c.pad_h, c.pad_h), value=fill)
        cols = F.unfold(xp, (s.KH, s.KW), dilation=(c.dil_h, c.dil_w), stride=(c.stride_h, c.stride_w))
        cols = cols.view(s.N, 1, s.C_in, s.KH * s.KW, ho * wo)
        wt = torch.from_numpy(w).to(dtype).view(1, s.C_out, s.C_in, s.KH * s.KW, 1)
        sums = cols + wt                                           # [N, CO, C, taps, L]
        return sums.amax(dim=3) if want_max else sums.amin(dim=3)  # [N, CO, C, L]

    m = base(w_min, False) if mode != "max" else None
    M = base(w_max, True) if mode != "min" else None
    acc = torch.zeros((s.N, s.C_out, ho * wo), dtype=dtype)
    for ci in range(s.C_in):
        if two:
            a = torch.from_numpy(alpha[ci]).to(dtype).view(1, -1, 1) if alpha is not None else 1.0
            b = torch.from_numpy(beta[ci]).to(dtype).view(1, -1, 1) if beta is not None else 1.0
            term = a * m[:, :, ci] + b * M[:, :, ci]
        else:
            term = m[:, :, ci] if mode == "min" else M[:, :, ci]
        acc = acc + term
    return acc.view(s.N, s.C_out, ho, wo).numpy()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("stride,pad,dil,k", [(1, 1, 1, 3), (2, 1, 1, 3), (1, 2, 2, 3), (1, 0, 1, 2), (2, 2, 1, 5)])
def test_forward_equals_unfold_formulation(mode, stride, pad, dil, k):
    s, x, w1, w2, a, b, _ = _layer(3, k=k, stride=stride, pad=pad, dil=dil, H=9, W=8)
    wmn, wmx = _kernels(mode, w1, w2)
    y = osum.forward(s, mode, x, wmn, wmx, a, b)
    ref = _unfold_reference(s, mode, x, wmn, wmx, a, b)
    assert np.array_equal(y, ref)          # same fp32 operations in the same order
    y1 = osum.forward(s, mode, x, wmn, wmx)  # alpha = beta = None: all ones
    assert np.array_equal(y1, _unfold_reference(s, mode, x, wmn, wmx, None, None))


def test_one_by_one_kernel_closed_form():
    """KH = KW = 1: both base operators are x + w, so y = sum_c (alpha + beta)[c, co] * (x[c] + w[co, c])."""
    s, x, w1, _, a, b, _ = _layer(5, k=1, pad=0, integer=True)
    y = osum.forward(s, "compound", x, w1, w1, a, b)
    ref = np.einsum("co,nchw->nohw", (a + b).astype(np.float64), x.astype(np.float64)) \
        + np.einsum("co,oc->o", (a + b).astype(np.float64), w1[:, :, 0, 0].astype(np.float64))[None, :, None, None]
    assert np.array_equal(y.astype(np.float64), ref)   # small integers: every operation is exact
    ymin = osum.forward(s, "min", x, w1, None)
    assert np.array_equal(ymin.astype(np.float64),
                          x.astype(np.float64).sum(1)[:, None] + w1[:, :, 0, 0].astype(np.float64).sum(1)[None, :, None, None])


def test_zero_kernel_is_pooling():
    """w == 0: MaxPlus2d is a max-pool of the channel (padding never wins = -inf padding of F.max_pool2d),
    MinPlus2d is minus the max-pool of -x."""
    s, x, _, _, a, b, _ = _layer(6, integer=True, H=8, W=8)
    z = np.zeros((s.C_out, s.C_in, 3, 3), np.float32)
    xt = torch.from_numpy(x)
    mx = F.max_pool2d(xt, 3, stride=1, padding=1).numpy().astype(np.float64)       # [N, C, H, W]
    mn = (-F.max_pool2d(-xt, 3, stride=1, padding=1)).numpy().astype(np.float64)
    y = osum.forward(s, "parallel", x, z, z, a, b)
    ref = np.einsum("co,nchw->nohw", a.astype(np.float64), mn) + np.einsum("co,nchw->nohw", b.astype(np.float64), mx)
    assert np.array_equal(y.astype(np.float64), ref)
    assert np.array_equal(osum.forward(s, "max", x, None, z).astype(np.float64), np.repeat(mx.sum(1)[:, None], s.C_out, 1))


@pytest.mark.parametrize("mode", ["compound", "parallel"])
def test_single_input_channel_reduces_to_full_window_layer(mode):
    """With C_in = 1 the channel sum has one term: the layer is the full-window compound / parallel
    operator (whose oracle is pinned on its own) with alpha[0, :], beta[0, :] as per-c_out coefficients."""
    s, x, w1, w2, a, b, _ = _layer(7, C=1, stride=2, pad=1)
    wmn, wmx = _kernels(mode, w1, w2)
    y = osum.forward(s, mode, x, wmn, wmx, a, b)
    r = orc.forward(s, mode, x, w_min=wmn, w_max=wmx, alpha=a[0], beta=b[0])
    assert np.array_equal(y, r["y"])
    gy = np.random.default_rng(0).standard_normal(y.shape).astype(np.float32)
    g = osum.backward(s, mode, x, gy, wmn, wmx, a, b)
    gx = orc.backward_input(s, mode, gy, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=a[0], beta=b[0])
    g1, g2 = orc.backward_weight(s, mode, gy, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=a[0], beta=b[0])
    ga, gb = orc.backward_alpha_beta(s, mode, gy, r["y_min"], r["y_max"])
    assert np.allclose(g["grad_x"], gx, rtol=0, atol=1e-12)
    assert np.allclose(g["grad_w_min"], g1, rtol=0, atol=1e-12)
    if mode == "parallel":
        assert np.allclose(g["grad_w_max"], g2, rtol=0, atol=1e-12)
    assert np.allclose(g["grad_alpha"][0], ga, rtol=0, atol=1e-12) and np.allclose(g["grad_beta"][0], gb, rtol=0, atol=1e-12)


def test_all_ties_pick_the_lowest_valid_tap():
    """x == 1, w == 0 on a 3x3 map with pad 1: every tap of every window ties, so the winner is the lowest
    valid tap.  Worked by hand, the winners of the 9 windows are [[4,3,3],[1,0,0],[1,0,0]]: tap 0 four
    times, taps 1 and 3 twice, tap 4 once; with gy == 1 these counts are grad_w.  Window (oh, ow) with
    winner tap (i, j) reads input pixel (oh - 1 + i, ow - 1 + j): (0,0) four times, (0,1) and (1,0) twice,
    (1,1) once - that is grad_x."""
    s = orc.Shape(1, 1, 3, 3, 1, 3, 3, 1, 1, 1)
    x = np.ones((1, 1, 3, 3), np.float32)
    w = np.zeros((1, 1, 3, 3), np.float32)
    gy = np.ones((1, 1, 3, 3), np.float32)
    for mode in ("min", "max"):
        wmn, wmx = _kernels(mode, w, w)
        g = osum.backward(s, mode, x, gy, wmn, wmx)
        gw = g["grad_w_min"] if mode == "min" else g["grad_w_max"]
        assert gw.reshape(9).tolist() == [4, 2, 0, 2, 1, 0, 0, 0, 0]
        assert g["grad_x"].reshape(3, 3).tolist() == [[4, 2, 0], [2, 1, 0], [0, 0, 0]]
    assert np.array_equal(osum.forward(s, "min", x, w, None), np.ones((1, 1, 3, 3), np.float32))


@pytest.mark.parametrize("integer", [False, True])
def test_invariants_of_the_layer_equations(integer):
    s, x, w1, w2, a, b, _ = _layer(9, integer=integer, stride=1, pad=1)
    one, zero = np.ones_like(a), np.zeros_like(a)
    # degenerate coefficient pairs of Sec. 3.3 give the single-branch layers (i) and (ii)
    assert np.array_equal(osum.forward(s, "parallel", x, w1, w2, one, zero), osum.forward(s, "min", x, w1, None))
    assert np.array_equal(osum.forward(s, "parallel", x, w1, w2, zero, one), osum.forward(s, "max", x, None, w2))
    # compound is parallel with W1 == W2
    assert np.array_equal(osum.forward(s, "compound", x, w1, w1, a, b), osum.forward(s, "parallel", x, w1, w1, a, b))
    # linear in (alpha, beta): a power-of-two scale is exact in fp32
    y = osum.forward(s, "parallel", x, w1, w2, a, b)
    assert np.array_equal(osum.forward(s, "parallel", x, w1, w2, 2 * a, 2 * b), 2 * y)
    # duality: MinPlus-Sum(x, w) = -MaxPlus-Sum(-x, -w)
    assert np.array_equal(osum.forward(s, "min", x, w1, None), -osum.forward(s, "max", -x, None, -w1))
    # a sum layer shifts by C_in * c (the full-window layers shift by c): exact on integer data
    if integer:
        assert np.array_equal(osum.forward(s, "max", x + 8, None, w2), osum.forward(s, "max", x, None, w2) + 8 * s.C_in)
    # every (c_in, c_out, pixel, branch) deposits its whole gradient once
    gy = np.random.default_rng(1).standard_normal(y.shape).astype(np.float32)
    g = osum.backward(s, "parallel", x, gy, w1, w2, a, b)
    per_co = gy.astype(np.float64).sum(axis=(0, 2, 3))
    assert np.isclose(g["grad_x"].sum(), (per_co * (a.astype(np.float64) + b.astype(np.float64)).sum(0)).sum(), rtol=1e-12, atol=1e-9)
    assert np.allclose(g["grad_w_min"].sum(axis=(2, 3)), (a.T.astype(np.float64) * per_co[:, None]), rtol=1e-12, atol=1e-9)
    assert np.allclose(g["grad_w_max"].sum(axis=(2, 3)), (b.T.astype(np.float64) * per_co[:, None]), rtol=1e-12, atol=1e-9)


@pytest.mark.parametrize("mode", MODES)
def test_backward_against_finite_differences(mode):
    """L = sum(gy * y) is piecewise linear in x and w and linear in alpha, beta; where no window winner
    changes within +-h, the central difference of the fp64 unfold formulation is the exact gradient."""
    s, x, w1, w2, a, b, rng = _layer(11, N=1, C=2, H=5, W=5, CO=2)
    wmn, wmx = _kernels(mode, w1, w2)
    two = mode in ("compound", "parallel")
    y = osum.forward(s, mode, x, wmn, wmx, a, b)
    gy = rng.standard_normal(y.shape).astype(np.float32)
    g = osum.backward(s, mode, x, gy, wmn, wmx, a, b)

    def loss(xv, w1v, w2v, av, bv):
        wa, wb = _kernels(mode, w1v, w2v)
        yv = _unfold_reference(s, mode, xv, wa, wb, av if two else None, bv if two else None, dtype=torch.float64)
        return float((gy.astype(np.float64) * yv).sum())

    base = [x.astype(np.float64), w1.astype(np.float64), w2.astype(np.float64), a.astype(np.float64), b.astype(np.float64)]
    h = 2.0 ** -12

    def fd(which, pos):
        p, m = [v.copy() for v in base], [v.copy() for v in base]
        p[which][pos] += h
        m[which][pos] -= h
        # a kink inside +-h shows as a mismatch between the one-sided slopes
        l0, lp, lm = loss(*base), loss(*p), loss(*m)
        if abs((lp - l0) - (l0 - lm)) > 1e-9:
            return None
        return (lp - lm) / (2 * h)

    checked = 0
    for pos in itertools.product(range(1), range(2), range(5), range(5)):
        d = fd(0, pos)
        if d is not None:
            assert abs(d - g["grad_x"][pos]) < 1e-6
            checked += 1
    assert checked >= 30
    for which, key in ((1, "grad_w_min"), (2, "grad_w_max")):
        if g[key] is None or (mode == "compound" and which == 2) or (mode == "min" and which == 2) or (mode == "max" and which == 1):
            continue
        for pos in itertools.product(range(2), range(2), range(3), range(3)):
            d = fd(which, pos)
            if d is not None:
                assert abs(d - g[key][pos]) < 1e-6
                checked += 1
    if two:
        for pos in itertools.product(range(2), range(2)):
            assert abs(fd(3, pos) - g["grad_alpha"][pos]) < 1e-6
            assert abs(fd(4, pos) - g["grad_beta"][pos]) < 1e-6
    assert checked >= 50


def test_rejects_bad_requests():
    s, x, w1, w2, a, b, _ = _layer(12)
    with pytest.raises(ValueError):
        osum.forward(s, "parallel", x, w1, None)                       # parallel needs both kernels
    with pytest.raises(ValueError):
        osum.forward(orc.Shape(1, 1, 4, 4, 1, 3, 3, 1, 3, 1), "max", np.zeros((1, 1, 4, 4), np.float32), None,
                     np.zeros((1, 1, 3, 3), np.float32))               # pad 3 > dil*(k-1): a window of padding only
