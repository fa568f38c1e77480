"""Pins for the oracle's mixed layers (paper Sec. 3.1: (iii) MinPlus-Max-Conv2d = max over input channels
of the min-plus operator, (vi) MaxPlus-Min-Conv2d = min over input channels of the max-plus operator).
None of them re-types the oracle's loops: an enumeration that reduces a [C_in, taps] table with numpy's
argmin / argmax, an unfold formulation with torch ops, pooling through a library routine for zero kernels,
the single-channel case that falls back on the already pinned layers (iv) / (v), 1x1 kernels, the
min/max duality, ordering between the four full-window layers, and finite differences of the gradients.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import brute
from oracle import tconv_oracle as orc

LAYERS = ["minplus_max", "maxplus_min"]


def _layer(seed, N=2, C=3, H=7, W=6, CO=4, k=3, stride=1, pad=1, dil=1, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        draw = lambda shape: rng.integers(-3, 4, shape).astype(np.float32)
    else:
        draw = lambda shape: rng.standard_normal(shape).astype(np.float32)
    return orc.Shape(N, C, H, W, CO, k, k, stride, pad, dil), draw((N, C, H, W)), draw((CO, C, k, k)), rng


GEOS = [(1, 1, 1, 3), (2, 1, 1, 3), (1, 2, 2, 3), (1, 0, 1, 2), (2, 2, 1, 5), (1, 0, 1, 1)]


@pytest.mark.parametrize("layer", LAYERS)
@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("stride,pad,dil,k", GEOS)
def test_enumeration(layer, integer, stride, pad, dil, k):
    """Values and winners against the table enumeration; integer data make ties the common case, so the
    lowest-tap / lowest-channel rule is exercised."""
    s, x, w, _ = _layer(5 + k, N=2, C=3, H=6, W=7, CO=3, k=k, stride=stride, pad=pad, dil=dil, integer=integer)
    r = orc.forward_mixed(s, layer, x, w)
    y, idx = brute.forward_mixed(x, w, layer == "minplus_max", stride, pad, dil)
    assert np.array_equal(r["y"].view(np.int32), y.view(np.int32))
    assert np.array_equal(r["idx"], idx)


@pytest.mark.parametrize("layer", LAYERS)
@pytest.mark.parametrize("stride,pad,dil,k", GEOS)
def test_unfold_formulation(layer, stride, pad, dil, k):
    """The layer equation with torch ops: pad with the inner operator's identity, unfold, add the kernel,
    reduce the taps, then the channels (torch's argmin / argmax return the first extremum)."""
    s, x, w, _ = _layer(11, N=2, C=4, H=9, W=8, CO=5, k=k, stride=stride, pad=pad, dil=dil, integer=True)
    outer_max = layer == "minplus_max"
    xp = F.pad(torch.from_numpy(x), (pad, pad, pad, pad), value=float("inf") if outer_max else float("-inf"))
    cols = F.unfold(xp, (k, k), dilation=dil, stride=stride).view(s.N, 1, s.C_in, k * k, -1)
    sums = cols + torch.from_numpy(w).view(1, s.C_out, s.C_in, k * k, 1)
    if outer_max:
        v, t = sums.min(dim=3)
        yv, c = v.max(dim=2)
    else:
        v, t = sums.max(dim=3)
        yv, c = v.min(dim=2)
    ho, wo = orc.out_shape(s)
    r = orc.forward_mixed(s, layer, x, w)
    assert np.array_equal(r["y"], yv.view(s.N, s.C_out, ho, wo).numpy())
    # values only: torch documents first-occurrence only for argmin/argmax, so winners go through them
    ta = sums.argmin(dim=3) if outer_max else sums.argmax(dim=3)
    va = torch.gather(sums, 3, ta.unsqueeze(3)).squeeze(3)
    ca = va.argmax(dim=2) if outer_max else va.argmin(dim=2)
    kk = ca * (k * k) + torch.gather(ta, 2, ca.unsqueeze(2)).squeeze(2)
    assert np.array_equal(r["idx"], kk.view(s.N, s.C_out, ho, wo).numpy().astype(np.int32))


@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 2, 2), (2, 0, 1)])
def test_zero_kernel_is_pooling_then_channel_reduction(stride, pad, dil):
    """W == 0: the inner operator is min / max pooling (library routine; -max_pool(-x) is min pooling with
    +inf padding), the outer one a reduction over channels, the same for every output channel."""
    s, x, _, _ = _layer(3, N=2, C=5, H=10, W=9, CO=2, stride=stride, pad=pad, dil=dil)
    w = np.zeros((s.C_out, s.C_in, 3, 3), np.float32)
    xt = torch.from_numpy(x)
    maxpool = F.max_pool2d(xt, 3, stride=stride, padding=0, dilation=dil) if pad == 0 else \
        F.max_pool2d(F.pad(xt, (pad,) * 4, value=float("-inf")), 3, stride=stride, dilation=dil)
    minpool = -(F.max_pool2d(-xt, 3, stride=stride, dilation=dil) if pad == 0 else
                F.max_pool2d(F.pad(-xt, (pad,) * 4, value=float("-inf")), 3, stride=stride, dilation=dil))
    a = orc.forward_mixed(s, "minplus_max", x, w)["y"]
    b = orc.forward_mixed(s, "maxplus_min", x, w)["y"]
    for co in range(s.C_out):
        assert np.array_equal(a[:, co], minpool.amax(dim=1).numpy())
        assert np.array_equal(b[:, co], maxpool.amin(dim=1).numpy())


@pytest.mark.parametrize("integer", [False, True])
def test_single_input_channel_is_the_plain_layer(integer):
    """C_in = 1: the outer reduction has one operand, so (iii) is layer (iv) and (vi) is layer (v)."""
    s, x, w, _ = _layer(8, C=1, integer=integer)
    a = orc.forward_mixed(s, "minplus_max", x, w)
    b = orc.forward_mixed(s, "maxplus_min", x, w)
    rmin = orc.forward(s, "min", x, w_min=w)
    rmax = orc.forward(s, "max", x, w_max=w)
    assert np.array_equal(a["y"], rmin["y"]) and np.array_equal(a["idx"], rmin["idx_min"])
    assert np.array_equal(b["y"], rmax["y"]) and np.array_equal(b["idx"], rmax["idx_max"])


def test_1x1_kernel_swaps_the_roles():
    """1x1 kernels: the inner operator has one operand, so (iii) is the plain max-plus layer (v) and (vi)
    the plain min-plus layer (iv), winners included (k = c)."""
    s, x, w, _ = _layer(9, C=5, k=1, pad=0, integer=True)
    a = orc.forward_mixed(s, "minplus_max", x, w)
    b = orc.forward_mixed(s, "maxplus_min", x, w)
    rmax = orc.forward(s, "max", x, w_max=w)
    rmin = orc.forward(s, "min", x, w_min=w)
    assert np.array_equal(a["y"], rmax["y"]) and np.array_equal(a["idx"], rmax["idx_max"])
    assert np.array_equal(b["y"], rmin["y"]) and np.array_equal(b["idx"], rmin["idx_min"])


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 2, 2)])
def test_duality_and_ordering(integer, stride, pad, dil):
    """(iii)(x, w) = -(vi)(-x, -w) with the same winners (negation is exact and keeps the scan order), and
    min-layer <= (iii), (vi) <= max-layer for the same kernel: min over everything <= max_c min_t,
    min_c max_t <= max over everything."""
    s, x, w, _ = _layer(21, stride=stride, pad=pad, dil=dil, integer=integer)
    a = orc.forward_mixed(s, "minplus_max", x, w)
    b = orc.forward_mixed(s, "maxplus_min", -x, -w)
    assert np.array_equal(a["y"], -b["y"]) and np.array_equal(a["idx"], b["idx"])
    lo = orc.forward(s, "min", x, w_min=w)["y"]
    hi = orc.forward(s, "max", x, w_max=w)["y"]
    c = orc.forward_mixed(s, "maxplus_min", x, w)
    for r in (a, c):
        assert (lo <= r["y"]).all() and (r["y"] <= hi).all()


@pytest.mark.parametrize("layer", LAYERS)
def test_index_reproduces_value_and_is_in_window(layer):
    s, x, w, _ = _layer(4, N=2, C=4, H=9, W=9, CO=3, stride=2, pad=1)
    r = orc.forward_mixed(s, layer, x, w)
    ho, wo = orc.out_shape(s)
    for n, co, oh, ow in itertools.product(range(s.N), range(s.C_out), range(ho), range(wo)):
        c, t = divmod(int(r["idx"][n, co, oh, ow]), 9)
        i, j = divmod(t, 3)
        ih, iw = oh * 2 - 1 + i, ow * 2 - 1 + j
        assert 0 <= ih < s.H and 0 <= iw < s.W
        assert r["y"][n, co, oh, ow] == np.float32(x[n, c, ih, iw]) + np.float32(w[co, c, i, j])


def test_bf16_output_rounding_matches_library_cast():
    s, x, w, _ = _layer(6)
    for layer in LAYERS:
        full = orc.forward_mixed(s, layer, x, w)
        rb = orc.forward_mixed(s, layer, x, w, out_bf16=True)
        assert np.array_equal(rb["y"], torch.from_numpy(full["y"]).to(torch.bfloat16).float().numpy())
        assert np.array_equal(rb["idx"], full["idx"])


@pytest.mark.parametrize("layer", LAYERS)
def test_backward_against_finite_differences(layer):
    """The gradient flows through the one winning tap, so the backward of layer (iv) / (v) applied to the
    mixed layer's indices is its backward; L = sum(gy * y) is piecewise linear and the central difference
    is exact wherever no winner changes within +-h."""
    s, x, w, rng = _layer(31, N=1, C=3, H=5, W=5, CO=2)
    outer_max = layer == "minplus_max"
    r = orc.forward_mixed(s, layer, x, w)
    gyf = rng.standard_normal(r["y"].shape).astype(np.float32)
    gy = gyf.astype(np.float64)
    mode, kw = ("min", dict(idx_min=r["idx"])) if outer_max else ("max", dict(idx_max=r["idx"]))
    gx = orc.backward_input(s, mode, gyf, **kw)
    g1, g2 = orc.backward_weight(s, mode, gyf, **kw)
    gw = g1 if outer_max else g2

    def loss(xv, wv):
        y, i = brute.forward_mixed(xv, wv, outer_max, 1, 1, 1, dtype=np.float64)
        return (gy * y).sum(), i

    h = 2.0 ** -10
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    checked = 0
    for pos in itertools.product(range(1), range(3), range(5), range(5)):
        xp, xm = x64.copy(), x64.copy()
        xp[pos] += h
        xm[pos] -= h
        (lp, sp), (lm, sm) = loss(xp, w64), loss(xm, w64)
        if np.array_equal(sp, sm):
            assert abs((lp - lm) / (2 * h) - gx[pos]) < 1e-6
            checked += 1
    assert checked >= 40
    checked = 0
    for pos in itertools.product(range(2), range(3), range(3), range(3)):
        wp, wm = w64.copy(), w64.copy()
        wp[pos] += h
        wm[pos] -= h
        (lp, sp), (lm, sm) = loss(x64, wp), loss(x64, wm)
        if np.array_equal(sp, sm):
            assert abs((lp - lm) / (2 * h) - gw[pos]) < 1e-6
            checked += 1
    assert checked >= 30


def test_rejects_window_that_can_lie_in_padding():
    s = orc.Shape(1, 1, 4, 4, 1, 3, 3, 1, 3, 1)
    with pytest.raises(ValueError):
        orc.forward_mixed(s, "minplus_max", np.zeros((1, 1, 4, 4), np.float32), np.zeros((1, 1, 3, 3), np.float32))
