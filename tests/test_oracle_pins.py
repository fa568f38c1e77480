"""Pins for the CPU oracle: everything here checks the oracle against something other than itself.

Hand-worked fixtures (tests/golden), an independent enumerate-then-argmax brute
force, library routines in the special cases that reduce to them (max-pool,
unfold + amax), closed forms, algebraic invariants of the max-plus / min-plus
semirings (paper Sec. 3.1) and of the compound / parallel definitions (Sec. 3.3),
and finite differences for the backward pass.
"""
import itertools
import json
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import brute
from oracle import tconv_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


def _shape(d, **over):
    d = dict(d, **over)
    return orc.Shape(d["N"], d["C_in"], d["H"], d["W"], d["C_out"], d["KH"], d["KW"],
                     d["stride"], d["pad"], d["dil"])


def _f(a):
    return np.asarray(a, np.float32)


def _example_c_data():
    x = np.empty((1, 2, 3, 3), np.float32)
    w = np.empty((2, 2, 3, 3), np.float32)
    for c, h, ww in itertools.product(range(2), range(3), range(3)):
        x[0, c, h, ww] = ((7 * c + 3 * h + 5 * ww) % 11) - 5
    for o, c, i, j in itertools.product(range(2), range(2), range(3), range(3)):
        w[o, c, i, j] = ((5 * o + 3 * c + 2 * i + 4 * j) % 7) - 3
    return x, w


# ---------------------------------------------------------------- hand-worked fixtures

def test_example_a_1x1():
    g = _gold("example_a_1x1.json")
    s, x, w = _shape(g["shape"]), _f(g["x"]), _f(g["w"])
    r = orc.forward(s, "max", x, w_max=w)
    assert np.array_equal(r["y"], _f(g["max"]["y"])) and np.array_equal(r["idx_max"], g["max"]["idx"])
    r = orc.forward(s, "min", x, w_min=w)
    assert np.array_equal(r["y"], _f(g["min"]["y"])) and np.array_equal(r["idx_min"], g["min"]["idx"])
    r = orc.forward(s, "compound", x, w_min=w)
    assert np.array_equal(r["y"], _f(g["compound_y"]))


def test_example_b_3x3_zero_kernel():
    g = _gold("example_b_3x3_pool.json")
    s, x = _shape(g["shape"]), _f(g["x"])
    w = np.zeros((1, 1, 3, 3), np.float32)
    r = orc.forward(s, "max", x, w_max=w)
    assert np.array_equal(r["y"], _f(g["max"]["y"])) and np.array_equal(r["idx_max"], g["max"]["idx"])
    r = orc.forward(s, "min", x, w_min=w)
    assert np.array_equal(r["y"], _f(g["min"]["y"])) and np.array_equal(r["idx_min"], g["min"]["idx"])
    ones = np.ones_like(x)
    for mode, key, wk in (("max", "idx_max", "w_max"), ("min", "idx_min", "w_min")):
        r = orc.forward(s, mode, ones, **{wk: w})
        assert np.array_equal(r[key], g["all_ones_idx"]), "all-tie case must keep the lowest VALID tap"


def test_example_c_forward_backward():
    g = _gold("example_c_2ch_2filters.json")
    s = _shape(g["shape"])
    x, w = _example_c_data()
    gy = np.ones((1, 2, 3, 3), np.float32)
    for mode, wk, ik in (("max", "w_max", "idx_max"), ("min", "w_min", "idx_min")):
        r = orc.forward(s, mode, x, **{wk: w})
        assert np.array_equal(r["y"][0], _f(g[mode]["y"]))
        assert np.array_equal(r[ik][0], g[mode]["idx"])
        gx = orc.backward_input(s, mode, gy, **{ik: r[ik]})
        assert np.array_equal(gx[0], np.asarray(g[mode]["grad_x_ones"], np.float64))
        gmn, gmx = orc.backward_weight(s, mode, gy, **{ik: r[ik]})
        gw = gmx if mode == "max" else gmn
        assert np.array_equal(gw, np.asarray(g[mode]["grad_w_ones"], np.float64))
        # the fixture itself against the independent enumerator
        yb, ib = brute.forward(x, w, mode == "max", 1, 1, 1)
        assert np.array_equal(yb[0], _f(g[mode]["y"])) and np.array_equal(ib[0], g[mode]["idx"])
    r = orc.forward(s, "compound", x, w_min=w)
    assert np.array_equal(r["y"][0], _f(g["compound_y"]))
    gx = orc.backward_input(s, "compound", gy, idx_min=r["idx_min"], idx_max=r["idx_max"])
    assert np.array_equal(gx[0], np.asarray(g["max"]["grad_x_ones"], np.float64)
                          + np.asarray(g["min"]["grad_x_ones"], np.float64))
    gw, none = orc.backward_weight(s, "compound", gy, idx_min=r["idx_min"], idx_max=r["idx_max"])
    assert none is None
    assert np.array_equal(gw, np.asarray(g["max"]["grad_w_ones"], np.float64)
                          + np.asarray(g["min"]["grad_w_ones"], np.float64))
    s2 = _shape(g["shape"], stride=2)
    r = orc.forward(s2, "max", x, w_max=w)
    assert np.array_equal(r["y"][0], _f(g["stride2_max"]["y"]))
    assert np.array_equal(r["idx_max"][0], g["stride2_max"]["idx"])


# ---------------------------------------------------------------- brute force on tiny inputs

def _tiny_cases():
    rng = np.random.default_rng(1234)
    cases = []
    for t in range(60):
        KH, KW = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        stride, dil = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        pad = int(rng.integers(0, 3))
        pad = min(pad, dil * (KH - 1), dil * (KW - 1))
        N, C, CO = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        H = int(rng.integers(max(1, dil * (KH - 1) + 1 - 2 * pad), 7))
        W = int(rng.integers(max(1, dil * (KW - 1) + 1 - 2 * pad), 7))
        cases.append((t, N, C, H, W, CO, KH, KW, stride, pad, dil))
    return cases


@pytest.mark.parametrize("case", _tiny_cases(), ids=lambda c: "t%d" % c[0])
def test_brute_force_tiny(case):
    t, N, C, H, W, CO, KH, KW, stride, pad, dil = case
    rng = np.random.default_rng(100 + t)
    integer = (t % 3 == 0)  # integer data: exact adds, many ties
    if integer:
        x = rng.integers(-3, 4, (N, C, H, W)).astype(np.float32)
        w1 = rng.integers(-3, 4, (CO, C, KH, KW)).astype(np.float32)
        w2 = rng.integers(-3, 4, (CO, C, KH, KW)).astype(np.float32)
    else:
        x = rng.standard_normal((N, C, H, W)).astype(np.float32)
        w1 = rng.uniform(-1, 1, (CO, C, KH, KW)).astype(np.float32)
        w2 = rng.uniform(-1, 1, (CO, C, KH, KW)).astype(np.float32)
    alpha = rng.uniform(-1, 1, CO).astype(np.float32)
    beta = rng.uniform(-1, 1, CO).astype(np.float32)
    s = orc.Shape(N, C, H, W, CO, KH, KW, stride, pad, dil)
    ymx1, imx1 = brute.forward(x, w1, True, stride, pad, dil)
    ymn1, imn1 = brute.forward(x, w1, False, stride, pad, dil)
    ymx2, imx2 = brute.forward(x, w2, True, stride, pad, dil)
    gy = rng.standard_normal(ymx1.shape).astype(np.float32)

    r = orc.forward(s, "max", x, w_max=w1)
    assert np.array_equal(r["y"].view(np.int32), ymx1.view(np.int32)) and np.array_equal(r["idx_max"], imx1)
    assert r["y_min"] is None and r["idx_min"] is None
    r = orc.forward(s, "min", x, w_min=w1)
    assert np.array_equal(r["y"].view(np.int32), ymn1.view(np.int32)) and np.array_equal(r["idx_min"], imn1)

    for mode, wmn, wmx, ymn, imn, ymx, imx in (
            ("compound", w1, w1, ymn1, imn1, ymx1, imx1),
            ("parallel", w1, w2, ymn1, imn1, ymx2, imx2)):
        for a, b in ((None, None), (alpha, beta)):
            r = orc.forward(s, mode, x, w_min=wmn, w_max=wmx, alpha=a, beta=b)
            assert np.array_equal(r["y_min"].view(np.int32), ymn.view(np.int32))
            assert np.array_equal(r["y_max"].view(np.int32), ymx.view(np.int32))
            assert np.array_equal(r["idx_min"], imn) and np.array_equal(r["idx_max"], imx)
            assert np.array_equal(r["y"].view(np.int32), brute.combine(ymn, ymx, a, b).view(np.int32))
            ga = gy if a is None else gy.astype(np.float64) * a[None, :, None, None].astype(np.float64)
            gb = gy if b is None else gy.astype(np.float64) * b[None, :, None, None].astype(np.float64)
            gx_mn, gw_mn = brute.scatter_backward(x.shape, w1.shape, imn, ga, stride, pad, dil)
            gx_mx, gw_mx = brute.scatter_backward(x.shape, w1.shape, imx, gb, stride, pad, dil)
            gx = orc.backward_input(s, mode, gy, idx_min=imn, idx_max=imx, alpha=a, beta=b)
            np.testing.assert_allclose(gx, gx_mn + gx_mx, rtol=1e-12, atol=1e-12)
            g1, g2 = orc.backward_weight(s, mode, gy, idx_min=imn, idx_max=imx, alpha=a, beta=b)
            if mode == "compound":
                assert g2 is None
                np.testing.assert_allclose(g1, gw_mn + gw_mx, rtol=1e-12, atol=1e-12)
            else:
                np.testing.assert_allclose(g1, gw_mn, rtol=1e-12, atol=1e-12)
                np.testing.assert_allclose(g2, gw_mx, rtol=1e-12, atol=1e-12)

    # single-branch backward: no alpha / beta scaling
    gx_b, gw_b = brute.scatter_backward(x.shape, w1.shape, imx1, gy, stride, pad, dil)
    np.testing.assert_allclose(orc.backward_input(s, "max", gy, idx_max=imx1, alpha=alpha, beta=beta), gx_b,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.backward_weight(s, "max", gy, idx_max=imx1)[1], gw_b, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- library special cases

@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 2, 2), (1, 0, 1), (2, 0, 2)])
def test_zero_kernel_is_channel_max_of_maxpool(stride, pad, dil):
    """w == 0: y_max = max over channels of max_pool2d(x) (-inf padded); y_min by duality."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 3, 9, 8)).astype(np.float32)
    s = orc.Shape(2, 3, 9, 8, 2, 3, 3, stride, pad, dil)
    w = np.zeros((2, 3, 3, 3), np.float32)
    xt = torch.from_numpy(x)
    xp = F.pad(xt, (pad, pad, pad, pad), value=float("-inf"))
    ref = F.max_pool2d(xp, 3, stride=stride, padding=0, dilation=dil).amax(dim=1, keepdim=True)
    r = orc.forward(s, "max", x, w_max=w)
    assert np.array_equal(r["y"], ref.expand(-1, 2, -1, -1).numpy())
    xn = F.pad(-xt, (pad, pad, pad, pad), value=float("-inf"))
    refmin = -F.max_pool2d(xn, 3, stride=stride, padding=0, dilation=dil).amax(dim=1, keepdim=True)
    r = orc.forward(s, "min", x, w_min=w)
    assert np.array_equal(r["y"], refmin.expand(-1, 2, -1, -1).numpy())


@pytest.mark.parametrize("stride,pad,dil,k", [(1, 1, 1, 3), (2, 1, 1, 3), (1, 2, 2, 3), (1, 0, 1, 2), (2, 2, 1, 5)])
def test_unfold_formulation(stride, pad, dil, k):
    """The three-step description of App. A.1.1: unfold, broadcast add, reduce; torch ops only."""
    rng = np.random.default_rng(11)
    N, C, H, W, CO = 2, 3, 10, 9, 4
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.uniform(-1, 1, (CO, C, k, k)).astype(np.float32)
    s = orc.Shape(N, C, H, W, CO, k, k, stride, pad, dil)
    ho, wo = orc.out_shape(s)
    for mode, fill, red, arg in (("max", float("-inf"), torch.amax, torch.argmax),
                                 ("min", float("inf"), torch.amin, torch.argmin)):
        xp = F.pad(torch.from_numpy(x), (pad, pad, pad, pad), value=fill)
        cols = F.unfold(xp, k, dilation=dil, padding=0, stride=stride)          # [N, K, L]
        sums = cols[:, None, :, :] + torch.from_numpy(w).reshape(1, CO, -1, 1)   # [N, CO, K, L]
        yref = red(sums, dim=2).reshape(N, CO, ho, wo).numpy()
        iref = arg(sums, dim=2).reshape(N, CO, ho, wo).numpy()
        r = orc.forward(s, mode, x, **{"w_" + mode: w})
        assert np.array_equal(r["y"], yref)
        # random data: the extremum is unique, so argmax needs no tie rule
        assert np.array_equal(r["idx_" + mode], iref)


def test_1x1_single_channel_is_broadcast_add():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 1, 5, 6)).astype(np.float32)
    w = rng.uniform(-1, 1, (3, 1, 1, 1)).astype(np.float32)
    s = orc.Shape(2, 1, 5, 6, 3, 1, 1)
    for mode in ("max", "min"):
        r = orc.forward(s, mode, x, **{"w_" + mode: w})
        assert np.array_equal(r["y"], x + w.reshape(1, 3, 1, 1))
        assert not r["idx_" + mode].any()


def test_bf16_output_rounding_matches_library_cast():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 2, 6, 6)).astype(np.float32)
    w = rng.uniform(-1, 1, (3, 2, 3, 3)).astype(np.float32)
    s = orc.Shape(1, 2, 6, 6, 3, 3, 3, 1, 1, 1)
    full = orc.forward(s, "compound", x, w_min=w)
    r = orc.forward(s, "compound", x, w_min=w, out_bf16=True)
    for key in ("y", "y_min", "y_max"):
        ref = torch.from_numpy(full[key]).to(torch.bfloat16).to(torch.float32).numpy()
        assert np.array_equal(r[key], ref)
    assert np.array_equal(r["idx_min"], full["idx_min"]) and np.array_equal(r["idx_max"], full["idx_max"])


# ---------------------------------------------------------------- invariants

def _rand_layer(seed, N=2, C=3, H=8, W=7, CO=4, k=3, stride=1, pad=1, dil=1, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        x = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
        w = rng.integers(-4, 5, (CO, C, k, k)).astype(np.float32)
        w2 = rng.integers(-4, 5, (CO, C, k, k)).astype(np.float32)
    else:
        x = rng.standard_normal((N, C, H, W)).astype(np.float32)
        w = rng.uniform(-1, 1, (CO, C, k, k)).astype(np.float32)
        w2 = rng.uniform(-1, 1, (CO, C, k, k)).astype(np.float32)
    return orc.Shape(N, C, H, W, CO, k, k, stride, pad, dil), x, w, w2, rng


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 2, 2)])
def test_duality_and_ordering(integer, stride, pad, dil):
    """min-plus(x, w) = -max-plus(-x, -w) with identical indices; y_max >= y_min for a shared kernel."""
    s, x, w, _, _ = _rand_layer(21, stride=stride, pad=pad, dil=dil, integer=integer)
    mx = orc.forward(s, "max", x, w_max=w)
    mn = orc.forward(s, "min", x, w_min=w)
    dual = orc.forward(s, "max", -x, w_max=-w)
    assert np.array_equal(mn["y"], -dual["y"]) and np.array_equal(mn["idx_min"], dual["idx_max"])
    assert (mx["y"] >= mn["y"]).all()


def test_shift_equivariance_exact_on_integers():
    """x + c or w + c shifts both outputs by c and leaves the indices alone (c a power of two, integer data)."""
    s, x, w, _, _ = _rand_layer(22, integer=True)
    base = orc.forward(s, "compound", x, w_min=w)
    for c in (8.0, -16.0):
        for xs, ws in ((x + np.float32(c), w), (x, w + np.float32(c))):
            r = orc.forward(s, "compound", xs, w_min=ws)
            assert np.array_equal(r["y_min"], base["y_min"] + np.float32(c))
            assert np.array_equal(r["y_max"], base["y_max"] + np.float32(c))
            assert np.array_equal(r["idx_min"], base["idx_min"]) and np.array_equal(r["idx_max"], base["idx_max"])


def test_monotone_in_x():
    s, x, w, _, rng = _rand_layer(23)
    bump = np.abs(rng.standard_normal(x.shape)).astype(np.float32)
    lo = orc.forward(s, "compound", x, w_min=w)
    hi = orc.forward(s, "compound", x + bump, w_min=w)
    assert (hi["y_min"] >= lo["y_min"]).all() and (hi["y_max"] >= lo["y_max"]).all()


@pytest.mark.parametrize("integer", [False, True])
def test_degeneracy_and_shared_kernel(integer):
    """(alpha, beta) = (1, 0) -> min-plus, (0, 1) -> max-plus (Sec. 3.3); compound(W) == parallel(W, W)."""
    s, x, w, w2, _ = _rand_layer(24, integer=integer)
    one, zero = np.ones(s.C_out, np.float32), np.zeros(s.C_out, np.float32)
    mn = orc.forward(s, "min", x, w_min=w)
    mx = orc.forward(s, "max", x, w_max=w2)
    p10 = orc.forward(s, "parallel", x, w_min=w, w_max=w2, alpha=one, beta=zero)
    p01 = orc.forward(s, "parallel", x, w_min=w, w_max=w2, alpha=zero, beta=one)
    assert np.array_equal(p10["y"], mn["y"] + np.float32(0)) and np.array_equal(p01["y"], mx["y"] + np.float32(0))
    cp = orc.forward(s, "compound", x, w_min=w)
    pp = orc.forward(s, "parallel", x, w_min=w, w_max=w)
    for key in cp:
        assert np.array_equal(cp[key], pp[key])
    # compound accepts the kernel through either pointer
    cp2 = orc.forward(s, "compound", x, w_max=w)
    for key in cp:
        assert np.array_equal(cp[key], cp2[key])


@pytest.mark.parametrize("stride,pad,dil", [(1, 1, 1), (2, 1, 1), (1, 2, 2)])
def test_indices_are_valid_and_reproduce_the_value(stride, pad, dil):
    s, x, w, w2, _ = _rand_layer(25, stride=stride, pad=pad, dil=dil)
    r = orc.forward(s, "parallel", x, w_min=w, w_max=w2)
    ho, wo = orc.out_shape(s)
    for key, wt, yk in (("idx_min", w, "y_min"), ("idx_max", w2, "y_max")):
        idx = r[key]
        assert idx.min() >= 0 and idx.max() < s.K
        for n, co, oh, ow in itertools.product(range(s.N), range(s.C_out), range(ho), range(wo)):
            k = int(idx[n, co, oh, ow])
            c, rem = divmod(k, 9)
            i, j = divmod(rem, 3)
            ih, iw = oh * stride - pad + i * dil, ow * stride - pad + j * dil
            assert 0 <= ih < s.H and 0 <= iw < s.W
            assert np.float32(x[n, c, ih, iw] + wt[co, c, i, j]) == r[yk][n, co, oh, ow]


def test_gradient_mass_conservation():
    """Each output deposits its whole gradient once per branch: sum grad_x = sum grad_w = sum of branch gradients."""
    s, x, w, w2, rng = _rand_layer(26)
    r = orc.forward(s, "parallel", x, w_min=w, w_max=w2)
    gy = rng.standard_normal(r["y"].shape).astype(np.float32)
    alpha = rng.uniform(-1, 1, s.C_out).astype(np.float32)
    beta = rng.uniform(-1, 1, s.C_out).astype(np.float32)
    total = (gy.astype(np.float64) * (alpha.astype(np.float64) + beta.astype(np.float64))[None, :, None, None]).sum()
    gx = orc.backward_input(s, "parallel", gy, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=alpha, beta=beta)
    g1, g2 = orc.backward_weight(s, "parallel", gy, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=alpha, beta=beta)
    assert abs(gx.sum() - total) < 1e-9 and abs(g1.sum() + g2.sum() - total) < 1e-9


def test_spatial_translation_of_interior():
    """Shifting x by one stride step shifts interior outputs by one pixel."""
    s, x, w, _, _ = _rand_layer(27, H=10, W=10, stride=2, pad=1)
    r0 = orc.forward(s, "max", x, w_max=w)
    xs = np.roll(x, shift=(2, 2), axis=(2, 3))
    r1 = orc.forward(s, "max", xs, w_max=w)
    assert np.array_equal(r1["y"][:, :, 2:-1, 2:-1], r0["y"][:, :, 1:-2, 1:-2])
    assert np.array_equal(r1["idx_max"][:, :, 2:-1, 2:-1], r0["idx_max"][:, :, 1:-2, 1:-2])


# ---------------------------------------------------------------- finite differences

@pytest.mark.parametrize("mode", ["max", "min", "compound", "parallel"])
def test_backward_against_finite_differences(mode):
    """L = sum(gy * y) is piecewise linear; where no winner changes within +-h the central difference is exact."""
    s, x, w, w2, rng = _rand_layer(31, N=1, C=2, H=5, W=5, CO=2)
    alpha = rng.uniform(0.25, 1, s.C_out).astype(np.float32)
    beta = rng.uniform(-1, -0.25, s.C_out).astype(np.float32)
    wmn, wmx = (w, w2) if mode == "parallel" else (w, w)

    def loss(xv, wmnv, wmxv):
        tot, sig = 0.0, []
        if mode != "max":
            y, i = brute.forward(xv, wmnv, False, 1, 1, 1, dtype=np.float64)
            coef = alpha[None, :, None, None].astype(np.float64) if mode in ("compound", "parallel") else 1.0
            tot += (gy * coef * y).sum()
            sig.append(i)
        if mode != "min":
            y, i = brute.forward(xv, wmxv, True, 1, 1, 1, dtype=np.float64)
            coef = beta[None, :, None, None].astype(np.float64) if mode in ("compound", "parallel") else 1.0
            tot += (gy * coef * y).sum()
            sig.append(i)
        return tot, np.stack(sig)

    r = orc.forward(s, mode, x, w_min=wmn if mode != "max" else None, w_max=wmx if mode != "min" else None,
                    alpha=alpha, beta=beta)
    gy = rng.standard_normal(r["y"].shape).astype(np.float64)
    gyf = gy.astype(np.float32)
    gy = gyf.astype(np.float64)
    gx = orc.backward_input(s, mode, gyf, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=alpha, beta=beta)
    g1, g2 = orc.backward_weight(s, mode, gyf, idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=alpha, beta=beta)
    h = 2.0 ** -10
    x64, wmn64, wmx64 = x.astype(np.float64), wmn.astype(np.float64), wmx.astype(np.float64)
    checked = 0
    for pos in itertools.product(range(1), range(2), range(5), range(5)):
        xp, xm = x64.copy(), x64.copy()
        xp[pos] += h
        xm[pos] -= h
        (lp, sp), (lm, sm) = loss(xp, wmn64, wmx64), loss(xm, wmn64, wmx64)
        if np.array_equal(sp, sm):
            assert abs((lp - lm) / (2 * h) - gx[pos]) < 1e-6
            checked += 1
    assert checked >= 25
    # kernel gradients, a sample of taps
    checked = 0
    for pos in itertools.product(range(2), range(2), range(3), range(3)):
        if mode == "compound":
            wp, wm = wmn64.copy(), wmn64.copy()
            wp[pos] += h
            wm[pos] -= h
            (lp, sp), (lm, sm) = loss(x64, wp, wp), loss(x64, wm, wm)
            ref = g1[pos]
        elif mode == "parallel":
            wp, wm = wmx64.copy(), wmx64.copy()
            wp[pos] += h
            wm[pos] -= h
            (lp, sp), (lm, sm) = loss(x64, wmn64, wp), loss(x64, wmn64, wm)
            ref = g2[pos]
        else:
            wp, wm = wmn64.copy(), wmn64.copy()
            wp[pos] += h
            wm[pos] -= h
            (lp, sp), (lm, sm) = loss(x64, wp, wp), loss(x64, wm, wm)
            ref = (g2 if mode == "max" else g1)[pos]
        if np.array_equal(sp, sm):
            assert abs((lp - lm) / (2 * h) - ref) < 1e-6
            checked += 1
    assert checked >= 18


# ---------------------------------------------------------------- argument checking and counts

def test_rejects_window_that_can_lie_in_padding():
    s = orc.Shape(1, 1, 4, 4, 1, 3, 3, 1, 3, 1)
    with pytest.raises(ValueError):
        orc.forward(s, "max", np.zeros((1, 1, 4, 4), np.float32), w_max=np.zeros((1, 1, 3, 3), np.float32))


def test_pair_count_formula():
    """adds = K_h K_w C_in C_out H_out W_out per image for the max / min channel layers (Sec. 4.1)."""
    from paper_2504_06881_amd.inputs import CONFIGS
    c = CONFIGS["cfg3a"]
    assert c.candidates == 64 * (3 * 3 * 64 * 64 * 56 * 56) and c.pairs == 2 * c.candidates
    c = CONFIGS["cfg3b"]
    assert c.out_hw == (14, 14) and c.candidates == 64 * 1152 * 256 * 14 * 14
    assert CONFIGS["cfg4b"].out_hw == (64, 64)
    assert CONFIGS["cfg1"].pairs == 2 * 8 * 16 * 16 * 27


# ---------------------------------------------------------------- gradient of the combine step

@pytest.mark.parametrize("mode", ["compound", "parallel"])
def test_alpha_beta_gradient_against_finite_differences(mode):
    """L = sum(gy * (alpha*y_min + beta*y_max)) is linear in alpha and beta (Sec. 3.3), so a central
    difference of the fp64 brute-force forward in one alpha[c] / beta[c] is the exact gradient."""
    s, x, w, w2, rng = _rand_layer(41, N=2, C=2, H=5, W=4, CO=3)
    wmn, wmx = (w, w2) if mode == "parallel" else (w, w)
    alpha = rng.uniform(-1, 1, s.C_out)
    beta = rng.uniform(-1, 1, s.C_out)
    r = orc.forward(s, mode, x, w_min=wmn, w_max=wmx)
    gy = rng.standard_normal(r["y"].shape).astype(np.float32)
    ga, gb = orc.backward_alpha_beta(s, mode, gy, r["y_min"], r["y_max"])
    ymn, _ = brute.forward(x.astype(np.float64), wmn.astype(np.float64), False, 1, 1, 1, dtype=np.float64)
    ymx, _ = brute.forward(x.astype(np.float64), wmx.astype(np.float64), True, 1, 1, 1, dtype=np.float64)

    def loss(a, b):
        return (gy.astype(np.float64) * (a[None, :, None, None] * ymn + b[None, :, None, None] * ymx)).sum()

    h = 0.125
    for c in range(s.C_out):
        e = np.zeros(s.C_out)
        e[c] = h
        assert abs((loss(alpha + e, beta) - loss(alpha - e, beta)) / (2 * h) - ga[c]) < 1e-5
        assert abs((loss(alpha, beta + e) - loss(alpha, beta - e)) / (2 * h) - gb[c]) < 1e-5


def test_alpha_beta_gradient_special_cases():
    """gy == 1 turns the gradients into plain per-channel sums of the branch outputs (library sum);
    a gy that is non-zero in one channel only leaves every other channel's gradient at zero; and the
    gradients of the degenerate pairs (1, 0) / (0, 1) of Sec. 3.3 are those of the single branches."""
    s, x, w, _, rng = _rand_layer(42, N=3, C=2, H=6, W=5, CO=4, integer=True)
    r = orc.forward(s, "compound", x, w_min=w, w_max=w)
    ones = np.ones(r["y"].shape, np.float32)
    ga, gb = orc.backward_alpha_beta(s, "compound", ones, r["y_min"], r["y_max"])
    assert np.array_equal(ga, r["y_min"].astype(np.float64).sum(axis=(0, 2, 3)))   # integers: exact
    assert np.array_equal(gb, r["y_max"].astype(np.float64).sum(axis=(0, 2, 3)))
    gy = np.zeros(r["y"].shape, np.float32)
    gy[:, 2] = rng.standard_normal(gy[:, 2].shape).astype(np.float32)
    ga, gb = orc.backward_alpha_beta(s, "compound", gy, r["y_min"], r["y_max"])
    assert ga[2] != 0 and gb[2] != 0
    assert not ga[[0, 1, 3]].any() and not gb[[0, 1, 3]].any()
    # y_min, y_max do not depend on alpha / beta: swapping the two branch tensors swaps the two gradients
    ga2, gb2 = orc.backward_alpha_beta(s, "compound", gy, r["y_max"], r["y_min"])
    assert np.array_equal(ga2, gb) and np.array_equal(gb2, ga)
    with pytest.raises(ValueError):
        orc.backward_alpha_beta(s, "max", gy, r["y_min"], r["y_max"])
