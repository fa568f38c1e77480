"""Pins of the extension oracle (oracle/text_oracle.c): zero padding, epilogue, half-precision contract.

None of these re-types the oracle's loop nest: zero padding is pinned against the already pinned main oracle run on an
explicitly padded input, against the unfold formulation of App. A.1.1 written with library routines (F.unfold pads
with zeros by itself) and a hand-worked fixture; the epilogue against elementwise numpy fp32 arithmetic on the main
oracle's outputs; the half-precision arithmetic against numpy's correctly rounded float16 type."""
import json
import os

import numpy as np
import pytest

from oracle import tconv_oracle as orc
from oracle import text_oracle as ext

HERE = os.path.dirname(os.path.abspath(__file__))
MODES = ("max", "min", "compound", "parallel")


def draw(rng, s, mode, integer=False):
    xs, ws = (s.N, s.C_in, s.H, s.W), (s.C_out, s.C_in, s.KH, s.KW)
    if integer:
        x = rng.integers(-3, 4, xs).astype(np.float32)
        w1 = rng.integers(-3, 4, ws).astype(np.float32)
        w2 = rng.integers(-3, 4, ws).astype(np.float32)
    else:
        x = rng.standard_normal(xs).astype(np.float32)
        w1 = rng.uniform(-1, 1, ws).astype(np.float32)
        w2 = rng.uniform(-1, 1, ws).astype(np.float32)
    w_min = None if mode == "max" else w1
    w_max = None if mode == "min" else (w1 if mode == "compound" else w2)
    if mode == "max":
        w_max = w1
    ho, wo = s.out_hw
    gy = rng.standard_normal((s.N, s.C_out, ho, wo)).astype(np.float32)
    alpha = rng.uniform(-1, 1, s.C_out).astype(np.float32) if mode in ("compound", "parallel") else None
    beta = rng.uniform(-1, 1, s.C_out).astype(np.float32) if mode in ("compound", "parallel") else None
    return x, w_min, w_max, gy, alpha, beta


SHAPES = [
    ext.Shape(2, 3, 6, 7, 4, 3, 3, 1, 1, 1),
    ext.Shape(1, 2, 7, 5, 3, 3, 3, 2, 1, 1),
    ext.Shape(1, 2, 8, 8, 2, 3, 3, 1, 2, 2),
    ext.Shape(1, 3, 5, 6, 2, 5, 5, 1, 2, 1),
    ext.Shape(2, 1, 4, 4, 3, 2, 3, 1, 1, 1),
    ext.Shape(1, 2, 3, 3, 2, 3, 3, 1, 2, 1),     # padding 2 under a 3x3 window: corner windows hold one real tap
    ext.Shape(1, 4, 9, 9, 5, 1, 1, 1, 0, 1),
]


def main_shape(s, pad=None, H=None, W=None):
    return orc.Shape(s.N, s.C_in, s.H if H is None else H, s.W if W is None else W, s.C_out, s.KH, s.KW, s.stride,
                     s.pad if pad is None else pad, s.dil)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("integer", [False, True])
def test_identity_padding_equals_the_main_oracle(mode, integer):
    rng = np.random.default_rng(5)
    for s in SHAPES:
        x, w_min, w_max, gy, alpha, beta = draw(rng, s, mode, integer)
        a = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=False)
        b = orc.forward(main_shape(s), mode, x, w_min, w_max, alpha, beta)
        for k in ("y", "y_min", "y_max", "idx_min", "idx_max"):
            assert (a[k] is None) == (b[k] is None)
            if a[k] is not None:
                assert np.array_equal(a[k], b[k]), (s, k)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("integer", [False, True])
def test_zero_padding_equals_the_main_oracle_on_a_padded_input(mode, integer):
    """Zero padding = no padding on an input that was padded with zeros beforehand: same candidates, same tap
    numbers.  Gradients: the padded input's gradient cropped to the image, and the same kernel gradient."""
    rng = np.random.default_rng(6)
    for s in SHAPES:
        if s.pad == 0:
            continue
        x, w_min, w_max, gy, alpha, beta = draw(rng, s, mode, integer)
        p = s.pad
        xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
        sp = main_shape(s, pad=0, H=s.H + 2 * p, W=s.W + 2 * p)
        a = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=True)
        b = orc.forward(sp, mode, xp, w_min, w_max, alpha, beta)
        for k in ("y", "y_min", "y_max", "idx_min", "idx_max"):
            if a[k] is not None:
                assert np.array_equal(a[k], b[k]), (s, k)
        ga = ext.backward(s, mode, gy, a["idx_min"], a["idx_max"], alpha, beta)
        gxp = orc.backward_input(sp, mode, gy, b["idx_min"], b["idx_max"], alpha, beta)
        gwn, gwx = orc.backward_weight(sp, mode, gy, b["idx_min"], b["idx_max"], alpha, beta)
        assert np.array_equal(ga["grad_x"], gxp[:, :, p:p + s.H, p:p + s.W])
        for got, want in ((ga["grad_w_min"], gwn), (ga["grad_w_max"], gwx)):
            assert (got is None) == (want is None)
            if got is not None:
                assert np.array_equal(got, want)
        # what fell into the padding is exactly what the cropped gradient lacks
        lost = gxp.sum() - gxp[:, :, p:p + s.H, p:p + s.W].sum()
        assert np.isclose(ga["grad_x"].sum() + lost, gxp.sum())


@pytest.mark.parametrize("integer", [False, True])
def test_zero_padding_equals_the_unfold_formulation(integer):
    """App. A.1.1: unfold the (zero-padded) input into columns, add the kernel row, reduce over the column."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(7)
    for s in SHAPES:
        for mode in ("max", "min"):
            x, w_min, w_max, gy, alpha, beta = draw(rng, s, mode, integer)
            w = w_max if mode == "max" else w_min
            cols = F.unfold(torch.from_numpy(x), (s.KH, s.KW), dilation=s.dil, padding=s.pad, stride=s.stride).numpy()
            sums = cols[:, None, :, :] + w.reshape(s.C_out, -1)[None, :, :, None]      # [N, C_out, K, L], fp32 adds
            ho, wo = s.out_hw
            val = (sums.max(axis=2) if mode == "max" else sums.min(axis=2)).reshape(s.N, s.C_out, ho, wo)
            arg = (sums.argmax(axis=2) if mode == "max" else sums.argmin(axis=2)).reshape(s.N, s.C_out, ho, wo)
            a = ext.forward(s, mode, x, w_min, w_max, pad_zero=True)
            assert np.array_equal(a["y"], val.astype(np.float32))
            assert np.array_equal(a["idx_" + mode], arg.astype(np.int32))   # numpy returns the first extremum: lowest k


def test_zero_padding_hand_worked_fixture():
    g = json.load(open(os.path.join(HERE, "golden", "example_b_zero_padding.json")))
    x = np.array(g["x"], np.float32).reshape(1, 1, 3, 3)
    w = np.zeros((1, 1, 3, 3), np.float32)
    s = ext.Shape(1, 1, 3, 3, 1, 3, 3, 1, 1, 1)
    a = ext.forward(s, "max", x, None, w, pad_zero=True)
    b = ext.forward(s, "min", x, w, None, pad_zero=True)
    assert a["y"][0, 0].tolist() == g["max_y"] and a["idx_max"][0, 0].tolist() == g["max_idx"]
    assert b["y"][0, 0].tolist() == g["min_y"] and b["idx_min"][0, 0].tolist() == g["min_idx"]
    # a padded winner has no input element: with gy = 1 only the centre window's gradient (k = 0 -> x[0, 0]) arrives
    gb = ext.backward(s, "min", np.ones((1, 1, 3, 3), np.float32), idx_min=b["idx_min"])
    want = np.zeros((3, 3)); want[0, 0] = 1.0
    assert gb["grad_x"][0, 0].tolist() == want.tolist()
    assert gb["grad_w_min"].sum() == 9.0 and gb["grad_w_min"][0, 0, 0, 0] == 6.0


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("pad_zero", [False, True])
def test_epilogue_is_the_elementwise_chain(mode, pad_zero):
    """y of the epilogue = ((y0 + bias) * scale + shift) + residual in separately rounded fp32 operations on the bare
    layer's y0 (numpy float32 arithmetic rounds every operation); branch outputs and indices are the bare layer's."""
    rng = np.random.default_rng(8)
    for s in SHAPES[:5]:
        x, w_min, w_max, gy, alpha, beta = draw(rng, s, mode)
        ho, wo = s.out_hw
        bias = rng.standard_normal(s.C_out).astype(np.float32)
        scale = rng.uniform(0.5, 2, s.C_out).astype(np.float32)
        shift = rng.standard_normal(s.C_out).astype(np.float32)
        res = rng.standard_normal((s.N, s.C_out, ho, wo)).astype(np.float32)
        bare = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=pad_zero)
        y0 = bare["y"]
        bc = lambda v: v[None, :, None, None]
        for use in [(1, 0, 0), (0, 1, 0), (0, 0, 1), (1, 1, 1), (1, 1, 0)]:
            t = y0.copy()
            if use[0]:
                t = (t + bc(bias)).astype(np.float32)
            if use[1]:
                t = ((t * bc(scale)).astype(np.float32) + bc(shift)).astype(np.float32)
            if use[2]:
                t = (t + res).astype(np.float32)
            a = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=pad_zero, bias=bias if use[0] else None,
                            scale=scale if use[1] else None, shift=shift if use[1] else None,
                            residual=res if use[2] else None)
            assert np.array_equal(a["y"], t), (s, use)
            for k in ("y_min", "y_max", "idx_min", "idx_max"):
                if a[k] is not None:
                    assert np.array_equal(a[k], bare[k])
        # neutral elements leave y untouched; scale without shift adds nothing
        ones, zeros = np.ones(s.C_out, np.float32), np.zeros(s.C_out, np.float32)
        a = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=pad_zero, bias=zeros, scale=ones, shift=zeros,
                        residual=np.zeros_like(res))
        assert np.array_equal(a["y"], (y0 + np.float32(0)).astype(np.float32))
        a = ext.forward(s, mode, x, w_min, w_max, alpha, beta, pad_zero=pad_zero, scale=scale)
        assert np.array_equal(a["y"], ((y0 * bc(scale)).astype(np.float32) + np.float32(0)).astype(np.float32))
        assert np.allclose(ext.backward_bias(s, gy), gy.astype(np.float64).sum(axis=(0, 2, 3)))


# ---------------------------------------------------------------- half precision

def test_half_conversions_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in list(range(0, 65536, 7)) + [0x0001, 0x03ff, 0x0400, 0x7bff, 0x7c00, 0xfbff, 0xfc00, 0x8000]:
        v = ext.half_to_double(b)
        assert (np.isnan(v) and np.isnan(ref[b])) or v == ref[b], hex(b)
    rng = np.random.default_rng(9)
    vals = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-8, 5, 2000),
                           [0.0, 65504.0, 65519.99, 65520.0, 1e-8, 2.0 ** -25, 2.0 ** -24, 3 * 2.0 ** -25,
                            1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -14 - 2.0 ** -25]])
    # exact midpoints between neighbouring halves: ties must go to the even mantissa
    h = rng.integers(0x0001, 0x7bfe, 500).astype(np.uint16)
    mid = (h.view(np.float16).astype(np.float64) + (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)) / 2
    vals = np.concatenate([vals, mid, -mid])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    for v, w in zip(vals, want):
        assert ext.double_to_half(float(v)) == int(w), v


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("pad_zero", [False, True])
@pytest.mark.parametrize("coarse", [False, True])
def test_half_forward_against_numpy_float16(mode, pad_zero, coarse):
    """Candidates formed with numpy's float16 add (correctly rounded), reduced with amax / first argmax; the combine in
    float32, rounded to float16.  coarse: values on a grid of 1/4 with a wide range, so that rounded sums tie."""
    rng = np.random.default_rng(10 + coarse)
    for s in SHAPES[:6]:
        if pad_zero is False and (s.pad > s.dil * (s.KH - 1)):
            continue
        x, w_min, w_max, gy, alpha, beta = draw(rng, s, mode)
        if coarse:
            q = lambda a: None if a is None else (np.round(a * 4) * 512).astype(np.float32)
            x, w_min, w_max = q(x), q(w_min), q(w_max)
        h = lambda a: None if a is None else a.astype(np.float16)
        xh, wmn, wmx = h(x), h(w_min), h(w_max)
        got = ext.forward_f16(s, mode, xh, wmn, wmx, alpha, beta, pad_zero=pad_zero)
        ho, wo = s.out_hw
        K = s.C_in * s.KH * s.KW
        # candidate table [N, K, Ho, Wo] of inputs (float16) with a validity mask
        tab = np.zeros((s.N, K, ho, wo), np.float16)
        ok = np.zeros((K, ho, wo), bool)
        for c in range(s.C_in):
            for i in range(s.KH):
                for j in range(s.KW):
                    k = (c * s.KH + i) * s.KW + j
                    for oh in range(ho):
                        for ow in range(wo):
                            ih, iw = oh * s.stride - s.pad + i * s.dil, ow * s.stride - s.pad + j * s.dil
                            if 0 <= ih < s.H and 0 <= iw < s.W:
                                tab[:, k, oh, ow] = xh[:, c, ih, iw]
                                ok[k, oh, ow] = True
                            elif pad_zero:
                                ok[k, oh, ow] = True
        res = {}
        for br, w in (("min", wmn), ("max", wmx)):
            if w is None or (mode == "max" and br == "min") or (mode == "min" and br == "max"):
                continue
            sums = tab[:, None] + w.reshape(s.C_out, K)[None, :, :, None, None]      # float16 arithmetic
            assert sums.dtype == np.float16
            f = sums.astype(np.float32)
            f[:, :, ~ok] = np.inf if br == "min" else -np.inf
            res[br] = ((f.min(axis=2), f.argmin(axis=2)) if br == "min" else (f.max(axis=2), f.argmax(axis=2)))
        if mode in ("max", "min"):
            v, i = res[mode]
            assert np.array_equal(got["y"], v.astype(np.float16))
            assert np.array_equal(got["idx_" + mode], i.astype(np.int32))
        else:
            (vn, i_n), (vx, i_x) = res["min"], res["max"]
            bc = lambda a: a[None, :, None, None]
            comb = ((bc(alpha) * vn).astype(np.float32) + (bc(beta) * vx).astype(np.float32)).astype(np.float32)
            assert np.array_equal(got["y"], comb.astype(np.float16))
            assert np.array_equal(got["y_min"], vn.astype(np.float16)) and np.array_equal(got["y_max"], vx.astype(np.float16))
            assert np.array_equal(got["idx_min"], i_n.astype(np.int32)) and np.array_equal(got["idx_max"], i_x.astype(np.int32))


def test_half_duality_and_ordering():
    rng = np.random.default_rng(12)
    s = SHAPES[0]
    x, w_min, w_max, _, _, _ = draw(rng, s, "parallel")
    xh, w = x.astype(np.float16), w_min.astype(np.float16)
    mx = ext.forward_f16(s, "max", xh, None, w)
    mn = ext.forward_f16(s, "min", -xh, -w, None)
    assert np.array_equal(mx["y"], -mn["y"]) and np.array_equal(mx["idx_max"], mn["idx_min"])
    both = ext.forward_f16(s, "compound", xh, w, None)
    assert (both["y_max"].astype(np.float32) >= both["y_min"].astype(np.float32)).all()


# ---------------------------------------------------------------- gradient rules of a residual block

def _block_loss64(x, wa, wb, sa, ha, sb, hb, gy):
    """sum(gy * block(x)) in float64 by enumeration: block = conv_b(conv_a(x)*sa + ha)*sb + hb + x, both convs
    parallel-mode 3x3 / pad 1 with alpha = beta = 1 (Sec. 5 TCNN BasicBlock with the batch norms folded to affines)."""
    import brute

    def conv(v, w):
        y_min, _ = brute.forward(v, w[0], False, 1, 1, 1, dtype=np.float64)
        y_max, _ = brute.forward(v, w[1], True, 1, 1, 1, dtype=np.float64)
        return y_min + y_max

    a = conv(x, wa) * sa[None, :, None, None] + ha[None, :, None, None]
    b = conv(a, wb) * sb[None, :, None, None] + hb[None, :, None, None] + x
    return float(np.sum(gy.astype(np.float64) * b))


def test_residual_block_gradient_rules_against_finite_differences():
    """How the fused layers compose into a training step (the rule bench.py's end-to-end workload uses): the gradient of
    a fused layer's bare output is scale*g, passed to the backward call as alpha = beta = scale; grad_shift is the bias
    gradient of g; grad_scale is sum g*(y_min + y_max); the shortcut adds g to the block input's gradient.  Checked on
    the oracle's own forward / backward calls against central differences of a float64 enumeration of the block."""
    rng = np.random.Generator(np.random.PCG64(991))
    N, C, H, W = 2, 3, 5, 6
    s = ext.Shape(N, C, H, W, C, 3, 3, 1, 1, 1)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    wa = (rng.random((2, C, C, 3, 3), dtype=np.float32) * 2 - 1) * np.float32(0.5)
    wb = (rng.random((2, C, C, 3, 3), dtype=np.float32) * 2 - 1) * np.float32(0.5)
    sa, sb = (rng.uniform(0.3, 0.9, C).astype(np.float32) for _ in range(2))
    ha, hb = (rng.standard_normal(C).astype(np.float32) * np.float32(0.1) for _ in range(2))
    gy = rng.standard_normal((N, C, H, W)).astype(np.float32)
    ones = np.ones(C, np.float32)
    # forward through the fused layers
    fa = ext.forward(s, "parallel", x, wa[0], wa[1], ones, ones, scale=sa, shift=ha)
    fb = ext.forward(s, "parallel", fa["y"], wb[0], wb[1], ones, ones, scale=sb, shift=hb, residual=x)
    # backward by the rules
    gb = ext.backward(s, "parallel", gy, fb["idx_min"], fb["idx_max"], alpha=sb, beta=sb)
    g_hb = ext.backward_bias(s, gy)
    g_sb = np.sum(gy.astype(np.float64) * (fb["y_min"].astype(np.float64) + fb["y_max"]), axis=(0, 2, 3))
    g_mid = gb["grad_x"].astype(np.float32)
    ga = ext.backward(s, "parallel", g_mid, fa["idx_min"], fa["idx_max"], alpha=sa, beta=sa)
    g_ha = ext.backward_bias(s, g_mid)
    g_sa = np.sum(g_mid.astype(np.float64) * (fa["y_min"].astype(np.float64) + fa["y_max"]), axis=(0, 2, 3))
    g_x = ga["grad_x"] + gy
    args = dict(x=x, wa=wa, wb=wb, sa=sa, ha=ha, sb=sb, hb=hb)
    analytic = dict(x=g_x, wa=np.stack([ga["grad_w_min"], ga["grad_w_max"]]),
                    wb=np.stack([gb["grad_w_min"], gb["grad_w_max"]]), sa=g_sa, ha=g_ha, sb=g_sb, hb=g_hb)
    h = 2.0 ** -20   # small: a scale or shift moves every pixel of its channel, and a change of winner inside the
                     # interval would mix two slopes (the enumeration is float64, so the difference stays exact)
    for name in ("x", "wa", "wb", "sa", "ha", "sb", "hb"):
        flat = analytic[name].reshape(-1)
        for e in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            hi = {k: v.astype(np.float64).copy() for k, v in args.items()}
            lo = {k: v.astype(np.float64).copy() for k, v in args.items()}
            hi[name].reshape(-1)[e] += h
            lo[name].reshape(-1)[e] -= h
            fd = (_block_loss64(gy=gy, **hi) - _block_loss64(gy=gy, **lo)) / (2 * h)
            # the function is piecewise linear: away from a change of winner the central difference is exact
            assert abs(fd - flat[e]) <= 1e-4 * max(1.0, abs(fd)), (name, int(e), fd, float(flat[e]))
