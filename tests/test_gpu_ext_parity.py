"""GPU parity of the layer extensions against the extension oracle: zero padding (App. A.1.1), the fused epilogue
(bias of App. A.2, batch norm + shortcut of the Sec. 5 residual blocks) and the bias gradient.  Outputs and winners
bit for bit, gradients within 1e-5."""
import os

import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS, LayerCfg, make_inputs
from test_gpu_parity import BOTH_TN, KNOBS, MODES, RAGGED, RAGGED_LARGE, TILED, _random_layers

pytestmark = pytest.mark.gpu


def _check_ext(cfg, ep_kind="", alpha_beta=None, integer=False, kernel=None, tn=(None,), backward=True):
    inp = make_inputs(cfg, alpha_beta=alpha_beta, integer=integer)
    ep = hs.draw_epilogue(cfg, ep_kind)
    ref = hs.run_oracle_ext(cfg, inp, ep, backward=backward)
    old = {k: os.environ.pop(k, None) for k in KNOBS}
    try:
        if kernel:
            os.environ["TCONV_FORWARD_KERNEL"] = kernel
        for t in tn:
            os.environ.pop("TCONV_FWD_TN", None)
            os.environ["TCONV_FWD_KSPLIT"] = "1" if t == "ks" else "0" if t else ""
            if not t:
                os.environ.pop("TCONV_FWD_KSPLIT")
            elif t != "ks":
                os.environ["TCONV_FWD_TN"] = str(t)
            hip = hs.run_hip_ext(cfg, inp, ep, backward=backward)
            what = f"[{cfg.name} {cfg.mode} {cfg.dtype} pad={cfg.pad_mode} ep={ep_kind} int={integer} k={kernel} tn={t}] "
            hs.assert_forward_bit_exact(hip, ref, what=what)
            if backward:
                for k in ("grad_x", "grad_w_min", "grad_w_max", "grad_bias"):
                    if ref.get(k) is not None:
                        hs.assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k)
    finally:
        for k in KNOBS:
            os.environ.pop(k, None)
            if old[k] is not None:
                os.environ[k] = old[k]


ZERO_SHAPES = [c for c in RAGGED if c.pad > 0 and c.name not in ("r_cin300", "r_cin350", "r_cin130")]


@pytest.mark.parametrize("cfg", ZERO_SHAPES, ids=lambda c: c.name)
def test_zero_padding_ragged_shapes(cfg):
    cfg = cfg.with_(pad_mode="zero")
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) in TILED
    tn = BOTH_TN if tiled else (None,)
    for mode in MODES:
        _check_ext(cfg.with_(mode=mode), alpha_beta="random" if mode in ("compound", "parallel") else None, tn=tn)
        _check_ext(cfg.with_(mode=mode), integer=True, tn=tn)   # integer data: padded and real taps tie all the time
    if tiled:
        _check_ext(cfg.with_(mode="compound"), kernel="generic")
        _check_ext(cfg.with_(mode="parallel"), integer=True, kernel="generic")


@pytest.mark.parametrize("cfg", RAGGED_LARGE[:3], ids=lambda c: c.name)
def test_zero_padding_large_ragged_shapes(cfg):
    for mode in ("compound", "parallel", "max"):
        _check_ext(cfg.with_(mode=mode, pad_mode="zero"), integer=(mode == "parallel"))


@pytest.mark.parametrize("mode", MODES)
def test_zero_padding_bf16_storage(mode):
    for base in (RAGGED[0], RAGGED[2], RAGGED[4]):
        cfg = base.with_(mode=mode, dtype="bf16", pad_mode="zero")
        _check_ext(cfg, tn=BOTH_TN)
        _check_ext(cfg, integer=True, tn=BOTH_TN)


@pytest.mark.parametrize("pad_mode", ["identity", "zero"])
@pytest.mark.parametrize("cfg", [RAGGED[0], RAGGED[1], RAGGED[2], RAGGED[4], RAGGED[10], RAGGED[12]], ids=lambda c: c.name)
def test_epilogue_ragged_shapes(cfg, pad_mode):
    cfg = cfg.with_(pad_mode=pad_mode)
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) in TILED
    tn = BOTH_TN if tiled else (None,)
    for mode in MODES:
        ab = "random" if mode in ("compound", "parallel") else None
        for kind in ("b", "a", "s", "r", "bar"):
            _check_ext(cfg.with_(mode=mode), ep_kind=kind, alpha_beta=ab, tn=tn, backward=(kind == "bar"))
    _check_ext(cfg.with_(mode="parallel", dtype="bf16"), ep_kind="bar", tn=tn, backward=False)
    _check_ext(cfg.with_(mode="compound"), ep_kind="bar", kernel="generic", backward=False)


def test_epilogue_full_size_block_layer():
    """A 16-channel 32 x 32 layer of the ResNet-20-style stack at the benchmark batch, with batch norm and shortcut fused."""
    cfg = LayerCfg("r20_block", 256, 16, 32, 32, 16, mode="parallel", seed=5, w_range=0.1)
    _check_ext(cfg, ep_kind="ar")
    _check_ext(cfg.with_(pad_mode="zero"), ep_kind="bar")


def test_fused_forward_without_an_epilogue_is_the_plain_forward():
    cfg = RAGGED[0].with_(mode="compound")
    inp = make_inputs(cfg, alpha_beta="random")
    a = hs.run_hip(cfg, inp, backward=False)
    b = hs.run_hip_ext(cfg, inp, None, backward=False)
    for k in ("y", "y_min", "y_max", "idx_min", "idx_max"):
        assert np.array_equal(hs.bits(a[k]) if a[k].dtype != np.int32 else a[k],
                              hs.bits(b[k]) if b[k].dtype != np.int32 else b[k])


def test_extension_error_paths():
    import torch
    z = torch.zeros(4096, device="cuda")
    zi = torch.zeros(4096, device="cuda", dtype=torch.int32)
    d = tb.Desc.from_cfg(CONFIGS["cfg1"].with_(mode="minplus_max", pad_mode="zero"))
    with pytest.raises(tb.TconvError) as e:   # the mixed layers keep identity padding
        tb.tconv_forward(d, z, z, None, None, None, z, None, None, zi, None)
    assert e.value.status == -4
    d = tb.Desc.from_cfg(CONFIGS["cfg1"].with_(mode="max"))
    with pytest.raises(tb.TconvError) as e:   # a shift needs its scale
        tb.tconv_forward_fused(d, z, None, z, None, None, z, None, None, None, zi, shift=z)
    assert e.value.status == -1
    d = tb.Desc.from_cfg(CONFIGS["cfg1"].with_(mode="max", pad_mode="zero"))
    with pytest.raises(tb.TconvError) as e:   # the Sum-channel layers keep identity padding
        tb.tconv_sum_forward(d, z, None, z, None, None, z)
    assert e.value.status == -4


@pytest.mark.parametrize("stride", [1, 2])
def test_residual_block_training_step(stride):
    """One Sec. 5 TCNN BasicBlock, forward and backward, chained through the library the way bench.py's end-to-end
    workload chains it (batch norm as a fused scale / shift, shortcut as the fused residual: the block input, or at a
    stage boundary every second pixel with zero-filled new channels; gradient of a fused layer = tconv_backward with
    alpha = beta = scale, tconv_backward_bias, tconv_backward_alpha_beta), against the same chain of oracle calls."""
    import torch
    from oracle import text_oracle as ext
    dev = torch.device("cuda:0")
    rng = np.random.Generator(np.random.PCG64(4242 + stride))
    N, C, H, W = 3, 6, 12, 16
    Co = C * stride
    Ho, Wo = H // stride, W // stride
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = lambda co, ci: ((rng.random((2, co, ci, 3, 3), dtype=np.float32) * 2 - 1) * np.float32(0.1))
    wa, wb = w(Co, C), w(Co, Co)
    sa, sb = (rng.uniform(0.2, 0.4, Co).astype(np.float32) for _ in range(2))
    ha, hb = (rng.standard_normal(Co).astype(np.float32) * np.float32(0.1) for _ in range(2))
    gy = rng.standard_normal((N, Co, Ho, Wo)).astype(np.float32)
    short = x if stride == 1 else np.concatenate([x[:, :, ::2, ::2], np.zeros((N, Co - C, Ho, Wo), np.float32)], 1)
    ones = np.ones(Co, np.float32)
    # ---- oracle chain
    s_a = ext.Shape(N, C, H, W, Co, 3, 3, stride, 1, 1)
    s_b = ext.Shape(N, Co, Ho, Wo, Co, 3, 3, 1, 1, 1)
    fa = ext.forward(s_a, "parallel", x, wa[0], wa[1], ones, ones, scale=sa, shift=ha)
    fb = ext.forward(s_b, "parallel", fa["y"], wb[0], wb[1], ones, ones, scale=sb, shift=hb, residual=short)
    gb = ext.backward(s_b, "parallel", gy, fb["idx_min"], fb["idx_max"], alpha=sb, beta=sb)
    g_mid = gb["grad_x"].astype(np.float32)
    ga = ext.backward(s_a, "parallel", g_mid, fa["idx_min"], fa["idx_max"], alpha=sa, beta=sa)
    g_short = gy if stride == 1 else None
    g_x = ga["grad_x"].copy()
    if stride == 1:
        g_x += gy
    else:
        g_x[:, :, ::2, ::2] += gy[:, :C]
    want = dict(y=fb["y"], g_x=g_x, gwa_min=ga["grad_w_min"], gwb_max=gb["grad_w_max"],
                g_hb=ext.backward_bias(s_b, gy), g_ha=ext.backward_bias(s_a, g_mid),
                g_sb=np.sum(gy.astype(np.float64) * (fb["y_min"].astype(np.float64) + fb["y_max"]), axis=(0, 2, 3)),
                g_sa=np.sum(g_mid.astype(np.float64) * (fa["y_min"].astype(np.float64) + fa["y_max"]), axis=(0, 2, 3)))
    # ---- the same chain through the C ABI
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    d_a = tb.Desc(N, C, H, W, Co, 3, 3, (stride, stride), (1, 1), (1, 1), "parallel")
    d_b = tb.Desc(N, Co, Ho, Wo, Co, 3, 3, (1, 1), (1, 1), (1, 1), "parallel")

    def fused(d, xin, wpair, scale, shift, residual):
        osh = (N, Co, Ho, Wo)
        o = {k: torch.empty(osh, device=dev) for k in ("y", "y_min", "y_max")}
        o.update({k: torch.empty(osh, device=dev, dtype=torch.int32) for k in ("idx_min", "idx_max")})
        tb.tconv_forward_fused(d, xin, up(wpair[0]), up(wpair[1]), None, None, o["y"], o["y_min"], o["y_max"],
                               o["idx_min"], o["idx_max"], scale=up(scale), shift=up(shift), residual=residual)
        return o

    def backward(d, g, o, scale, xshape, wshape):
        r = dict(gx=torch.empty(xshape, device=dev), gw_min=torch.empty(wshape, device=dev),
                 gw_max=torch.empty(wshape, device=dev), gh=torch.empty(Co, device=dev),
                 ga=torch.empty(Co, device=dev), gb=torch.empty(Co, device=dev))
        sc = up(scale)
        ws = lambda op: hs.scratch(tb.tconv_workspace_bytes(d, op), dev)
        tb.tconv_backward(d, g, sc, sc, o["idx_min"], o["idx_max"], r["gx"], r["gw_min"], r["gw_max"], ws("backward"))
        tb.tconv_backward_bias(d, g, r["gh"], ws("backward_bias"))
        tb.tconv_backward_alpha_beta(d, g, o["y_min"], o["y_max"], r["ga"], r["gb"], ws("backward_alpha_beta"))
        return r

    oa = fused(d_a, up(x), wa, sa, ha, None)
    ob = fused(d_b, oa["y"], wb, sb, hb, up(short))
    rb = backward(d_b, up(gy), ob, sb, (N, Co, Ho, Wo), (Co, Co, 3, 3))
    ra = backward(d_a, rb["gx"], oa, sa, (N, C, H, W), (Co, C, 3, 3))
    gx = ra["gx"].clone()
    if stride == 1:
        gx += up(gy)
    else:
        gx[:, :, ::2, ::2] += up(gy)[:, :C]
    torch.cuda.synchronize()
    got = dict(y=ob["y"], g_x=gx, gwa_min=ra["gw_min"], gwb_max=rb["gw_max"], g_hb=rb["gh"], g_ha=ra["gh"],
               g_sb=rb["ga"] + rb["gb"], g_sa=ra["ga"] + ra["gb"])
    got = {k: v.cpu().numpy() for k, v in got.items()}
    assert np.array_equal(hs.bits(got["y"]), hs.bits(want["y"])), "block output differs"
    for k in ("g_x", "gwa_min", "gwb_max", "g_hb", "g_ha", "g_sb", "g_sa"):
        a, b = got[k].astype(np.float64), np.asarray(want[k], np.float64)
        tol = 2e-5 * max(1.0, float(np.max(np.abs(b))))
        assert np.max(np.abs(a - b)) <= tol, (k, float(np.max(np.abs(a - b))), tol)


@pytest.mark.parametrize("cfg", _random_layers(30, 20250611 + hs.SEED_SHIFT), ids=lambda c: c.name)
def test_random_layers_with_zero_padding_and_epilogue(cfg):
    """Random shapes in every form of the tiled kernel: zero padding, and the fused epilogue (bias, scale / shift,
    shortcut) with either padding, fp32 and bf16 storage."""
    mode = MODES[cfg.seed % 4]
    ab = "random" if mode in ("compound", "parallel") else None
    _check_ext(cfg.with_(mode=mode, pad_mode="zero"), alpha_beta=ab, tn=BOTH_TN)
    _check_ext(cfg.with_(mode=mode, pad_mode="zero"), integer=True, alpha_beta=ab, tn=BOTH_TN)
    pm = ("identity", "zero")[cfg.seed // 4 % 2]
    _check_ext(cfg.with_(mode=mode, pad_mode=pm), ep_kind="bar", alpha_beta=ab, tn=BOTH_TN)
    _check_ext(cfg.with_(mode=MODES[(cfg.seed + 1) % 4], pad_mode=pm, dtype="bf16"), ep_kind="bar", tn=BOTH_TN, backward=False)
