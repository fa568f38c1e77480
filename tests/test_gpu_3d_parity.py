"""GPU parity of the three-dimensional layers (tconv3d_forward / tconv3d_backward_input / tconv3d_backward_weight)
against their CPU oracle: outputs and winners bit for bit, gradients within 1e-5 of the size of their summands."""
import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS_3D, Layer3dCfg, make_3d_inputs

pytestmark = pytest.mark.gpu
MODES = ("max", "min", "compound", "parallel", "minplus_max", "maxplus_min")


def _check(cfg, alpha_beta=None, integer=False):
    inp = make_3d_inputs(cfg, alpha_beta=alpha_beta, integer=integer)
    ref = hs.run_oracle_3d(cfg, inp)
    hip = hs.run_hip_3d(cfg, inp)
    what = f"[3d {cfg.name} {cfg.mode} ab={alpha_beta} int={integer}] "
    hs.assert_forward_bit_exact(hip, ref, what=what)
    hs.assert_grad_close(hip["grad_x"], ref["grad_x"], ref["grad_x_scale"], what + "grad_x")
    for k in ("grad_w_min", "grad_w_max"):
        if ref[k] is not None:
            hs.assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k)


SHAPES = [
    Layer3dCfg("v_333", 2, 3, 6, 7, 9, 4, seed=130),
    Layer3dCfg("v_333_s2", 2, 4, 9, 8, 11, 5, stride=(2, 2, 2), seed=131),
    Layer3dCfg("v_mixed_geo", 2, 3, 7, 9, 10, 3, k=(2, 3, 1), stride=(1, 2, 1), pad=(1, 0, 0), seed=132),
    Layer3dCfg("v_dil", 1, 2, 9, 8, 12, 3, k=(3, 2, 3), stride=(1, 1, 2), pad=(2, 1, 2), dil=(2, 1, 2), seed=133),
    Layer3dCfg("v_p0", 2, 2, 5, 5, 5, 3, pad=(0, 0, 0), seed=134),
    Layer3dCfg("v_111", 2, 5, 3, 4, 5, 4, k=(1, 1, 1), pad=(0, 0, 0), seed=135),
    Layer3dCfg("v_one", 1, 1, 1, 1, 1, 1, seed=136),                       # 26 of 27 taps are padding
    Layer3dCfg("v_deep", 1, 40, 4, 5, 6, 3, seed=137),                     # K = 1080
    Layer3dCfg("v_wide", 1, 8, 4, 4, 4, 70, seed=138),
    Layer3dCfg("v_ragged_w", 2, 3, 5, 6, 13, 6, pad=(1, 0, 1), seed=139),    # W_out = 13: moved last segment
    Layer3dCfg("v_p2", 1, 3, 3, 4, 6, 9, pad=(2, 2, 1), seed=140),
]


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: c.name)
def test_three_dimensional_layers(cfg):
    for mode in MODES:
        c = cfg.with_(mode=mode)
        _check(c, alpha_beta="random" if mode in ("compound", "parallel") else None)
        _check(c, integer=True)


def test_plain_kernel_on_3x3x3_shapes():
    """The register-resident 3 x 3 x 3 kernel is the default on these shapes; the plain kernel must agree too."""
    import os
    old = os.environ.get("TCONV_FORWARD_KERNEL")
    os.environ["TCONV_FORWARD_KERNEL"] = "generic"
    try:
        for cfg in (SHAPES[0], SHAPES[4]):
            for mode in ("max", "compound", "parallel"):
                _check(cfg.with_(mode=mode), alpha_beta="random" if mode != "max" else None)
            _check(cfg.with_(mode="compound"), integer=True)
    finally:
        if old is None:
            os.environ.pop("TCONV_FORWARD_KERNEL", None)
        else:
            os.environ["TCONV_FORWARD_KERNEL"] = old


@pytest.mark.parametrize("kb", ["2", "12"])
def test_input_gradient_boxes_under_a_small_lds_budget(kb):
    """TCONV_BWD3_LDS_KB shrinks the LDS box of the input-gradient kernel: channel chunks (fewer channels than C_in per
    box), several boxes per volume, ragged last boxes."""
    import os
    os.environ["TCONV_BWD3_LDS_KB"] = kb
    try:
        for cfg in (SHAPES[0], SHAPES[1], SHAPES[3], SHAPES[7], SHAPES[9]):
            _check(cfg.with_(mode="compound"), alpha_beta="random")
            _check(cfg.with_(mode="parallel"), integer=True)
            _check(cfg.with_(mode="min"))
    finally:
        os.environ.pop("TCONV_BWD3_LDS_KB", None)


def test_larger_layer():
    cfg = CONFIGS_3D["c3d_main"].with_(N=2)
    print(f"[3d] {cfg.name} pairs={cfg.pairs:.3e}", flush=True)
    _check(cfg)
    _check(cfg.with_(mode="parallel"), alpha_beta="random")


def test_error_paths():
    import torch
    z = torch.zeros(256, device="cuda")
    zi = torch.zeros(256, device="cuda", dtype=torch.int32)
    d = tb.Desc3d(1, 2, 4, 4, 4, 2, 3, 3, 3, pad=(1, 1, 1), mode="parallel")
    with pytest.raises(tb.TconvError) as e:   # parallel needs both kernels
        tb.tconv3d_forward(d, z, z, None, None, None, z, None, None, zi, zi)
    assert e.value.status == -1
    with pytest.raises(tb.TconvError) as e:   # a window could lie wholly in the depth padding
        tb.tconv3d_out_shape(tb.Desc3d(1, 2, 4, 4, 4, 2, 3, 3, 3, pad=(3, 1, 1)))
    assert e.value.status == -2
    with pytest.raises(tb.TconvError) as e:   # fp32 only
        tb.tconv3d_out_shape(tb.Desc3d(1, 2, 4, 4, 4, 2, 3, 3, 3, pad=(1, 1, 1), dtype="bf16"))
    assert e.value.status == -4


def _random_3d_layers(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        k = tuple(int(v) for v in rng.choice([1, 2, 3, 3], size=3))
        st = tuple(int(v) for v in rng.choice([1, 1, 2], size=3))
        dl = tuple(int(v) for v in rng.choice([1, 1, 2], size=3))
        pad = tuple(int(rng.integers(0, d * (kk - 1) + 1)) for kk, d in zip(k, dl))
        dims = tuple(int(v) for v in rng.integers(1, 14, size=3))
        cin, cout = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        cfg = Layer3dCfg(f"vrnd{len(out)}", int(rng.integers(1, 3)), cin, dims[0], dims[1], dims[2], cout, k=k,
                         stride=st, pad=pad, dil=dl, seed=6000 + len(out))
        if min(cfg.out) < 1 or not all(hs.every_window_has_a_tap(*a) for a in zip(dims, k, st, pad, dl)):
            continue
        out.append(cfg)
    return out


@pytest.mark.parametrize("cfg", _random_3d_layers(40, 20250615 + hs.SEED_SHIFT), ids=lambda c: c.name)
def test_random_volumes(cfg):
    mode = MODES[cfg.seed % 6]
    ab = "random" if mode in ("compound", "parallel") else None
    _check(cfg.with_(mode=mode), alpha_beta=ab)
    _check(cfg.with_(mode=mode), alpha_beta=ab, integer=True)
