"""GPU parity of the binary16 layers (dtype f16: one binary16-rounded add per candidate, comparisons on the rounded
sums, lowest k on ties) against the half-precision contract of the extension oracle: outputs and winners bit for bit,
fp32 gradients within 1e-5.  Rounded sums tie all the time in binary16, so every case also tests the tie rule."""
import os

import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS, LayerCfg, make_inputs
from test_gpu_parity import MODES, RAGGED, RAGGED_LARGE, _random_layers

pytestmark = pytest.mark.gpu


def _check16(cfg, alpha_beta=None, integer=False, kernel=None, backward=True):
    inp = make_inputs(cfg, alpha_beta=alpha_beta, integer=integer)
    ref = hs.run_oracle_f16(cfg, inp, backward=backward)
    old = os.environ.pop("TCONV_FORWARD_KERNEL", None)
    try:
        if kernel:
            os.environ["TCONV_FORWARD_KERNEL"] = kernel
        hip = hs.run_hip_f16(cfg, inp, backward=backward)
    finally:
        os.environ.pop("TCONV_FORWARD_KERNEL", None)
        if old is not None:
            os.environ["TCONV_FORWARD_KERNEL"] = old
    what = f"[f16 {cfg.name} {cfg.mode} pad={cfg.pad_mode} ab={alpha_beta} int={integer} k={kernel}] "
    hs.assert_forward_bit_exact(hip, ref, what=what)
    if backward:
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            if ref.get(k) is not None:
                hs.assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k)


F16_SHAPES = [c for c in RAGGED if c.name not in ("r_cin300", "r_cin350", "r_cin260_s2")]


@pytest.mark.parametrize("cfg", F16_SHAPES, ids=lambda c: c.name)
def test_f16_ragged_shapes(cfg):
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg, dtype="f16")) != "generic"
    for mode in MODES:
        c = cfg.with_(mode=mode)
        _check16(c, alpha_beta="random" if mode in ("compound", "parallel") else None)
        _check16(c, integer=True, backward=False)
        if tiled:
            _check16(c, kernel="generic", backward=False)
    if cfg.pad > 0:
        _check16(cfg.with_(mode="compound", pad_mode="zero"))
        _check16(cfg.with_(mode="parallel", pad_mode="zero"), integer=True)


# Shapes the packed kernel takes (even W, even left margin dilation - pad): odd channel counts on both sides, a shifted
# last segment, dilation 2 with pad 2 and pad 0, a lone channel, many images.
PACKED_SHAPES = [
    LayerCfg("h_odd", 3, 5, 19, 24, 7, seed=61),
    LayerCfg("h_odd_cout1", 2, 3, 9, 10, 1, seed=62),
    LayerCfg("h_d2", 2, 5, 18, 26, 6, pad=2, dil=2, seed=63),
    LayerCfg("h_d2_p0", 2, 4, 18, 26, 5, pad=0, dil=2, seed=64),
    LayerCfg("h_cin1", 3, 1, 12, 16, 9, seed=65),
    LayerCfg("h_many", 130, 7, 14, 20, 10, seed=66),
    LayerCfg("h_deep", 1, 131, 8, 12, 5, seed=67),
]


@pytest.mark.parametrize("cfg", PACKED_SHAPES, ids=lambda c: c.name)
def test_f16_packed_kernel_shapes(cfg):
    assert tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg, dtype="f16")) == "tiled3x3_f16"
    for mode in MODES:
        c = cfg.with_(mode=mode)
        _check16(c, alpha_beta="random" if mode in ("compound", "parallel") else None, backward=(mode == "compound"))
        _check16(c, integer=True, backward=False)
    if cfg.pad > 0:
        _check16(cfg.with_(mode="compound", pad_mode="zero"), backward=False)
        _check16(cfg.with_(mode="parallel", pad_mode="zero"), integer=True, backward=False)
        _check16(cfg.with_(mode="min", pad_mode="zero"), backward=False)


@pytest.mark.parametrize("cfg", RAGGED_LARGE[:2], ids=lambda c: c.name)
def test_f16_large_ragged_shapes(cfg):
    for mode in ("compound", "parallel", "min"):
        _check16(cfg.with_(mode=mode), backward=(mode == "compound"))


def test_f16_benchmark_layer_slice():
    """A four-image slice of the headline classification layer: w ~ U(-0.1, 0.1) against x ~ N(0, 1) in binary16."""
    _check16(CONFIGS["cfg2_main"].with_(N=4, name="cfg2_n4"))
    _check16(CONFIGS["cfg3b"].with_(N=2, name="cfg3b_n2"), backward=False)
    _check16(CONFIGS["cfg3a"].with_(N=2, name="cfg3a_n2"), backward=False)
    _check16(CONFIGS["cfg4b"].with_(N=1, C_out=32, name="cfg4b_n1_c32"), backward=False)


def test_f16_error_paths():
    import torch
    z = torch.zeros(4096, device="cuda", dtype=torch.float16)
    zi = torch.zeros(4096, device="cuda", dtype=torch.int32)
    d = tb.Desc.from_cfg(CONFIGS["cfg1"].with_(mode="minplus_max"), dtype="f16")
    with pytest.raises(tb.TconvError) as e:   # no binary16 mixed layers
        tb.tconv_forward(d, z, z, None, None, None, z, None, None, zi, None)
    assert e.value.status == -4
    d = tb.Desc.from_cfg(CONFIGS["cfg1"].with_(mode="max"), dtype="f16")
    with pytest.raises(tb.TconvError) as e:   # no epilogue in the binary16 contract
        tb.tconv_forward_fused(d, z, None, z, None, None, z, None, None, None, zi, bias=torch.zeros(8, device="cuda"))
    assert e.value.status == -4


@pytest.mark.parametrize("cfg", _random_layers(30, 20250612 + hs.SEED_SHIFT), ids=lambda c: c.name)
def test_random_layers(cfg):
    """Random shapes in binary16: the packed kernel where it applies (stride 1, core columns at an even element),
    else the generic kernel; real and integer data."""
    mode = MODES[cfg.seed % 4]
    ab = "random" if mode in ("compound", "parallel") else None
    _check16(cfg.with_(mode=mode, dtype="f16"), alpha_beta=ab)
    _check16(cfg.with_(mode=mode, dtype="f16"), alpha_beta=ab, integer=True)
