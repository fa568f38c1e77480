"""GPU parity of the layer extensions against the extension oracle: zero padding (App. A.1.1), the fused epilogue
(bias of App. A.2, batch norm + shortcut of the Sec. 5 residual blocks) and the bias gradient.  Outputs and winners
bit for bit, gradients within 1e-5."""
import os

import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS, LayerCfg, make_inputs
from test_gpu_parity import BOTH_TN, KNOBS, MODES, RAGGED, RAGGED_LARGE

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
            if t:
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
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) == "tiled3x3"
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
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) == "tiled3x3"
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
