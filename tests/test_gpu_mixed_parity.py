"""GPU parity of the mixed layers (paper Sec. 3.1: (iii) MinPlus-Max-Conv2d, (vi) MaxPlus-Min-Conv2d): the HIP
path through the C ABI against the CPU oracle on the same seeded inputs.  Outputs and winning taps must
match bit for bit; gradients (the plain single-branch backward on the layer's indices) within 1e-5 of the
magnitude of their summands.
"""
import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS, make_inputs
from test_gpu_parity import BOTH_TN, RAGGED, RAGGED_LARGE, _check, _random_layers

pytestmark = pytest.mark.gpu

MIXED = ("minplus_max", "maxplus_min")


@pytest.mark.parametrize("kernel", [None, "generic"])
@pytest.mark.parametrize("mode", MIXED)
def test_cfg1(mode, kernel):
    cfg = CONFIGS["cfg1"].with_(mode=mode)
    _check(cfg, kernel=kernel)
    _check(cfg, integer=True, kernel=kernel)          # ties everywhere: lowest tap, lowest channel
    _check(cfg, branch_outputs=False, kernel=kernel)


@pytest.mark.parametrize("cfg", RAGGED, ids=lambda c: c.name)
def test_ragged_shapes(cfg):
    tiled = tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) in ("tiled3x3", "tiled3x3_split")
    tn = BOTH_TN if tiled else (None,)
    for mode in MIXED:
        _check(cfg.with_(mode=mode), tn=tn)
        _check(cfg.with_(mode=mode), integer=True, tn=tn)


@pytest.mark.parametrize("cfg", RAGGED_LARGE[:2], ids=lambda c: c.name)
def test_ragged_shapes_that_pick_four_channels_per_lane(cfg):
    for mode in MIXED:
        _check(cfg.with_(mode=mode))
        _check(cfg.with_(mode=mode), integer=True)


@pytest.mark.parametrize("cfg", [RAGGED[0], RAGGED[2], RAGGED[4], RAGGED[10]], ids=lambda c: c.name)
def test_generic_kernel_on_ragged_shapes(cfg):
    for mode in MIXED:
        _check(cfg.with_(mode=mode), kernel="generic")
        _check(cfg.with_(mode=mode), integer=True, kernel="generic")


@pytest.mark.parametrize("mode", MIXED)
def test_bf16_storage(mode):
    for base in (RAGGED[0], RAGGED[2], RAGGED[4], CONFIGS["cfg1"]):
        cfg = base.with_(mode=mode, dtype="bf16")
        _check(cfg, tn=BOTH_TN)
        _check(cfg, integer=True, tn=BOTH_TN)


@pytest.mark.parametrize("name", ["cfg2_main", "cfg3b"])
@pytest.mark.parametrize("mode", MIXED)
def test_full_size_configs(name, mode):
    """Every output of a full-size layer (stride 1 and stride 2) against the oracle."""
    cfg = CONFIGS[name].with_(mode=mode)
    print(f"[full] {name} {mode} pairs={cfg.pairs:.3e}", flush=True)
    _check(cfg)


def test_kernel_selection_and_error_paths():
    import torch
    cfg = CONFIGS["cfg2_main"].with_(mode="minplus_max")
    assert tb.tconv_forward_kernel_name(tb.Desc.from_cfg(cfg)) == "tiled3x3"
    small = CONFIGS["cfg1"].with_(mode="maxplus_min")
    d = tb.Desc.from_cfg(small)
    z = torch.zeros(16, device="cuda")
    zi = torch.zeros(16, device="cuda", dtype=torch.int32)
    with pytest.raises(tb.TconvError) as e:   # (vi) lives on the max side: w_max and idx_max are required
        tb.tconv_forward(d, z, z, None, None, None, z, None, None, zi, zi)
    assert e.value.status == -1
    with pytest.raises(tb.TconvError) as e:
        tb.tconv_forward(d, z, None, z, None, None, z, None, None, zi, None)
    assert e.value.status == -1
    with pytest.raises(tb.TconvError) as e:   # no combine step, so no alpha / beta gradient
        tb.tconv_backward_alpha_beta(d, z, z, z, z, z)
    assert e.value.status == -1
    with pytest.raises(tb.TconvError) as e:   # no Sum-channel variant of a mixed layer
        tb.tconv_sum_forward(d, z, z, z, None, None, z)
    assert e.value.status == -1


@pytest.mark.parametrize("cfg", _random_layers(30, 20250610 + hs.SEED_SHIFT), ids=lambda c: c.name)
def test_random_layers_in_every_form(cfg):
    mode = MIXED[cfg.seed % 2]
    _check(cfg.with_(mode=mode), tn=BOTH_TN)
    _check(cfg.with_(mode=mode), integer=True, tn=BOTH_TN)
    _check(cfg.with_(mode=MIXED[1 - cfg.seed % 2], dtype="bf16"), integer=True, tn=BOTH_TN)
