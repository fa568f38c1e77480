"""GPU parity of the one-dimensional layers (tconv1d_forward / tconv1d_backward_input / tconv1d_backward_weight)
against their CPU oracle: outputs and winners bit for bit, gradients within 1e-5 of the size of their summands.
Covers both two-dimensional views the library chooses between (three channels as the rows of a 3 x 3 window,
and the one-row image) and the long-window kernel of the one-row image."""
import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS_1D, Layer1dCfg, make_1d_inputs

pytestmark = pytest.mark.gpu
MODES = ("max", "min", "compound", "parallel", "minplus_max", "maxplus_min")


def _check(cfg, alpha_beta=None, integer=False):
    inp = make_1d_inputs(cfg, alpha_beta=alpha_beta, integer=integer)
    ref = hs.run_oracle_1d(cfg, inp)
    hip = hs.run_hip_1d(cfg, inp)
    what = f"[1d {cfg.name} {cfg.mode} {cfg.dtype} ab={alpha_beta} int={integer}] "
    hs.assert_forward_bit_exact(hip, ref, what=what)
    hs.assert_grad_close(hip["grad_x"], ref["grad_x"], ref["grad_x_scale"], what + "grad_x")
    for k in ("grad_w_min", "grad_w_max"):
        if ref[k] is not None:
            hs.assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k)


SHAPES = [
    Layer1dCfg("l_k3_c6", 2, 6, 100, 8, seed=100),                       # three-rows view, tiled kernel
    Layer1dCfg("l_k3_c9_ragged", 3, 9, 203, 7, seed=101),                # L_out not a multiple of 8
    Layer1dCfg("l_k3_c12_s2", 2, 12, 131, 5, stride=2, seed=102),        # three-rows view, stride 2
    Layer1dCfg("l_k3_c3_p0", 2, 3, 64, 4, pad=0, seed=103),
    Layer1dCfg("l_k3_c5", 2, 5, 90, 6, seed=104),                        # C_in not a multiple of 3: one-row image
    Layer1dCfg("l_k3_d2", 2, 6, 77, 4, pad=2, dil=2, seed=105),          # dilation: one-row image
    Layer1dCfg("l_k5", 2, 4, 60, 6, K=5, pad=2, seed=106),
    Layer1dCfg("l_k80_s4", 2, 1, 2000, 8, K=80, stride=4, pad=38, seed=107),   # raw-waveform stem
    Layer1dCfg("l_k1", 2, 7, 33, 5, K=1, pad=0, seed=108),
    Layer1dCfg("l_short", 3, 6, 5, 4, seed=109),                         # L_out < one pixel segment
    Layer1dCfg("l_one", 1, 1, 1, 1, K=1, pad=0, seed=110),
    Layer1dCfg("l_k3_c300", 1, 300, 40, 6, seed=111),                    # deep input
]


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: c.name)
def test_one_dimensional_layers(cfg):
    for mode in MODES:
        c = cfg.with_(mode=mode)
        _check(c, alpha_beta="random" if mode in ("compound", "parallel") else None)
        _check(c, integer=True)


# shapes of the long-window kernel: every stride it takes, windows that are and are not whole chunks of 8 taps,
# several input channels, outputs past one workgroup of 256, channel counts that are not multiples of 8
LONG = [
    Layer1dCfg("w_k80_s4_ragged", 2, 1, 2103, 9, K=80, stride=4, pad=38, seed=120),
    Layer1dCfg("w_k80_s4_p0", 1, 1, 1500, 8, K=80, stride=4, pad=0, seed=121),
    Layer1dCfg("w_k19_s2_c2", 1, 2, 733, 3, K=19, stride=2, pad=9, seed=122),
    Layer1dCfg("w_k8_s1_c3", 2, 3, 270, 17, K=8, stride=1, pad=3, seed=123),
    Layer1dCfg("w_k64_s1_maxpad", 1, 1, 64, 1, K=64, stride=1, pad=63, seed=124),
    Layer1dCfg("w_k33_s8", 1, 1, 4100, 2, K=33, stride=8, pad=16, seed=125),
    Layer1dCfg("w_k12_s4_c4", 1, 4, 90, 5, K=12, stride=4, pad=11, seed=126),
    Layer1dCfg("w_k9_s1", 1, 1, 257, 4, K=9, stride=1, pad=0, seed=127),
    Layer1dCfg("w_k25_s2_c8", 2, 8, 600, 24, K=25, stride=2, pad=12, seed=128),
]


@pytest.mark.parametrize("cfg", LONG, ids=lambda c: c.name)
def test_long_window_kernel(cfg):
    for mode in ("max", "min", "compound", "parallel"):
        c = cfg.with_(mode=mode)
        d = tb.Desc1d(c.N, c.C_in, c.L, c.C_out, c.K, c.stride, c.pad, c.dil, c.mode, c.dtype)
        assert tb.tconv1d_forward_kernel_name(d) == "row1d"
        _check(c, alpha_beta="random" if mode in ("compound", "parallel") else None)
        _check(c, integer=True)


def test_full_size_stem():
    cfg = CONFIGS_1D["c1d_stem"].with_(N=4)
    print(f"[1d stem] {cfg.name} pairs={cfg.pairs:.3e}", flush=True)
    d = tb.Desc1d(cfg.N, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil, cfg.mode, cfg.dtype)
    assert tb.tconv1d_forward_kernel_name(d) == "row1d"
    _check(cfg)
    _check(cfg.with_(mode="parallel"), alpha_beta="random")


@pytest.mark.parametrize("mode", ["max", "compound", "parallel"])
def test_bf16_storage(mode):
    for base in (SHAPES[0], SHAPES[4], SHAPES[6]):
        _check(base.with_(mode=mode, dtype="bf16"))


def test_full_size_layer():
    cfg = CONFIGS_1D["c1d_main"].with_(N=8)
    print(f"[1d full] {cfg.name} pairs={cfg.pairs:.3e}", flush=True)
    _check(cfg)
    d = tb.Desc1d(cfg.N, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil, cfg.mode, cfg.dtype)
    assert tb.tconv1d_forward_kernel_name(d) in ("tiled3x3", "tiled3x3_split")


def test_error_paths():
    import torch
    z = torch.zeros(64, device="cuda")
    zi = torch.zeros(64, device="cuda", dtype=torch.int32)
    d = tb.Desc1d(1, 3, 16, 2, 3, pad=1, mode="parallel")
    with pytest.raises(tb.TconvError) as e:   # parallel needs both kernels
        tb.tconv1d_forward(d, z, z, None, None, None, z, None, None, zi, zi)
    assert e.value.status == -1
    with pytest.raises(tb.TconvError) as e:
        tb.tconv1d_backward_input(d, z, None, None, zi, None, z)
    assert e.value.status == -1


def _random_1d_layers(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        k = int(rng.choice([1, 2, 3, 3, 3, 4, 5, 7, 9, 15]))
        s_, d = int(rng.choice([1, 1, 2, 3, 4])), int(rng.integers(1, 3))
        pad = int(rng.integers(0, d * (k - 1) + 1))
        cin, cout = int(rng.choice([1, 2, 3, 5, 6, 9, 12, 13])), int(rng.integers(1, 12))
        L = int(rng.integers(1, 300))
        cfg = Layer1dCfg(f"lrnd{len(out)}_k{k}s{s_}d{d}p{pad}_{cin}x{L}_{cout}", int(rng.integers(1, 4)), cin, L, cout,
                         K=k, stride=s_, pad=pad, dil=d, seed=5000 + len(out))
        if cfg.L_out < 1 or not hs.every_window_has_a_tap(L, k, s_, pad, d):
            continue
        out.append(cfg)
    return out


@pytest.mark.parametrize("cfg", _random_1d_layers(40, 20250614 + hs.SEED_SHIFT), ids=lambda c: c.name)
def test_random_sequences(cfg):
    mode = MODES[cfg.seed % 6]
    ab = "random" if mode in ("compound", "parallel") else None
    _check(cfg.with_(mode=mode), alpha_beta=ab)
    _check(cfg.with_(mode=mode), alpha_beta=ab, integer=True)
