"""The entry point that allocates nothing (tconv_backward_weight_noalloc) against tconv_backward_weight with a
workspace: same kernels, same summation order, so the two must agree bit for bit - on two calls in a row, the second on
a smaller layer (the library's fixed scratch array keeps the first call's contents), and both within the parity bar of
the oracle."""
import numpy as np
import pytest

import harness as hs
from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import LayerCfg, make_inputs

pytestmark = pytest.mark.gpu


def _both(cfg, seed):
    import torch
    dev = torch.device("cuda:0")
    inp = make_inputs(cfg, alpha_beta="random" if cfg.mode in ("compound", "parallel") else None, seed=seed)
    ref = hs.run_oracle(cfg, inp)
    d = tb.Desc.from_cfg(cfg)
    up = lambda a, dt=None: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    gy, alpha, beta = up(inp["gy"]), up(inp["alpha"]), up(inp["beta"])
    idx_min, idx_max = up(ref["idx_min"]), up(ref["idx_max"])       # the oracle's winners: the gradient alone is under test
    wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
    new = lambda want: torch.full(wshape, float("nan"), device=dev) if want else None
    want_min, want_max = cfg.mode != "max", cfg.mode in ("max", "parallel")
    a_min, a_max, b_min, b_max = new(want_min), new(want_max), new(want_min), new(want_max)
    ws = hs.scratch(tb.tconv_workspace_bytes(d, "backward_weight"), dev)
    tb.tconv_backward_weight(d, gy, alpha, beta, idx_min, idx_max, a_min, a_max, ws)
    tb.tconv_backward_weight_noalloc(d, gy, alpha, beta, idx_min, idx_max, b_min, b_max)
    torch.cuda.synchronize()
    for name, a, b in (("grad_w_min", a_min, b_min), ("grad_w_max", a_max, b_max)):
        if a is None:
            continue
        a, b = a.cpu().numpy(), b.cpu().numpy()
        assert np.array_equal(hs.bits(a), hs.bits(b)), f"{cfg.name} {cfg.mode} {name}: the two entry points differ"
        hs.assert_grad_close(b, ref[name], ref[name + "_scale"], f"[{cfg.name} {cfg.mode} noalloc] {name}")


@pytest.mark.parametrize("mode", ["parallel", "compound", "max", "min"])
def test_no_alloc_entry_point_twice_the_second_call_smaller(mode):
    big = LayerCfg("na_big", 12, 9, 21, 26, 11, mode=mode, seed=61)
    small = LayerCfg("na_small", 3, 4, 9, 10, 5, stride=2, mode=mode, seed=62)
    _both(big, 61)
    _both(small, 62)
    _both(big, 63)


def test_no_alloc_entry_point_rejects_what_its_array_cannot_hold():
    import torch
    # 1 slice x 600 channels x 8100 taps x 8 bytes = 38.9 MB of partial histograms: over the 32 MiB array
    d = tb.Desc(1, 900, 4, 4, 600, 3, 3, pad=(1, 1), mode="compound")
    assert tb.tconv_workspace_bytes(d, "backward_weight") > 32 << 20
    z = torch.zeros(8, device="cuda")
    zi = torch.zeros(8, device="cuda", dtype=torch.int32)
    with pytest.raises(tb.TconvError) as e:
        tb.tconv_backward_weight_noalloc(d, z, None, None, zi, zi, z, z)
    assert e.value.status == -3
