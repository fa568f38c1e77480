"""The library's calls inside a captured HIP graph: every entry point only enqueues kernels (its zero fills are
kernels, not memsets), so a step can be captured once and replayed.  Each replay is checked against the eager
result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2504_06881_amd import binding as tb
from paper_2504_06881_amd.inputs import CONFIGS, DW_CONFIGS, make_depthwise_inputs, make_inputs

pytestmark = pytest.mark.gpu


def _replay_and_compare(step, outputs, scratch):
    import torch
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outputs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in outputs:                      # poison, so that a replay that does nothing cannot pass
            t.fill_(-7 if t.dtype in (torch.int32, torch.uint8) else float("nan"))
        scratch.normal_()                      # unrelated eager work between the replays
        _ = (scratch * 2).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outputs, ref):
            if got.dtype in (torch.int32, torch.uint8):
                assert torch.equal(got, want), f"replay {rep}: integer output differs"
            else:
                # sums with atomics round differently from run to run: by a few ulp of the partial sums, whose size
                # the largest element of the tensor stands for (an element may be a small rest of large summands)
                atol = 1e-5 * max(1.0, float(want.abs().max()))
                assert torch.allclose(got, want, rtol=1e-5, atol=atol), f"replay {rep}: output differs"


def test_hot_path_step_in_a_graph():
    import torch
    dev = torch.device("cuda:0")
    cfg = CONFIGS["cfg1"].with_(N=8, C_in=12, C_out=12, H=24, W=24, mode="parallel")
    inp = make_inputs(cfg, alpha_beta="random")
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    up = lambda a: torch.from_numpy(a).to(dev)
    x, w1, w2, gy, al, be = (up(inp[k]) for k in ("x", "w_min", "w_max", "gy", "alpha", "beta"))
    osh = (cfg.N, cfg.C_out, ho, wo)
    y, ymn, ymx = (torch.empty(osh, device=dev) for _ in range(3))
    imn, imx = (torch.empty(osh, device=dev, dtype=torch.int32) for _ in range(2))
    gx, g1, g2 = torch.empty_like(x), torch.empty_like(w1), torch.empty_like(w2)
    ga, gb = torch.empty_like(al), torch.empty_like(be)

    def step():
        tb.tconv_forward(d, x, w1, w2, al, be, y, ymn, ymx, imn, imx)
        tb.tconv_backward_input(d, gy, al, be, imn, imx, gx)
        tb.tconv_backward_weight(d, gy, al, be, imn, imx, g1, g2)
        tb.tconv_backward_alpha_beta(d, gy, ymn, ymx, ga, gb)

    _replay_and_compare(step, [y, ymn, ymx, imn, imx, gx, g1, g2, ga, gb], torch.empty(1 << 16, device=dev))


def test_depthwise_step_in_a_graph():
    import torch
    dev = torch.device("cuda:0")
    cfg = DW_CONFIGS["dw_small"].with_(N=4, C_in=12, C_out=12, H=32, W=32)
    inp = make_depthwise_inputs(cfg)
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    up = lambda a: torch.from_numpy(a).to(dev)
    x, w, gy, al, be = (up(inp[k]) for k in ("x", "w_min", "gy", "alpha", "beta"))
    osh = (cfg.N, cfg.C_out, ho, wo)
    y = torch.empty(osh, device=dev)
    idx = torch.empty(osh, device=dev, dtype=torch.uint8)
    gx, gw, ga, gb = torch.empty_like(x), torch.empty_like(w), torch.empty_like(al), torch.empty_like(be)

    def step():
        tb.tconv_depthwise_forward(d, x, w, w, al, be, y, idx)
        tb.tconv_depthwise_backward(d, x, w, w, al, be, gy, idx, gx, gw, None, ga, gb)

    _replay_and_compare(step, [y, idx, gx, gw, ga, gb], torch.empty(1 << 16, device=dev))
