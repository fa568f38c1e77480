#!/usr/bin/env python3
"""Benchmark of the tropical-convolution hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
tconv_forward + tconv_backward (input and kernel gradient) of the headline layer - the largest
single-GPU layer of the benchmark configurations, the segmentation-encoder layer
x [8,128,128,128] -> 128 channels, 3x3, stride 1, pad 1, compound mode, fp32 - with the inputs
resident in HBM before the timed region.  The same run measures every other layer the forward bar
is stated on ("layers": forward time and fraction of the fp32 vector peak, backward GB/s on
rotating buffers).

Prints ONE JSON line:
  metric / value : add+compare pairs per second of the step (dense pair count / step time), GOPS
  roofline       : the forward kernel against the fp32 vector-ALU peak, measured live with HIP events around
                   every forward launch of the timed region
  cpu_baseline   : the CPU oracle timed on this machine's host cores on a bounded sample of the same workload
Extra keys give the forward-only rate and the achieved HBM GB/s of the two backward calls.
--workload takes any single-layer configuration name (cfg2_main, cfg3a, cfg4b, ...) or cfg5, the 19
layers of a ResNet-20-style net run back to back (one step = all layers, forward and backward).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published machine figures
N_CU, CLOCK_HZ = 256, 2.4e9
LANE_OPS_PER_S = N_CU * 64 * CLOCK_HZ           # one fp32 VALU lane-instruction per lane per clock: 39.32e12
HBM_PEAK_GBS = 8000.0


# HBM-side bytes per launch of the forward kernel (fetched + written), measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this script and scaled by what a plain device copy reads on the same counters.  Every entry
# names the summary under profiles/ that holds the command and the raw figures.  Keyed by (workload, mode, dtype, op).
MEASURED_FORWARD_TRAFFIC = {
    ("cfg4a", "compound", "f32", "full"): (142.4e6 + 335.5e6, "profiles/bench_cfg4a_all_kernels.md"),
    ("cfg4a", "compound", "bf16", "full"): (84.6e6 + 234.9e6, "profiles/bench_cfg4a_bf16_all_kernels.md"),
    ("cfg4a", "compound", "f16", "full"): (58.1e6 + 234.9e6, "profiles/bench_cfg4a_f16_all_kernels.md"),
    ("cfg4b", "compound", "f32", "full"): (156.7e6 + 176.2e6, "profiles/bench_cfg4b_all_kernels.md"),
    ("cfg2_main", "compound", "f32", "full"): (53.4e6 + 167.8e6, "profiles/bench_cfg2_main_all_kernels.md"),
    ("cfg3a", "parallel", "f32", "full"): (56.6e6 + 256.9e6, "profiles/bench_cfg3a_all_kernels.md"),
    ("cfg3b", "parallel", "f32", "full"): (70.7e6 + 70.6e6, "profiles/bench_cfg3b_all_kernels.md"),
    ("cfg3c", "parallel", "f32", "full"): (73.6e6 + 66.1e6, "profiles/bench_cfg3c_all_kernels.md"),
    ("cfg2_main", "minplus_max", "f32", "full"): (52.4e6 + 100.7e6, "profiles/bench_cfg2_main_minplus_max_all_kernels.md"),
    ("cfg2_main", "compound", "f32", "sum"): (37.7e6 + 34.6e6, "profiles/bench_sum_cfg2_main_all_kernels.md"),
    ("c1d_main", "compound", "f32", "1d"): (305.1e6 + 983.1e6, "profiles/bench_c1d_main_all_kernels.md"),
    ("c1d_stem", "compound", "f32", "1d"): (11.0e6 + 655.4e6, "profiles/bench_c1d_stem_all_kernels.md"),
}

# The layers the forward bar is stated on (large 3 x 3 layers), the HBM-judged stem, and the bf16-storage variant.
BAR_LAYERS = [("cfg2_main", None), ("cfg2_stem", None), ("cfg3a", None), ("cfg3b", None), ("cfg3c", None),
              ("cfg4a", None), ("cfg4b", None), ("cfg4a", "bf16"), ("cfg4b", "bf16"),
              ("cfg2_main", "f16"), ("cfg3a", "f16"), ("cfg4a", "f16"), ("cfg4b", "f16")]
ROTATE_BYTES = 600e6   # backward calls are timed on rotating operand sets larger than the 256 MB last-level cache


def calibrate_copy(torch, dev) -> None:
    """--calibrate-copy: a plain 256 MiB device copy, three times; what FETCH_SIZE / WRITE_SIZE read for it fixes the
    unit of those counters in the same profiler run."""
    src = torch.empty(64 * 1024 * 1024, device=dev)  # 256 MiB
    src.normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def alu_peak_pairs_per_s(mode: str) -> float:
    """Plain fp32 VALU roofline in pairs/s: one v_add_f32 and one v_max/min_f32 per pair,
    except compound where one add feeds both branches (3 lane-instructions per 2 pairs)."""
    instr_per_pair = {"max": 2.0, "min": 2.0, "parallel": 2.0, "compound": 1.5,
                      "minplus_max": 2.0, "maxplus_min": 2.0}[mode]
    return LANE_OPS_PER_S / instr_per_pair


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4a",
                    help="headline workload: a single-layer configuration (cfg4a: the largest single-GPU layer, "
                         "x[8,128,128,128] -> 128 channels, compound, fp32; cfg2_main, cfg3a, ...) or cfg5, the 19 "
                         "layers of a ResNet-20-style net")
    ap.add_argument("--op", default="full", choices=["full", "sum", "dw", "1d", "3d"],
                    help="full: the full-window layers (the headline path); sum: the Sum-channel layers "
                         "(tconv_sum_forward / tconv_sum_backward) on the same shapes; dw: the depthwise layers "
                         "(tconv_depthwise_forward / tconv_depthwise_backward; --workload dw_main | dw_s2 | dw_16 | dw_8); "
                         "1d: the one-dimensional layers (tconv1d_*; --workload c1d_main | c1d_stem); "
                         "3d: the three-dimensional layers (tconv3d_*; --workload c3d_main)")
    ap.add_argument("--mode", default=None,
                    choices=["max", "min", "compound", "parallel", "minplus_max", "maxplus_min"],
                    help="run the workload's shape as another layer of the family (default: the configuration's own)")
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16", "f16"],
                    help="f32; bf16: storage type of x, kernels and outputs, fp32 arithmetic; f16: binary16 storage AND "
                         "arithmetic (the packed 16-bit vector path, its own numeric contract)")
    ap.add_argument("--no-graph", action="store_true",
                    help="multi-layer workloads (cfg5): launch every step eagerly instead of replaying a HIP graph")
    ap.add_argument("--recompute-branch-outputs", action="store_true",
                    help="cfg5net: the forward pass stores no y_min / y_max (12 instead of 20 bytes per output) and "
                         "tconv_backward_params_recompute forms them again from the winners; default: stored and read "
                         "by tconv_backward_params (the faster step: 2.29 against 2.48 ms)")
    ap.add_argument("--no-layers", action="store_true",
                    help="leave out the per-layer table of the other bar layers (profiling runs)")
    ap.add_argument("--separate-backward", action="store_true",
                    help="a step calls tconv_backward_input and tconv_backward_weight instead of the one-call tconv_backward")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target wall time of the oracle sample")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the hot path has no multi-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2504_06881_amd import binding as tb
    from paper_2504_06881_amd.inputs import CONFIGS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    tb.load()  # fails loudly if libtconv.so has not been built
    if args.op == "dw":
        return bench_depthwise(args, torch, tb)
    if args.op == "1d":
        return bench_1d(args, torch, tb)
    if args.op == "3d":
        return bench_3d(args, torch, tb)
    from paper_2504_06881_amd.inputs import resnet20_layers
    if args.workload == "cfg5net":
        return bench_net(args, torch, tb)
    if args.workload == "cfg5":
        # the 19 tropical conv layers of a ResNet-20-style net on [256, 3, 32, 32] (the end-to-end configuration);
        # the batch-norm / residual glue of the net is not part of the hot path and is not run
        cfgs = resnet20_layers(256)
        wl_name = "cfg5: the 19 parallel-mode 3x3 layers of a ResNet-20-style net on x[256,3,32,32], f32"
    else:
        cfgs = [CONFIGS[args.workload]]
        if args.mode:
            cfgs = [cfgs[0].with_(mode=args.mode)]
        if args.dtype:
            cfgs = [cfgs[0].with_(dtype=args.dtype)]
        c0 = cfgs[0]
        wl_name = (f"{c0.name}: x[{c0.N},{c0.C_in},{c0.H},{c0.W}] -> {c0.C_out}ch 3x3 s{c0.stride} p{c0.pad} "
                   f"d{c0.dil} {c0.mode} {c0.dtype}")
    dev = torch.device("cuda:0")

    class Layer:
        """Device buffers and the calls of one layer.  rotate: number of operand sets (gy, idx, gradients) for the
        cold-cache timing of the backward calls."""

        def __init__(self, cfg, op, rotate=1):
            self.cfg = cfg
            self.op = op
            self.inp = inp = make_inputs(cfg)
            self.d = d = tb.Desc.from_cfg(cfg)
            ho, wo = tb.tconv_out_shape(d)
            tdt = {"bf16": torch.bfloat16, "f16": torch.float16}.get(cfg.dtype, torch.float32)

            def up(a, dt=torch.float32):
                return None if a is None else torch.from_numpy(a).to(dev).to(dt).contiguous()

            self.x = up(inp["x"], tdt)
            if cfg.mode == "compound":
                self.w_min = self.w_max = up(inp["w_min"], tdt)
            else:
                self.w_min, self.w_max = up(inp["w_min"], tdt), up(inp["w_max"], tdt)
            osh = (cfg.N, cfg.C_out, ho, wo)
            do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")
            self.y = torch.empty(osh, device=dev, dtype=tdt)
            self.y_min = torch.empty(osh, device=dev, dtype=tdt) if do_min else None
            self.y_max = torch.empty(osh, device=dev, dtype=tdt) if do_max else None
            wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
            gy0 = up(inp["gy"])
            self.sets = []
            for r in range(rotate):
                self.sets.append(dict(
                    gy=gy0 if r == 0 else gy0.clone(),
                    idx_min=torch.empty(osh, device=dev, dtype=torch.int32) if do_min else None,
                    idx_max=torch.empty(osh, device=dev, dtype=torch.int32) if do_max else None,
                    gx=torch.empty(tuple(inp["x"].shape), device=dev),
                    gw_min=torch.empty(wshape, device=dev) if do_min else None,
                    gw_max=(torch.empty(wshape, device=dev)
                            if cfg.mode in ("max", "parallel", "maxplus_min") else None)))
            self.n_out = cfg.N * cfg.C_out * ho * wo
            # algorithmic HBM bytes of the backward calls: gy + idx per output per branch, grad written once
            self.bytes_bi = self.n_out * (4 + 4 * cfg.branches) + inp["x"].size * 4
            self.bytes_bw = self.n_out * (4 + 4 * cfg.branches) + cfg.C_out * cfg.K * 4 * (2 if cfg.mode == "parallel" else 1)
            # one pass over gy / idx serving both gradients
            self.bytes_b = self.bytes_bi + self.bytes_bw - self.n_out * (4 + 4 * cfg.branches)
            wsz = tb.tconv_workspace_bytes(d, "forward") if op == "full" else 0
            self.ws_f = torch.empty(max(wsz, 1), device=dev, dtype=torch.uint8) if wsz else None
            wsz = tb.tconv_workspace_bytes(d, "backward") if op == "full" else 0
            self.ws_b = torch.empty(max(wsz // 8, 1), device=dev, dtype=torch.float64) if wsz else None
            if op == "sum":
                two = cfg.mode in ("compound", "parallel")
                g = torch.Generator(device="cpu")
                g.manual_seed(cfg.seed + 1000)
                cshape = (cfg.C_in, cfg.C_out)
                self.alpha = torch.rand(cshape, generator=g).to(dev) if two else None
                self.beta = torch.rand(cshape, generator=g).to(dev) if two else None
                self.ga = torch.empty(cshape, device=dev) if two else None
                self.gb = torch.empty(cshape, device=dev) if two else None
                # the backward pass re-reads x and gy instead of index tensors
                self.bytes_bi = (inp["x"].size + self.n_out) * 4 + inp["x"].size * 4
                self.bytes_bw = (inp["x"].size + self.n_out) * 4
                self.bytes_b = self.bytes_bi + self.bytes_bw

        def fwd(self, r=0):
            s = self.sets[r]
            if self.op == "sum":
                return tb.tconv_sum_forward(self.d, self.x, self.w_min, self.w_max, self.alpha, self.beta, self.y)
            tb.tconv_forward(self.d, self.x, self.w_min, self.w_max, None, None, self.y, self.y_min, self.y_max,
                             s["idx_min"], s["idx_max"], self.ws_f)

        def bwd_in(self, r=0):
            s = self.sets[r]
            if self.op == "sum":
                return tb.tconv_sum_backward(self.d, self.x, self.w_min, self.w_max, self.alpha, self.beta, s["gy"],
                                             s["gx"], None, None, None, None)
            tb.tconv_backward_input(self.d, s["gy"], None, None, s["idx_min"], s["idx_max"], s["gx"])

        def bwd_w(self, r=0):
            s = self.sets[r]
            if self.op == "sum":
                return tb.tconv_sum_backward(self.d, self.x, self.w_min, self.w_max, self.alpha, self.beta, s["gy"],
                                             None, s["gw_min"], s["gw_max"], self.ga, self.gb)
            tb.tconv_backward_weight(self.d, s["gy"], None, None, s["idx_min"], s["idx_max"], s["gw_min"],
                                     s["gw_max"], self.ws_b)

        def bwd(self, r=0):
            """Both gradients: the one-call entry point (the Sum-channel layers: one call for all five gradients)."""
            s = self.sets[r]
            if self.op == "sum":
                return tb.tconv_sum_backward(self.d, self.x, self.w_min, self.w_max, self.alpha, self.beta, s["gy"],
                                             s["gx"], s["gw_min"], s["gw_max"], self.ga, self.gb)
            if args.separate_backward:
                self.bwd_in(r)
                return self.bwd_w(r)
            tb.tconv_backward(self.d, s["gy"], None, None, s["idx_min"], s["idx_max"], s["gx"], s["gw_min"],
                              s["gw_max"], self.ws_b)

        def rotate_count(self):
            set_bytes = self.n_out * (4 + 4 * self.cfg.branches)
            return int(ROTATE_BYTES // set_bytes) + 2

    if args.op == "sum" and any(c.dtype != "f32" for c in cfgs):
        print("bench.py: the Sum-channel layers are fp32 only", file=sys.stderr)
        return 2

    # HIP events on the stream the kernels are launched on (torch's current stream)
    def ev():
        return torch.cuda.Event(enable_timing=True)

    def time_loop(fn, reps):
        """Average milliseconds per call of fn(i), i = 0 .. reps - 1, one event pair around the whole loop."""
        e0, e1 = ev(), ev()
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def cold_backward(cfg, op):
        """Backward calls of one layer on rotating operand sets, so that neither gy nor idx of a call is still in the
        last-level cache from the call that wrote or last read them.  Returns (ms_bwd_input, ms_bwd_weight, ms_both, layer)."""
        probe = Layer(cfg, op)
        R = probe.rotate_count()
        del probe
        L = Layer(cfg, op, rotate=R)
        for r in range(R):
            L.fwd(r)                       # valid winners in every set
        torch.cuda.synchronize()
        reps = max(2 * R, 8)
        for r in range(R):                 # warm-up of the three call paths
            L.bwd_in(r); L.bwd_w(r); L.bwd(r)
        torch.cuda.synchronize()
        t_bi = time_loop(lambda i: L.bwd_in(i % R), reps)
        t_bw = time_loop(lambda i: L.bwd_w(i % R), reps)
        t_b = time_loop(lambda i: L.bwd(i % R), reps)
        return t_bi, t_bw, t_b, L

    layers = [Layer(c, args.op) for c in cfgs]

    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for _ in range(args.warmup):
        for L in layers:
            L.fwd(); L.bwd()
    torch.cuda.synchronize()
    # The timed region carries HIP events around the dominant (forward) kernel only: an event costs about 10 us of
    # stream time on this stack.  The backward calls are timed in a pass of their own afterwards, on rotating buffers.
    graph = None
    if len(layers) > 1 and not args.no_graph:
        # The multi-layer step is some 60 launches of 20 - 100 us each, which the Python launch path cannot always
        # feed fast enough: the whole step (every layer, forward and backward) is captured once in a HIP graph
        # and replayed.  The library records no memset (its zero fills are kernels), so it is capture-safe.
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for L in layers:
                L.fwd(); L.bwd()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for L in layers:
                L.fwd(); L.bwd()
        graph.replay()
        torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if graph is not None:
            graph.replay()
            continue
        for L in layers:
            e = [ev(), ev()]
            e[0].record(); L.fwd(); e[1].record(); L.bwd()
            marks.append((L, e))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    if graph is not None:
        # events cannot sit inside a graph, and around eager launches of 20 - 100 us kernels they would time the launch
        # gaps: the forward launches of all layers are captured in a graph of their own and its replays are timed
        fgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(fgraph):
            for L in layers:
                L.fwd()
        fgraph.replay()
        torch.cuda.synchronize()
        t_f = time_loop(lambda i: fgraph.replay(), args.steps)
    else:
        t_f = sum(m[0].elapsed_time(m[1]) for _, m in marks) / args.steps   # ms per step, all layers
    # backward calls: on the operand sets of the step (warm: what a training step sees right after its forward
    # pass) and, for single layers, on rotating sets (cold: every byte from HBM)
    aux_steps = min(args.steps, 10)
    aux = []
    for _ in range(aux_steps):
        for L in layers:
            e = [ev() for _ in range(3)]
            L.fwd(); e[0].record(); L.bwd_in(); e[1].record(); L.bwd_w(); e[2].record()
            aux.append(e)
    torch.cuda.synchronize()
    t_bi = sum(m[0].elapsed_time(m[1]) for m in aux) / aux_steps
    t_bw = sum(m[1].elapsed_time(m[2]) for m in aux) / aux_steps

    pairs = sum(L.cfg.pairs for L in layers)
    value = pairs / (ms_step * 1e-3) / 1e9
    fwd_pairs_s = pairs / (t_f * 1e-3)
    # plain-form lane operations of the forward pass (2 per pair; compound 1.5) against the VALU issue rate
    lane_ops = sum(L.cfg.pairs * (LANE_OPS_PER_S / alu_peak_pairs_per_s(L.cfg.mode)) for L in layers)
    achieved = lane_ops / (t_f * 1e-3)
    # binary16 arithmetic: a packed instruction does two lane-operations, so the vector peak is twice the fp32 one
    peak_ops = LANE_OPS_PER_S * (2 if all(L.cfg.dtype == "f16" for L in layers) else 1)
    bytes_bi = sum(L.bytes_bi for L in layers)
    bytes_bw = sum(L.bytes_bw for L in layers)
    dtypes = {L.cfg.dtype for L in layers}
    traffic = (MEASURED_FORWARD_TRAFFIC.get((cfgs[0].name, cfgs[0].mode, cfgs[0].dtype, args.op))
               if len(cfgs) == 1 else None)

    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step"
                  + (" (Sum-channel layers)" if args.op == "sum" else ""),
        "value": round(value, 2),
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the arithmetic type: every add and compare is fp32 whatever the storage type, except the binary16 layers
        "dtype": "f16" if dtypes == {"f16"} else "f32",
        "storage": "f32" if dtypes == {"f32"} else ("f16" if dtypes == {"f16"} else "bf16"),
        "data": "synthetic",
        "config": {"workload": wl_name + (", forward + backward (all five gradients, one call)" if args.op == "sum" else
                                          ", forward + backward (grad_x and grad_w, "
                                          + ("two calls" if args.separate_backward else "one call") + ")")
                               + (", one HIP graph per step" if graph else ""),
                   "pairs_per_step": pairs,
                   "forward_kernel": (tb.tconv_sum_forward_kernel_name(layers[-1].d) if args.op == "sum"
                                      else tb.tconv_forward_kernel_name(layers[-1].d))},
        "forward_gops": round(fwd_pairs_s / 1e9, 2),
        "ms_forward": round(t_f, 4),
        "ms_backward_input": round(t_bi, 4),
        "ms_backward_weight": round(t_bw, 4),
        "backward_input_gbs": round(bytes_bi / (t_bi * 1e-3) / 1e9, 1),
        "backward_weight_gbs": round(bytes_bw / (t_bw * 1e-3) / 1e9, 1),
        # algorithmic lane-operations (one fp32 add or compare each) against the chip's fp32 VALU issue rate;
        # frac_best prices the same work at one packed add + one 3-operand compare per two pairs
        "roofline": {"bound": "alu", "kernel": "forward",
                     "achieved": round(achieved / 1e12, 3),
                     "peak": round(peak_ops / 1e12, 3), "unit": "Tlane-op/s",
                     "frac": round(achieved / peak_ops, 4), "frac_best": round(achieved / peak_ops / 2, 4),
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": traffic[1] if traffic else None},
    }
    if len(layers) == 1:
        cfg0 = layers[0].cfg
        del layers[0].sets[0]["gx"]
        c_bi, c_bw, c_b, Lc = cold_backward(cfg0, args.op)
        out["backward_cold"] = {
            "note": "backward calls on rotating operand sets (> 600 MB between two uses of a set): nothing served from "
                    "the last-level cache",
            "ms_backward_input": round(c_bi, 4), "ms_backward_weight": round(c_bw, 4), "ms_backward_both": round(c_b, 4),
            "backward_input_gbs": round(Lc.bytes_bi / (c_bi * 1e-3) / 1e9, 1),
            "backward_weight_gbs": round(Lc.bytes_bw / (c_bw * 1e-3) / 1e9, 1),
            "backward_both_gbs": round(Lc.bytes_b / (c_b * 1e-3) / 1e9, 1)}
        del Lc

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline([(L.cfg, L.inp) for L in layers], args.cpu_seconds, args.op,
                                           [(None if L.op != "sum" or L.alpha is None else L.alpha.cpu().numpy(),
                                             None if L.op != "sum" or L.beta is None else L.beta.cpu().numpy())
                                            for L in layers])

    if args.op == "full" and not args.no_layers and len(layers) == 1:
        # the other layers the bar is stated on, each measured the same way in this run: forward with events over a loop
        # of launches (milliseconds each), backward on rotating operand sets
        del layers
        torch.cuda.empty_cache()
        table = []
        for name, dt in BAR_LAYERS:
            cfg = CONFIGS[name] if dt is None else CONFIGS[name].with_(dtype=dt)
            c_bi, c_bw, c_b, L = cold_backward(cfg, "full")
            for _ in range(3):
                L.fwd()
            torch.cuda.synchronize()
            t = time_loop(lambda i: L.fwd(i % len(L.sets)), 10)
            ops = cfg.pairs * (LANE_OPS_PER_S / alu_peak_pairs_per_s(cfg.mode))
            lpeak = LANE_OPS_PER_S * (2 if cfg.dtype == "f16" else 1)   # packed 16-bit instructions: two per lane
            x_bytes = L.x.numel() * L.x.element_size()
            out_bytes = L.n_out * (L.y.element_size() * (1 + cfg.branches) + 4 * cfg.branches)
            table.append({
                "layer": name, "mode": cfg.mode, "storage": cfg.dtype, "pairs": cfg.pairs,
                "forward_kernel": tb.tconv_forward_kernel_name(L.d),
                "ms_forward": round(t, 4), "forward_gops": round(cfg.pairs / (t * 1e-3) / 1e9, 1),
                "frac": round(ops / (t * 1e-3) / lpeak, 4),
                "forward_hbm_gbs": round((x_bytes + out_bytes) / (t * 1e-3) / 1e9, 1),
                "ms_backward_input": round(c_bi, 4), "backward_input_gbs": round(L.bytes_bi / (c_bi * 1e-3) / 1e9, 1),
                "ms_backward_weight": round(c_bw, 4), "backward_weight_gbs": round(L.bytes_bw / (c_bw * 1e-3) / 1e9, 1),
                "ms_backward_both": round(c_b, 4), "backward_both_gbs": round(L.bytes_b / (c_b * 1e-3) / 1e9, 1)})
            del L
            torch.cuda.empty_cache()
        # the 19-layer stack: forward launches replayed from one HIP graph (no launch gaps inside the timed region)
        stack = [Layer(c, "full") for c in resnet20_layers(256)]
        for _ in range(2):
            for L in stack:
                L.fwd(); L.bwd()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for L in stack:
                L.fwd(); L.bwd()
        torch.cuda.current_stream().wait_stream(side)
        gf, gs = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(gf):
            for L in stack:
                L.fwd()
        with torch.cuda.graph(gs):
            for L in stack:
                L.fwd(); L.bwd()
        gf.replay(); gs.replay()
        torch.cuda.synchronize()
        t_f5 = time_loop(lambda i: gf.replay(), 10)
        t_s5 = time_loop(lambda i: gs.replay(), 10)
        p5 = sum(L.cfg.pairs for L in stack)
        table.append({"layer": "cfg5 (19 layers, batch 256, HIP graph replays)", "mode": "parallel", "storage": "f32",
                      "pairs": p5, "ms_forward": round(t_f5, 4), "forward_gops": round(p5 / (t_f5 * 1e-3) / 1e9, 1),
                      "frac": round(p5 * 2.0 / (t_f5 * 1e-3) / LANE_OPS_PER_S, 4),
                      "ms_step": round(t_s5, 4), "step_gops": round(p5 / (t_s5 * 1e-3) / 1e9, 1)})
        del stack, gf, gs
        torch.cuda.empty_cache()
        # the same net as ONE end-to-end training step (fused batch-norm / shortcut epilogues, head, all gradients)
        import copy
        nargs = copy.copy(args)
        nargs.steps, nargs.warmup, nargs.no_cpu_baseline = 10, 3, True
        net = bench_net(nargs, torch, tb, emit=False)
        table.append({"layer": "cfg5net (end-to-end training step of the ResNet-20-style net, glue included)",
                      "mode": "parallel", "storage": "f32", "pairs": net["config"]["pairs_per_step"],
                      "ms_forward": net["ms_forward"], "ms_backward": net["ms_backward"],
                      "ms_step": net["ms_per_step"], "step_gops": net["value"], "frac": net["roofline"]["frac"],
                      "graph_replays_checked_against_eager": net["config"]["graph_replays_checked_against_eager"]})
        torch.cuda.empty_cache()
        # the Sum-channel compound layer on the cfg2 shape (what the paper's networks are built from)
        Ls = Layer(CONFIGS["cfg2_main"], "sum")
        for _ in range(3):
            Ls.fwd(); Ls.bwd()
        torch.cuda.synchronize()
        t_sf = time_loop(lambda i: Ls.fwd(), 10)
        t_sb = time_loop(lambda i: Ls.bwd(), 10)
        ps = Ls.cfg.pairs
        table.append({"layer": "cfg2_main as a Sum-channel layer (tconv_sum_forward / tconv_sum_backward, all five "
                               "gradients)", "mode": "compound", "storage": "f32", "pairs": ps,
                      "forward_kernel": tb.tconv_sum_forward_kernel_name(Ls.d),
                      "ms_forward": round(t_sf, 4), "forward_gops": round(ps / (t_sf * 1e-3) / 1e9, 1),
                      "frac": round(ps * 1.5 / (t_sf * 1e-3) / LANE_OPS_PER_S, 4),
                      "ms_backward": round(t_sb, 4), "step_gops": round(ps / ((t_sf + t_sb) * 1e-3) / 1e9, 1)})
        del Ls
        torch.cuda.empty_cache()
        # the 19 layers of the ResNet-20 stack as Sum-channel layers (batch 256), back to back
        sstack = [Layer(c, "sum") for c in resnet20_layers(256)]
        for _ in range(2):
            for L in sstack:
                L.fwd(); L.bwd()
        torch.cuda.synchronize()

        def sum_fwd_all(i):
            for L in sstack:
                L.fwd()

        def sum_bwd_all(i):
            for L in sstack:
                L.bwd()

        t_ssf = time_loop(sum_fwd_all, 5)
        t_ssb = time_loop(sum_bwd_all, 5)
        pss = sum(L.cfg.pairs for L in sstack)
        table.append({"layer": "cfg5 as Sum-channel layers (19 layers, batch 256, launches back to back)",
                      "mode": "parallel", "storage": "f32", "pairs": pss, "ms_forward": round(t_ssf, 4),
                      "forward_gops": round(pss / (t_ssf * 1e-3) / 1e9, 1),
                      "frac": round(pss * 2.0 / (t_ssf * 1e-3) / LANE_OPS_PER_S, 4), "ms_backward": round(t_ssb, 4),
                      "step_gops": round(pss / ((t_ssf + t_ssb) * 1e-3) / 1e9, 1)})
        del sstack
        out["layers"] = table
    print(json.dumps(out), flush=True)
    return 0


def bench_net(args, torch, tb, emit: bool = True):
    """--workload cfg5net: ONE end-to-end training step of the all-tropical ResNet-20-style net (Sec. 5 TCNN BasicBlock:
    TropConv -> BN -> TropConv -> BN -> + shortcut, no ReLU), [256, 3, 32, 32] synthetic images, every conv in parallel
    mode.  Forward: 19 tconv_forward_fused calls chained layer to layer (batch norm folded to a per-channel scale and
    shift, the shortcut added in the kernel that writes y), global average pool, a 10-way linear head and a squared
    loss.  Backward: through the head, then per layer tconv_backward_input and tconv_backward_params (both kernel
    tensors, the shift and the scale from one pass over gy; the batch-norm scale enters as the branch coefficients).  Pool, head, loss, the shortcut's subsampling / channel padding and the
    gradient adds at the shortcuts are torch glue: inside the timed step, outside the pair count."""
    from paper_2504_06881_amd.inputs import resnet20_layers, make_inputs
    dev = torch.device("cuda:0")
    cfgs = resnet20_layers(256)
    g = torch.Generator(device="cpu")
    g.manual_seed(4)
    f32 = torch.float32

    class L:
        pass

    layers = []
    for cfg in cfgs:
        o = L()
        o.cfg, o.d = cfg, tb.Desc.from_cfg(cfg)
        inp = make_inputs(cfg)
        o.w_min = torch.from_numpy(inp["w_min"]).to(dev)
        o.w_max = torch.from_numpy(inp["w_max"]).to(dev)
        ho, wo = tb.tconv_out_shape(o.d)
        osh = (cfg.N, cfg.C_out, ho, wo)
        o.scale = (0.2 + 0.2 * torch.rand(cfg.C_out, generator=g)).to(dev)   # a branch sum doubles the scale of x
        o.shift = (0.2 * torch.rand(cfg.C_out, generator=g) - 0.1).to(dev)
        o.y = torch.empty(osh, device=dev)
        o.y_min, o.y_max = torch.empty(osh, device=dev), torch.empty(osh, device=dev)
        o.idx_min = torch.empty(osh, device=dev, dtype=torch.int32)
        o.idx_max = torch.empty(osh, device=dev, dtype=torch.int32)
        o.gx = torch.empty((cfg.N, cfg.C_in, cfg.H, cfg.W), device=dev)
        o.gw_min, o.gw_max = torch.empty_like(o.w_min), torch.empty_like(o.w_max)
        o.gshift, o.ga, o.gb = (torch.empty(cfg.C_out, device=dev) for _ in range(3))
        o.gscale = torch.empty(cfg.C_out, device=dev)
        nb = tb.tconv_workspace_bytes(o.d, "backward_params")
        o.ws = torch.empty(max(nb // 8, 1), device=dev, dtype=torch.float64)
        layers.append(o)
    x0 = torch.from_numpy(make_inputs(cfgs[0])["x"]).to(dev)
    n_cls = 10
    w_fc = ((torch.rand(n_cls, 64, generator=g) - 0.5) * 0.2).to(dev)
    b_fc = torch.zeros(n_cls, device=dev)
    target = torch.randn(256, n_cls, generator=g).to(dev)
    # blocks: (first conv, second conv) pairs after the stem; the shortcut of a block whose first conv has stride 2
    # takes every second pixel and pads the new channels with zeros
    blocks = [(layers[1 + 2 * b], layers[2 + 2 * b]) for b in range(9)]
    for a, b in blocks:
        a.sc = torch.zeros_like(b.y) if a.cfg.stride == 2 else None   # the padded channels stay zero
        a.gsc = torch.zeros_like(a.gx) if a.cfg.stride == 2 else None  # the skipped pixels stay zero
    head = L()

    stored = not args.recompute_branch_outputs

    def conv(o, x, residual):
        o.x_in = x
        tb.tconv_forward_fused(o.d, x, o.w_min, o.w_max, None, None, o.y, o.y_min if stored else None,
                               o.y_max if stored else None, o.idx_min, o.idx_max, scale=o.scale, shift=o.shift,
                               residual=residual)

    def forward():
        conv(layers[0], x0, None)
        x = layers[0].y
        for a, b in blocks:
            if a.sc is not None:
                a.sc[:, :a.cfg.C_in].copy_(x[:, :, ::2, ::2])
            conv(a, x, None)
            conv(b, a.y, a.sc if a.sc is not None else x)
            x = b.y
        return x

    def head_step(x):
        pooled = x.mean(dim=(2, 3))
        logits = torch.addmm(b_fc, pooled, w_fc.t())
        diff = logits - target
        head.loss = (diff * diff).mean()
        dlogits = diff * (2.0 / diff.numel())
        head.gw = dlogits.t() @ pooled
        head.gb = dlogits.sum(0)
        dpool = dlogits @ w_fc
        head.g = (dpool * (1.0 / (x.shape[2] * x.shape[3])))[:, :, None, None].expand_as(x).contiguous()

    def conv_backward(o, gy, need_gx=True):
        if need_gx:
            tb.tconv_backward_input(o.d, gy, o.scale, o.scale, o.idx_min, o.idx_max, o.gx)
        if stored:
            tb.tconv_backward_params(o.d, gy, o.scale, o.scale, o.idx_min, o.idx_max, o.y_min, o.y_max, o.gw_min,
                                     o.gw_max, o.ga, o.gb, o.gshift, o.ws)
        else:
            tb.tconv_backward_params_recompute(o.d, o.x_in, o.w_min, o.w_max, gy, o.scale, o.scale, o.idx_min, o.idx_max,
                                               o.gw_min, o.gw_max, o.ga, o.gb, o.gshift, o.ws)
        torch.add(o.ga, o.gb, out=o.gscale)

    def backward():
        gy = head.g
        for a, b in reversed(blocks):
            conv_backward(b, gy)
            conv_backward(a, b.gx)
            if a.gsc is not None:
                a.gsc[:, :, ::2, ::2].copy_(gy[:, :a.cfg.C_in])
                a.gx.add_(a.gsc)
            else:
                a.gx.add_(gy)
            gy = a.gx
        conv_backward(layers[0], gy, need_gx=False)

    def step_eager():
        head_step(forward())
        backward()

    def checksum():
        return [float(head.loss), float(layers[0].gw_min.double().abs().sum()), float(layers[5].gscale.double().sum()),
                float(layers[18].gw_max.double().abs().sum()), float(blocks[3][0].gx.double().abs().sum())]

    for _ in range(max(args.warmup, 2)):
        step_eager()
    torch.cuda.synchronize()
    ref = checksum()
    g_f = g_b = None
    graph_ok = False
    if not args.no_graph:
        # the forward and backward chains of library launches (and the elementwise glue between them) replay from HIP
        # graphs; the head (a reduction and three small matrix products) stays eager between the two
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_eager()
        torch.cuda.current_stream().wait_stream(side)
        g_f, g_b = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_f):
            xo = forward()
        head_step(xo)
        with torch.cuda.graph(g_b):
            backward()
        graph_ok = True
        for _ in range(3):   # replays against the eager step, with eager work in between
            g_f.replay(); head_step(xo); g_b.replay()
            torch.cuda.synchronize()
            got = checksum()
            if any(abs(a - b) > 1e-6 * max(1.0, abs(b)) for a, b in zip(got, ref)):
                graph_ok = False
            step_eager()
            torch.cuda.synchronize()

    def step():
        if graph_ok:
            g_f.replay(); head_step(xo); g_b.replay()
        else:
            step_eager()

    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def timed(fn, reps=10):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_f = timed(g_f.replay if graph_ok else forward)
    t_b = timed(g_b.replay if graph_ok else backward)
    pairs = sum(c.pairs for c in cfgs)
    achieved = pairs * 2.0 / (t_f * 1e-3)
    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step",
        "value": round(pairs / (ms_step * 1e-3) / 1e9, 2), "unit": "GOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "storage": "f32", "data": "synthetic",
        "config": {"workload": "cfg5net: one training step of the all-tropical ResNet-20-style net on x[256,3,32,32], "
                               "19 parallel-mode 3x3 layers with fused batch-norm scale/shift and shortcut, pool + "
                               "linear head + squared loss, all gradients; glue inside the time, outside the pair count"
                               + (", forward and backward chains replayed from HIP graphs" if graph_ok else ", eager"),
                   "pairs_per_step": pairs, "graph_replays_checked_against_eager": graph_ok},
        "ms_forward": round(t_f, 4), "ms_backward": round(t_b, 4),
        "forward_gops": round(pairs / (t_f * 1e-3) / 1e9, 2),
        "loss": ref[0],
        "roofline": {"bound": "alu", "kernel": "forward chain (19 fused layers and the shortcut copies)",
                     "achieved": round(achieved / 1e12, 3), "peak": round(LANE_OPS_PER_S / 1e12, 3),
                     "unit": "Tlane-op/s", "frac": round(achieved / LANE_OPS_PER_S, 4), "traffic": None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline([(c, make_inputs(c)) for c in cfgs], args.cpu_seconds, "full",
                                           [(None, None)] * len(cfgs))
        out["cpu_baseline"]["sample"] += " (the 19 layers' forward and backward calls; no glue)"
    if not emit:
        return out
    print(json.dumps(out), flush=True)
    return 0


def bench_1d(args, torch, tb) -> int:
    """One one-dimensional layer: tconv1d_forward, tconv1d_backward_input, tconv1d_backward_weight per step; the
    forward pass is judged against the plain fp32 VALU form, as for the two-dimensional layers."""
    from paper_2504_06881_amd.inputs import CONFIGS_1D, make_1d_inputs
    cfg = CONFIGS_1D[args.workload if args.workload in CONFIGS_1D else "c1d_main"]
    if args.mode:
        cfg = cfg.with_(mode=args.mode)
    dev = torch.device("cuda:0")
    inp = make_1d_inputs(cfg)
    d = tb.Desc1d(cfg.N, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil, cfg.mode, cfg.dtype)
    lo = tb.tconv1d_out_len(d)
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    x, gy = up(inp["x"]), up(inp["gy"])
    w_min = up(inp["w_min"])
    w_max = w_min if cfg.mode == "compound" else up(inp["w_max"])
    do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")
    osh = (cfg.N, cfg.C_out, lo)
    new = lambda dt=torch.float32: torch.empty(osh, device=dev, dtype=dt)
    y, y_min, y_max = new(), (new() if do_min else None), (new() if do_max else None)
    i_min, i_max = (new(torch.int32) if do_min else None), (new(torch.int32) if do_max else None)
    gx = torch.empty_like(x)
    wshape = (cfg.C_out, cfg.C_in, cfg.K)
    g1 = torch.empty(wshape, device=dev) if do_min else None
    g2 = torch.empty(wshape, device=dev) if (do_max and cfg.mode != "compound") else None
    fwd = lambda: tb.tconv1d_forward(d, x, w_min, w_max, None, None, y, y_min, y_max, i_min, i_max)
    bwd_i = lambda: tb.tconv1d_backward_input(d, gy, None, None, i_min, i_max, gx)
    bwd_w = lambda: tb.tconv1d_backward_weight(d, gy, None, None, i_min, i_max, g1, g2)
    for _ in range(args.warmup):
        fwd(); bwd_i(); bwd_w()
    torch.cuda.synchronize()
    # events around the forward kernel only inside the timed region; the backward calls are timed in a short
    # pass of their own afterwards (an event costs about 10 us of stream time)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [ev(), ev()]
        e[0].record(); fwd(); e[1].record(); bwd_i(); bwd_w()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_f = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    ms_step = wall * 1e3 / args.steps
    aux_steps, aux = min(args.steps, 10), []
    for _ in range(aux_steps):
        e = [ev() for _ in range(3)]
        fwd(); e[0].record(); bwd_i(); e[1].record(); bwd_w(); e[2].record()
        aux.append(e)
    torch.cuda.synchronize()
    t_bi = sum(m[0].elapsed_time(m[1]) for m in aux) / aux_steps
    t_bw = sum(m[1].elapsed_time(m[2]) for m in aux) / aux_steps
    pairs = cfg.pairs
    achieved = pairs * (LANE_OPS_PER_S / alu_peak_pairs_per_s(cfg.mode)) / (t_f * 1e-3)
    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step (one-dimensional layer)",
        "value": round(pairs / (ms_step * 1e-3) / 1e9, 2), "unit": "GOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: x[{cfg.N},{cfg.C_in},{cfg.L}] -> {cfg.C_out}ch k{cfg.K} s{cfg.stride} "
                               f"p{cfg.pad} d{cfg.dil} {cfg.mode} f32, fwd+bwd_input+bwd_weight",
                   "pairs_per_step": pairs, "forward_kernel": tb.tconv1d_forward_kernel_name(d)},
        "forward_gops": round(pairs / (t_f * 1e-3) / 1e9, 2),
        "ms_forward": round(t_f, 4), "ms_backward_input": round(t_bi, 4), "ms_backward_weight": round(t_bw, 4),
        "roofline": {"bound": "alu", "kernel": "forward", "achieved": round(achieved / 1e12, 3),
                     "peak": round(LANE_OPS_PER_S / 1e12, 3), "unit": "Tlane-op/s",
                     "frac": round(achieved / LANE_OPS_PER_S, 4), "frac_best": round(achieved / LANE_OPS_PER_S / 2, 4),
                     "traffic": (MEASURED_FORWARD_TRAFFIC.get((cfg.name, cfg.mode, "f32", "1d")) or (None, None))[0],
                     "traffic_source": (MEASURED_FORWARD_TRAFFIC.get((cfg.name, cfg.mode, "f32", "1d")) or (None, None))[1]},
    }
    if not args.no_cpu_baseline:
        from oracle import tconv1d_oracle as o1
        from oracle import tconv_oracle as orc

        def run(n_img):
            t = time.perf_counter()
            s = o1.Shape1d(n_img, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil)
            r = o1.forward(s, cfg.mode, inp["x"][:n_img], inp["w_min"], inp["w_max"])
            o1.backward(s, cfg.mode, inp["gy"][:n_img], r["idx_min"], r["idx_max"])
            return time.perf_counter() - t

        t1 = run(1)
        n_img = int(max(1, min(cfg.N, args.cpu_seconds / max(t1, 1e-6))))
        reps, total = 0, 0.0
        while reps == 0 or (total < args.cpu_seconds and reps < 50):
            total += run(n_img)
            reps += 1
        out["cpu_baseline"] = {"value": round(pairs / cfg.N * n_img * reps / total / 1e9, 3), "unit": "GOPS",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {n_img} of {cfg.N} signals of the same layer, forward + backward, "
                                         f"{reps} repetitions, {total:.1f} s of wall time"}
    print(json.dumps(out), flush=True)
    return 0


def bench_3d(args, torch, tb) -> int:
    """One three-dimensional layer: tconv3d_forward, tconv3d_backward_input, tconv3d_backward_weight per step."""
    from paper_2504_06881_amd.inputs import CONFIGS_3D, make_3d_inputs
    cfg = CONFIGS_3D[args.workload if args.workload in CONFIGS_3D else "c3d_main"]
    if args.mode:
        cfg = cfg.with_(mode=args.mode)
    dev = torch.device("cuda:0")
    inp = make_3d_inputs(cfg)
    d = tb.Desc3d(cfg.N, cfg.C_in, cfg.D, cfg.H, cfg.W, cfg.C_out, cfg.k[0], cfg.k[1], cfg.k[2], tuple(cfg.stride),
                  tuple(cfg.pad), tuple(cfg.dil), cfg.mode)
    out3 = tb.tconv3d_out_shape(d)
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    x, gy = up(inp["x"]), up(inp["gy"])
    w_min = up(inp["w_min"])
    w_max = w_min if cfg.mode == "compound" else up(inp["w_max"])
    do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")
    osh = (cfg.N, cfg.C_out) + out3
    new = lambda dt=torch.float32: torch.empty(osh, device=dev, dtype=dt)
    y, y_min, y_max = new(), (new() if do_min else None), (new() if do_max else None)
    i_min, i_max = (new(torch.int32) if do_min else None), (new(torch.int32) if do_max else None)
    gx = torch.empty_like(x)
    wshape = (cfg.C_out, cfg.C_in) + tuple(cfg.k)
    g1 = torch.empty(wshape, device=dev) if do_min else None
    g2 = torch.empty(wshape, device=dev) if (do_max and cfg.mode != "compound") else None
    fwd = lambda: tb.tconv3d_forward(d, x, w_min, w_max, None, None, y, y_min, y_max, i_min, i_max)
    bwd_i = lambda: tb.tconv3d_backward_input(d, gy, None, None, i_min, i_max, gx)
    bwd_w = lambda: tb.tconv3d_backward_weight(d, gy, None, None, i_min, i_max, g1, g2)
    for _ in range(args.warmup):
        fwd(); bwd_i(); bwd_w()
    torch.cuda.synchronize()
    # events around the forward kernel only inside the timed region; the backward calls are timed in a short
    # pass of their own afterwards (an event costs about 10 us of stream time)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [ev(), ev()]
        e[0].record(); fwd(); e[1].record(); bwd_i(); bwd_w()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_f = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    ms_step = wall * 1e3 / args.steps
    aux_steps, aux = min(args.steps, 10), []
    for _ in range(aux_steps):
        e = [ev() for _ in range(3)]
        fwd(); e[0].record(); bwd_i(); e[1].record(); bwd_w(); e[2].record()
        aux.append(e)
    torch.cuda.synchronize()
    t_bi = sum(m[0].elapsed_time(m[1]) for m in aux) / aux_steps
    t_bw = sum(m[1].elapsed_time(m[2]) for m in aux) / aux_steps
    pairs = cfg.pairs
    achieved = pairs * (LANE_OPS_PER_S / alu_peak_pairs_per_s(cfg.mode)) / (t_f * 1e-3)
    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step (three-dimensional layer)",
        "value": round(pairs / (ms_step * 1e-3) / 1e9, 2), "unit": "GOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: x[{cfg.N},{cfg.C_in},{cfg.D},{cfg.H},{cfg.W}] -> {cfg.C_out}ch "
                               f"k{cfg.k} s{cfg.stride} p{cfg.pad} d{cfg.dil} {cfg.mode} f32, fwd+bwd_input+bwd_weight",
                   "pairs_per_step": pairs, "forward_kernel": tb.tconv3d_forward_kernel_name(d)},
        "forward_gops": round(pairs / (t_f * 1e-3) / 1e9, 2),
        "ms_forward": round(t_f, 4), "ms_backward_input": round(t_bi, 4), "ms_backward_weight": round(t_bw, 4),
        "roofline": {"bound": "alu", "kernel": "forward", "achieved": round(achieved / 1e12, 3),
                     "peak": round(LANE_OPS_PER_S / 1e12, 3), "unit": "Tlane-op/s",
                     "frac": round(achieved / LANE_OPS_PER_S, 4), "frac_best": round(achieved / LANE_OPS_PER_S / 2, 4),
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import tconv3d_oracle as o3
        from oracle import tconv_oracle as orc

        def run(n_img):
            t = time.perf_counter()
            s = o3.Shape3d(n_img, cfg.C_in, cfg.D, cfg.H, cfg.W, cfg.C_out, cfg.k[0], cfg.k[1], cfg.k[2],
                           tuple(cfg.stride), tuple(cfg.pad), tuple(cfg.dil))
            r = o3.forward(s, cfg.mode, inp["x"][:n_img], inp["w_min"], inp["w_max"])
            o3.backward(s, cfg.mode, inp["gy"][:n_img], r["idx_min"], r["idx_max"])
            return time.perf_counter() - t

        t1 = run(1)
        n_img = int(max(1, min(cfg.N, args.cpu_seconds / max(t1, 1e-6))))
        reps, total = 0, 0.0
        while reps == 0 or (total < args.cpu_seconds and reps < 50):
            total += run(n_img)
            reps += 1
        out["cpu_baseline"] = {"value": round(pairs / cfg.N * n_img * reps / total / 1e9, 3), "unit": "GOPS",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {n_img} of {cfg.N} volumes of the same layer, forward + backward, "
                                         f"{reps} repetitions, {total:.1f} s of wall time"}
    print(json.dumps(out), flush=True)
    return 0


def bench_depthwise(args, torch, tb) -> int:
    """One depthwise layer: forward (writes y and the packed winner byte), backward w.r.t. the input, backward
    w.r.t. kernel and coefficients.  These layers are HBM bound: the roofline entry is the forward kernel's
    algorithmic bytes (x read once, y and one index byte written per output) against the HBM peak."""
    from paper_2504_06881_amd.inputs import DW_CONFIGS, make_depthwise_inputs
    name = args.workload if args.workload in DW_CONFIGS else "dw_main"
    cfg = DW_CONFIGS[name]
    if args.mode:
        if args.mode not in ("max", "min", "compound", "parallel"):
            print("bench.py: depthwise layers have the modes max, min, compound, parallel", file=sys.stderr)
            return 2
        cfg = cfg.with_(mode=args.mode)
    dev = torch.device("cuda:0")
    inp = make_depthwise_inputs(cfg)
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    x, gy, al, be = up(inp["x"]), up(inp["gy"]), up(inp["alpha"]), up(inp["beta"])
    w_min = up(inp["w_min"])
    w_max = w_min if cfg.mode == "compound" else up(inp["w_max"])
    two = cfg.mode in ("compound", "parallel")
    osh = (cfg.N, cfg.C_out, ho, wo)
    y = torch.empty(osh, device=dev)
    idx = torch.empty(osh, device=dev, dtype=torch.uint8)
    gx = torch.empty_like(x)
    wshape = (cfg.C_out, 1, cfg.KH, cfg.KW)
    g1 = torch.empty(wshape, device=dev) if cfg.mode != "max" else None
    g2 = torch.empty(wshape, device=dev) if cfg.mode in ("max", "parallel") else None
    ga = torch.empty(cfg.C_out, device=dev) if two else None
    gb = torch.empty(cfg.C_out, device=dev) if two else None
    fwd = lambda: tb.tconv_depthwise_forward(d, x, w_min, w_max, al, be, y, idx)
    # one backward call for every gradient, as a training step makes it
    bwd = lambda: tb.tconv_depthwise_backward(d, x, w_min, w_max, al, be, gy, idx, gx, g1, g2, ga, gb)
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [ev(), ev()]
        e[0].record(); fwd(); e[1].record(); bwd()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_f = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps
    ms_step = wall * 1e3 / args.steps
    aux_steps, aux = min(args.steps, 10), []   # the backward call, timed in a short pass of its own
    for _ in range(aux_steps):
        e = [ev(), ev()]
        fwd(); e[0].record(); bwd(); e[1].record()
        aux.append(e)
    torch.cuda.synchronize()
    t_b = sum(m[0].elapsed_time(m[1]) for m in aux) / aux_steps
    n_in, n_out = x.numel(), y.numel()
    pairs = n_out * cfg.KH * cfg.KW * (2 if two else 1)
    bytes_f = n_in * 4 + n_out * 5            # x read; y and one winner byte written
    # backward: gy and the winner byte read by the input-gradient and by the parameter-gradient kernel, x read for
    # the coefficient gradients, grad_x written
    bytes_b = 2 * n_out * 5 + n_in * 4 + (n_in * 4 if two else 0)
    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step (depthwise layer)",
        "value": round(pairs / (ms_step * 1e-3) / 1e9, 2), "unit": "GOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: depthwise x[{cfg.N},{cfg.C_in},{cfg.H},{cfg.W}] -> {cfg.C_out}ch 3x3 "
                               f"s{cfg.stride} p{cfg.pad} {cfg.mode} f32, forward + one backward call (all gradients)",
                   "pairs_per_step": pairs, "forward_kernel": tb.tconv_depthwise_forward_kernel_name(d)},
        "forward_gops": round(pairs / (t_f * 1e-3) / 1e9, 2),
        "ms_forward": round(t_f, 4), "ms_backward": round(t_b, 4),
        "backward_gbs": round(bytes_b / (t_b * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "kernel": "forward", "achieved": round(bytes_f / (t_f * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(bytes_f / (t_f * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import tconv_oracle as orc
        from oracle import tdw_oracle as odw

        def run(n_img):
            t = time.perf_counter()
            s = orc.Shape(n_img, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil)
            odw.forward(s, cfg.mode, inp["x"][:n_img], inp["w_min"], inp["w_max"], inp["alpha"], inp["beta"])
            odw.backward(s, cfg.mode, inp["x"][:n_img], inp["gy"][:n_img], inp["w_min"], inp["w_max"], inp["alpha"],
                         inp["beta"])
            return time.perf_counter() - t

        t1 = run(1)
        n_img = int(max(1, min(cfg.N, args.cpu_seconds / max(t1, 1e-6))))
        reps, total = 0, 0.0
        while reps == 0 or (total < args.cpu_seconds and reps < 50):
            total += run(n_img)
            reps += 1
        out["cpu_baseline"] = {"value": round(pairs / cfg.N * n_img * reps / total / 1e9, 3), "unit": "GOPS",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {n_img} of {cfg.N} images of the same layer, forward + backward, "
                                         f"{reps} repetitions, {total:.1f} s of wall time"}
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline(layers, target_s: float, op: str = "full", coefs=None):
    """The CPU oracle, as it stands, on a batch slice sized for about target_s seconds of CPU work."""
    from oracle import tconv_oracle as orc
    threads = orc.num_threads()
    if op == "sum":
        from oracle import tsum_oracle as osum
        threads = 1  # the Sum-channel oracle is a single-threaded loop nest
    n_full = layers[0][0].N
    per_image = sum(cfg.pairs for cfg, _ in layers) / n_full

    def run(n_img):
        t0 = time.perf_counter()
        for li, (cfg, inp) in enumerate(layers):
            s = orc.Shape(n_img, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil)
            xs, gys = inp["x"][:n_img], inp["gy"][:n_img]
            if op == "sum":
                a, b = coefs[li]
                osum.forward(s, cfg.mode, xs, inp["w_min"], inp["w_max"], a, b)
                osum.backward(s, cfg.mode, xs, gys, inp["w_min"], inp["w_max"], a, b)
                continue
            if cfg.mode in ("minplus_max", "maxplus_min"):  # single-branch layer; backward of the plain layer of its side
                side = "min" if cfg.mode == "minplus_max" else "max"
                f = orc.forward_mixed(s, cfg.mode, xs, inp["w_" + side])
                kw = {"idx_" + side: f["idx"]}
                orc.backward_input(s, side, gys, **kw)
                orc.backward_weight(s, side, gys, **kw)
                continue
            r = orc.forward(s, cfg.mode, xs, inp["w_min"], inp["w_max"])
            orc.backward_input(s, cfg.mode, gys, r["idx_min"], r["idx_max"])
            orc.backward_weight(s, cfg.mode, gys, r["idx_min"], r["idx_max"])
        return time.perf_counter() - t0

    t1 = run(1)  # calibrate on one image
    n_img = int(max(1, min(n_full, target_s / max(t1, 1e-6))))
    # repeat the slice until about target_s seconds of CPU work have been timed
    reps, total = 0, 0.0
    while reps == 0 or (total < target_s and reps < 50):
        total += run(n_img)
        reps += 1
    return {"value": round(per_image * n_img * reps / total / 1e9, 3), "unit": "GOPS", "cores": threads,
            "kind": "oracle", "sample": f"first {n_img} of {n_full} images of the same workload, forward + both "
                                        f"backward passes, {reps} repetitions, {total:.1f} s of wall time"}


if __name__ == "__main__":
    sys.exit(main())
