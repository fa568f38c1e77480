#!/usr/bin/env python3
"""Benchmark of the tropical-convolution hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
tconv_forward + tconv_backward_input + tconv_backward_weight of the headline
layer (benchmark configs[1]: x [128,64,32,32] -> 64 channels, 3x3, stride 1,
pad 1, compound mode, fp32), inputs resident in HBM before the timed region.

Prints ONE JSON line:
  metric / value : add+compare pairs per second of the step (dense pair count / step time), GOPS
  roofline       : the forward kernel against the fp32 vector-ALU peak, measured live with HIP events
  cpu_baseline   : the CPU oracle timed on this machine's host cores on a bounded sample of the same workload
Extra keys give the forward-only rate and the achieved HBM GB/s of the two backward calls.
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


def alu_peak_pairs_per_s(mode: str) -> float:
    """Plain fp32 VALU roofline in pairs/s: one v_add_f32 and one v_max/min_f32 per pair,
    except compound where one add feeds both branches (3 lane-instructions per 2 pairs)."""
    instr_per_pair = {"max": 2.0, "min": 2.0, "parallel": 2.0, "compound": 1.5}[mode]
    return LANE_OPS_PER_S / instr_per_pair


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2_main")
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
    cfg = CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    inp = make_inputs(cfg)
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def up(a, dt=torch.float32):
        return None if a is None else torch.from_numpy(a).to(dev).to(dt).contiguous()

    x = up(inp["x"], tdt)
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"], tdt)
    else:
        w_min, w_max = up(inp["w_min"], tdt), up(inp["w_max"], tdt)
    gy = up(inp["gy"])
    oshape = (cfg.N, cfg.C_out, ho, wo)
    do_min, do_max = cfg.mode != "max", cfg.mode != "min"
    y = torch.empty(oshape, device=dev, dtype=tdt)
    y_min = torch.empty(oshape, device=dev, dtype=tdt) if do_min else None
    y_max = torch.empty(oshape, device=dev, dtype=tdt) if do_max else None
    idx_min = torch.empty(oshape, device=dev, dtype=torch.int32) if do_min else None
    idx_max = torch.empty(oshape, device=dev, dtype=torch.int32) if do_max else None
    gx = torch.empty(tuple(inp["x"].shape), device=dev)
    wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
    gw_min = torch.empty(wshape, device=dev) if do_min else None
    gw_max = torch.empty(wshape, device=dev) if cfg.mode in ("max", "parallel") else None

    def fwd():
        tb.tconv_forward(d, x, w_min, w_max, None, None, y, y_min, y_max, idx_min, idx_max)

    def bwd_in():
        tb.tconv_backward_input(d, gy, None, None, idx_min, idx_max, gx)

    def bwd_w():
        tb.tconv_backward_weight(d, gy, None, None, idx_min, idx_max, gw_min, gw_max)

    # HIP events on the stream the kernels are launched on (torch's current stream)
    def ev():
        return torch.cuda.Event(enable_timing=True)

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, device=dev)  # 256 MiB
        src.normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        fwd(); bwd_in(); bwd_w()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [ev() for _ in range(4)]
        e[0].record(); fwd(); e[1].record(); bwd_in(); e[2].record(); bwd_w(); e[3].record()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_f = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps   # ms
    t_bi = sum(m[1].elapsed_time(m[2]) for m in marks) / args.steps
    t_bw = sum(m[2].elapsed_time(m[3]) for m in marks) / args.steps
    ms_step = wall * 1e3 / args.steps

    pairs = cfg.pairs
    value = pairs / (ms_step * 1e-3) / 1e9
    fwd_pairs_s = pairs / (t_f * 1e-3)
    peak = alu_peak_pairs_per_s(cfg.mode)
    n_out = cfg.N * cfg.C_out * ho * wo
    br = cfg.branches
    # algorithmic HBM bytes of the backward calls: gy + idx per output per branch, grad written once
    bytes_bi = n_out * (4 + 4 * br) + inp["x"].size * 4
    bytes_bw = n_out * (4 + 4 * br) + cfg.C_out * cfg.K * 4 * (2 if cfg.mode == "parallel" else 1)

    out = {
        "metric": "tropical-conv GOPS (add+max pairs/s), forward + backward step",
        "value": round(value, 2),
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16-storage/f32-arith",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: x[{cfg.N},{cfg.C_in},{cfg.H},{cfg.W}] -> {cfg.C_out}ch 3x3 "
                               f"s{cfg.stride} p{cfg.pad} d{cfg.dil} {cfg.mode} {cfg.dtype}, fwd+bwd_input+bwd_weight",
                   "pairs_per_step": pairs, "forward_kernel": tb.tconv_forward_kernel_name(d)},
        "forward_gops": round(fwd_pairs_s / 1e9, 2),
        "ms_forward": round(t_f, 4),
        "ms_backward_input": round(t_bi, 4),
        "ms_backward_weight": round(t_bw, 4),
        "backward_input_gbs": round(bytes_bi / (t_bi * 1e-3) / 1e9, 1),
        "backward_weight_gbs": round(bytes_bw / (t_bw * 1e-3) / 1e9, 1),
        # algorithmic lane-operations (one fp32 add or compare each) against the chip's fp32 VALU issue rate
        "roofline": {"bound": "alu", "kernel": "forward",
                     "achieved": round(fwd_pairs_s * (LANE_OPS_PER_S / peak) / 1e12, 3),
                     "peak": round(LANE_OPS_PER_S / 1e12, 3), "unit": "Tlane-op/s",
                     "frac": round(fwd_pairs_s / peak, 4), "traffic": None},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, args.cpu_seconds)
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline(cfg, inp, target_s: float):
    """The CPU oracle, as it stands, on a batch slice sized for about target_s seconds of CPU work."""
    from oracle import tconv_oracle as orc
    threads = orc.num_threads()
    per_image = cfg.pairs / cfg.N

    def run(n_img):
        s = orc.Shape(n_img, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil)
        xs, gys = inp["x"][:n_img], inp["gy"][:n_img]
        t0 = time.perf_counter()
        r = orc.forward(s, cfg.mode, xs, inp["w_min"], inp["w_max"])
        orc.backward_input(s, cfg.mode, gys, r["idx_min"], r["idx_max"])
        orc.backward_weight(s, cfg.mode, gys, r["idx_min"], r["idx_max"])
        return time.perf_counter() - t0

    t1 = run(1)  # calibrate on one image
    n_img = int(max(1, min(cfg.N, target_s / max(t1, 1e-6))))
    # repeat the slice until about target_s seconds of CPU work have been timed
    reps, total = 0, 0.0
    while reps == 0 or (total < target_s and reps < 50):
        total += run(n_img)
        reps += 1
    return {"value": round(per_image * n_img * reps / total / 1e9, 3), "unit": "GOPS", "cores": threads,
            "kind": "oracle", "sample": f"first {n_img} of {cfg.N} images of the same workload, forward + both "
                                        f"backward passes, {reps} repetitions, {total:.1f} s of wall time"}


if __name__ == "__main__":
    sys.exit(main())
