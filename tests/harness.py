"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle, compare.

The HIP side and the oracle side only meet here, on numpy arrays; both consume the
same seeded host buffers from ``paper_2504_06881_amd.inputs``.
"""
import os

import numpy as np

from oracle import tconv_oracle as orc
from paper_2504_06881_amd import binding as tb

GRAD_RTOL = 1e-5  # spec tolerance for fp32 gradients


MIXED = {"minplus_max": "min", "maxplus_min": "max"}   # mixed layer -> the side (kernel, index, output) it uses


def oracle_shape(cfg):
    return orc.Shape(cfg.N, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil,
                     stride_w=cfg.stride_hw[1], pad_w=cfg.pad_hw[1], dil_w=cfg.dil_hw[1])


def run_oracle(cfg, inp, backward=True):
    s = oracle_shape(cfg)
    m = cfg.mode
    if m in MIXED:
        # single-branch layer on the side of its operator; backward = the plain layer of that side
        side = MIXED[m]
        f = orc.forward_mixed(s, m, inp["x"], inp["w_" + side], out_bf16=(cfg.dtype == "bf16"))
        r = dict(y=f["y"], y_min=None, y_max=None, idx_min=None, idx_max=None)
        r["y_" + side], r["idx_" + side] = f["y"], f["idx"]
        m = side
    else:
        r = orc.forward(s, m, inp["x"], inp["w_min"], inp["w_max"], inp["alpha"], inp["beta"],
                        out_bf16=(cfg.dtype == "bf16"))
    if backward:
        kw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=inp["alpha"], beta=inp["beta"])
        r["grad_x"] = orc.backward_input(s, m, inp["gy"], **kw)
        r["grad_w_min"], r["grad_w_max"] = orc.backward_weight(s, m, inp["gy"], **kw)
        # magnitude of the summands of every gradient element: the scale of the tolerance
        ab = {k: (None if inp[k] is None else np.abs(inp[k])) for k in ("alpha", "beta")}
        kwa = dict(idx_min=r["idx_min"], idx_max=r["idx_max"], alpha=ab["alpha"], beta=ab["beta"])
        r["grad_x_scale"] = orc.backward_input(s, m, np.abs(inp["gy"]), **kwa)
        r["grad_w_min_scale"], r["grad_w_max_scale"] = orc.backward_weight(s, m, np.abs(inp["gy"]), **kwa)
        if m in ("compound", "parallel"):  # gradient of the combine step, from the branch outputs
            r["grad_alpha"], r["grad_beta"] = orc.backward_alpha_beta(s, m, inp["gy"], r["y_min"], r["y_max"])
            r["grad_alpha_scale"], r["grad_beta_scale"] = orc.backward_alpha_beta(
                s, m, np.abs(inp["gy"]), np.abs(r["y_min"]), np.abs(r["y_max"]))
    return r


def scratch(nbytes, dev):
    """A poisoned device buffer of nbytes (None for 0): the library must not rely on what a workspace holds."""
    import torch
    if not nbytes:
        return None
    t = torch.empty((nbytes + 7) // 8, device=dev, dtype=torch.float64)
    t.fill_(float("nan"))
    return t


# The random parity sweeps draw their layers from fixed seeds; TCONV_TEST_SEED_SHIFT=n (an integer) moves every one of
# them by n, for runs over other layers than the committed ones (pytest -m gpu -k random).
SEED_SHIFT = int(os.environ.get("TCONV_TEST_SEED_SHIFT", "0"))


def every_window_has_a_tap(size, k, stride, pad, dil):
    """One axis, written out: every output position has a tap inside the input.  A dilated window can straddle an
    input shorter than the dilation; such layers have no defined output and the library and the oracles reject them, so
    the random sweeps leave them out."""
    n = size + 2 * pad - dil * (k - 1) - 1
    return n >= 0 and all(any(0 <= o * stride - pad + t * dil < size for t in range(k))
                          for o in range(n // stride + 1))


def run_hip(cfg, inp, backward=True, branch_outputs=True, device="cuda:0", deterministic=True, fused=False,
            x_halfword_offset=False):
    """Forward (+ backward) through the C ABI; returns numpy arrays (bf16 outputs widened to fp32).
    deterministic: the parameter gradients get their workspaces (fixed-order fp64 sums); False: the atomic forms.
    fused: grad_x and the kernel gradients through the one-call tconv_backward instead of the two separate calls;
    "params": grad_x by tconv_backward_input and every parameter gradient, grad_bias included, by tconv_backward_params;
    "recompute": the same by tconv_backward_params_recompute after a forward pass without branch outputs."""
    import torch
    dev = torch.device(device)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    assert (ho, wo) == cfg.out_hw

    def up(a, dt=torch.float32):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()

    x = up(inp["x"], tdt)
    if x_halfword_offset:  # 16-bit storage: the same values one element into a larger buffer (address = 2 mod 4)
        big = torch.empty(x.numel() + 1, device=dev, dtype=tdt)
        big[1:].copy_(x.reshape(-1))
        x = big[1:].view(x.shape)
        assert x.data_ptr() % 4 == 2
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"], tdt)
    else:
        w_min, w_max = up(inp["w_min"], tdt), up(inp["w_max"], tdt)
    alpha, beta, gy = up(inp["alpha"]), up(inp["beta"]), up(inp["gy"])
    oshape = (cfg.N, cfg.C_out, ho, wo)
    do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")

    def poison(dt):  # outputs start from garbage: the library must overwrite, never accumulate
        t = torch.empty(oshape, device=dev, dtype=dt)
        if dt == torch.int32:
            t.fill_(-12345)
        else:
            t.fill_(float("nan"))
        return t

    y = poison(tdt)
    y_min = poison(tdt) if (do_min and branch_outputs) else None
    y_max = poison(tdt) if (do_max and branch_outputs) else None
    idx_min = poison(torch.int32) if do_min else None
    idx_max = poison(torch.int32) if do_max else None
    wsz = tb.tconv_workspace_bytes(d, "forward")
    ws = torch.empty(max(wsz, 1), device=dev, dtype=torch.uint8) if wsz else None
    tb.tconv_forward(d, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max, ws)
    out = dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
    if backward:
        gx = torch.full((cfg.N, cfg.C_in, cfg.H, cfg.W), float("nan"), device=dev)
        wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
        gw_min = torch.full(wshape, float("nan"), device=dev) if do_min else None
        gw_max = torch.full(wshape, float("nan"), device=dev) if cfg.mode in ("max", "parallel", "maxplus_min") else None
        if fused == "recompute":
            # the forward pass above kept no branch outputs; the combine-coefficient gradients come from the winners
            assert y_min is None and y_max is None
            tb.tconv_backward_input(d, gy, alpha, beta, idx_min, idx_max, gx)
            ab = cfg.mode in ("compound", "parallel")
            ga = torch.full((cfg.C_out,), float("nan"), device=dev) if ab else None
            gb = torch.full((cfg.C_out,), float("nan"), device=dev) if ab else None
            gbias = torch.full((cfg.C_out,), float("nan"), device=dev)
            ws_p = scratch(tb.tconv_workspace_bytes(d, "backward_params"), dev)
            tb.tconv_backward_params_recompute(d, x, w_min, w_max, gy, alpha, beta, idx_min, idx_max, gw_min, gw_max,
                                               ga, gb, gbias, ws_p)
            out.update(grad_alpha=ga, grad_beta=gb, grad_bias=gbias)
        elif fused == "params":
            # grad_x by its own call, every parameter gradient (kernels, combine coefficients, bias) by the one-call form
            tb.tconv_backward_input(d, gy, alpha, beta, idx_min, idx_max, gx)
            ab = cfg.mode in ("compound", "parallel") and branch_outputs
            ga = torch.full((cfg.C_out,), float("nan"), device=dev) if ab else None
            gb = torch.full((cfg.C_out,), float("nan"), device=dev) if ab else None
            gbias = torch.full((cfg.C_out,), float("nan"), device=dev)
            ws_p = scratch(tb.tconv_workspace_bytes(d, "backward_params"), dev) if deterministic else None
            tb.tconv_backward_params(d, gy, alpha, beta, idx_min, idx_max, y_min, y_max, gw_min, gw_max, ga, gb, gbias,
                                     ws_p)
            out.update(grad_alpha=ga, grad_beta=gb, grad_bias=gbias)
        elif fused:
            ws_b = scratch(tb.tconv_workspace_bytes(d, "backward"), dev) if deterministic else None
            tb.tconv_backward(d, gy, alpha, beta, idx_min, idx_max, gx, gw_min, gw_max, ws_b)
        else:
            tb.tconv_backward_input(d, gy, alpha, beta, idx_min, idx_max, gx)
            ws_w = scratch(tb.tconv_workspace_bytes(d, "backward_weight"), dev) if deterministic else None
            tb.tconv_backward_weight(d, gy, alpha, beta, idx_min, idx_max, gw_min, gw_max, ws_w)
        out.update(grad_x=gx, grad_w_min=gw_min, grad_w_max=gw_max)
        if cfg.mode in ("compound", "parallel") and branch_outputs and fused not in ("params", "recompute"):
            ga = torch.full((cfg.C_out,), float("nan"), device=dev)
            gb = torch.full((cfg.C_out,), float("nan"), device=dev)
            ws_ab = scratch(tb.tconv_workspace_bytes(d, "backward_alpha_beta"), dev) if deterministic else None
            tb.tconv_backward_alpha_beta(d, gy, y_min, y_max, ga, gb, ws_ab)
            out.update(grad_alpha=ga, grad_beta=gb)
    torch.cuda.synchronize()
    res = {}
    for k, v in out.items():
        if v is None:
            res[k] = None
        elif v.dtype == torch.bfloat16:
            res[k] = v.float().cpu().numpy()
        else:
            res[k] = v.cpu().numpy()
    return res


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.int32)


def assert_forward_bit_exact(hip, ref, keys=("y", "y_min", "y_max", "idx_min", "idx_max"), what=""):
    for k in keys:
        if ref.get(k) is None:
            assert hip.get(k) is None or k in ("y_min", "y_max"), f"{what}{k}: HIP wrote a dead branch"
            continue
        if hip.get(k) is None:
            continue  # optional output not requested
        a, b = hip[k], ref[k]
        assert a.shape == b.shape, f"{what}{k}: shape {a.shape} vs {b.shape}"
        same = np.array_equal(a, b) if a.dtype == np.int32 else np.array_equal(bits(a), bits(b))
        if not same:
            bad = np.argwhere((a != b) | (np.isnan(a.astype(np.float64)) != np.isnan(b.astype(np.float64))))
            first = tuple(bad[0])
            raise AssertionError(f"{what}{k}: {len(bad)} of {a.size} elements differ; first at {first}: "
                                 f"hip={a[first]!r} oracle={b[first]!r}")


# worst observed |hip - oracle| / |oracle| over the elements with |oracle| >= 1, per gradient tensor name; the test
# session prints the largest of them at its end (tests/conftest.py)
WORST_REL = {}


def assert_grad_close(a, b, scale, name, rtol=GRAD_RTOL, strict=True):
    """Three gates: |a - b| <= rtol * max(1, sum of |summands|) per element; the same bound in the max norm of b;
    and (strict) |a - b| <= rtol * |b| on every element with |b| >= 1, the plain relative tolerance.  The strict gate
    is left out only for sums combined with fp32 atomics across workgroups, where an element can be a small rest of
    large partial sums."""
    assert a.shape == b.shape, f"{name}: shape {a.shape} vs {b.shape}"
    assert np.isfinite(a).all(), f"{name}: non-finite values (output not overwritten?)"
    b = np.asarray(b, np.float64)
    err = np.abs(a.astype(np.float64) - b)
    bound = rtol * np.maximum(1.0, scale)
    if not (err <= bound).all():
        i = tuple(np.argwhere(err > bound)[0])
        raise AssertionError(f"{name}: element {i} hip={a[i]!r} oracle={b[i]!r} |err|={err[i]:.3e} "
                             f"> {bound[i]:.3e}")
    assert err.max() <= rtol * max(1.0, np.abs(b).max()), f"{name}: max-norm error {err.max():.3e}"
    big = np.abs(b) >= 1.0
    if big.any():
        rel = err[big] / np.abs(b[big])
        worst = float(rel.max())
        key = name.split("] ")[-1]
        WORST_REL[key] = max(WORST_REL.get(key, 0.0), worst)
        if strict:
            assert worst <= rtol, f"{name}: relative error {worst:.3e} on an element with |oracle| >= 1"


def assert_backward_close(hip, ref, what="", strict_params=True):
    """strict_params=False: the parameter gradients came from the atomic forms (fp32 atomics across workgroups), which
    the plain relative gate does not bind."""
    assert_grad_close(hip["grad_x"], ref["grad_x"], ref["grad_x_scale"], what + "grad_x")
    for k in ("grad_w_min", "grad_w_max"):
        if ref[k] is None:
            continue
        assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k, strict=strict_params)
    for k in ("grad_alpha", "grad_beta"):
        if ref.get(k) is not None and hip.get(k) is not None:
            assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k, strict=strict_params)


# ---------------------------------------------------------------- Sum-channel layers

def sum_coefficients(cfg, inp, kind):
    """alpha, beta [C_in, C_out] for the Sum-channel layers, drawn after everything make_inputs drew."""
    if kind is None or cfg.mode in ("max", "min"):
        return None, None
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 1000))
    shape = (cfg.C_in, cfg.C_out)
    if kind == "integer":
        return rng.integers(-2, 3, shape).astype(np.float32), rng.integers(-2, 3, shape).astype(np.float32)
    if kind == "one_parameter":   # beta = 1 - alpha (the one-parameter layers)
        a = rng.uniform(0, 1, shape).astype(np.float32)
        return a, (np.float32(1) - a).astype(np.float32)
    return rng.uniform(-1, 1, shape).astype(np.float32), rng.uniform(-1, 1, shape).astype(np.float32)


def run_oracle_sum(cfg, inp, alpha, beta, backward=True):
    from oracle import tsum_oracle as osum
    s = oracle_shape(cfg)
    r = {"y": osum.forward(s, cfg.mode, inp["x"], inp["w_min"], inp["w_max"], alpha, beta)}
    if cfg.dtype == "bf16":   # storage rounding of the output, as the library stores it (torch's cast)
        import torch
        r["y"] = torch.from_numpy(r["y"]).to(torch.bfloat16).float().numpy()
    if backward:
        r.update(osum.backward(s, cfg.mode, inp["x"], inp["gy"], inp["w_min"], inp["w_max"], alpha, beta))
        ab = [None if v is None else np.abs(v) for v in (alpha, beta)]
        sc = osum.backward(s, cfg.mode, inp["x"], np.abs(inp["gy"]), inp["w_min"], inp["w_max"], ab[0], ab[1])
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
        if r["grad_alpha"] is not None:
            # sum of |gy * m| is at most sum|gy| * (max|x| + max|w|)
            wmax = max(np.abs(v).max() for v in (inp["w_min"], inp["w_max"]) if v is not None)
            bound = np.abs(inp["gy"]).astype(np.float64).sum(axis=(0, 2, 3)) * float(np.abs(inp["x"]).max() + wmax)
            r["grad_alpha_scale"] = r["grad_beta_scale"] = np.broadcast_to(bound[None, :], r["grad_alpha"].shape)
    return r


def run_hip_sum(cfg, inp, alpha, beta, backward=True, device="cuda:0"):
    import torch
    dev = torch.device(device)
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)

    def up(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32   # storage of x, the kernels and y

    def ups(a):
        return None if a is None else up(a).to(tdt)

    def ws(backward_):
        n = tb.tconv_sum_workspace_bytes(d, backward_)
        return torch.empty(n, dtype=torch.uint8, device=dev) if n else None

    x, gy, al, be = ups(inp["x"]), up(inp["gy"]), up(alpha), up(beta)
    if cfg.mode == "compound":
        w_min = w_max = ups(inp["w_min"])
    else:
        w_min, w_max = ups(inp["w_min"]), ups(inp["w_max"])
    y = torch.full((cfg.N, cfg.C_out, ho, wo), float("nan"), device=dev, dtype=tdt)
    tb.tconv_sum_forward(d, x, w_min, w_max, al, be, y, ws(False))
    out = dict(y=y.float())
    if backward:
        two = cfg.mode in ("compound", "parallel")
        nan = lambda shape: torch.full(shape, float("nan"), device=dev)
        wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
        gx = nan((cfg.N, cfg.C_in, cfg.H, cfg.W))
        g1 = nan(wshape) if cfg.mode != "max" else None
        g2 = nan(wshape) if cfg.mode in ("max", "parallel") else None
        ga = nan((cfg.C_in, cfg.C_out)) if two else None
        gb = nan((cfg.C_in, cfg.C_out)) if two else None
        tb.tconv_sum_backward(d, x, w_min, w_max, al, be, gy, gx, g1, g2, ga, gb, ws(True))
        out.update(grad_x=gx, grad_w_min=g1, grad_w_max=g2, grad_alpha=ga, grad_beta=gb)
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}


def assert_sum_close(hip, ref, what=""):
    for k in ("grad_x", "grad_w_min", "grad_w_max", "grad_alpha", "grad_beta"):
        if ref.get(k) is None:
            continue
        # the parameter gradients of these layers are combined with fp32 atomics across workgroups
        assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k, strict=(k == "grad_x"))


# ---------------------------------------------------------------- depthwise layers

def run_oracle_dw(cfg, inp, backward=True):
    from oracle import tdw_oracle as odw
    s = oracle_shape(cfg)
    a, b = inp["alpha"], inp["beta"]
    y, tmin, tmax = odw.forward(s, cfg.mode, inp["x"], inp["w_min"], inp["w_max"], a, b, taps=True)
    r = dict(y=y, tap_min=tmin, tap_max=tmax)
    if backward:
        r.update(odw.backward(s, cfg.mode, inp["x"], inp["gy"], inp["w_min"], inp["w_max"], a, b))
        ab = [None if v is None else np.abs(v) for v in (a, b)]
        sc = odw.backward(s, cfg.mode, inp["x"], np.abs(inp["gy"]), inp["w_min"], inp["w_max"], ab[0], ab[1])
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
        if r["grad_alpha"] is not None:
            wmax = max(np.abs(v).max() for v in (inp["w_min"], inp["w_max"]) if v is not None)
            bound = np.abs(inp["gy"]).astype(np.float64).sum(axis=(0, 2, 3)) * float(np.abs(inp["x"]).max() + wmax)
            r["grad_alpha_scale"] = r["grad_beta_scale"] = bound
    return r


def run_hip_dw(cfg, inp, backward=True, save_idx=True, device="cuda:0"):
    import torch
    dev = torch.device(device)
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)

    def up(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    x, gy, al, be = up(inp["x"]), up(inp["gy"]), up(inp["alpha"]), up(inp["beta"])
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"])
    else:
        w_min, w_max = up(inp["w_min"]), up(inp["w_max"])
    oshape = (cfg.N, cfg.C_out, ho, wo)
    y = torch.full(oshape, float("nan"), device=dev)
    idx = torch.full(oshape, 0xEE, device=dev, dtype=torch.uint8) if save_idx else None
    tb.tconv_depthwise_forward(d, x, w_min, w_max, al, be, y, idx)
    out = dict(y=y, idx=idx)
    if backward:
        two = cfg.mode in ("compound", "parallel")
        nan = lambda shape: torch.full(shape, float("nan"), device=dev)
        wshape = (cfg.C_out, 1, cfg.KH, cfg.KW)
        gx = nan((cfg.N, cfg.C_in, cfg.H, cfg.W))
        g1 = nan(wshape) if cfg.mode != "max" else None
        g2 = nan(wshape) if cfg.mode in ("max", "parallel") else None
        ga = nan((cfg.C_out,)) if two else None
        gb = nan((cfg.C_out,)) if two else None
        tb.tconv_depthwise_backward(d, x, w_min, w_max, al, be, gy, idx, gx, g1, g2, ga, gb)
        out.update(grad_x=gx, grad_w_min=g1, grad_w_max=g2, grad_alpha=ga, grad_beta=gb)
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}


def assert_dw_close(hip, ref, mode, what="", backward=True):
    assert_forward_bit_exact(hip, ref, keys=("y",), what=what)
    if hip.get("idx") is not None:   # both winners in one byte: low nibble min-plus tap, high nibble max-plus tap
        if mode != "max":
            assert np.array_equal(hip["idx"] & 15, ref["tap_min"]), what + "min-plus winners"
        if mode != "min":
            assert np.array_equal(hip["idx"] >> 4, ref["tap_max"]), what + "max-plus winners"
    if backward:
        for k in ("grad_x", "grad_w_min", "grad_w_max", "grad_alpha", "grad_beta"):
            if ref.get(k) is None:
                continue
            # the parameter gradients of these layers are combined with fp32 atomics across workgroups
            assert_grad_close(hip[k], ref[k], ref[k + "_scale"], what + k, strict=(k == "grad_x"))


# ---------------------------------------------------------------- one-dimensional layers

def run_oracle_1d(cfg, inp, backward=True):
    from oracle import tconv1d_oracle as o1
    s = o1.Shape1d(cfg.N, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil)
    r = o1.forward(s, cfg.mode, inp["x"], inp["w_min"], inp["w_max"], inp["alpha"], inp["beta"])
    if cfg.dtype == "bf16":   # storage rounding of the outputs, as the library stores them
        import torch
        for k in ("y", "y_min", "y_max"):
            if r[k] is not None:
                r[k] = torch.from_numpy(r[k]).to(torch.bfloat16).float().numpy()
    if backward:
        kw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"])
        r.update(o1.backward(s, cfg.mode, inp["gy"], alpha=inp["alpha"], beta=inp["beta"], **kw))
        ab = {k: (None if inp[k] is None else np.abs(inp[k])) for k in ("alpha", "beta")}
        sc = o1.backward(s, cfg.mode, np.abs(inp["gy"]), alpha=ab["alpha"], beta=ab["beta"], **kw)
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
    return r


def run_hip_1d(cfg, inp, backward=True, device="cuda:0"):
    import torch
    dev = torch.device(device)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    d = tb.Desc1d(cfg.N, cfg.C_in, cfg.L, cfg.C_out, cfg.K, cfg.stride, cfg.pad, cfg.dil, cfg.mode, cfg.dtype)
    lo = tb.tconv1d_out_len(d)
    assert lo == cfg.L_out

    def up(a, dt=torch.float32):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()

    x = up(inp["x"], tdt)
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"], tdt)
    else:
        w_min, w_max = up(inp["w_min"], tdt), up(inp["w_max"], tdt)
    alpha, beta, gy = up(inp["alpha"]), up(inp["beta"]), up(inp["gy"])
    oshape = (cfg.N, cfg.C_out, lo)
    do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")
    nanf = lambda: torch.full(oshape, float("nan"), device=dev, dtype=tdt)
    bad = lambda: torch.full(oshape, -12345, device=dev, dtype=torch.int32)
    y, y_min, y_max = nanf(), (nanf() if do_min else None), (nanf() if do_max else None)
    idx_min, idx_max = (bad() if do_min else None), (bad() if do_max else None)
    wsz = tb.tconv1d_workspace_bytes(d, "forward")
    ws = torch.empty(max(wsz, 1), device=dev, dtype=torch.uint8) if wsz else None
    tb.tconv1d_forward(d, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max, ws)
    out = dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
    if backward:
        gx = torch.full((cfg.N, cfg.C_in, cfg.L), float("nan"), device=dev)
        tb.tconv1d_backward_input(d, gy, alpha, beta, idx_min, idx_max, gx)
        wshape = (cfg.C_out, cfg.C_in, cfg.K)
        gw_min = torch.full(wshape, float("nan"), device=dev) if do_min else None
        gw_max = torch.full(wshape, float("nan"), device=dev) if (do_max and cfg.mode != "compound") else None
        tb.tconv1d_backward_weight(d, gy, alpha, beta, idx_min, idx_max, gw_min, gw_max,
                                   scratch(tb.tconv1d_workspace_bytes(d, "backward_weight"), dev))
        out.update(grad_x=gx, grad_w_min=gw_min, grad_w_max=gw_max)
    torch.cuda.synchronize()
    return {k: (None if v is None else (v.float() if v.dtype == torch.bfloat16 else v).cpu().numpy())
            for k, v in out.items()}


# ---------------------------------------------------------------- three-dimensional layers

def run_oracle_3d(cfg, inp, backward=True):
    from oracle import tconv3d_oracle as o3
    s = o3.Shape3d(cfg.N, cfg.C_in, cfg.D, cfg.H, cfg.W, cfg.C_out, cfg.k[0], cfg.k[1], cfg.k[2], tuple(cfg.stride),
                   tuple(cfg.pad), tuple(cfg.dil))
    r = o3.forward(s, cfg.mode, inp["x"], inp["w_min"], inp["w_max"], inp["alpha"], inp["beta"])
    if backward:
        kw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"])
        r.update(o3.backward(s, cfg.mode, inp["gy"], alpha=inp["alpha"], beta=inp["beta"], **kw))
        ab = {k: (None if inp[k] is None else np.abs(inp[k])) for k in ("alpha", "beta")}
        sc = o3.backward(s, cfg.mode, np.abs(inp["gy"]), alpha=ab["alpha"], beta=ab["beta"], **kw)
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
    return r


def run_hip_3d(cfg, inp, backward=True, device="cuda:0"):
    import torch
    dev = torch.device(device)
    d = tb.Desc3d(cfg.N, cfg.C_in, cfg.D, cfg.H, cfg.W, cfg.C_out, cfg.k[0], cfg.k[1], cfg.k[2], tuple(cfg.stride),
                  tuple(cfg.pad), tuple(cfg.dil), cfg.mode)
    out3 = tb.tconv3d_out_shape(d)
    assert out3 == cfg.out
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)
    x, gy, alpha, beta = up(inp["x"]), up(inp["gy"]), up(inp["alpha"]), up(inp["beta"])
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"])
    else:
        w_min, w_max = up(inp["w_min"]), up(inp["w_max"])
    oshape = (cfg.N, cfg.C_out) + out3
    do_min, do_max = cfg.mode not in ("max", "maxplus_min"), cfg.mode not in ("min", "minplus_max")
    nanf = lambda: torch.full(oshape, float("nan"), device=dev)
    bad = lambda: torch.full(oshape, -12345, device=dev, dtype=torch.int32)
    y, y_min, y_max = nanf(), (nanf() if do_min else None), (nanf() if do_max else None)
    idx_min, idx_max = (bad() if do_min else None), (bad() if do_max else None)
    tb.tconv3d_forward(d, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max)
    out = dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
    if backward:
        gx = torch.full(tuple(inp["x"].shape), float("nan"), device=dev)
        tb.tconv3d_backward_input(d, gy, alpha, beta, idx_min, idx_max, gx)
        wshape = (cfg.C_out, cfg.C_in) + tuple(cfg.k)
        gw_min = torch.full(wshape, float("nan"), device=dev) if do_min else None
        gw_max = torch.full(wshape, float("nan"), device=dev) if (do_max and cfg.mode != "compound") else None
        tb.tconv3d_backward_weight(d, gy, alpha, beta, idx_min, idx_max, gw_min, gw_max,
                                   scratch(tb.tconv3d_workspace_bytes(d, "backward_weight"), dev))
        out.update(grad_x=gx, grad_w_min=gw_min, grad_w_max=gw_max)
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}


# ---------------------------------------------------------------- zero padding and the fused epilogue

def draw_epilogue(cfg, kind, seed=0):
    """bias / scale / shift [C_out] and residual [N, C_out, Ho, Wo] (fp32 host arrays; residual on the bf16 grid for
    bf16 storage).  kind: a string of the letters b (bias), a (affine scale + shift), s (scale only), r (residual)."""
    from paper_2504_06881_amd.inputs import to_bf16_grid
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 7000 + seed))
    ho, wo = cfg.out_hw
    ep = dict(bias=None, scale=None, shift=None, residual=None)
    if "b" in kind:
        ep["bias"] = rng.standard_normal(cfg.C_out).astype(np.float32)
    if "a" in kind or "s" in kind:
        ep["scale"] = rng.uniform(0.5, 2.0, cfg.C_out).astype(np.float32)
    if "a" in kind:
        ep["shift"] = rng.standard_normal(cfg.C_out).astype(np.float32)
    if "r" in kind:
        r = rng.standard_normal((cfg.N, cfg.C_out, ho, wo)).astype(np.float32)
        ep["residual"] = to_bf16_grid(r) if cfg.dtype == "bf16" else r
    return ep


def run_oracle_ext(cfg, inp, ep=None, backward=True):
    """The extension oracle: the layer's padding mode, the epilogue, and the backward pass through winners that may lie
    in the padding.  bf16 storage: outputs rounded to the bf16 grid, as the library stores them."""
    from oracle import text_oracle as ext
    from paper_2504_06881_amd.inputs import to_bf16_grid
    s = ext.Shape(cfg.N, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil)
    ep = ep or {}
    r = ext.forward(s, cfg.mode, inp["x"], inp["w_min"], inp["w_max"], inp["alpha"], inp["beta"],
                    pad_zero=(cfg.pad_mode == "zero"), bias=ep.get("bias"), scale=ep.get("scale"),
                    shift=ep.get("shift"), residual=ep.get("residual"))
    if cfg.dtype == "bf16":
        for k in ("y", "y_min", "y_max"):
            if r[k] is not None:
                r[k] = to_bf16_grid(r[k])
    if backward:
        kw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"])
        r.update(ext.backward(s, cfg.mode, inp["gy"], alpha=inp["alpha"], beta=inp["beta"], **kw))
        ab = {k: (None if inp[k] is None else np.abs(inp[k])) for k in ("alpha", "beta")}
        sc = ext.backward(s, cfg.mode, np.abs(inp["gy"]), alpha=ab["alpha"], beta=ab["beta"], **kw)
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
        r["grad_bias"] = ext.backward_bias(s, inp["gy"])
        r["grad_bias_scale"] = ext.backward_bias(s, np.abs(inp["gy"]))
    return r


def run_hip_ext(cfg, inp, ep=None, backward=True, device="cuda:0"):
    """tconv_forward_fused (+ tconv_backward and tconv_backward_bias) through the C ABI."""
    import torch
    dev = torch.device(device)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    d = tb.Desc.from_cfg(cfg)
    ho, wo = tb.tconv_out_shape(d)
    ep = ep or {}

    def up(a, dt=torch.float32):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()

    x = up(inp["x"], tdt)
    if cfg.mode == "compound":
        w_min = w_max = up(inp["w_min"], tdt)
    else:
        w_min, w_max = up(inp["w_min"], tdt), up(inp["w_max"], tdt)
    alpha, beta, gy = up(inp["alpha"]), up(inp["beta"]), up(inp["gy"])
    oshape = (cfg.N, cfg.C_out, ho, wo)
    do_min, do_max = cfg.mode != "max", cfg.mode != "min"
    nanf = lambda: torch.full(oshape, float("nan"), device=dev, dtype=tdt)
    bad = lambda: torch.full(oshape, -12345, device=dev, dtype=torch.int32)
    y, y_min, y_max = nanf(), (nanf() if do_min else None), (nanf() if do_max else None)
    idx_min, idx_max = (bad() if do_min else None), (bad() if do_max else None)
    ws = scratch(tb.tconv_workspace_bytes(d, "forward"), dev)
    tb.tconv_forward_fused(d, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max,
                           bias=up(ep.get("bias")), scale=up(ep.get("scale")), shift=up(ep.get("shift")),
                           residual=up(ep.get("residual"), tdt), workspace=ws)
    out = dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
    if backward:
        gx = torch.full((cfg.N, cfg.C_in, cfg.H, cfg.W), float("nan"), device=dev)
        wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
        gw_min = torch.full(wshape, float("nan"), device=dev) if do_min else None
        gw_max = torch.full(wshape, float("nan"), device=dev) if cfg.mode in ("max", "parallel") else None
        tb.tconv_backward(d, gy, alpha, beta, idx_min, idx_max, gx, gw_min, gw_max,
                          scratch(tb.tconv_workspace_bytes(d, "backward"), dev))
        gb = torch.full((cfg.C_out,), float("nan"), device=dev)
        tb.tconv_backward_bias(d, gy, gb, scratch(tb.tconv_workspace_bytes(d, "backward_bias"), dev))
        out.update(grad_x=gx, grad_w_min=gw_min, grad_w_max=gw_max, grad_bias=gb)
    torch.cuda.synchronize()
    return {k: (None if v is None else (v.float() if v.dtype == torch.bfloat16 else v).cpu().numpy())
            for k, v in out.items()}


# ---------------------------------------------------------------- binary16 arithmetic (dtype f16)

def run_oracle_f16(cfg, inp, backward=True):
    """The half-precision contract of the extension oracle on inputs rounded to binary16; the backward pass is the
    fp32-gradient routing of the main oracle (or of the extension oracle under zero padding) on its winners."""
    from oracle import text_oracle as ext
    s = ext.Shape(cfg.N, cfg.C_in, cfg.H, cfg.W, cfg.C_out, cfg.KH, cfg.KW, cfg.stride, cfg.pad, cfg.dil)
    h = lambda a: None if a is None else np.asarray(a, np.float32).astype(np.float16)
    r = ext.forward_f16(s, cfg.mode, h(inp["x"]), h(inp["w_min"]), h(inp["w_max"]), inp["alpha"], inp["beta"],
                        pad_zero=(cfg.pad_mode == "zero"))
    for k in ("y", "y_min", "y_max"):
        if r[k] is not None:
            r[k] = r[k].astype(np.float32)
    if backward:
        kw = dict(idx_min=r["idx_min"], idx_max=r["idx_max"])
        r.update(ext.backward(s, cfg.mode, inp["gy"], alpha=inp["alpha"], beta=inp["beta"], **kw))
        ab = {k: (None if inp[k] is None else np.abs(inp[k])) for k in ("alpha", "beta")}
        sc = ext.backward(s, cfg.mode, np.abs(inp["gy"]), alpha=ab["alpha"], beta=ab["beta"], **kw)
        for k in ("grad_x", "grad_w_min", "grad_w_max"):
            r[k + "_scale"] = sc[k]
    return r


def run_hip_f16(cfg, inp, backward=True, device="cuda:0"):
    import torch
    dev = torch.device(device)
    d = tb.Desc.from_cfg(cfg, dtype="f16")
    ho, wo = tb.tconv_out_shape(d)
    up16 = lambda a: None if a is None else torch.from_numpy(np.asarray(a, np.float32).astype(np.float16)).to(dev)
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)
    x = up16(inp["x"])
    if cfg.mode == "compound":
        w_min = w_max = up16(inp["w_min"])
    else:
        w_min, w_max = up16(inp["w_min"]), up16(inp["w_max"])
    alpha, beta, gy = up(inp["alpha"]), up(inp["beta"]), up(inp["gy"])
    oshape = (cfg.N, cfg.C_out, ho, wo)
    do_min, do_max = cfg.mode != "max", cfg.mode != "min"
    nanf = lambda: torch.full(oshape, float("nan"), device=dev, dtype=torch.float16)
    bad = lambda: torch.full(oshape, -12345, device=dev, dtype=torch.int32)
    y, y_min, y_max = nanf(), (nanf() if do_min else None), (nanf() if do_max else None)
    idx_min, idx_max = (bad() if do_min else None), (bad() if do_max else None)
    ws = scratch(tb.tconv_workspace_bytes(d, "forward"), dev)
    tb.tconv_forward(d, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max, ws)
    out = dict(y=y, y_min=y_min, y_max=y_max, idx_min=idx_min, idx_max=idx_max)
    if backward:
        gx = torch.full((cfg.N, cfg.C_in, cfg.H, cfg.W), float("nan"), device=dev)
        wshape = (cfg.C_out, cfg.C_in, cfg.KH, cfg.KW)
        gw_min = torch.full(wshape, float("nan"), device=dev) if do_min else None
        gw_max = torch.full(wshape, float("nan"), device=dev) if cfg.mode in ("max", "parallel") else None
        tb.tconv_backward(d, gy, alpha, beta, idx_min, idx_max, gx, gw_min, gw_max,
                          scratch(tb.tconv_workspace_bytes(d, "backward"), dev))
        out.update(grad_x=gx, grad_w_min=gw_min, grad_w_max=gw_max)
    torch.cuda.synchronize()
    return {k: (None if v is None else (v.float() if v.dtype == torch.float16 else v).cpu().numpy())
            for k, v in out.items()}
